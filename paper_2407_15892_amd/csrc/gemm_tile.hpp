// Block-tile bf16 GEMM main loop for gfx950 (MI355X), shared by the four
// contractions of the mini-sequence LM-head path (Algorithm 2 line 4 and
// Algorithm 4 lines 5, 7, 8 of the paper).
//
// One workgroup of 512 threads (8 wave64s, two per SIMD) owns a 256 x 256
// output tile.  Operand panels of 256 x 64 bf16 are brought from global memory
// straight into LDS (buffer loads with the LDS bit, 16 bytes per lane, no
// register staging), double buffered, and consumed by v_mfma_f32_32x32x16_bf16.
// The wave grid is 2 (A side) x 4 (B side): a wave accumulates 128 x 64, i.e.
// 4 x 2 MFMA tiles = 128 fp32 accumulator registers per lane.
//
// "A side" is the index that ends up spread over a lane's 16 accumulator
// registers, "B side" the index that ends up across the 32 lanes of a half
// wave.  Either operand may be stored K-contiguous (layout KC: X[index][k]) or
// K-strided (layout KS: X[k][index]).  KC panels are read from LDS with
// ds_read_b128; KS panels with the transposing ds_read_b64_tr_b16, so no
// operand is ever transposed in memory.
//
// Buffer resources give hardware range checking: a lane whose address lies
// beyond the matrix reads zeros instead of faulting, which is how ragged tile
// edges are handled without branches.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mst {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTile = 256;                   // block tile extent on both sides
constexpr int kBK = 64;                      // K step per LDS stage
constexpr int kThreads = 512;
constexpr int kPanelBytes = kTile * kBK * 2; // 32 KiB per operand per stage
constexpr int kStageBytes = 2 * kPanelBytes; // A panel then B panel
constexpr int kLdsBytes = 2 * kStageBytes;   // double buffered: 128 KiB
constexpr int kTA = 4;                       // MFMA tiles per wave, A side (128 rows)
constexpr int kTB = 2;                       // MFMA tiles per wave, B side (64 cols)
constexpr uint32_t kOutOfRange = 0xFFFFFF00u;  // byte offset beyond any buffer we describe

// raw buffer resource: base address, no stride, byte count, 32-bit data format
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// 16 bytes per lane from global memory into LDS at (m0 base + lane * 16).
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(voffset), "s"(rsrc) : "memory");
}

__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}

// Which index of a 32-wide MFMA tile the A-side row `i` (0..31) stands for.
// With `permute`, a lane's 16 accumulator registers cover 16 consecutive
// indices (16*(lane/32) + r) instead of the native 8*(r/4) + 4*(lane/32) + r%4,
// so that an epilogue can store 16 consecutive outputs per lane.
template <bool kPermute>
__device__ __forceinline__ int a_row_of_mfma_row(int i) {
  if (!kPermute) return i;
  return 16 * ((i >> 2) & 1) + 4 * (i >> 3) + (i & 3);
}
template <bool kPermute>
__device__ __forceinline__ int a_index_in_tile(int r, int lane) {   // accumulator register r -> A index within the 32-tile
  if (kPermute) return 16 * (lane >> 5) + r;
  return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
}

// ---------------------------------------------------------------------------
// K-contiguous operand: X[index][k], row stride ld elements.  LDS panel is
// [256 rows][64 k] with the eight 16-byte chunks of a row XOR-swizzled by
// (row % 8), which makes the b128 fragment reads bank-conflict free.
// ---------------------------------------------------------------------------
template <int kTilesPerWave, bool kPermute>
struct PanelKC {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t voff[4];   // this lane's global byte offset for k0 = 0, per issue slot
  uint32_t kelem;     // k element index of this lane's chunk within the stage
  uint32_t k_limit;   // number of valid k elements
  uint32_t slot0;     // wave-uniform: first 1 KiB slot of this wave in the panel
  uint32_t rd[4];     // fragment byte offsets within the panel, per k sub-step, tile 0

  // base: first row of the block's tile, k = 0.  rows_valid: rows of the matrix from there on.
  __device__ __forceinline__ void init(const void* base, uint32_t ld_elems, uint32_t rows_valid,
                                       uint32_t k_elems, int wave, int lane, int wave_side_index) {
    const uint32_t ld_bytes = ld_elems * 2;
    const uint32_t rows = rows_valid < (uint32_t)kTile ? rows_valid : (uint32_t)kTile;
    rsrc = make_rsrc(base, rows * ld_bytes);
    k_limit = k_elems;
    slot0 = wave * 4;
    const int chunk = (lane & 7) ^ (lane >> 3);
    kelem = chunk * 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t row = 8 * (slot0 + i) + (lane >> 3);
      voff[i] = row * ld_bytes + chunk * 16;
    }
    const int row0 = wave_side_index * (32 * kTilesPerWave) + a_row_of_mfma_row<kPermute>(lane & 31);
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) rd[kk] = row0 * 128 + (((2 * kk + (lane >> 5)) ^ (row0 & 7)) * 16);
  }
  __device__ __forceinline__ void issue(uint32_t panel_lds, uint32_t k0) const {
    const bool ok = (k0 + kelem) < k_limit;
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16(rsrc, ok ? voff[i] + k0 * 2 : kOutOfRange, panel_lds + (slot0 + i) * 1024);
  }
  __device__ __forceinline__ bf16x8 frag(const char* panel, int t, int kk) const {
    return *reinterpret_cast<const bf16x8*>(panel + rd[kk] + t * 4096);
  }
};

// ---------------------------------------------------------------------------
// K-strided operand: X[k][index], row stride ld elements.  LDS panel is
// [64 k][256 index]; the 16-byte chunks of row k are XOR-swizzled by
// 2 * (k % 4) so that the four k rows a transposing read touches fall into
// four different 32-byte bank groups.
// ---------------------------------------------------------------------------
template <int kTilesPerWave>
struct PanelKS {
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t voff[4];   // this lane's global byte offset for k0 = 0, per issue slot
  uint32_t ok_mask;   // bit i: the chunk of issue slot i lies inside the matrix' columns
  uint32_t ld_bytes;
  uint32_t slot0;
  uint32_t rd[kTilesPerWave];

  // base: &X[0][col0].  k_rows: rows of X.  cols_valid: columns of X from col0 on
  // (columns at or beyond it read as zero).
  __device__ __forceinline__ void init(const void* base, uint32_t ld_elems, uint32_t k_rows,
                                       uint32_t cols_valid, int wave, int lane, int wave_side_index) {
    ld_bytes = ld_elems * 2;
    const uint32_t last_cols = cols_valid < ld_elems ? cols_valid : ld_elems;
    rsrc = make_rsrc(base, (k_rows - 1) * ld_bytes + last_cols * 2);
    slot0 = wave * 4;
    ok_mask = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t krow = 2 * (slot0 + i) + (lane >> 5);
      const uint32_t chunk = (lane & 31) ^ (2 * (krow & 3));
      voff[i] = krow * ld_bytes + chunk * 16;
      ok_mask |= ((chunk * 8) < cols_valid ? 1u : 0u) << i;
    }
    const int g = lane >> 4, i16 = lane & 15;
#pragma unroll
    for (int t = 0; t < kTilesPerWave; ++t) {
      const int col = wave_side_index * (32 * kTilesPerWave) + 32 * t + 16 * (g & 1) + 4 * (i16 & 3);
      const int krow = 8 * (g >> 1) + (i16 >> 2);
      rd[t] = krow * 512 + (((col >> 3) ^ (2 * (i16 >> 2))) * 16) + (col & 7) * 2;
    }
  }
  __device__ __forceinline__ void issue(uint32_t panel_lds, uint32_t k0) const {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      dma16(rsrc, ((ok_mask >> i) & 1u) ? voff[i] + k0 * ld_bytes : kOutOfRange, panel_lds + (slot0 + i) * 1024);
  }
  // lane l receives index (l % 32) of tile t and k = 16 kk + 8 (l / 32) + 0..7, the MFMA operand layout
  __device__ __forceinline__ bf16x8 frag(const char* panel, int t, int kk) const {
    typedef __attribute__((address_space(3))) i16x4* lds_i16x4_ptr;
    const char* p = panel + rd[t] + kk * (16 * 512);
    i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(p));
    i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(p + 4 * 512));
    i16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
};

// ---------------------------------------------------------------------------
// Main loop: acc[t][u] += A-panel tile t  x  B-panel tile u over K.
// ---------------------------------------------------------------------------
template <class PanelA, class PanelB>
__device__ __forceinline__ void gemm_mainloop(f32x16 (&acc)[kTA][kTB], const PanelA& pa, const PanelB& pb,
                                              char* smem, int k_begin, int k_end) {
  const uint32_t lds0 = lds_addr_of(smem);
  const int nk = (k_end - k_begin + kBK - 1) / kBK;
  if (nk <= 0) return;
  pa.issue(lds0, k_begin);
  pb.issue(lds0 + kPanelBytes, k_begin);
  wait_all_loads();
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = (kt & 1) * kStageBytes;
    if (kt + 1 < nk) {
      const int nxt = kStageBytes - cur;
      pa.issue(lds0 + nxt, k_begin + (kt + 1) * kBK);
      pb.issue(lds0 + nxt + kPanelBytes, k_begin + (kt + 1) * kBK);
    }
    const char* a_panel = smem + cur;
    const char* b_panel = smem + cur + kPanelBytes;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      bf16x8 a[kTA], b[kTB];
#pragma unroll
      for (int t = 0; t < kTA; ++t) a[t] = pa.frag(a_panel, t, kk);
#pragma unroll
      for (int u = 0; u < kTB; ++u) b[u] = pb.frag(b_panel, u, kk);
#pragma unroll
      for (int t = 0; t < kTA; ++t)
#pragma unroll
        for (int u = 0; u < kTB; ++u)
          acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[t], b[u], acc[t][u], 0, 0, 0);
    }
    wait_all_loads();
    __syncthreads();
  }
}

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[kTA][kTB]) {
#pragma unroll
  for (int t = 0; t < kTA; ++t)
#pragma unroll
    for (int u = 0; u < kTB; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][u][r] = 0.f;
}

}  // namespace mst
