// Tile configuration and operand panels of the block-tile main loop (gemm_tile.hpp) for
// v_mfma_f32_16x16x32_bf16 tiles.
//
// On random operands a register-resident loop of the 16 x 16 x 32 instruction sustains about 15 % more flop
// per second than the 32 x 32 x 16 one on this power-limited chip, and inside the GEMMs of this library the
// difference was 4-6 % when both were built; every kernel uses 16 x 16 x 32.  Block tile 256 x 256, wave grid
// 2 x 4, wave tile 128 x 64; fragment and accumulator layout:
//
//   A fragment  lane l holds row (l % 16) of a 16-row tile, k = 8 * (l / 16) .. + 7 of a 32-wide k sub-step
//   B fragment  lane l holds column (l % 16), same k
//   accumulator register r of lane l is D[4 * (l / 16) + r][l % 16]               (4 registers per tile)
//
// so a wave tile is 8 x 4 MFMA tiles (128 accumulator registers), a K step of 64 is two k sub-steps, and a
// lane quarter g = l / 16 owns accumulator rows 4g..4g+3 of every tile.  With the A-side permutation (LDS row
// 16 t + 4 g + r of a 128-row block holds source row 32 g + 4 t + r) the 8 tiles x 4 registers of a lane
// cover 32 consecutive A indices: 64-byte bf16 stores per lane.
#pragma once
#include "gemm_tile.hpp"

namespace mst {

typedef __attribute__((ext_vector_type(4))) float f32x4;

template <int WA_, int WB_, int TA_, int TB_, int BK_, int NS_>
struct Cfg16 {
  static constexpr int WA = WA_, WB = WB_, TA = TA_, TB = TB_, BK = BK_, NS = NS_;
  static constexpr int kWaves = WA * WB, kThreads = 64 * kWaves;
  static constexpr int EA = 16 * TA * WA, EB = 16 * TB * WB;
  static constexpr int kPanelA = EA * BK * 2, kPanelB = EB * BK * 2;
  static constexpr int NSA = NS + 1, NSB = NS;
  static constexpr int kLds = NSA * kPanelA + NSB * kPanelB;
  static constexpr int kKK = BK / 32;            // MFMA k sub-steps per stage
  typedef f32x4 Acc;                             // accumulator of one 16 x 16 MFMA tile
  __device__ __forceinline__ static Acc mma(bf16x8 a, bf16x8 b, Acc c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};

// source row (within a block of 128 A rows) held by LDS / MFMA row m = 16 t + 4 g + r of the block
template <bool kPermute> __device__ __forceinline__ int a_row_of_block_row16(int m) {
  if (!kPermute) return m;
  return 32 * ((m >> 2) & 3) + 4 * (m >> 4) + (m & 3);
}
// K-contiguous panel [EXT rows][BK k]; LDS row = MFMA row order (a permutation, if any, is applied at the source)
template <class C, int EXT, int TILES, bool kPermute>
struct PanelKC16 {
  static constexpr int BK = C::BK;
  static constexpr int RB = BK * 2;
  static constexpr int CPR = BK / 8;
  static constexpr int RPS = 1024 / RB;
  static constexpr int NSLOT = EXT / RPS;
  static constexpr int SPW = NSLOT / C::kWaves;
  static_assert(NSLOT % C::kWaves == 0, "slots must divide over waves");
  static_assert(BK == 64, "row swizzle below is the one for 128-byte rows");
  static_assert(!kPermute || (EXT % 128 == 0 && TILES == 8), "the permutation works on blocks of 128 rows");
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t voff[SPW];
  uint32_t kelem[SPW];
  uint32_t k_limit, slot0;
  uint32_t rd[C::kKK];

  // XOR swizzle of the 16-byte chunk index.  ds_read_b128 serves 16 lanes (256 bytes, all 64 banks) per clock;
  // the 16 lanes of a quarter wave read 16 consecutive rows at one logical chunk, so the chunk index is XORed
  // with the row bits that do not already select a bank.
  __device__ __forceinline__ static int swz(int row) { return (row >> 1) & 7; }

  // `row_of(lrow)`: source row, relative to `base`, that LDS row lrow of the panel holds; rows >= rows_valid read zeros
  template <class RowOf>
  __device__ __forceinline__ void init_map(const void* base, uint32_t ld_elems, int rows_valid, uint32_t k_elems,
                                           int wave, int lane, int wave_side_index, RowOf row_of, bool uniform_base) {
    const uint32_t ld_bytes = ld_elems * 2;
    const uint32_t rows = rows_valid <= 0 ? 0u : (uint32_t)rows_valid;
    rsrc = uniform_base ? make_rsrc(base, rows * ld_bytes) : make_rsrc_uniform(base, rows * ld_bytes);
    k_limit = k_elems;
    slot0 = wave * SPW;
    const int rin = lane / CPR, p = lane % CPR;
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
      const uint32_t lrow = RPS * (slot0 + i) + rin;
      const int chunk = p ^ swz(lrow);
      kelem[i] = chunk * 8;
      voff[i] = (uint32_t)row_of((int)lrow) * ld_bytes + chunk * 16;
    }
    const int row0 = wave_side_index * (16 * TILES) + (lane & 15);
#pragma unroll
    for (int kk = 0; kk < C::kKK; ++kk) rd[kk] = row0 * RB + (((4 * kk + (lane >> 4)) ^ swz(row0)) * 16);
  }
  __device__ __forceinline__ void init(const void* base, uint32_t ld_elems, uint32_t rows_valid, uint32_t k_elems,
                                       int wave, int lane, int wave_side_index) {
    const int rows = rows_valid < (uint32_t)EXT ? (int)rows_valid : EXT;
    init_map(base, ld_elems, rows, k_elems, wave, lane, wave_side_index,
             [](int lrow) { return (lrow & ~127) + a_row_of_block_row16<kPermute>(lrow & 127); }, true);
  }
  __device__ __forceinline__ void issue_one(int i, uint32_t panel_lds, uint32_t k0) const {
    dma16(rsrc, (k0 + kelem[i]) < k_limit ? voff[i] + k0 * 2 : kOutOfRange, panel_lds + (slot0 + i) * 1024);
  }
  __device__ __forceinline__ void issue(uint32_t panel_lds, uint32_t k0) const {
#pragma unroll
    for (int i = 0; i < SPW; ++i) issue_one(i, panel_lds, k0);
  }
  __device__ __forceinline__ bf16x8 frag(const char* panel, int t, int kk) const {
    return *reinterpret_cast<const bf16x8*>(panel + rd[kk] + t * (16 * RB));
  }
};

// K-strided panel [BK k][EXT index], read with the transposing LDS read.  A quarter wave (16 lanes) feeds
// one 8-deep k group of a 16-wide tile: lane j of the quarter hands over the 4 consecutive indices
// 4 * (j % 4) .. + 3 at k row j / 4 (and, in a second read, 4 rows further).  kPermute (A side only): those
// 4 MFMA rows 16 t + 4 q + r read indices 32 q + 4 t + r of the 128-wide block, applied in the read addresses.
template <class C, int EXT, int TILES, bool kPermute = false>
struct PanelKS16 {
  static constexpr int BK = C::BK;
  static constexpr int RB = EXT * 2;
  static constexpr int CPR = EXT / 8;
  static constexpr int RPS = 1024 / RB;
  static constexpr int NSLOT = BK / RPS;
  static constexpr int SPW = NSLOT / C::kWaves;
  static_assert(NSLOT % C::kWaves == 0, "slots must divide over waves");
  static_assert(!kPermute || (EXT % 128 == 0 && TILES == 8), "the permutation works on blocks of 128 indices");
  __amdgpu_buffer_rsrc_t rsrc;
  uint32_t voff[SPW];
  uint32_t ok_mask, ld_bytes, slot0;
  uint32_t rd[TILES];

  // XOR swizzle of the 16-byte chunk index by the k row.  A quarter wave reads 4 k rows x 4 pieces of 8 bytes.
  // In memory order the 4 pieces of a row are 32 contiguous bytes (2 chunks), so rows must differ in chunk
  // bits 1-2; with the permutation the pieces are 64 bytes (4 chunks) apart, so rows must differ in bits 0-1.
  // The two lane quarters that are served in one clock read k rows 8 apart: in memory order bit 3 of the k row
  // moves them to the other 128-byte half of the 256-byte bank window.  (With the permutation both quarters
  // need the same 8-byte half of all 16 chunks of the window, which no 16-byte swizzle can separate.)
  __device__ __forceinline__ static uint32_t swz(uint32_t krow) {
    return kPermute ? (krow & 3) : (2 * (krow & 3)) ^ (8 * ((krow >> 3) & 1));
  }

  __device__ __forceinline__ void init(const void* base, uint32_t ld_elems, uint32_t k_rows, uint32_t cols_valid,
                                       int wave, int lane, int wave_side_index) {
    ld_bytes = ld_elems * 2;
    const uint32_t last_cols = cols_valid < ld_elems ? cols_valid : ld_elems;
    rsrc = make_rsrc(base, (k_rows - 1) * ld_bytes + last_cols * 2);
    slot0 = wave * SPW;
    ok_mask = 0;
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
      const uint32_t krow = RPS * (slot0 + i) + lane / CPR;
      const uint32_t chunk = (lane % CPR) ^ swz(krow);
      voff[i] = krow * ld_bytes + chunk * 16;
      ok_mask |= ((chunk * 8) < cols_valid ? 1u : 0u) << i;
    }
    const int g = lane >> 4, i16 = lane & 15, q = i16 & 3;
#pragma unroll
    for (int t = 0; t < TILES; ++t) {
      const int col = kPermute ? wave_side_index * 128 + 32 * q + 4 * t
                               : wave_side_index * (16 * TILES) + 16 * t + 4 * q;
      const int krow = 8 * g + (i16 >> 2);
      rd[t] = krow * RB + (((col >> 3) ^ swz(krow)) * 16) + (col & 7) * 2;
    }
  }
  __device__ __forceinline__ void issue_one(int i, uint32_t panel_lds, uint32_t k0) const {
    dma16(rsrc, ((ok_mask >> i) & 1u) ? voff[i] + k0 * ld_bytes : kOutOfRange, panel_lds + (slot0 + i) * 1024);
  }
  __device__ __forceinline__ void issue(uint32_t panel_lds, uint32_t k0) const {
#pragma unroll
    for (int i = 0; i < SPW; ++i) issue_one(i, panel_lds, k0);
  }
  __device__ __forceinline__ bf16x8 frag(const char* panel, int t, int kk) const {
    typedef __attribute__((address_space(3))) i16x4* lds_i16x4_ptr;
    const char* p = panel + rd[t] + kk * (32 * RB);
    i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(p));
    i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(p + 4 * RB));
    i16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
};

template <int TA, int TB>
__device__ __forceinline__ void zero_acc(f32x4 (&acc)[TA][TB]) {
#pragma unroll
  for (int t = 0; t < TA; ++t)
#pragma unroll
    for (int u = 0; u < TB; ++u)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[t][u][r] = 0.f;
}

}  // namespace mst
