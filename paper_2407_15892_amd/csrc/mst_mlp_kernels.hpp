// Device kernels of the mini-sequence MLP path (gfx950).
//
// Per mini-sequence (chunk) of C rows, following Algorithm 1 (forward) and
// Algorithm 3 (backward with recomputation) of the paper, for the block
// O = (silu(X Wg^T) * (X Wu^T)) Wd^T of Theorem 1 / Appendix C:
//
//   forward   k_mlp_gateup<false>  gate and up tiles of the same (token, i) range side by side in the MFMA
//                                  accumulators; A = silu(G) * U taken from them, bf16 to the workspace
//             k_mlp_gemm_nt        O_chunk = A Wd^T
//   backward  k_mlp_gemm_nn        dA = dO_chunk Wd
//             k_mlp_gateup<true>   gate and up tiles again; dG = dA U silu'(G), dU = dA silu(G), A
//             k_mlp_gemm_nn        dX_chunk = dG Wg + dU Wu   (two contractions into one accumulator)
//             k_bwd_gemm_dw        dWg += dG^T X, dWu += dU^T X, dWd += dO^T A   (the LM-head's kernel)
//
// All kernels use the 256 x 256 block tile main loop of gemm_tile.hpp and the XCD-aware workgroup
// remapping of mst_kernels.hpp.
#pragma once
#include "mst_kernels.hpp"

namespace mst {

// Workgroup -> tile mapping for a 2-D tile space cut into 8 x 4 (slow x fast) super-tiles: XCD x owns super-tiles
// x, x + 8, ... (row-major order of super-tiles), so the 32 workgroups resident on an XCD read 12 distinct operand
// panels, also when the whole grid is only 16 x 16 tiles.  Returns false for padding workgroups.
constexpr int kSuperSlow = 8, kSuperFast = 4;
__device__ __forceinline__ bool xcd_tile_super(int n_slow, int n_fast, int* slow, int* fast) {
  const int ss = (n_slow + kSuperSlow - 1) / kSuperSlow, sf = (n_fast + kSuperFast - 1) / kSuperFast;
  const int x = blockIdx.x % kNumXcd, q = blockIdx.x / kNumXcd;
  const int super = x + kNumXcd * (q / (kSuperSlow * kSuperFast));
  const int inner = q % (kSuperSlow * kSuperFast);
  if (super >= ss * sf) return false;
  *slow = (super / sf) * kSuperSlow + inner / kSuperFast;
  *fast = (super % sf) * kSuperFast + inner % kSuperFast;
  return *slow < n_slow && *fast < n_fast;
}
inline int xcd_grid_super(int n_slow, int n_fast) {
  const int ss = (n_slow + kSuperSlow - 1) / kSuperSlow, sf = (n_fast + kSuperFast - 1) / kSuperFast;
  return kNumXcd * ((ss * sf + kNumXcd - 1) / kNumXcd) * kSuperSlow * kSuperFast;
}

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
// logistic function; exp2 overflows to +inf for very negative g, whose reciprocal is 0
__device__ __forceinline__ float sigmoid_f(float g) { return fast_rcp(1.0f + fast_exp2(-g * kLog2e)); }

// ---------------------------------------------------------------------------
// gate / up projections of a chunk with the SwiGLU epilogue.
//   A side = intermediate index i, 128 per workgroup: the 256-row A panel holds, for each of the two
//   wave rows, 64 gate rows (MFMA tiles 0..3) and the 64 up rows of the same i (tiles 4..7), so gate and
//   up values of one (token, i) sit in the same lane and register of accumulators t and t + 4.
//   B side = chunk rows (tokens).  A lane owns 4 tokens and 16 consecutive i for each: 32-byte stores.
//   kBackward: dAG holds dA on entry and receives dG (same element, same lane); dU and A are written.
// ---------------------------------------------------------------------------
constexpr int kGateUpI = 128;   // intermediate indices per workgroup
template <bool kBackward>
__global__ __launch_bounds__(kThreads) void k_mlp_gateup(
    const __bf16* __restrict__ Xc, const __bf16* __restrict__ Wg, const __bf16* __restrict__ Wu,
    int rows, int d, int I, int n_st, int n_it,
    __bf16* __restrict__ A, __bf16* __restrict__ dAG, __bf16* __restrict__ dU) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int it, st;
  if (!xcd_tile_super(n_it, n_st, &it, &st)) return;
  const int i0 = it * kGateUpI, s0 = st * kTile;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave >> 2, wb = wave & 3;

  f32x4 acc[kTA16][kTB16];
  zero_acc<kTA16, kTB16>(acc);
  PanelKC16<Tile16, kTile, kTA16, true> pa;
  PanelKC16<Tile16, kTile, kTB16, false> pb;
  {
    // A panel, per wave row of 128 LDS rows: MFMA tiles 0..3 are gate rows, tiles 4..7 the up rows of the same 64
    // intermediate indices; LDS row 16 t + 4 g + r holds index 16 g + 4 (t % 4) + r, so that a lane's gate value
    // acc[t][u][r] and up value acc[t + 4][u][r] belong to the same index and its 16 indices are consecutive.
    // As a loader, wave w fills LDS rows 32 w .. 32 w + 31 (tiles 2 (w % 4), 2 (w % 4) + 1 of wave row w / 4).
    const int q = wave & 3;
    const int ib = i0 + 64 * (wave >> 2);                       // first index of the loader's wave row
    const __bf16* src = (q < 2 ? Wg : Wu) + (size_t)ib * d;
    int valid = I - ib;
    if (valid > 64) valid = 64;
    pa.init_map(src, d, valid, d, wave, lane, wa,
                [](int lrow) { const int m = lrow & 127; return 16 * ((m >> 2) & 3) + 4 * ((m >> 4) & 3) + (m & 3); }, false);
  }
  pb.init(Xc + (size_t)s0 * d, d, rows - s0, d, wave, lane, wb);
  gemm_mainloop_pp<Tile16>(acc, pa, pb, smem, 0, d, wa);

  const int ib = i0 + 64 * wa + 16 * (lane >> 4);              // this lane's 16 consecutive intermediate indices
#pragma unroll
  for (int u = 0; u < kTB16; ++u) {
    const int s_local = s0 + wb * 64 + 16 * u + (lane & 15);
    if (s_local >= rows || ib >= I) continue;                  // I % 8 == 0: a group of 8 is inside or outside
    const size_t off = (size_t)s_local * I + ib;
    const bool hi_ok = ib + 8 < I;
    bf16x8 da[2];
    if (kBackward) {
      da[0] = *reinterpret_cast<const bf16x8*>(dAG + off);
      if (hi_ok) da[1] = *reinterpret_cast<const bf16x8*>(dAG + off + 8);
    }
    bf16x8 a_o[2], g_o[2], u_o[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) {                             // index ib + e: tile e / 4, register e % 4
      const float g = acc[e >> 2][u][e & 3], up = acc[4 + (e >> 2)][u][e & 3];
      const float sg = sigmoid_f(g);
      const float act = g * sg;                                // silu(g)
      a_o[e >> 3][e & 7] = (__bf16)(act * up);
      if (kBackward) {
        const float dav = (float)da[e >> 3][e & 7];
        g_o[e >> 3][e & 7] = (__bf16)(dav * up * (sg * (1.0f + g * (1.0f - sg))));   // dA * U * silu'(G)
        u_o[e >> 3][e & 7] = (__bf16)(dav * act);                                    // dA * silu(G)
      }
    }
    *reinterpret_cast<bf16x8*>(A + off) = a_o[0];
    if (hi_ok) *reinterpret_cast<bf16x8*>(A + off + 8) = a_o[1];
    if (kBackward) {
      *reinterpret_cast<bf16x8*>(dAG + off) = g_o[0];
      *reinterpret_cast<bf16x8*>(dU + off) = u_o[0];
      if (hi_ok) {
        *reinterpret_cast<bf16x8*>(dAG + off + 8) = g_o[1];
        *reinterpret_cast<bf16x8*>(dU + off + 8) = u_o[1];
      }
    }
  }
}

// epilogue of the two plain GEMMs: a lane holds, for each of its rows s, 32 consecutive n (A side, permuted),
// i.e. 64 contiguous bytes of bf16, and the lanes of a wave instruction hold 16 different rows.  Stored directly,
// every instruction would be 64 separate 16-byte writes; instead the bf16 tile is staged in LDS (free after the main
// loop; rows padded by 16 bytes, which spreads the 16 rows of a quarter wave over all banks) and every wave
// instruction then writes two whole rows of the tile.
template <class T>
__device__ __forceinline__ void store_rows_bf16(const f32x4 (&acc)[T::TA][T::TB], __bf16* __restrict__ out, int ldo,
                                                int rows, int N, int s0, int n0, int wa, int wb, int wave, int lane,
                                                char* smem) {
  static_assert(T::TA == 8 && T::EA == 256, "one 128-wide permuted block per wave row, two wave rows");
  constexpr int kStageRow = T::EA * 2 + 16;
#pragma unroll
  for (int u = 0; u < T::TB; ++u) {
    const int row = wb * (16 * T::TB) + 16 * u + (lane & 15);
    char* srow = smem + row * kStageRow + (wa * 128 + 32 * (lane >> 4)) * 2;
#pragma unroll
    for (int p = 0; p < 4; ++p) {                    // tiles 2p and 2p + 1: n = nb + 8p .. + 7
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (__bf16)acc[2 * p + (e >> 2)][u][e & 3];
      *reinterpret_cast<bf16x8*>(srow + 16 * p) = o;
    }
  }
  __syncthreads();
  const int col = (lane & 31) * 8;                   // 8 entries = 16 bytes per lane, 32 lanes per row
  const bool col_ok = n0 + col < N;                  // N % 8 == 0
  constexpr int kRowsPerWave = T::EB / T::kWaves;
#pragma unroll
  for (int i = 0; i < kRowsPerWave / 2; ++i) {
    const int row = kRowsPerWave * wave + 2 * i + (lane >> 5);
    if (s0 + row < rows && col_ok)
      *reinterpret_cast<bf16x8*>(out + (size_t)(s0 + row) * ldo + n0 + col) =
          *reinterpret_cast<const bf16x8*>(smem + row * kStageRow + col * 2);
  }
}

// ---------------------------------------------------------------------------
// out[s][n] = sum_k P[s][k] Q[n][k]      (both operands K-contiguous; used for O_chunk = A Wd^T)
//   A side = n (rows of Q, permuted so a lane holds 32 consecutive n), B side = s (rows of P)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_mlp_gemm_nt(
    const __bf16* __restrict__ P, int ldp, const __bf16* __restrict__ Q, int ldq, int rows, int N, int K,
    int n_st, int n_nt, __bf16* __restrict__ out, int ldo) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int nt, st;
  if (!xcd_tile_super(n_nt, n_st, &nt, &st)) return;
  const int n0 = nt * kTile, s0 = st * kTile;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave >> 2, wb = wave & 3;

  f32x4 acc[kTA16][kTB16];
  zero_acc<kTA16, kTB16>(acc);
  PanelKC16<Tile16, kTile, kTA16, true> pa;
  PanelKC16<Tile16, kTile, kTB16, false> pb;
  pa.init(Q + (size_t)n0 * ldq, ldq, N - n0, K, wave, lane, wa);
  pb.init(P + (size_t)s0 * ldp, ldp, rows - s0, K, wave, lane, wb);
  gemm_mainloop_pp<Tile16>(acc, pa, pb, smem, 0, K, wa);
  store_rows_bf16<Tile16>(acc, out, ldo, rows, N, s0, n0, wa, wb, wave, lane, smem);
}

// ---------------------------------------------------------------------------
// out[s][n] = sum_k P1[s][k] Q1[k][n] (+ sum_k P2[s][k] Q2[k][n])   (Q K-strided)
//   used for dA = dO Wd (one term, K = d) and dX = dG Wg + dU Wu (two terms, K = I each)
//   A side = n (columns of Q, read transposed with the row permutation, so a lane holds 32 consecutive n
//   and stores 64 bytes), B side = s (rows of P).  T: Tile16, or Tile16HalfB for a partly filled last round.
// ---------------------------------------------------------------------------
template <class T>
__global__ __launch_bounds__(kThreads) void k_mlp_gemm_nn(
    const __bf16* __restrict__ P1, const __bf16* __restrict__ Q1,
    const __bf16* __restrict__ P2, const __bf16* __restrict__ Q2,
    int ldp, int ldq, int rows, int N, int K, int n_st, int n_nt, __bf16* __restrict__ out, int ldo) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int nt, st;
  if (!xcd_tile_super(n_nt, n_st, &nt, &st)) return;
  const int n0 = nt * T::EA, s0 = st * T::EB;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave / T::WB, wb = wave % T::WB;

  f32x4 acc[T::TA][T::TB];
  zero_acc<T::TA, T::TB>(acc);
  {
    PanelKS16<T, T::EA, T::TA, true> pa;
    PanelKC16<T, T::EB, T::TB, false> pb;
    pa.init(Q1 + n0, ldq, K, N - n0, wave, lane, wa);
    pb.init(P1 + (size_t)s0 * ldp, ldp, rows - s0, K, wave, lane, wb);
    gemm_mainloop_pp<T>(acc, pa, pb, smem, 0, K, wa);
  }
  if (P2 != nullptr) {
    PanelKS16<T, T::EA, T::TA, true> pa;
    PanelKC16<T, T::EB, T::TB, false> pb;
    pa.init(Q2 + n0, ldq, K, N - n0, wave, lane, wa);
    pb.init(P2 + (size_t)s0 * ldp, ldp, rows - s0, K, wave, lane, wb);
    gemm_mainloop_pp<T>(acc, pa, pb, smem, 0, K, wa);
  }
  store_rows_bf16<T>(acc, out, ldo, rows, N, s0, n0, wa, wb, wave, lane, smem);
}

// ---------------------------------------------------------------------------
// the three weight gradients of a chunk from one launch: dWg (+)= dG^T X, dWu (+)= dU^T X, dWd (+)= dO^T A.
//   Each is a tile space of its own (the LM-head's dW tile body); the workgroup index selects the problem.
//   One launch instead of three leaves one partly filled last round of workgroups instead of three
//   (3 x 896 tiles = 10.5 rounds of 256 instead of 3 x 4 at the Llama3-8B shape).
// ---------------------------------------------------------------------------
struct DwProblem {
  const __bf16* G; int ldg;      // [rows][ldg], V columns used
  const __bf16* H; int ldh;      // [rows][ldh], d columns used
  int d, V, n_vt, n_jt, grid;    // grid = xcd_grid_2d(n_vt, n_jt)
  float* dW;                     // [V][d]
};
struct DwProblems { DwProblem p[3]; };
template <bool kStoreOnly>   // the first chunk only stores; later chunks add to the stored sums; `more`: another chunk follows
__global__ __launch_bounds__(kThreads) void k_mlp_dw3(DwProblems ps, int rows, int more) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int b = blockIdx.x, which = 0;
  if (b >= ps.p[0].grid) { b -= ps.p[0].grid; which = 1; if (b >= ps.p[1].grid) { b -= ps.p[1].grid; which = 2; } }
  const DwProblem& q = ps.p[which];
  int vt, jt;
  // 8 x 4 rectangles walked group by group of 4 fast tiles (measured 0.7 % faster here than the LM-head's 4 x 8 bands)
  if (!xcd_tile_of_block<8, 4, 4>(b, q.n_vt, q.n_jt, &vt, &jt)) return;
  dw_tile(q.G, q.ldg, q.ldg, q.H, q.ldh, rows, q.d, q.V, vt, jt, kStoreOnly ? 0 : 1, more, 1.0f, q.dW, q.d, smem);
}

}  // namespace mst
