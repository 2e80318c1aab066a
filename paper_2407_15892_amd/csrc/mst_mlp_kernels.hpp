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
//   wave rows, 64 gate rows (MFMA tiles 0, 1) and the 64 up rows of the same i (tiles 2, 3), so gate and
//   up values of one (token, i) sit in the same lane and register of accumulators t and t + 2.
//   B side = chunk rows (tokens).  A lane owns one token and 16 consecutive i per tile: 32-byte stores.
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

  f32x16 acc[kTA][kTB];
  zero_acc<kTA, kTB>(acc);
  PanelKC<Tile, kTile, kTA, true> pa;
  PanelKC<Tile, kTile, kTB, false> pb;
  {
    // as a loader, wave w brings in MFMA tile w of the A panel: wave row w / 4, tile w % 4 of that row
    const int t_l = wave & 3;
    const int ib = i0 + 64 * (wave >> 2) + 32 * (t_l & 1);
    const __bf16* src = (t_l < 2 ? Wg : Wu) + (size_t)ib * d;
    pa.init_tile32(src, d, I - ib, d, wave, lane, wa);
  }
  pb.init(Xc + (size_t)s0 * d, d, rows - s0, d, wave, lane, wb);
  gemm_mainloop_pp<Tile>(acc, pa, pb, smem, 0, d, wa);

#pragma unroll
  for (int u = 0; u < kTB; ++u) {
    const int s_local = s0 + wb * 64 + 32 * u + (lane & 31);
    if (s_local >= rows) continue;
    const size_t row_off = (size_t)s_local * I;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int ib = i0 + 64 * wa + 32 * t + 16 * (lane >> 5);
      if (ib >= I) continue;                       // I % 8 == 0: a group of 8 is inside or outside
      const bool hi_ok = ib + 8 < I;
      bf16x8 da_lo, da_hi;
      if (kBackward) {
        da_lo = *reinterpret_cast<const bf16x8*>(dAG + row_off + ib);
        if (hi_ok) da_hi = *reinterpret_cast<const bf16x8*>(dAG + row_off + ib + 8);
      }
      bf16x8 a_lo, a_hi, g_lo, g_hi, u_lo, u_hi;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float g = acc[t][u][r], up = acc[t + 2][u][r];
        const float s = sigmoid_f(g);
        const float act = g * s;                                   // silu(g)
        const float a = act * up;
        if (r < 8) a_lo[r] = (__bf16)a; else a_hi[r - 8] = (__bf16)a;
        if (kBackward) {
          const float da = (float)(r < 8 ? da_lo[r] : da_hi[r - 8]);
          const float dg = da * up * (s * (1.0f + g * (1.0f - s)));  // dA * U * silu'(G)
          const float du = da * act;                                 // dA * silu(G)
          if (r < 8) { g_lo[r] = (__bf16)dg; u_lo[r] = (__bf16)du; } else { g_hi[r - 8] = (__bf16)dg; u_hi[r - 8] = (__bf16)du; }
        }
      }
      *reinterpret_cast<bf16x8*>(A + row_off + ib) = a_lo;
      if (hi_ok) *reinterpret_cast<bf16x8*>(A + row_off + ib + 8) = a_hi;
      if (kBackward) {
        *reinterpret_cast<bf16x8*>(dAG + row_off + ib) = g_lo;
        *reinterpret_cast<bf16x8*>(dU + row_off + ib) = u_lo;
        if (hi_ok) {
          *reinterpret_cast<bf16x8*>(dAG + row_off + ib + 8) = g_hi;
          *reinterpret_cast<bf16x8*>(dU + row_off + ib + 8) = u_hi;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------
// out[s][n] = sum_k P[s][k] Q[n][k]      (both operands K-contiguous; used for O_chunk = A Wd^T)
//   A side = n (rows of Q, permuted so a lane holds 16 consecutive n), B side = s (rows of P)
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

  f32x16 acc[kTA][kTB];
  zero_acc<kTA, kTB>(acc);
  PanelKC<Tile, kTile, kTA, true> pa;
  PanelKC<Tile, kTile, kTB, false> pb;
  pa.init(Q + (size_t)n0 * ldq, ldq, N - n0, K, wave, lane, wa);
  pb.init(P + (size_t)s0 * ldp, ldp, rows - s0, K, wave, lane, wb);
  gemm_mainloop_pp<Tile>(acc, pa, pb, smem, 0, K, wa);

#pragma unroll
  for (int u = 0; u < kTB; ++u) {
    const int s_local = s0 + wb * 64 + 32 * u + (lane & 31);
    if (s_local >= rows) continue;
    __bf16* orow = out + (size_t)s_local * ldo;
#pragma unroll
    for (int t = 0; t < kTA; ++t) {
      const int nb = n0 + wa * 128 + 32 * t + 16 * (lane >> 5);
      bf16x8 lo, hi;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (r < 8) lo[r] = (__bf16)acc[t][u][r]; else hi[r - 8] = (__bf16)acc[t][u][r];
      }
      if (nb < N) *reinterpret_cast<bf16x8*>(orow + nb) = lo;          // N % 8 == 0
      if (nb + 8 < N) *reinterpret_cast<bf16x8*>(orow + nb + 8) = hi;
    }
  }
}

// ---------------------------------------------------------------------------
// out[s][n] = sum_k P1[s][k] Q1[k][n] (+ sum_k P2[s][k] Q2[k][n])   (Q K-strided)
//   used for dA = dO Wd (one term, K = d) and dX = dG Wg + dU Wu (two terms, K = I each)
//   A side = n (columns of Q, read transposed with the row permutation, so a lane holds 16 consecutive n
//   and stores 32 bytes), B side = s (rows of P).  T: Tile, or TileHalfB for a partly filled last round.
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

  f32x16 acc[T::TA][T::TB];
  zero_acc<T::TA, T::TB>(acc);
  {
    PanelKS<T, T::EA, T::TA, true> pa;
    PanelKC<T, T::EB, T::TB, false> pb;
    pa.init(Q1 + n0, ldq, K, N - n0, wave, lane, wa);
    pb.init(P1 + (size_t)s0 * ldp, ldp, rows - s0, K, wave, lane, wb);
    gemm_mainloop_pp<T>(acc, pa, pb, smem, 0, K, wa);
  }
  if (P2 != nullptr) {
    PanelKS<T, T::EA, T::TA, true> pa;
    PanelKC<T, T::EB, T::TB, false> pb;
    pa.init(Q2 + n0, ldq, K, N - n0, wave, lane, wa);
    pb.init(P2 + (size_t)s0 * ldp, ldp, rows - s0, K, wave, lane, wb);
    gemm_mainloop_pp<T>(acc, pa, pb, smem, 0, K, wa);
  }

#pragma unroll
  for (int u = 0; u < T::TB; ++u) {
    const int s_local = s0 + wb * (32 * T::TB) + 32 * u + (lane & 31);
    if (s_local >= rows) continue;
    __bf16* orow = out + (size_t)s_local * ldo;
#pragma unroll
    for (int t = 0; t < T::TA; ++t) {
      const int nb = n0 + wa * (32 * T::TA) + 32 * t + 16 * (lane >> 5);
      bf16x8 lo, hi;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (r < 8) lo[r] = (__bf16)acc[t][u][r]; else hi[r - 8] = (__bf16)acc[t][u][r];
      }
      if (nb < N) *reinterpret_cast<bf16x8*>(orow + nb) = lo;          // N % 8 == 0
      if (nb + 8 < N) *reinterpret_cast<bf16x8*>(orow + nb + 8) = hi;
    }
  }
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
__global__ __launch_bounds__(kThreads) void k_mlp_dw3(DwProblems ps, int rows, int accumulate) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int b = blockIdx.x, which = 0;
  if (b >= ps.p[0].grid) { b -= ps.p[0].grid; which = 1; if (b >= ps.p[1].grid) { b -= ps.p[1].grid; which = 2; } }
  const DwProblem& q = ps.p[which];
  int vt, jt;
  if (!xcd_tile_2d(q.n_vt, q.n_jt, &vt, &jt, b)) return;
  dw_tile(q.G, q.ldg, q.ldg, q.H, q.ldh, rows, q.d, q.V, vt, jt, accumulate, 1.0f, q.dW, q.d, smem);
}

}  // namespace mst
