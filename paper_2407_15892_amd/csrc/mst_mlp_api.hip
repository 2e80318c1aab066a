// Host side of the mini-sequence MLP library: argument validation, the chunk
// schedule over the M mini-sequences (Algorithm 1 lines 1-5 and Algorithm 3
// lines 1-7 of the paper: partition, loop, concatenate / accumulate), workspace
// carving, launches, and the optional per-kernel event timing.
#include "../../include/mst_mlp.h"
#include "host_util.hpp"
#include "mst_mlp_kernels.hpp"

#include <mutex>

namespace {

using namespace mst;
using mst_host::misaligned;

struct Plan {
  int64_t S, d, I;
  int M;
  int C;            // rows per chunk = ceil(S / M)
  int n_chunks;     // non-empty chunks
  int n_dt, n_it;   // 256-wide tiles of d and of I
  int n_it128;      // 128-wide tiles of I (gate/up kernel)
  size_t slot;      // bytes of one chunk-sized bf16 [C, I] buffer
};

mst_status make_plan(int64_t S, int64_t d, int64_t I, int32_t M, Plan* p) {
  if (S <= 0 || d <= 0 || I <= 0) return MST_ERR_BAD_SHAPE;
  if (d % 8 != 0 || I % 8 != 0) return MST_ERR_BAD_SHAPE;
  if (M < 1 || (int64_t)M > S) return MST_ERR_BAD_M;
  if (I * d >= (int64_t(1) << 31) || d >= (int64_t(1) << 22) || I >= (int64_t(1) << 22)) return MST_ERR_BAD_SHAPE;
  const int64_t C = (S + M - 1) / M;
  if (C * I >= (int64_t(1) << 30) || C * d >= (int64_t(1) << 30)) return MST_ERR_BAD_SHAPE;
  p->S = S; p->d = d; p->I = I; p->M = M;
  p->C = (int)C;
  p->n_chunks = (int)((S + C - 1) / C);
  p->n_dt = (int)((d + kTile - 1) / kTile);
  p->n_it = (int)((I + kTile - 1) / kTile);
  p->n_it128 = (int)((I + kGateUpI - 1) / kGateUpI);
  p->slot = mst_host::align_up((size_t)C * I * 2, 256);
  return MST_OK;
}

mst_host::Profiler g_prof;
struct Scope : mst_host::Scope {
  Scope(hipStream_t s, int k) : mst_host::Scope(g_prof, s, k) {}
};

mst_host::PerDeviceOnce g_attr_once;
bool set_kernel_attributes() {   // on the current device
  bool ok = true;
  auto set = [&ok](const void* f) {
    if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess) ok = false;
  };
  set((const void*)k_mlp_gateup<false>);
  set((const void*)k_mlp_gateup<true>);
  set((const void*)k_mlp_gemm_nt);
  set((const void*)k_mlp_gemm_nn<Tile16>);
  set((const void*)k_mlp_gemm_nn<Tile16HalfB>);
  set((const void*)k_mlp_dw3<false>);
  set((const void*)k_mlp_dw3<true>);
  return ok;
}

mst_status check_launch() { return hipGetLastError() == hipSuccess ? MST_OK : MST_ERR_LAUNCH; }

mst_status prepare_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MST_ERR_NO_DEVICE;
  if (!g_attr_once.run(dev, set_kernel_attributes)) {
    (void)hipGetLastError();
    return MST_ERR_LAUNCH;
  }
  return MST_OK;
}

int rows_of(const Plan& p, int i) {
  const int64_t r0 = (int64_t)i * p.C;
  return (int)((p.S - r0) < p.C ? (p.S - r0) : p.C);
}


constexpr int kNumCu = 256;   // MI355X compute units; one workgroup is resident per CU

// Tail of the workgroup grid.  A GEMM of n_a x n_b block tiles runs in rounds of kNumCu workgroups; when the
// last round would be at most half full, the tiles of that round (whole tile rows of the A side, else whole
// tile columns of the B side) are cut in two along the B side (256 x 128 tiles) and launched separately, so
// that the last round is full and shorter.
struct Tail { int a_tail, b_tail; };
Tail tail_split(int n_a, int n_b) {
  const int total = n_a * n_b, rem = total % kNumCu;
  if (total < kNumCu || rem == 0 || 2 * rem > kNumCu) return {0, 0};
  if (rem % n_b == 0) return {rem / n_b, 0};
  if (rem % n_a == 0) return {0, rem / n_a};
  return {0, 0};
}

// out[rows][N] (+)= P1 Q1 (+ P2 Q2), Q: [K][ldq] with N columns used
void launch_nn(hipStream_t st, const __bf16* P1, const __bf16* Q1, const __bf16* P2, const __bf16* Q2,
               int ldp, int ldq, int rows, int N, int K, __bf16* out, int ldo) {
  const int n_nt = (N + kTile - 1) / kTile, n_st = (rows + kTile - 1) / kTile;
  const Tail tl = tail_split(n_nt, n_st);
  const int nt_full = n_nt - tl.a_tail;        // only a split of the A side (columns of Q) is used here
  const int n_full = tl.a_tail ? nt_full * kTile : N;
  hipLaunchKernelGGL(k_mlp_gemm_nn<Tile16>, dim3(xcd_grid_super(nt_full, n_st)), dim3(kThreads), kLdsBytes, st,
                     P1, Q1, P2, Q2, ldp, ldq, rows, n_full, K, n_st, nt_full, out, ldo);
  if (tl.a_tail) {
    const int n_sh = (rows + Tile16HalfB::EB - 1) / Tile16HalfB::EB;
    hipLaunchKernelGGL(k_mlp_gemm_nn<Tile16HalfB>, dim3(xcd_grid_super(tl.a_tail, n_sh)), dim3(kThreads),
                       Tile16HalfB::kLds, st, P1, Q1 + n_full, P2, Q2 ? Q2 + n_full : Q2, ldp, ldq, rows, N - n_full, K,
                       n_sh, tl.a_tail, out + n_full, ldo);
  }
}

DwProblem dw_problem(const __bf16* G, int ldg, const __bf16* H, int ldh, int d, int V, float* dW) {
  DwProblem q;
  q.G = G; q.ldg = ldg; q.H = H; q.ldh = ldh; q.d = d; q.V = V;
  q.n_vt = (V + kTile - 1) / kTile;
  q.n_jt = (d + kTile - 1) / kTile;
  q.grid = xcd_grid_2d(q.n_vt, q.n_jt);
  q.dW = dW;
  return q;
}

}  // namespace

extern "C" {

const char* mst_mlp_version(void) { return "mst-mlp 0.1 (gfx950)"; }

int32_t mst_mlp_suggest_m(int64_t S, int64_t d, int64_t I) {
  if (S <= 0 || d <= 0 || I <= 0) return 0;
  int64_t m = (2 * S + d) / (2 * d);             // S / d to the nearest integer: chunk size C = d
  if (m < 1) m = 1;
  if (m > S) m = S;
  if (m > 0x7fffffff) m = 0x7fffffff;
  return (int32_t)m;
}

mst_status mst_mlp_workspace_bytes(int64_t S, int64_t d, int64_t I, int32_t M, size_t* fwd_bytes, size_t* bwd_bytes) {
  Plan p;
  mst_status s = make_plan(S, d, I, M, &p);
  if (s != MST_OK) return s;
  if (fwd_bytes) *fwd_bytes = p.slot;
  if (bwd_bytes) *bwd_bytes = 3 * p.slot;
  return MST_OK;
}

mst_status mst_mlp_fwd(const void* X, const void* Wg, const void* Wu, const void* Wd,
                       int64_t S, int64_t d, int64_t I, int32_t M,
                       void* workspace, size_t workspace_bytes, void* O, void* stream) {
  Plan p;
  mst_status s = make_plan(S, d, I, M, &p);
  if (s != MST_OK) return s;
  if (!X || !Wg || !Wu || !Wd || !O) return MST_ERR_NULL_POINTER;
  if (!workspace || workspace_bytes < p.slot) return MST_ERR_WORKSPACE;
  if (misaligned(X, 16) || misaligned(Wg, 16) || misaligned(Wu, 16) || misaligned(Wd, 16) || misaligned(O, 16) ||
      misaligned(workspace, 256))
    return MST_ERR_ALIGNMENT;
  if ((s = prepare_device()) != MST_OK) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const __bf16* Xb = static_cast<const __bf16*>(X);
  const __bf16* Wgb = static_cast<const __bf16*>(Wg);
  const __bf16* Wub = static_cast<const __bf16*>(Wu);
  const __bf16* Wdb = static_cast<const __bf16*>(Wd);
  __bf16* Ob = static_cast<__bf16*>(O);
  __bf16* A = static_cast<__bf16*>(workspace);
  // Algorithm 1: loop over the mini-sequences; O_i lands in its row range of O (the concatenation of line 5)
  for (int i = 0; i < p.n_chunks; ++i) {
    const int64_t r0 = (int64_t)i * p.C;
    const int rows = rows_of(p, i), n_st = (rows + kTile - 1) / kTile;
    {
      Scope sc(st, MST_MLP_K_GATEUP);
      hipLaunchKernelGGL(k_mlp_gateup<false>, dim3(xcd_grid_super(p.n_it128, n_st)), dim3(kThreads), kLdsBytes, st,
                         Xb + r0 * p.d, Wgb, Wub, rows, (int)p.d, (int)p.I, n_st, p.n_it128,
                         A, (__bf16*)nullptr, (__bf16*)nullptr);
    }
    {
      Scope sc(st, MST_MLP_K_DOWN);
      hipLaunchKernelGGL(k_mlp_gemm_nt, dim3(xcd_grid_super(p.n_dt, n_st)), dim3(kThreads), kLdsBytes, st,
                         A, (int)p.I, Wdb, (int)p.I, rows, (int)p.d, (int)p.I, n_st, p.n_dt, Ob + r0 * p.d, (int)p.d);
    }
  }
  return check_launch();
}

mst_status mst_mlp_bwd(const void* X, const void* Wg, const void* Wu, const void* Wd, const void* dO,
                       int64_t S, int64_t d, int64_t I, int32_t M,
                       void* workspace, size_t workspace_bytes,
                       void* dX, float* dWg, float* dWu, float* dWd, void* stream) {
  Plan p;
  mst_status s = make_plan(S, d, I, M, &p);
  if (s != MST_OK) return s;
  if (!X || !Wg || !Wu || !Wd || !dO || !dX || !dWg || !dWu || !dWd) return MST_ERR_NULL_POINTER;
  if (!workspace || workspace_bytes < 3 * p.slot) return MST_ERR_WORKSPACE;
  if (misaligned(X, 16) || misaligned(Wg, 16) || misaligned(Wu, 16) || misaligned(Wd, 16) || misaligned(dO, 16) ||
      misaligned(dX, 16) || misaligned(dWg, 16) || misaligned(dWu, 16) || misaligned(dWd, 16) || misaligned(workspace, 256))
    return MST_ERR_ALIGNMENT;
  if ((s = prepare_device()) != MST_OK) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const __bf16* Xb = static_cast<const __bf16*>(X);
  const __bf16* Wgb = static_cast<const __bf16*>(Wg);
  const __bf16* Wub = static_cast<const __bf16*>(Wu);
  const __bf16* Wdb = static_cast<const __bf16*>(Wd);
  const __bf16* dOb = static_cast<const __bf16*>(dO);
  __bf16* dXb = static_cast<__bf16*>(dX);
  char* ws = static_cast<char*>(workspace);
  __bf16* bufG = reinterpret_cast<__bf16*>(ws);               // dA, then dG in place
  __bf16* bufU = reinterpret_cast<__bf16*>(ws + p.slot);      // dU
  __bf16* bufA = reinterpret_cast<__bf16*>(ws + 2 * p.slot);  // A
  const int dI = (int)p.I, dd = (int)p.d;

  // Algorithm 3: loop over the mini-sequences; dX_i lands in its row range, the weight gradients accumulate
  for (int i = 0; i < p.n_chunks; ++i) {
    const int64_t r0 = (int64_t)i * p.C;
    const int rows = rows_of(p, i), n_st = (rows + kTile - 1) / kTile;
    const __bf16* Xc = Xb + r0 * p.d;
    const __bf16* dOc = dOb + r0 * p.d;
    const int acc = i > 0 ? 1 : 0;
    {
      Scope sc(st, MST_MLP_K_DA);
      launch_nn(st, dOc, Wdb, nullptr, nullptr, dd, dI, rows, dI, dd, bufG, dI);
    }
    {
      Scope sc(st, MST_MLP_K_GATEUP_BWD);
      hipLaunchKernelGGL(k_mlp_gateup<true>, dim3(xcd_grid_super(p.n_it128, n_st)), dim3(kThreads), kLdsBytes, st,
                         Xc, Wgb, Wub, rows, dd, dI, n_st, p.n_it128, bufA, bufG, bufU);
    }
    {
      Scope sc(st, MST_MLP_K_DX);
      launch_nn(st, bufG, Wgb, bufU, Wub, dI, dd, rows, dd, dI, dXb + r0 * p.d, dd);
    }
    {
      Scope sc(st, MST_MLP_K_DW);
      DwProblems ps;
      ps.p[0] = dw_problem(bufG, dI, Xc, dd, dd, dI, dWg);     // dWg [I][d] (+)= dG^T X
      ps.p[1] = dw_problem(bufU, dI, Xc, dd, dd, dI, dWu);     // dWu [I][d] (+)= dU^T X
      ps.p[2] = dw_problem(dOc, dd, bufA, dI, dI, dd, dWd);    // dWd [d][I] (+)= dO^T A
      hipLaunchKernelGGL(acc ? k_mlp_dw3<false> : k_mlp_dw3<true>, dim3(ps.p[0].grid + ps.p[1].grid + ps.p[2].grid),
                         dim3(kThreads), kLdsBytes, st, ps, rows, i + 1 < p.n_chunks ? 1 : 0);
    }
  }
  return check_launch();
}

mst_status mst_mlp_profile_enable(int every) {
  g_prof.enable(every);
  return MST_OK;
}

mst_status mst_mlp_profile_collect(double* ms_per_kind, int64_t* launches_per_kind, int64_t* issued_per_kind) {
  return g_prof.collect(MST_MLP_PROFILE_KINDS, ms_per_kind, launches_per_kind, issued_per_kind) ? MST_OK : MST_ERR_LAUNCH;
}

const char* mst_mlp_profile_kind_name(int kind) {
  static const char* names[MST_MLP_PROFILE_KINDS] = {"gateup", "down", "da", "gateup_bwd", "dx", "dw"};
  return (kind >= 0 && kind < MST_MLP_PROFILE_KINDS) ? names[kind] : "?";
}

}  // extern "C"
