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
  if (I * d >= (int64_t(1) << 31)) return MST_ERR_BAD_SHAPE;
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

std::once_flag g_attr_once;
hipError_t g_attr_err = hipSuccess;
void set_kernel_attributes() {
  auto set = [](const void* f) {
    hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess && g_attr_err == hipSuccess) g_attr_err = e;
  };
  set((const void*)k_mlp_gateup<false>);
  set((const void*)k_mlp_gateup<true>);
  set((const void*)k_mlp_gemm_nt);
  set((const void*)k_mlp_gemm_nn);
  set((const void*)k_bwd_gemm_dw);
}

mst_status check_launch() { return hipGetLastError() == hipSuccess ? MST_OK : MST_ERR_LAUNCH; }

mst_status prepare_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MST_ERR_NO_DEVICE;
  std::call_once(g_attr_once, set_kernel_attributes);
  if (g_attr_err != hipSuccess) return MST_ERR_LAUNCH;
  return MST_OK;
}

int rows_of(const Plan& p, int i) {
  const int64_t r0 = (int64_t)i * p.C;
  return (int)((p.S - r0) < p.C ? (p.S - r0) : p.C);
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
      misaligned(dX, 16) || misaligned(dWg, 4) || misaligned(dWu, 4) || misaligned(dWd, 4) || misaligned(workspace, 256))
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
  const long long* no_count = nullptr;

  // Algorithm 3: loop over the mini-sequences; dX_i lands in its row range, the weight gradients accumulate
  for (int i = 0; i < p.n_chunks; ++i) {
    const int64_t r0 = (int64_t)i * p.C;
    const int rows = rows_of(p, i), n_st = (rows + kTile - 1) / kTile;
    const __bf16* Xc = Xb + r0 * p.d;
    const __bf16* dOc = dOb + r0 * p.d;
    const int acc = i > 0 ? 1 : 0;
    {
      Scope sc(st, MST_MLP_K_DA);
      hipLaunchKernelGGL(k_mlp_gemm_nn, dim3(xcd_grid_super(p.n_it, n_st)), dim3(kThreads), kLdsBytes, st,
                         dOc, Wdb, (const __bf16*)nullptr, (const __bf16*)nullptr, dd, dI, rows, dI, dd,
                         n_st, p.n_it, bufG, dI);
    }
    {
      Scope sc(st, MST_MLP_K_GATEUP_BWD);
      hipLaunchKernelGGL(k_mlp_gateup<true>, dim3(xcd_grid_super(p.n_it128, n_st)), dim3(kThreads), kLdsBytes, st,
                         Xc, Wgb, Wub, rows, dd, dI, n_st, p.n_it128, bufA, bufG, bufU);
    }
    {
      Scope sc(st, MST_MLP_K_DX);
      hipLaunchKernelGGL(k_mlp_gemm_nn, dim3(xcd_grid_super(p.n_dt, n_st)), dim3(kThreads), kLdsBytes, st,
                         (const __bf16*)bufG, Wgb, (const __bf16*)bufU, Wub, dI, dd, rows, dd, dI,
                         n_st, p.n_dt, dXb + r0 * p.d, dd);
    }
    {
      Scope sc(st, MST_MLP_K_DW);
      hipLaunchKernelGGL(k_bwd_gemm_dw, dim3(xcd_grid_2d(p.n_it, p.n_dt)), dim3(kThreads), kLdsBytes, st,
                         (const __bf16*)bufG, dI, Xc, rows, dd, dI, p.n_it, p.n_dt, acc, 0, no_count, 1.0f, dWg);
    }
    {
      Scope sc(st, MST_MLP_K_DW);
      hipLaunchKernelGGL(k_bwd_gemm_dw, dim3(xcd_grid_2d(p.n_it, p.n_dt)), dim3(kThreads), kLdsBytes, st,
                         (const __bf16*)bufU, dI, Xc, rows, dd, dI, p.n_it, p.n_dt, acc, 0, no_count, 1.0f, dWu);
    }
    {
      Scope sc(st, MST_MLP_K_DW);
      hipLaunchKernelGGL(k_bwd_gemm_dw, dim3(xcd_grid_2d(p.n_dt, p.n_it)), dim3(kThreads), kLdsBytes, st,
                         dOc, dd, (const __bf16*)bufA, rows, dI, dd, p.n_dt, p.n_it, acc, 0, no_count, 1.0f, dWd);
    }
  }
  return check_launch();
}

mst_status mst_mlp_profile_enable(int enable) {
  g_prof.enable(enable != 0);
  return MST_OK;
}

mst_status mst_mlp_profile_collect(double* ms_per_kind, int64_t* launches_per_kind) {
  return g_prof.collect(MST_MLP_PROFILE_KINDS, ms_per_kind, launches_per_kind) ? MST_OK : MST_ERR_LAUNCH;
}

const char* mst_mlp_profile_kind_name(int kind) {
  static const char* names[MST_MLP_PROFILE_KINDS] = {"gateup", "down", "da", "gateup_bwd", "dx", "dw"};
  return (kind >= 0 && kind < MST_MLP_PROFILE_KINDS) ? names[kind] : "?";
}

}  // extern "C"
