// Block-tile bf16 GEMM main loop for gfx950 (MI355X), shared by the contractions of the mini-sequence
// LM-head path (Algorithm 2 line 4 and Algorithm 4 lines 5, 7, 8 of the paper) and of the mini-sequence MLP
// path (Algorithms 1 and 3).
//
// One workgroup of 512 threads (8 wave64s, two per SIMD) owns a 256 x 256 output tile.  Operand panels of
// 256 x 64 bf16 are brought from global memory straight into LDS (buffer loads with the LDS bit, 16 bytes
// per lane, no register staging), three stages deep for the A operand and two for the B operand (all 160 KB
// of LDS), and consumed by MFMA instructions.  The wave grid is 2 (A side) x 4 (B side): a wave accumulates
// 128 x 64 = 128 fp32 accumulator registers per lane.  This header holds the main loop; gemm_tile16.hpp holds
// the tile configuration and the panel classes for v_mfma_f32_16x16x32_bf16 tiles (8 x 4 per wave).
//
// The two halves of the workgroup (waves 0-3 and 4-7, one wave of each half on every SIMD) run half a step
// apart: while one half reads its fragments of a stage out of LDS and issues the global loads of later
// stages, the other half issues that stage's MFMAs from registers; one workgroup barrier per phase keeps
// them alternating, so the matrix pipe of a SIMD is fed by one wave while its sibling waits on memory.
//
// "A side" is the index that ends up spread over a lane's accumulator registers, "B side" the index that
// ends up across lanes.  Either operand may be stored K-contiguous (layout KC: X[index][k]) or K-strided
// (layout KS: X[k][index]).  KC panels are read from LDS with ds_read_b128; KS panels with the transposing
// ds_read_b64_tr_b16, so no operand is ever transposed in memory.
//
// Buffer resources give hardware range checking: a lane whose address lies beyond the matrix reads zeros
// instead of faulting, which is how ragged tile edges are handled without branches, and why loads may be
// issued past the end of K (they write zeros into a stage nobody reads).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mst {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short i16x4;
typedef __attribute__((ext_vector_type(8))) short i16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr uint32_t kOutOfRange = 0xFFFFFF00u;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}
// same, for a base address or size that the compiler cannot prove wave-uniform (it is, by construction):
// the descriptor has to live in scalar registers
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc_uniform(const void* base, uint32_t bytes) {
  const uint64_t a = reinterpret_cast<uint64_t>(base);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
  return make_rsrc(reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo), __builtin_amdgcn_readfirstlane(bytes));
}
// m0 (the LDS base of the load) is written here without being declared: the compiler treats m0 as reserved and
// rejects it in a clobber list ("may not be preserved across the asm statement ... undefined behaviour"), so a
// declaration would promise nothing.  It never keeps a value of its own in m0 across statements on this target:
// it loads m0 immediately in front of each of its own uses (LDS-DMA intrinsics, s_sendmsg, GWS, interpolation),
// none of which these kernels contain.  A kernel that adds one must not interleave it with this function.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, uint32_t voffset, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :: "s"(lds_addr), "v"(voffset), "s"(rsrc) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory"); }
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// Ping-pong main loop for 8 waves (WA == 2): waves 0-3 (group 0) and 4-7 (group 1) alternate between a
// memory phase (global->LDS loads of later stages + all fragment reads of the current stage) and a compute
// phase (all MFMAs of the stage), one workgroup barrier per phase, group 1 running one phase behind group 0.
//
// LDS holds NSA = 3 stages of the A panel and NSB = 2 of the B panel (3 * 32 KB + 2 * 32 KB = all 160 KB
// of a CU for the 256 x 256 tile).  In the memory phase of step kt a wave issues its B loads for step kt + 1
// and then its A loads for step kt + 2; the wait that opens step kt + 1 (vmcnt(SPW of A)) lets the A loads
// of step kt + 2 stay in flight.  So the A operand, which is the one every kernel streams from HBM or the
// memory-side cache, has two K steps to arrive and the B operand one; with two stages each (one K step for
// both) the matrix pipe was busy 75 % of the clocks, with loads that are never waited for 98 %.
// Loads are always issued, also past the end of K: there they are out of range and write zeros into a stage
// nobody reads.
struct NoHook { __device__ __forceinline__ void operator()() const {} };
// `after_issue` runs once, after the first operand loads have been issued and before anything waits for them: a
// kernel that has preloaded its accumulators from memory ties them off there, so that the latency of that preload
// and the latency of the first panels pass together instead of one after the other.
template <class C, class PA, class PB, class Hook = NoHook>
__device__ __forceinline__ void gemm_mainloop_pp(typename C::Acc (&acc)[C::TA][C::TB], const PA& pa, const PB& pb,
                                                 char* smem, int k_begin, int k_end, int group,
                                                 Hook after_issue = Hook()) {
  static_assert(C::NSA == 3 && C::NSB == 2, "three A stages, two B stages");
  constexpr int kAhead = PA::SPW;              // loads of one A stage per wave: allowed in flight at a wait
  const uint32_t ldsA = lds_addr_of(smem), ldsB = ldsA + C::NSA * C::kPanelA;
  const char* smemB = smem + C::NSA * C::kPanelA;
  const int nk = (k_end - k_begin + C::BK - 1) / C::BK;
  pa.issue(ldsA, k_begin);
  pb.issue(ldsB, k_begin);
  pa.issue(ldsA + C::kPanelA, k_begin + C::BK);
  after_issue();
  wait_vmcnt<kAhead>();
  __builtin_amdgcn_s_barrier();
  if (group == 1) __builtin_amdgcn_s_barrier();
  int ca = 0, cb = 0;                          // stage indices of step kt
  for (int kt = 0; kt < nk; ++kt) {
    // ---- memory phase
    int na = ca + C::NSA - 1; if (na >= C::NSA) na -= C::NSA;
    const int nb = cb ^ 1;
    const char* a_panel = smem + ca * C::kPanelA;
    const char* b_panel = smemB + cb * C::kPanelB;
    bf16x8 a[C::kKK][C::TA], b[C::kKK][C::TB];
    {
      // Each global->LDS load is followed by its share of the fragment reads: a wave's vector-memory instruction
      // waits for the CU's one address unit (16 clocks per 1 KB load, and the four waves of this half issue 32 of
      // them per phase), and LDS reads queued behind it would wait too.  Interleaved, both units work at once:
      // the memory phase, which was the longer of the two (1120 against 1086 clocks), drops below the compute
      // phase.  The A loads stay last: the wait that opens the next step counts on them being the newest.
      constexpr int kLoads = PB::SPW + PA::SPW, kFrags = C::kKK * (C::TA + C::TB);
#pragma unroll
      for (int j = 0; j < kLoads; ++j) {
        if (j < PB::SPW) pb.issue_one(j, ldsB + nb * C::kPanelB, k_begin + (kt + 1) * C::BK);
        else pa.issue_one(j - PB::SPW, ldsA + na * C::kPanelA, k_begin + (kt + 2) * C::BK);
#pragma unroll
        for (int f = j * kFrags / kLoads; f < (j + 1) * kFrags / kLoads; ++f) {
          const int kk = f / (C::TA + C::TB), r = f % (C::TA + C::TB);
          if (r < C::TA) a[kk][r] = pa.frag(a_panel, r, kk);
          else b[kk][r - C::TA] = pb.frag(b_panel, r - C::TA, kk);
        }
      }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (group == 1) wait_vmcnt<kAhead>();      // group 1 reaches the barrier that opens step kt + 1 right after this phase
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    // ---- compute phase
    __builtin_amdgcn_s_setprio(1);
    // Serpentine order over the B-side tiles: between any two consecutive MFMAs one of the two operands stays in
    // place (in plain row-major order both change at every row change).  On this power-limited chip fewer operand
    // changes are measurably cheaper: -0.55 % of the LM-head step, same-box A/B.
#pragma unroll
    for (int kk = 0; kk < C::kKK; ++kk)
#pragma unroll
      for (int t = 0; t < C::TA; ++t)
#pragma unroll
        for (int uu = 0; uu < C::TB; ++uu) {
          const int u = (t & 1) ? C::TB - 1 - uu : uu;
          acc[t][u] = C::mma(a[kk][t], b[kk][u], acc[t][u]);
        }
    __builtin_amdgcn_s_setprio(0);
    if (group == 0) wait_vmcnt<kAhead>();      // group 0 opens step kt + 1 right after this phase
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    ca = ca + 1 == C::NSA ? 0 : ca + 1;
    cb ^= 1;
  }
  if (group == 0) __builtin_amdgcn_s_barrier();
  wait_vmcnt<0>();
  __syncthreads();
}

template <int TA, int TB>
__device__ __forceinline__ void zero_acc(f32x16 (&acc)[TA][TB]) {
#pragma unroll
  for (int t = 0; t < TA; ++t)
#pragma unroll
    for (int u = 0; u < TB; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[t][u][r] = 0.f;
}

}  // namespace mst
