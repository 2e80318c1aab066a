// Host side of the mini-sequence LM-head + cross-entropy library: argument
// validation, the chunk schedule over the M mini-sequences (Algorithm 2 lines
// 1-3 and Algorithm 4 lines 1-4 of the paper: partition, then loop; for the
// backward also the choice between that loop and blocks of rows x vocabulary
// windows of the same size), workspace carving, launches, and the optional
// per-kernel event timing.
#include "../../include/mst_lmhead.h"
#include "host_util.hpp"
#include "mst_kernels.hpp"

#include <atomic>
#include <mutex>

namespace {

using namespace mst;

constexpr int kNumCu = 256;          // MI355X compute units; only steers the schedule choices (splits, blocks)
constexpr int kMaxDhSplit = 16;
constexpr int kMaxWindows = 64;      // most vocabulary windows the block schedule considers

// Override of the backward order, per calling thread: a caller that forces an order cannot change the
// summation order of a call another thread is making at the same time.
thread_local int t_bwd_schedule = MST_BWD_SCHEDULE_AUTO;

using mst_host::align_up;
using mst_host::misaligned;

struct Plan {
  int64_t S, d, V;
  int M;
  int C;            // rows per chunk = ceil(S / M)
  int n_chunks;     // non-empty chunks = ceil(S / C)
  int64_t fwd_group_rows;   // rows whose log-sum-exp partials are merged by one launch: a whole number of chunks
  int ldg;          // leading dimension of the dlogits workspace (V rounded up to 8)
  int n_vt;         // vocabulary tiles
  int n_jt;         // hidden tiles
  int n_st;         // row tiles of a full chunk
  int dh_split;     // splits of the dH contraction over V
  int dh_ksteps;    // K steps (of kBK) per split
  // forward workspace (byte offsets)
  size_t f_nll, f_tgt, f_part, f_total;
  // backward workspace: two dlogits slots of one chunk each (bf16), contiguous
  size_t b_slot;      // bytes of one slot = C * ldg * 2
  size_t b_total;     // 2 * b_slot: what the call needs when lse and n_valid are supplied
  size_t b_ctl;       // offset of the control block used when n_valid is not supplied (aligned, after the slots)
  size_t b_lse;       // offset of the lse scratch used when lse is not supplied
  size_t b_fwd;       // offset of the forward region used when lse is not supplied
  size_t b_total_max; // bytes needed when neither lse nor n_valid is supplied
  // Block schedule of the backward pass (used when blk_use): the same b_total bytes hold dlogits of blk_rows rows
  // by blk_win_tiles * kTile vocabulary entries (bf16, leading dimension blk_ldg) and, behind it, fp32 dH sums of
  // blk_rows x d.  blk_n_rb row blocks x blk_n_win vocabulary windows cover S x V.
  bool blk_use;
  bool blk_fused;     // dH and dW of a block from one launch
  int blk_rows, blk_n_rb, blk_win_tiles, blk_n_win, blk_ldg;
  size_t blk_acc;     // byte offset of the dH sums
  double est_pairs_us, est_blocks_us;   // the cost model's figures (for the record; see choose_schedule)
};

// ------------------------------------------------------------------ backward schedule
// Both schedules recompute each logit once and keep at most b_total bytes of dlogits alive; they differ in
// which block of the S x V dlogits matrix is alive at a time and therefore in how often the fp32 gradients
// are read back and rewritten:
//   pairs   (Algorithm 4 as printed, two mini-sequences per dW pass): blocks of 2C rows x all of V.
//           dW is read and rewritten once per pair after the first; dH is final after each chunk.
//   blocks  R rows x one window of the vocabulary, R as large as the same bytes allow (dlogits of the block
//           plus fp32 dH sums of its rows).  dW of a window accumulates over the row blocks (none to add when
//           R covers S), dH of a row block accumulates over the windows (S*d*4 bytes, far smaller than dW when
//           V >> d).
// The estimate counts rounds of kNumCu workgroups per launch at a nominal time per K step, plus the fp32
// gradient traffic at a nominal bandwidth; it only has to rank the candidates.
constexpr double kUsPerKStep = 1.5;      // one 256 x 256 x 64 block-tile step with one workgroup per CU
constexpr double kRmwBytesPerUs = 4.0e6; // fp32 read-modify-write streams next to a running GEMM
double rounds_us(int64_t tiles, int64_t k) {
  return (double)((tiles + kNumCu - 1) / kNumCu) * (double)((k + kBK - 1) / kBK) * kUsPerKStep;
}

void choose_schedule(Plan* p, int forced) {
  const int64_t S = p->S, d = p->d, V = p->V, C = p->C;
  const int n_vt = p->n_vt, n_jt = p->n_jt;
  // pairs
  double pairs = 0.0;
  for (int ia = 0; ia < p->n_chunks; ia += 2) {
    int64_t rows_pair = 0;
    for (int i = ia; i < ia + 2 && i < p->n_chunks; ++i) {
      const int64_t rows = (S - (int64_t)i * C) < C ? (S - (int64_t)i * C) : C;
      const int64_t n_st = (rows + kTile - 1) / kTile;
      rows_pair += rows;
      pairs += rounds_us(n_st * n_vt, d);                                                  // dlogits
      pairs += rounds_us(n_st * n_jt * p->dh_split, (int64_t)p->dh_ksteps * kBK);           // dH
      if (p->dh_split > 1) pairs += 2.0 * (double)(p->dh_split * rows * d * 4) / kRmwBytesPerUs;
    }
    pairs += rounds_us((int64_t)n_vt * n_jt, rows_pair);                                   // dW
    pairs += (double)((ia > 0 ? 8 : 4) * V * d) / kRmwBytesPerUs;
  }
  p->est_pairs_us = pairs;
  // blocks: for every window count, the largest row block that fits, then rows balanced over the blocks
  p->blk_use = false;
  p->blk_fused = false;
  p->est_blocks_us = 0.0;
  double best = 0.0;
  for (int n_win = 2; n_win <= kMaxWindows && n_win <= n_vt; ++n_win) {
    const int win_tiles = (n_vt + n_win - 1) / n_win;
    const int n_win_eff = (n_vt + win_tiles - 1) / win_tiles;
    if (n_win_eff != n_win) continue;                       // same partition as a smaller count
#ifdef MST_FORCE_WINDOWS                                    // measurement builds: rank by measurement, not by the model
    if (n_win != MST_FORCE_WINDOWS) continue;
#endif
    const int64_t ldg_w = (int64_t)win_tiles * kTile;
    const int64_t per_row = ldg_w * 2 + (int64_t)n_jt * kTile * 4;   // dlogits + fp32 dH sums (whole column tiles)
    if (p->b_total < 256 + (size_t)per_row * kTile) continue;
    int64_t R = (int64_t)((p->b_total - 256) / (size_t)per_row) / kTile * kTile;
    const int64_t S_up = (S + kTile - 1) / kTile * kTile;
    if (R > S_up) R = S_up;
    const int n_rb = (int)((S + R - 1) / R);
    R = ((S + n_rb - 1) / n_rb + kTile - 1) / kTile * kTile;
    if (R * ldg_w >= (int64_t(1) << 30) || R * d >= (int64_t(1) << 30)) continue;   // 32-bit offsets inside a block
    double t = 0.0;
    for (int rb = 0; rb < n_rb; ++rb) {
      const int64_t rows = (S - rb * R) < R ? (S - rb * R) : R;
      const int64_t n_st = (rows + kTile - 1) / kTile;
      for (int w = 0; w < n_win; ++w) {
        const int64_t tiles_w = (w + 1) * win_tiles <= n_vt ? win_tiles : n_vt - w * win_tiles;
        const int64_t cols = tiles_w * kTile < V - (int64_t)w * ldg_w ? tiles_w * kTile : V - (int64_t)w * ldg_w;
        t += rounds_us(n_st * tiles_w, d);                                                 // dlogits
        t += (double)((w > 0 ? 4 : 0) + (w + 1 < n_win ? 4 : 2)) * (double)(rows * d) / kRmwBytesPerUs;
        t += (double)((rb > 0 ? 8 : 4) * cols * d) / kRmwBytesPerUs;
        t += rounds_us(n_st * n_jt, cols) + rounds_us(tiles_w * n_jt, rows);               // dH, dW
      }
    }
    // One launch for the dH and the dW tiles of a block: a partly filled last round of dH workgroups is topped up
    // with dW tiles, and one launch boundary per block goes away.  Measured: -0.25 to -0.4 % of the step where both
    // tile counts fill whole rounds anyway (configs 2 and 3: 512 and 1008 tiles), -1.5 to -2 % where they do not
    // (Gemma shape: 896 dH tiles = 3.5 rounds; config 5: 496).  The automatic choice always takes it; the block
    // shapes are ranked as separate launches.
    const bool fuse = forced == MST_BWD_SCHEDULE_BLOCKS_FUSED || forced == MST_BWD_SCHEDULE_AUTO;
    const double t_pick = t;
    if (!p->blk_use || t_pick < best) {
      best = t_pick;
      p->blk_use = true;
      p->blk_fused = fuse;
      p->blk_rows = (int)R; p->blk_n_rb = n_rb; p->blk_win_tiles = win_tiles; p->blk_n_win = n_win;
      p->blk_ldg = (int)ldg_w;
      p->blk_acc = align_up((size_t)R * ldg_w * 2, 256);
    }
  }
  p->est_blocks_us = best;
  if (forced == MST_BWD_SCHEDULE_PAIRS) p->blk_use = false;
  else if (forced == MST_BWD_SCHEDULE_AUTO && p->blk_use && !(best < pairs)) p->blk_use = false;
  // MST_BWD_SCHEDULE_BLOCKS and _BLOCKS_FUSED keep the best block shape whenever one fits
}

// `forced`: one of the MST_BWD_SCHEDULE_* values; only the backward's block shape depends on it.
// `fwd_cap`: if non-zero, the forward's groups of mini-sequences are shortened until the forward workspace fits
// into that many bytes (one mini-sequence per group at least; the caller checks f_total against the cap).
mst_status make_plan(int64_t S, int64_t d, int64_t V, int32_t M, Plan* p, int forced = MST_BWD_SCHEDULE_AUTO,
                     size_t fwd_cap = 0) {
  if (S <= 0 || d <= 0 || V <= 0) return MST_ERR_BAD_SHAPE;
  if (d % 8 != 0) return MST_ERR_BAD_SHAPE;
  if (M < 1 || (int64_t)M > S) return MST_ERR_BAD_M;
  if (V * d >= (int64_t(1) << 31) || d >= (int64_t(1) << 22)) return MST_ERR_BAD_SHAPE;
  const int64_t C = (S + M - 1) / M;
  const int64_t ldg = (V + 7) / 8 * 8;
  if (C * ldg >= (int64_t(1) << 30) || C * d >= (int64_t(1) << 30)) return MST_ERR_BAD_SHAPE;
  p->S = S; p->d = d; p->V = V; p->M = M;
  p->C = (int)C;
  p->n_chunks = (int)((S + C - 1) / C);
  p->ldg = (int)ldg;
  p->n_vt = (int)((V + kTile - 1) / kTile);
  p->n_jt = (int)((d + kTile - 1) / kTile);
  p->n_st = (int)((C + kTile - 1) / kTile);
  // dH: few output tiles, long contraction -> split V so that the workgroups fill whole rounds of kNumCu
  // (one workgroup is resident per CU).  Among the split counts that fit (at most kMaxDhSplit, at most one per
  // K step, partials must fit into the dlogits slot that is free at that moment) take the one with the fullest
  // rounds, with a small penalty per split for the fp32 partials it adds.
  const int out_tiles = p->n_st * p->n_jt;
  const int ksteps = (int)((V + kBK - 1) / kBK);
  const int64_t room = (C * ldg * 2) / (C * d * 4);
  int split = 1;
  double best = -1.0;
  for (int s = 1; s <= kMaxDhSplit && s <= ksteps && (s == 1 || s <= room); ++s) {
    const int wgs = out_tiles * s;
    const int rounds = (wgs + kNumCu - 1) / kNumCu;
    const double score = (double)wgs / ((double)rounds * kNumCu) - 0.002 * s;
    if (score > best) { best = score; split = s; }
  }
  p->dh_ksteps = (ksteps + split - 1) / split;
  p->dh_split = (ksteps + p->dh_ksteps - 1) / p->dh_ksteps;

  // Forward: one GEMM launch per mini-sequence; the (max, sum) pairs per row and vocabulary tile of a group of
  // consecutive mini-sequences are merged by one launch.  A group is as many chunks as fit, with their pairs,
  // into half of one fp32 logits chunk (all of them at the paper-shaped configurations).
  {
    const int64_t per_chunk = ((int64_t)p->n_vt * 8 + 4) * C;
    int64_t g = (C * ldg * 2) / per_chunk;
    if (fwd_cap) {
      const int64_t fixed = (int64_t)sizeof(Control) + (S * 4 + 255) / 256 * 256 + 512;   // control, nll, padding
      const int64_t by_cap = ((int64_t)fwd_cap - fixed) / per_chunk;
      if (g > by_cap) g = by_cap;
    }
    if (g < 1) g = 1;
    if (g > p->n_chunks) g = p->n_chunks;
    p->fwd_group_rows = g * C;
  }
  size_t off = sizeof(Control);
  p->f_nll = off;  off = align_up(off + (size_t)S * 4, 256);
  p->f_tgt = off;  off = align_up(off + (size_t)p->fwd_group_rows * 4, 256);
  p->f_part = off; off = align_up(off + (size_t)p->n_vt * p->fwd_group_rows * 8, 256);
  p->f_total = off;

  p->b_slot = (size_t)C * ldg * 2;
  p->b_total = 2 * p->b_slot;
  p->b_ctl = align_up(p->b_total, 256);
  p->b_lse = p->b_ctl + sizeof(Control);
  p->b_fwd = p->b_lse + align_up((size_t)S * 4, 256);
  p->b_total_max = p->b_fwd + p->f_total;
  choose_schedule(p, forced);
  return MST_OK;
}

// ------------------------------------------------------------------ profiling
mst_host::Profiler g_prof;
struct Scope : mst_host::Scope {
  Scope(hipStream_t s, int k) : mst_host::Scope(g_prof, s, k) {}
};

mst_host::PerDeviceOnce g_attr_once, g_shape_once;
// The tile maps and the schedule's cost model are written for the whole chip: kNumCu compute units in kNumXcd
// XCDs.  A partitioned device (fewer compute units behind one HIP device) would be mis-tiled, so it is refused.
bool device_is_whole_chip(int dev) {
  int cus = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
  return cus == kNumCu;
}
bool set_kernel_attributes() {   // on the current device
  bool ok = true;
  auto set = [&ok](const void* f) {
    if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes) != hipSuccess) ok = false;
  };
  set((const void*)k_fwd_gemm_lse);
  set((const void*)k_bwd_gemm_dlogits);
  set((const void*)k_bwd_gemm_dh);
  set((const void*)k_bwd_gemm_dw<false>);
  set((const void*)k_bwd_gemm_dw<true>);
  set((const void*)k_bwd_gemm_dh_dw<false>);
  set((const void*)k_bwd_gemm_dh_dw<true>);
  return ok;
}

mst_status check_launch() { return hipGetLastError() == hipSuccess ? MST_OK : MST_ERR_LAUNCH; }

mst_status prepare_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MST_ERR_NO_DEVICE;
  if (!g_shape_once.run(dev, [dev] { return device_is_whole_chip(dev); })) {
    (void)hipGetLastError();
    return MST_ERR_NO_DEVICE;
  }
  if (!g_attr_once.run(dev, set_kernel_attributes)) {
    (void)hipGetLastError();
    return MST_ERR_LAUNCH;
  }
  return MST_OK;
}

// forward pass over all chunks: writes lse (if non-null) and nll (if non-null)
// `queue`: eight zeroed ints for the persistent forward launches (nullptr: one workgroup per tile)
mst_status run_forward_chunks(const Plan& p, const __bf16* H, const __bf16* W, const int32_t* labels,
                              int ignore_index, char* ws, float* lse, float* nll, hipStream_t st, int* queue = nullptr) {
  int queue_base = 0;
  float* tgt = reinterpret_cast<float*>(ws + p.f_tgt);
  float2* part = reinterpret_cast<float2*>(ws + p.f_part);
  const size_t stride = (size_t)p.fwd_group_rows;
  for (int64_t g0 = 0; g0 < p.S; g0 += p.fwd_group_rows) {
    const int64_t g_rows = (p.S - g0) < p.fwd_group_rows ? (p.S - g0) : p.fwd_group_rows;
    {
      // One launch for the group's mini-sequences.  Rows are independent and no logits are stored, so the row tiles
      // of the launch need not respect the boundaries between the mini-sequences of the group: a mini-sequence
      // shorter than a 256-row tile costs no idle tile rows, and every row's result is bit-identical for every M.
      const int n_st = (int)((g_rows + kTile - 1) / kTile);
      Scope sc(st, MST_K_FWD_GEMM_LSE);
      const int tiles = xcd_grid_2d(p.n_vt, n_st);
      const int grid = queue && tiles > kNumCu ? kNumCu : tiles;
      hipLaunchKernelGGL(k_fwd_gemm_lse, dim3(grid), dim3(kThreads), kLdsBytes, st,
                         H + g0 * p.d, W, labels + g0, (int)g_rows, (int)p.d, (int)p.V, n_st, p.n_vt,
                         part, stride, tgt, queue, queue_base);
      queue_base += tiles / kNumXcd + grid;
    }
    {
      Scope sc(st, MST_K_LSE_FINALIZE);
      hipLaunchKernelGGL(k_lse_finalize, dim3((unsigned)((g_rows + kFinRows - 1) / kFinRows)), dim3(kFinRows * kFinGroups), 0, st,
                         part, stride, p.n_vt, tgt, labels + g0, (int)g_rows, (int)p.V, ignore_index,
                         lse ? lse + g0 : nullptr, nll ? nll + g0 : nullptr);
    }
  }
  return check_launch();
}

mst_status check_forward_alignment(const void* H, const void* W, const int32_t* labels, const float* loss,
                                   const float* lse, const int64_t* n_valid) {
  if (misaligned(H, 16) || misaligned(W, 16) || misaligned(lse, 4) || misaligned(labels, 4) || misaligned(loss, 4) ||
      misaligned(n_valid, 8))
    return MST_ERR_ALIGNMENT;
  return MST_OK;
}

// label scan, the chunk loop, the loss: everything the forward call enqueues, on workspace `ws` of p.f_total bytes
mst_status enqueue_forward(const Plan& p, const void* H, const void* W, const int32_t* labels, int32_t ignore_index,
                           char* ws, float* loss, float* lse, int64_t* n_valid, void* stream) {
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  Control* ctl = reinterpret_cast<Control*>(ws);
  float* nll = reinterpret_cast<float*>(ws + p.f_nll);
  {
    Scope sc(st, MST_K_LABEL_SCAN);
    hipLaunchKernelGGL(k_label_scan, dim3(1), dim3(1024), 0, st, labels, (long long)p.S, (int)p.V, ignore_index, ctl);
  }
  const mst_status s = run_forward_chunks(p, static_cast<const __bf16*>(H), static_cast<const __bf16*>(W), labels,
                                          ignore_index, ws, lse, nll, st, ctl->queue);
  if (s != MST_OK) return s;
  {
    Scope sc(st, MST_K_LOSS_REDUCE);
    hipLaunchKernelGGL(k_loss_reduce, dim3(1), dim3(1024), 0, st, nll, (long long)p.S, ctl, loss,
                       reinterpret_cast<long long*>(n_valid));
  }
  return check_launch();
}

// Scratch of the entry point that allocates nothing: one array per GPU, part of the code object, alive until
// the process ends.  Its name is only a host-side handle; the device address is asked for once per device
// (with that device current) and kept, and only that address is ever handed to a kernel.
__device__ __align__(256) static unsigned char scratch[MST_STATIC_SCRATCH_BYTES];
std::mutex g_scratch_mu;
char* g_scratch_ptr[mst_host::PerDeviceOnce::kMaxDevices] = {};
char* static_scratch_of_current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= mst_host::PerDeviceOnce::kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = static_cast<char*>(ptr);
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

const char* mst_strerror(mst_status s) {
  switch (s) {
    case MST_OK: return "ok";
    case MST_ERR_NULL_POINTER: return "a required pointer is NULL";
    case MST_ERR_BAD_SHAPE: return "bad shape: S, d, V must be positive, d % 8 == 0, d < 2^22, V*d < 2^31, ceil(S/M)*V < 2^30";
    case MST_ERR_BAD_M: return "M must satisfy 1 <= M <= S";
    case MST_ERR_WORKSPACE: return "workspace is NULL or too small (see mst_workspace_bytes)";
    case MST_ERR_ALIGNMENT: return "pointer alignment: H, W, dH 16 bytes; workspace 256 bytes; lse, dW 4 bytes";
    case MST_ERR_LAUNCH: return "the HIP runtime refused a kernel launch or attribute";
    case MST_ERR_NO_DEVICE: return "no current HIP device, or it is not a whole 256-CU gfx950 chip";
    default: return "unknown status";
  }
}

const char* mst_version(void) { return "mst-lmhead 0.1 (gfx950)"; }

int32_t mst_suggest_m(int64_t S, int64_t d, int64_t V) {
  if (S <= 0 || d <= 0 || V <= 0) return 0;
  int64_t m = (2 * V + d) / (2 * d);             // V / d to the nearest integer
  const int64_t by_rows = S / kTile;             // most chunks that still have one full block tile of rows
  if (m > by_rows) m = by_rows;
  if (m < 1) m = 1;
  if (m > 0x7fffffff) m = 0x7fffffff;
  return (int32_t)m;
}

mst_status mst_mfma_probe(int32_t blocks, int32_t iters, float scale, float* sink, void* stream) {
  if (blocks < 1 || blocks > (1 << 20) || iters < 1 || iters > (1 << 20)) return MST_ERR_BAD_SHAPE;
  if (!sink) return MST_ERR_NULL_POINTER;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MST_ERR_NO_DEVICE;
  hipLaunchKernelGGL(k_mfma_probe, dim3(blocks), dim3(kThreads), 0, reinterpret_cast<hipStream_t>(stream),
                     sink, iters, scale);
  return check_launch();
}

mst_status mst_shift_labels(const int32_t* labels_in, int64_t B, int64_t L, int32_t ignore_index,
                            int32_t* labels_out, void* stream) {
  if (B <= 0 || L <= 0 || B >= (int64_t(1) << 40) / L) return MST_ERR_BAD_SHAPE;
  if (!labels_in || !labels_out) return MST_ERR_NULL_POINTER;
  if (misaligned(labels_in, 4) || misaligned(labels_out, 4)) return MST_ERR_ALIGNMENT;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MST_ERR_NO_DEVICE;
  const long long n = (long long)(B * L);
  hipLaunchKernelGGL(k_shift_labels, dim3((unsigned)((n + 255) / 256)), dim3(256), 0,
                     reinterpret_cast<hipStream_t>(stream), labels_in, n, (long long)L, ignore_index, labels_out);
  return check_launch();
}

mst_status mst_workspace_bytes(int64_t S, int64_t d, int64_t V, int32_t M, size_t* fwd_bytes, size_t* bwd_bytes) {
  Plan p;
  mst_status s = make_plan(S, d, V, M, &p);
  if (s != MST_OK) return s;
  if (fwd_bytes) *fwd_bytes = p.f_total;
  if (bwd_bytes) *bwd_bytes = p.b_total;
  return MST_OK;
}

mst_status mst_lmhead_ce_fwd(const void* H, const void* W, const int32_t* labels, int64_t S, int64_t d, int64_t V,
                             int32_t ignore_index, int32_t M, void* workspace, size_t workspace_bytes,
                             float* loss, float* lse, int64_t* n_valid, void* stream) {
  Plan p;
  mst_status s = make_plan(S, d, V, M, &p);
  if (s != MST_OK) return s;
  if (!H || !W || !labels || !loss) return MST_ERR_NULL_POINTER;
  if (!workspace || workspace_bytes < p.f_total) return MST_ERR_WORKSPACE;
  if (misaligned(workspace, 256)) return MST_ERR_ALIGNMENT;
  if ((s = check_forward_alignment(H, W, labels, loss, lse, n_valid)) != MST_OK) return s;
  if ((s = prepare_device()) != MST_OK) return s;
  return enqueue_forward(p, H, W, labels, ignore_index, static_cast<char*>(workspace), loss, lse, n_valid, stream);
}

mst_status mst_lmhead_ce_fwd_static(const void* H, const void* W, const int32_t* labels, int64_t S, int64_t d, int64_t V,
                                    int32_t ignore_index, int32_t M, float* loss, float* lse, int64_t* n_valid,
                                    void* stream) {
  Plan p;
  mst_status s = make_plan(S, d, V, M, &p, MST_BWD_SCHEDULE_AUTO, (size_t)MST_STATIC_SCRATCH_BYTES);
  if (s != MST_OK) return s;
  if (!H || !W || !labels || !loss) return MST_ERR_NULL_POINTER;
  if (p.f_total > (size_t)MST_STATIC_SCRATCH_BYTES) return MST_ERR_WORKSPACE;   // one mini-sequence alone is too large
  if ((s = check_forward_alignment(H, W, labels, loss, lse, n_valid)) != MST_OK) return s;
  if ((s = prepare_device()) != MST_OK) return s;
  char* ws = static_scratch_of_current_device();
  if (!ws) return MST_ERR_LAUNCH;
  return enqueue_forward(p, H, W, labels, ignore_index, ws, loss, lse, n_valid, stream);
}

mst_status mst_lmhead_ce_bwd(const void* H, const void* W, const int32_t* labels, int64_t S, int64_t d, int64_t V,
                             int32_t ignore_index, int32_t M, float grad_loss, const float* lse,
                             const int64_t* n_valid, void* workspace, size_t workspace_bytes,
                             void* dH, float* dW, void* stream) {
  Plan p;
  mst_status s = make_plan(S, d, V, M, &p, t_bwd_schedule);
  if (s != MST_OK) return s;
  if (!H || !W || !labels || !dH || !dW) return MST_ERR_NULL_POINTER;
  const size_t need = !lse ? p.b_total_max : (!n_valid ? p.b_lse : p.b_total);
  if (!workspace || workspace_bytes < need) return MST_ERR_WORKSPACE;
  if (misaligned(H, 16) || misaligned(W, 16) || misaligned(dH, 16) || misaligned(workspace, 256) ||
      misaligned(lse, 4) || misaligned(dW, 16) || misaligned(labels, 4) || misaligned(n_valid, 8))
    return MST_ERR_ALIGNMENT;
  if ((s = prepare_device()) != MST_OK) return s;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  const __bf16* Hb = static_cast<const __bf16*>(H);
  const __bf16* Wb = static_cast<const __bf16*>(W);
  const long long* nv = reinterpret_cast<const long long*>(n_valid);
  if (!nv) {
    Control* ctl = reinterpret_cast<Control*>(ws + p.b_ctl);
    Scope sc(st, MST_K_LABEL_SCAN);
    hipLaunchKernelGGL(k_label_scan, dim3(1), dim3(1024), 0, st, labels, (long long)S, (int)V, ignore_index, ctl);
    nv = &ctl->n_valid_checked;   // -1 if a label is outside [0, V): dH and dW then come out NaN
  }
  if (!lse) {
    // no saved log-sum-exp: run the forward's pass first, in the tail of the workspace
    float* lse_tmp = reinterpret_cast<float*>(ws + p.b_lse);
    s = run_forward_chunks(p, Hb, Wb, labels, ignore_index, ws + p.b_fwd, lse_tmp, nullptr, st);
    if (s != MST_OK) return s;
    lse = lse_tmp;
  }
  __bf16* slot[2] = {reinterpret_cast<__bf16*>(ws), reinterpret_cast<__bf16*>(ws + p.b_slot)};
  __bf16* dHb = static_cast<__bf16*>(dH);

  auto rows_of = [&](int i) { const int64_t r0 = (int64_t)i * p.C; return (int)((p.S - r0) < p.C ? (p.S - r0) : p.C); };
  auto dlogits = [&](int i, __bf16* G) {
    const int64_t r0 = (int64_t)i * p.C;
    const int rows = rows_of(i), n_st = (rows + kTile - 1) / kTile;
    Scope sc(st, MST_K_BWD_GEMM_DLOGITS);
    hipLaunchKernelGGL(k_bwd_gemm_dlogits, dim3(xcd_grid_2d(p.n_vt, n_st)), dim3(kThreads), kLdsBytes, st,
                       Hb + r0 * p.d, Wb, labels + r0, lse + r0, rows, (int)p.d, (int)p.V, 0, (int)p.V, ignore_index,
                       n_st, p.n_vt, G, p.ldg);
  };
  auto grad_h = [&](int i, const __bf16* G, void* partial_space) {
    const int64_t r0 = (int64_t)i * p.C;
    const int rows = rows_of(i), n_st = (rows + kTile - 1) / kTile;
    float* partial = static_cast<float*>(partial_space);
    {
      Scope sc(st, MST_K_BWD_GEMM_DH);
      hipLaunchKernelGGL(k_bwd_gemm_dh, dim3(xcd_grid(n_st * p.n_jt * p.dh_split)), dim3(kThreads), kLdsBytes, st,
                         G, p.ldg, Wb, rows, (int)p.d, (int)p.V, n_st, p.n_jt, p.dh_split, p.dh_ksteps, kDhSplit,
                         nv, grad_loss, partial, p.C, dHb + r0 * p.d);
    }
    if (p.dh_split > 1) {
      Scope sc(st, MST_K_BWD_DH_REDUCE);
      const size_t n = (size_t)rows * p.d;
      hipLaunchKernelGGL(k_bwd_dh_reduce, dim3((unsigned)((n / 8 + 255) / 256)), dim3(256), 0, st,
                         partial, p.dh_split, (size_t)p.C * p.d, n, nv, grad_loss, dHb + r0 * p.d);
    }
  };
  auto grad_w = [&](int i_first, int i_last, int rows) {
    const int64_t r0 = (int64_t)i_first * p.C;
    Scope sc(st, MST_K_BWD_GEMM_DW);
    hipLaunchKernelGGL(i_first > 0 ? k_bwd_gemm_dw<false> : k_bwd_gemm_dw<true>, dim3(xcd_grid_2d(p.n_vt, p.n_jt)),
                       dim3(kThreads), kLdsBytes, st,
                       slot[0], p.ldg, Hb + r0 * p.d, rows, (int)p.d, (int)p.V, p.n_vt, p.n_jt,
                       i_last == p.n_chunks - 1 ? 1 : 0, nv, grad_loss, dW);
  };

  if (p.blk_use) {
    // Block schedule: for each block of rows, walk the vocabulary windows.  Per (row block, window):
    //   dlogits of the block -> workspace | dH sums of the row block (+)= G W_window | dW_window (+)= G^T H_block
    // dH of a row block is final after its last window, dW of a window after the last row block; both
    // accumulate in a fixed order.
    __bf16* G = reinterpret_cast<__bf16*>(ws);
    float* dh_sums = reinterpret_cast<float*>(ws + p.blk_acc);
    for (int rb = 0; rb < p.blk_n_rb; ++rb) {
      const int64_t r0 = (int64_t)rb * p.blk_rows;
      const int rows = (int)((p.S - r0) < p.blk_rows ? (p.S - r0) : p.blk_rows);
      const int n_st = (rows + kTile - 1) / kTile;
      for (int w = 0; w < p.blk_n_win; ++w) {
        const int t0 = w * p.blk_win_tiles;
        const int tiles_w = t0 + p.blk_win_tiles <= p.n_vt ? p.blk_win_tiles : p.n_vt - t0;
        const int64_t v_base = (int64_t)t0 * kTile;
        const int Vw = (int)((p.V - v_base) < (int64_t)tiles_w * kTile ? (p.V - v_base) : (int64_t)tiles_w * kTile);
        {
          Scope sc(st, MST_K_BWD_GEMM_DLOGITS);
          hipLaunchKernelGGL(k_bwd_gemm_dlogits, dim3(xcd_grid_2d(tiles_w, n_st)), dim3(kThreads), kLdsBytes, st,
                             Hb + r0 * p.d, Wb + v_base * p.d, labels + r0, lse + r0, rows, (int)p.d, Vw, (int)v_base,
                             (int)p.V, ignore_index, n_st, tiles_w, G, p.blk_ldg);
        }
        const int mode = w == 0 ? kDhFirst : (w == p.blk_n_win - 1 ? kDhLast : kDhAdd);
        const int dw_last = rb == p.blk_n_rb - 1 ? 1 : 0;
        if (p.blk_fused) {
          Scope sc(st, MST_K_BWD_GEMM_DH_DW);
          const int dh_grid = xcd_grid_2d(n_st, p.n_jt);
          hipLaunchKernelGGL(rb > 0 ? k_bwd_gemm_dh_dw<false> : k_bwd_gemm_dh_dw<true>,
                             dim3(dh_grid + xcd_grid_2d(tiles_w, p.n_jt)), dim3(kThreads), kLdsBytes, st,
                             G, p.blk_ldg, Wb + v_base * p.d, Hb + r0 * p.d, rows, (int)p.d, Vw, n_st, tiles_w, p.n_jt,
                             dh_grid, mode, dw_last, nv, grad_loss, dh_sums, p.blk_rows, dHb + r0 * p.d,
                             dW + v_base * p.d);
        } else {
          {
            Scope sc(st, MST_K_BWD_GEMM_DH);
            hipLaunchKernelGGL(k_bwd_gemm_dh, dim3(xcd_grid_2d(n_st, p.n_jt)), dim3(kThreads), kLdsBytes, st,
                               G, p.blk_ldg, Wb + v_base * p.d, rows, (int)p.d, Vw, n_st, p.n_jt, 1, (Vw + kBK - 1) / kBK, mode,
                               nv, grad_loss, dh_sums, p.blk_rows, dHb + r0 * p.d);
          }
          {
            Scope sc(st, MST_K_BWD_GEMM_DW);
            hipLaunchKernelGGL(rb > 0 ? k_bwd_gemm_dw<false> : k_bwd_gemm_dw<true>, dim3(xcd_grid_2d(tiles_w, p.n_jt)),
                               dim3(kThreads), kLdsBytes, st,
                               G, p.blk_ldg, Hb + r0 * p.d, rows, (int)p.d, Vw, tiles_w, p.n_jt,
                               dw_last, nv, grad_loss, dW + v_base * p.d);
          }
        }
      }
    }
    return check_launch();
  }

  // Algorithm 4's loop over mini-sequences, two at a time: the chunk pair (A, B) shares one dW pass.
  //   dlogits(A) -> slot 0 | dH(A), partials in slot 1 | dlogits(B) -> slot 1 | dW += [G_A; G_B]^T [H_A; H_B]
  //   | dH(B), partials in slot 0
  for (int ia = 0; ia < p.n_chunks; ia += 2) {
    const int ib = ia + 1;
    dlogits(ia, slot[0]);
    grad_h(ia, slot[0], slot[1]);
    if (ib < p.n_chunks) {
      dlogits(ib, slot[1]);
      grad_w(ia, ib, p.C + rows_of(ib));
      grad_h(ib, slot[1], slot[0]);
    } else {
      grad_w(ia, ia, rows_of(ia));
    }
  }
  return check_launch();
}

mst_status mst_set_bwd_schedule(int32_t schedule) {
  if (schedule < MST_BWD_SCHEDULE_AUTO || schedule > MST_BWD_SCHEDULE_BLOCKS_FUSED) return MST_ERR_BAD_SHAPE;
  t_bwd_schedule = schedule;
  return MST_OK;
}

mst_status mst_bwd_schedule_info(int64_t S, int64_t d, int64_t V, int32_t M, int64_t* info) {
  return mst_bwd_schedule_info_for(S, d, V, M, t_bwd_schedule, info);
}

mst_status mst_bwd_schedule_info_for(int64_t S, int64_t d, int64_t V, int32_t M, int32_t schedule, int64_t* info) {
  if (!info) return MST_ERR_NULL_POINTER;
  if (schedule < MST_BWD_SCHEDULE_AUTO || schedule > MST_BWD_SCHEDULE_BLOCKS_FUSED) return MST_ERR_BAD_SHAPE;
  Plan p;
  const mst_status s = make_plan(S, d, V, M, &p, schedule);
  if (s != MST_OK) return s;
  info[0] = p.blk_use ? (p.blk_fused ? MST_BWD_SCHEDULE_BLOCKS_FUSED : MST_BWD_SCHEDULE_BLOCKS) : MST_BWD_SCHEDULE_PAIRS;
  info[1] = p.blk_use ? p.blk_rows : 2 * (int64_t)p.C;
  info[2] = p.blk_use ? p.blk_n_rb : (p.n_chunks + 1) / 2;
  info[3] = p.blk_use ? (int64_t)p.blk_win_tiles * kTile : p.V;
  info[4] = p.blk_use ? p.blk_n_win : 1;
  info[5] = p.blk_use ? 1 : p.dh_split;
  info[6] = (int64_t)p.est_pairs_us;
  info[7] = (int64_t)p.est_blocks_us;
  return MST_OK;
}

int32_t mst_tile_of_workgroup(int32_t n_slow, int32_t n_fast, int32_t order, int32_t workgroup, int32_t* slow,
                              int32_t* fast) {
  if (n_slow < 1 || n_fast < 1 || workgroup < 0 || !slow || !fast || order < 0 || order > 1) return -1;
  if (workgroup >= xcd_grid_2d(n_slow, n_fast)) return -1;
  int s = 0, f = 0;
  const bool ok = order == 0
      ? xcd_tile_of_block<kXcdRectSlow, kXcdRectFast, kXcdSuper>(workgroup, n_slow, n_fast, &s, &f)
      : xcd_tile_of_block<kXcdRectSlow, kXcdRectFast, kXcdRectFast>(workgroup, n_slow, n_fast, &s, &f);
  *slow = s;
  *fast = f;
  return ok ? 1 : 0;
}

int32_t mst_tile_grid(int32_t n_slow, int32_t n_fast) {
  if (n_slow < 1 || n_fast < 1 || (int64_t)xcd_grid_2d(n_slow, 1) * n_fast > 0x7fffffff) return -1;
  return xcd_grid_2d(n_slow, n_fast);
}

mst_status mst_profile_enable(int every) {
  g_prof.enable(every);
  return MST_OK;
}

mst_status mst_profile_collect(double* ms_per_kind, int64_t* launches_per_kind, int64_t* issued_per_kind) {
  return g_prof.collect(MST_PROFILE_KINDS, ms_per_kind, launches_per_kind, issued_per_kind) ? MST_OK : MST_ERR_LAUNCH;
}

const char* mst_profile_kind_name(int kind) {
  static const char* names[MST_PROFILE_KINDS] = {
      "label_scan", "fwd_gemm_lse", "lse_finalize", "loss_reduce",
      "bwd_gemm_dlogits", "bwd_gemm_dh", "bwd_dh_reduce", "bwd_gemm_dw", "bwd_gemm_dh_dw"};
  return (kind >= 0 && kind < MST_PROFILE_KINDS) ? names[kind] : "?";
}

}  // extern "C"
