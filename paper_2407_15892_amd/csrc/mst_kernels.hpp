// Device kernels of the mini-sequence LM-head + cross-entropy path (gfx950).
//
// Per mini-sequence (chunk) of C rows, following Algorithm 2 (forward) and
// Algorithm 4 (backward with recomputation) of the paper:
//
//   forward   k_fwd_gemm_lse     logits tile = W_tile H_chunk^T in MFMA accumulators; per row the
//                                running max / sum-exp of the tile's 256 vocabulary entries and the
//                                target logit are taken from the accumulators; no logits are stored
//             k_lse_finalize     per row: combine the per-vocab-tile partials into lse, nll
//   backward  k_bwd_gemm_dlogits logits tile again; softmax - onehot via the saved lse; bf16 to workspace
//             k_bwd_gemm_dh      dH_chunk = dlogits W       (contraction over V, split, fixed-order reduce)
//             k_bwd_gemm_dw      dW (+)= dlogits^T H_chunk  (contraction over the chunk's rows)
//
// All kernels use the 256 x 256 block tile main loop of gemm_tile.hpp.  The
// linear workgroup id is remapped so that each of the 8 XCDs (which receive
// workgroups round-robin and own a private L2) works on a contiguous range of
// the tile space: workgroups that share an operand panel then share an L2.
#pragma once
#include "gemm_tile.hpp"
#include "gemm_tile16.hpp"

namespace mst {

// tile configuration: 2 x 4 waves, wave tile 128 x 64, K step 64, LDS stages 3 (A) + 2 (B), 8 x 4 tiles of
// v_mfma_f32_16x16x32_bf16 per wave (on random operands this power-limited chip sustains more flop/s with it than
// with v_mfma_f32_32x32x16_bf16, whose only advantage -- 128-byte instead of 64-byte row pieces in fp32 epilogues --
// went away when the fp32 intermediates moved to accumulator order)
typedef Cfg16<2, 4, 8, 4, 64, 2> Tile16;
constexpr int kTA16 = Tile16::TA, kTB16 = Tile16::TB;
// same wave grid, half as wide on the B side: 256 x 128 block tile, wave tile 128 x 32
typedef Cfg16<2, 4, 8, 2, 64, 2> Tile16HalfB;
constexpr int kTile = 256;             // Tile16::EA == Tile16::EB
constexpr int kBK = Tile16::BK;
constexpr int kThreads = Tile16::kThreads;
constexpr int kLdsBytes = Tile16::kLds;
static_assert(Tile16::EA == kTile && Tile16::EB == kTile && kLdsBytes == 5 * 32768, "square 256 x 256 block tile, all of LDS");

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kMasked = -1.0e30f;     // stands for -infinity in max / sum-exp without producing NaN
constexpr int kNumXcd = 8;

// Control block in the workspace, written by k_label_scan (n_valid is its first member).
struct Control {
  long long n_valid;    // rows whose label is neither ignored nor out of range
  int bad_labels;       // rows whose label is outside [0, V) and not the ignore value
  int pad0;
  long long n_valid_checked;   // n_valid, or -1 if bad_labels > 0: what a caller (or the backward pass) is handed
  int queue[8];         // per-XCD tile queues of the persistent forward launch (see TileFeed); zeroed by the label scan
  int pad[50];
};
static_assert(sizeof(Control) == 256, "control block is one 256-byte line");

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// gamma = grad_loss / N_valid (Algorithm 4 lines 9-10 and the mean of the loss), 0 when nothing is valid.
// A negative count is the forward's (or the label scan's) report of a label outside [0, V): the gradients
// are then NaN throughout, like the loss.
__device__ __forceinline__ float gamma_of(const long long* __restrict__ n_valid, float grad_loss) {
  const long long nv = *n_valid;
  if (nv < 0) return __builtin_nanf("");
  return nv > 0 ? (float)((double)grad_loss / (double)nv) : 0.f;
}

// XCD-aware remap of the linear workgroup id to a work item; returns -1 for padding workgroups.
__device__ __forceinline__ int xcd_work_item(int total) {
  const int per_xcd = (total + kNumXcd - 1) / kNumXcd;
  const int b = blockIdx.x;
  const int w = (b % kNumXcd) * per_xcd + b / kNumXcd;
  return w < total ? w : -1;
}
inline int xcd_grid(int total) { return kNumXcd * ((total + kNumXcd - 1) / kNumXcd); }

// Remap for a 2-D tile space (n_slow x n_fast) in which every tile reads one panel per coordinate.  Each XCD owns a
// contiguous range of the slow coordinate.  Its 32 resident workgroups (one "round") form a kRectSlow x kRectFast
// rectangle of tiles (12 distinct panels for 32 workgroups; a 1 x 32 strip would read 33), and the rounds walk
//   for each super-group of kSuper fast tiles:  for each band of kRectSlow slow tiles of the XCD:  for each kRectFast
//   fast tiles of the super-group
// With kSuper > kRectFast consecutive rounds keep the same slow panels while the fast panels of a super-group, which
// all XCDs walk at the same time, stay in the memory-side cache for the XCD's whole slow range: in the forward kernel
// (slow = vocabulary, fast = rows; W, 1 GB, cannot stay in any cache) W is streamed from HBM once per 8192 rows
// instead of once per 1024 (forward pass -2.4 % against kSuper = kRectFast, -6 % against 8 x 4 rectangles walked
// fast-group by fast-group).  With kSuper = kRectFast the fast panels are the ones kept from round to round; the
// dlogits kernel, whose window of W is in the memory-side cache anyway, is 2 % faster that way.  Returns false for
// padding workgroups.
template <int kRectSlow, int kRectFast, int kSuper>
__host__ __device__ inline bool xcd_tile_of_block(int block, int n_slow, int n_fast, int* slow, int* fast) {
  static_assert(kSuper % kRectFast == 0, "a super-group is a whole number of rectangles");
  const int x = block % kNumXcd;
  int q = block / kNumXcd;
  const int spx = (n_slow + kNumXcd - 1) / kNumXcd;          // slow tiles per XCD
  if (q >= spx * n_fast) return false;
  const int per_super = spx * kSuper;                        // super-group of fast tiles
  const int sup = q / per_super;
  q -= sup * per_super;
  const int f0 = sup * kSuper;
  const int fs = n_fast - f0 < kSuper ? n_fast - f0 : kSuper;
  const int per_band = kRectSlow * fs;                       // band of kRectSlow slow tiles
  const int band = q / per_band;
  q -= band * per_band;
  const int s0 = band * kRectSlow;
  const int ss = spx - s0 < kRectSlow ? spx - s0 : kRectSlow;
  const int per_rect = ss * kRectFast;                       // rectangle: ss x (up to kRectFast) tiles
  const int rect = q / per_rect;
  q -= rect * per_rect;
  const int g0 = rect * kRectFast;
  const int gs = fs - g0 < kRectFast ? fs - g0 : kRectFast;
  const int sl = q / gs;
  *slow = x * spx + s0 + sl;
  *fast = f0 + g0 + (q - sl * gs);
  return *slow < n_slow;
}
constexpr int kXcdRectSlow = 4, kXcdRectFast = 8, kXcdSuper = 32;
// a kernel that serves several tile spaces passes its own workgroup index as `block`
__device__ __forceinline__ bool xcd_tile_2d(int n_slow, int n_fast, int* slow, int* fast, int block = -1) {
  return xcd_tile_of_block<kXcdRectSlow, kXcdRectFast, kXcdSuper>(block < 0 ? (int)blockIdx.x : block, n_slow, n_fast, slow, fast);
}
// the same with the fast panels kept from round to round
__device__ __forceinline__ bool xcd_tile_2d_fast_major(int n_slow, int n_fast, int* slow, int* fast) {
  return xcd_tile_of_block<kXcdRectSlow, kXcdRectFast, kXcdRectFast>((int)blockIdx.x, n_slow, n_fast, slow, fast);
}
__host__ __device__ inline int xcd_grid_2d(int n_slow, int n_fast) { return kNumXcd * ((n_slow + kNumXcd - 1) / kNumXcd) * n_fast; }

// Persistent workgroups that pull their tiles from per-XCD queues instead of owning one tile each.
//
// A launch of `grid` tiles in the maps above gives XCD x the workgroup indices x, x + 8, x + 16, ...: a list of
// per_xcd = grid / 8 entries that its 32 resident workgroups take in order.  Here the launch has one workgroup per
// compute unit, and workgroup b (on XCD b % 8, as the hardware deals them out) takes the next entry of its XCD's
// list with an atomic add on queue[b % 8] -- the same order, so the rectangles of tiles that share operand panels
// in an XCD's L2 are the same -- and, when that list is used up, goes on to the lists of the other XCDs: an XCD
// that runs faster than the others (they differ by several per cent) takes over work of the slower ones, and the
// launch ends with all compute units busy instead of with the slowest XCD.  Nobody waits for anybody: a workgroup
// leaves when it has found all 8 lists used up.
//
// The counters are not reset between launches.  Every workgroup fails exactly once on every list, so a launch
// leaves each counter at its old value + per_xcd + number of workgroups, which the host adds up into `base` for the
// next launch on the same counters.  Thread 0 fetches; the index reaches the other threads through one LDS word in
// the third A stage.  The fetch for the tile after this one is issued at the start of a tile and collected behind
// the first operand loads of its main loop.
//
// Only the forward launch works this way.  It runs 250 rounds of tiles at the benchmark shape, so a difference of a
// few per cent between XCDs adds up to several whole tiles (forward pass -2.3 %, same-box A/B); the backward launches
// run 2 to 8 rounds, the difference never reaches one tile, and the queue bought nothing there (dlogits -0.2 %,
// dH + dW 0).

// The lane index, opaque to the compiler.  In a persistent kernel everything a tile body derives from the lane index
// alone (panel offsets, output offsets) is invariant over the loop over tiles; hoisted out of it, those values would
// have to live through the main loop, whose accumulators and fragments leave no registers free, and be spilled -- and
// each reload (a vector-memory operation) would wait for the operand loads issued before it.  Read through this
// function inside the loop they are recomputed per tile instead, which costs nothing next to a tile.
__device__ __forceinline__ int lane_index_per_tile() {
  int lane = (int)(threadIdx.x & 63);
  asm volatile("" : "+v"(lane));
  return lane;
}

constexpr int kFeedWordOffset = 2 * 32768;
struct TileFeed {
  int* queue;
  int base, per_xcd, x, visited;
  int pending;          // wave 0: the index fetched for the tile after the current one (uniform, lives in a scalar register)
  int raw;              // thread 0: the atomic's result on its way back
  char* smem;
  __device__ __forceinline__ void init(int* q, int base_, int per_xcd_, char* smem_) {
    queue = q; base = base_; per_xcd = per_xcd_; smem = smem_;
    x = (int)(blockIdx.x % kNumXcd); visited = 0; pending = 0; raw = 0;
    issue();
    resolve();
  }
  // Thread 0 asks for the next entry of the current list.  Called at the start of a tile; resolve() is called behind
  // the main loop's first operand loads, where the wave waits for memory anyway, and moves the answer into a scalar
  // register (a vector register kept across the tile would be spilled, and the spill would wait for the answer at
  // once).  Only wave 0 takes part.
  __device__ __forceinline__ void issue() {
    if (threadIdx.x == 0) raw = atomicAdd(queue + x, 1);        // nothing may touch the result before resolve()
  }
  __device__ __forceinline__ void resolve() {
    if (__builtin_amdgcn_readfirstlane(threadIdx.x >> 6) == 0) pending = __builtin_amdgcn_readfirstlane(raw) - base;
  }
  // index of the next tile in the launch's static map, or -1 when every list is used up; all threads call it
  __device__ __forceinline__ int next() {
    int* word = reinterpret_cast<int*>(smem + kFeedWordOffset);
    __syncthreads();                         // the previous tile's epilogue may still be reading LDS
    if (threadIdx.x == 0) {
      int t = pending;
      while (t >= per_xcd) {
        if (++visited == kNumXcd) { t = -1; break; }
        x = (x + 1) % kNumXcd;
        t = atomicAdd(queue + x, 1) - base;
      }
      *word = t < 0 ? -1 : t * kNumXcd + x;
    }
    __syncthreads();
    const int block = __builtin_amdgcn_readfirstlane(*word);
    __syncthreads();                         // a tile body may write this part of LDS before its first barrier
    return block;
  }
};

// ---------------------------------------------------------------------------
// label scan: N_valid and range check.  One workgroup, integer sums only.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void k_label_scan(const int* __restrict__ labels, long long S, int V,
                                                     int ignore_index, Control* ctl) {
  __shared__ long long s_valid[16];
  __shared__ int s_bad[16];
  long long nv = 0;
  int nb = 0;
  for (long long i = threadIdx.x; i < S; i += 1024) {
    const int y = labels[i];
    if (y != ignore_index) {
      if ((unsigned)y < (unsigned)V) ++nv; else ++nb;
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    nv += __shfl_xor(nv, o);
    nb += __shfl_xor(nb, o);
  }
  if ((threadIdx.x & 63) == 0) { s_valid[threadIdx.x >> 6] = nv; s_bad[threadIdx.x >> 6] = nb; }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long tv = 0; int tb = 0;
    for (int i = 0; i < 16; ++i) { tv += s_valid[i]; tb += s_bad[i]; }
    ctl->n_valid = tv;
    ctl->bad_labels = tb;
    ctl->n_valid_checked = tb > 0 ? -1 : tv;
  }
  if (threadIdx.x < kNumXcd) ctl->queue[threadIdx.x] = 0;
}

// register-resident MFMA loop: the matrix-core rate the chip sustains without any data movement
__global__ __launch_bounds__(kThreads) void k_mfma_probe(float* sink, int iters, float scale) {
  constexpr int kTA = 4, kTB = 2;          // 4 x 2 tiles of 32 x 32: 128 accumulator registers, as in the GEMM kernels
  f32x16 acc[kTA][kTB];
  zero_acc<kTA, kTB>(acc);
  bf16x8 a[8], b[8];
  uint32_t s = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      s = s * 1664525u + 1013904223u;
      a[i][e] = (__bf16)(scale * ((int)(s >> 8) % 20001 - 10000) * 1e-4f);
      s = s * 1664525u + 1013904223u;
      b[i][e] = (__bf16)(scale * ((int)(s >> 8) % 20001 - 10000) * 1e-4f);
    }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int t = 0; t < kTA; ++t)
#pragma unroll
        for (int u = 0; u < kTB; ++u)
          acc[t][u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(t + 4 * kk) & 7], b[(u + 2 * t + 4 * kk) & 7], acc[t][u], 0, 0, 0);
  }
  float tot = 0.f;
#pragma unroll
  for (int t = 0; t < kTA; ++t)
#pragma unroll
    for (int u = 0; u < kTB; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) tot += acc[t][u][r];
  if (tot == 1.2345e-30f) *sink = tot;
}

// next-token alignment: the label of position t of a sequence is the token at t + 1; the last position has none
__global__ __launch_bounds__(256) void k_shift_labels(const int* __restrict__ in, long long n, long long L,
                                                      int ignore_index, int* __restrict__ out) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  out[i] = (i % L == L - 1) ? ignore_index : in[i + 1];
}

// ---------------------------------------------------------------------------
// forward: logits tile + running log-sum-exp partials + target logit
//   A side = vocabulary (W rows), B side = chunk rows (H rows): a lane owns one
//   row s and 32 consecutive vocabulary entries, so the row reduction is in-lane
//   plus exchanges with the other three lane quarters and the other wave row.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_fwd_gemm_lse(
    const __bf16* __restrict__ Hc, const __bf16* __restrict__ W, const int* __restrict__ labels_c,
    int rows, int d, int V, int n_st, int n_vt, float2* __restrict__ part, size_t part_stride,
    float* __restrict__ tgt, int* __restrict__ queue, int queue_base) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave >> 2, wb = wave & 3;
  TileFeed feed;
  if (queue) feed.init(queue, queue_base, xcd_grid_2d(n_vt, n_st) / kNumXcd, smem);
  for (int block = queue ? feed.next() : (int)blockIdx.x; block >= 0; block = queue ? feed.next() : -1) {
  int vt, st;                                        // an XCD's resident workgroups: 4 vocabulary x 8 row tiles
  if (!xcd_tile_2d(n_vt, n_st, &vt, &st, block)) {   // padding entry of the map
    if (queue) { feed.issue(); feed.resolve(); }
    continue;
  }
  if (queue) feed.issue();
  const int lane = lane_index_per_tile();
  const int v0 = vt * kTile, s0 = st * kTile;

  f32x4 acc[kTA16][kTB16];
  zero_acc<kTA16, kTB16>(acc);
  PanelKC16<Tile16, kTile, kTA16, true> pa;
  PanelKC16<Tile16, kTile, kTB16, false> pb;
  pa.init(W + (size_t)v0 * d, d, V - v0, d, wave, lane, wa);
  pb.init(Hc + (size_t)s0 * d, d, rows - s0, d, wave, lane, wb);
  gemm_mainloop_pp<Tile16>(acc, pa, pb, smem, 0, d, wa, [&]() { if (queue) feed.resolve(); });

  // a lane (quarter g, column c) holds, for each of its 4 rows s, the 32 consecutive vocabulary entries
  // va + 4 t + r (t = 0..7, r = 0..3)
  const int g = lane >> 4, c = lane & 15;
  const int va = v0 + wa * 128 + 32 * g;
  if (v0 + kTile > V) {                              // ragged last vocabulary tile: mask entries >= V
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (va + 4 * t + r >= V) {
#pragma unroll
          for (int u = 0; u < kTB16; ++u) acc[t][u][r] = kMasked;
        }
  }

  float2* xch = reinterpret_cast<float2*>(smem);     // [wb][u][16] pairs from the wa == 1 waves
  float m_u[kTB16], l_u[kTB16];
#pragma unroll
  for (int u = 0; u < kTB16; ++u) {
    float m = kMasked;
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) m = fmaxf(m, acc[t][u][r]);
    float l = 0.f;
    // subtract before scaling: with the masking sentinel, a fused (z * log2e - m * log2e)
    // would leave a huge rounding residue when z == m == sentinel
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) l += fast_exp2((acc[t][u][r] - m) * kLog2e);
    // the four lane quarters hold four 32-entry slices of the same rows
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
      const float m2 = __shfl_xor(m, o), l2 = __shfl_xor(l, o);
      const float mm = fmaxf(m, m2);
      l = l * fast_exp2((m - mm) * kLog2e) + l2 * fast_exp2((m2 - mm) * kLog2e);
      m = mm;
    }
    m_u[u] = m;
    l_u[u] = l;

    // target logit straight from the accumulator that holds it
    const int s_local = s0 + wb * 64 + 16 * u + c;
    const int y = s_local < rows ? labels_c[s_local] : -1;
    const int rel = y - (v0 + wa * 128);
    if (rel >= 0 && rel < 128 && y < V && (rel >> 5) == g) {
      const int t_sel = (rel & 31) >> 2, r_sel = rel & 3;
      float val = 0.f;
#pragma unroll
      for (int t = 0; t < kTA16; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (t == t_sel && r == r_sel) val = acc[t][u][r];
      tgt[s_local] = val;
    }
  }
  // the main loop ended with a barrier, LDS is free
  if (wa == 1 && lane < 16) {
#pragma unroll
    for (int u = 0; u < kTB16; ++u) xch[(wb * kTB16 + u) * 16 + lane] = make_float2(m_u[u], l_u[u]);
  }
  __syncthreads();
  if (wa == 0 && lane < 16) {
#pragma unroll
    for (int u = 0; u < kTB16; ++u) {
      const float2 o = xch[(wb * kTB16 + u) * 16 + lane];
      const float mm = fmaxf(m_u[u], o.x);
      const float l = l_u[u] * fast_exp2((m_u[u] - mm) * kLog2e) + o.y * fast_exp2((o.x - mm) * kLog2e);
      const int s_local = s0 + wb * 64 + 16 * u + lane;
      if (s_local < rows) part[(size_t)vt * part_stride + s_local] = make_float2(mm, l);
    }
  }
  }
}

// per row: combine the vocab-tile partials into lse and nll.  A workgroup owns 64 rows; its 16
// waves each fold every 16th vocabulary tile in ascending order, then the 16 partial results are
// folded in wave order: the combination order is fixed, so lse is reproducible bit for bit.
constexpr int kFinRows = 64;
constexpr int kFinGroups = 16;
__global__ __launch_bounds__(kFinRows * kFinGroups) void k_lse_finalize(
    const float2* __restrict__ part, size_t part_stride, int n_vt, const float* __restrict__ tgt,
    const int* __restrict__ labels_c, int rows, int V, int ignore_index,
    float* __restrict__ lse_c, float* __restrict__ nll_c) {
  __shared__ float2 sh[kFinGroups][kFinRows];
  const int r = threadIdx.x & (kFinRows - 1), g = threadIdx.x / kFinRows;
  const int s = blockIdx.x * kFinRows + r;
  float m = kMasked, l = 0.f;
  if (s < rows) {
    for (int vt = g; vt < n_vt; vt += kFinGroups) {
      const float2 p = part[(size_t)vt * part_stride + s];
      const float mm = fmaxf(m, p.x);
      l = l * fast_exp2((m - mm) * kLog2e) + p.y * fast_exp2((p.x - mm) * kLog2e);
      m = mm;
    }
  }
  sh[g][r] = make_float2(m, l);
  __syncthreads();
  if (g != 0 || s >= rows) return;
  for (int q = 1; q < kFinGroups; ++q) {
    const float2 p = sh[q][r];
    const float mm = fmaxf(m, p.x);
    l = l * fast_exp2((m - mm) * kLog2e) + p.y * fast_exp2((p.x - mm) * kLog2e);
    m = mm;
  }
  const float log_l = __builtin_amdgcn_logf(l) * kLn2;     // v_log_f32 is log2
  const float lse = m + log_l;
  const int y = labels_c[s];
  const bool valid = (y != ignore_index) && ((unsigned)y < (unsigned)V);
  if (lse_c) lse_c[s] = lse;
  // nll = lse - z_y as (m - z_y) + log l: for a confidently predicted label (z_y = m or close to it) the first term is
  // exact and the small second one keeps its relative precision, where m + log l would round it to the grid of m
  if (nll_c) nll_c[s] = valid ? (m - tgt[s]) + log_l : 0.f;
}

// loss = sum(nll) / n_valid, fixed summation order, fp64 accumulation.  One workgroup.
__global__ __launch_bounds__(1024) void k_loss_reduce(const float* __restrict__ nll, long long S,
                                                      const Control* __restrict__ ctl,
                                                      float* __restrict__ loss, long long* __restrict__ n_valid_out) {
  __shared__ double sh[1024];
  double a = 0.0;
  for (long long i = threadIdx.x; i < S; i += 1024) a += (double)nll[i];
  sh[threadIdx.x] = a;
  __syncthreads();
  for (int o = 512; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const long long nv = ctl->n_valid;
    if (ctl->bad_labels > 0) {
      *loss = __builtin_nanf("");
      if (n_valid_out) *n_valid_out = -1;
    } else {
      *loss = nv > 0 ? (float)(sh[0] / (double)nv) : 0.f;
      if (n_valid_out) *n_valid_out = nv;
    }
  }
}

// ---------------------------------------------------------------------------
// backward 1: recompute the logits tile, write softmax - onehot as bf16
//   (kept unscaled so that the label entry p - 1 stays within 2^-9 of -1, its nearest bf16 neighbour in most
//   rows; the factor gamma = grad_loss / N_valid is applied in fp32 by the two gradient GEMMs)
// ---------------------------------------------------------------------------
// The kernel works on a window of the vocabulary: W points at the window's first row, V is the number of
// vocabulary entries from there on, G column 0 is the window's first entry; v_base is that entry's absolute
// index and V_all the whole vocabulary (both only for the labels).  The row-chunk schedule passes the whole
// vocabulary (v_base = 0, V = V_all).
__global__ __launch_bounds__(kThreads) void k_bwd_gemm_dlogits(
    const __bf16* __restrict__ Hc, const __bf16* __restrict__ W, const int* __restrict__ labels_c,
    const float* __restrict__ lse_c, int rows, int d, int V, int v_base, int V_all, int ignore_index, int n_st, int n_vt,
    __bf16* __restrict__ G, int ldg) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int vt, st;                                        // an XCD's resident workgroups: 4 vocabulary x 8 row tiles
  if (!xcd_tile_2d_fast_major(n_vt, n_st, &vt, &st)) return;
  const int v0 = vt * kTile, s0 = st * kTile;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave >> 2, wb = wave & 3;

  f32x4 acc[kTA16][kTB16];
  zero_acc<kTA16, kTB16>(acc);
  PanelKC16<Tile16, kTile, kTA16, true> pa;
  PanelKC16<Tile16, kTile, kTB16, false> pb;
  pa.init(W + (size_t)v0 * d, d, V - v0, d, wave, lane, wa);
  pb.init(Hc + (size_t)s0 * d, d, rows - s0, d, wave, lane, wb);
  gemm_mainloop_pp<Tile16>(acc, pa, pb, smem, 0, d, wa);

  // Epilogue in two steps.  A lane holds 64 contiguous bytes of each of its 4 token rows, and the lanes of a wave
  // instruction hold 16 different rows: stored directly, every instruction is 64 separate 16-byte writes, and the
  // 8192 of them per tile cost 9 us (the whole difference to the forward kernel).  So the bf16 tile is first
  // staged in LDS (free after the main loop; rows padded to 528 bytes, which spreads the 16 rows of a quarter wave
  // over all banks), then every wave instruction writes two whole 512-byte rows.
  constexpr int kStageRow = kTile * 2 + 16;
  const int va = v0 + wa * 128 + 32 * (lane >> 4);   // this lane's 32 consecutive vocabulary entries start here
  if (v0 + kTile > V) {                              // ragged last vocabulary tile: entries >= V must come out as 0
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        if (va + 4 * t + r >= V) {
#pragma unroll
          for (int u = 0; u < kTB16; ++u) acc[t][u][r] = kMasked;
        }
  }
#pragma unroll
  for (int u = 0; u < kTB16; ++u) {
    const int row = wb * 64 + 16 * u + (lane & 15);
    const int s_local = s0 + row;
    if (s_local >= rows) continue;
    const int y_abs = labels_c[s_local];
    const bool valid = (y_abs != ignore_index) && ((unsigned)y_abs < (unsigned)V_all);
    // z - lse is formed first and scaled afterwards: where a class dominates (z close to lse) the difference is exact,
    // so p - 1 at a confidently predicted label keeps full precision, and a one-class vocabulary gives exactly 0.
    // An ignored row takes lse = +infinity: every p is then exp2(-infinity) = 0 without a select per element, and
    // its label index is moved out of range so that nothing is subtracted.
    const float lse_s = valid ? lse_c[s_local] : __builtin_inff();
    const int y_lane = valid ? y_abs - v_base - va : -1;   // the label's position among this lane's 32 entries, if it is there
    char* srow = smem + row * kStageRow + (wa * 128 + 32 * (lane >> 4)) * 2;
#pragma unroll
    for (int p = 0; p < kTA16 / 2; ++p) {            // tiles 2p and 2p + 1: entries va + 8p .. + 7
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e)
        o[e] = (__bf16)fast_exp2((acc[2 * p + (e >> 2)][u][e & 3] - lse_s) * kLog2e);
      *reinterpret_cast<bf16x8*>(srow + 16 * p) = o;
    }
    // The label's entry, p - 1, is patched in afterwards by the one lane that holds it (a lane holds 32 of the V
    // entries of its row, so for most waves nobody does and the branch is skipped): a compare and a select per
    // element of every row would cost a third of this epilogue's instructions.
    if ((unsigned)y_lane < 32u) {
      float z_y = 0.f;
#pragma unroll
      for (int t = 0; t < kTA16; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (4 * t + r == y_lane) z_y = acc[t][u][r];
      *reinterpret_cast<__bf16*>(srow + 2 * y_lane) = (__bf16)(fast_exp2((z_y - lse_s) * kLog2e) - 1.0f);
    }
  }
  __syncthreads();
  {
    const int col = (lane & 31) * 8;                 // 8 entries = 16 bytes per lane, 32 lanes per row
    const bool col_ok = v0 + col < ldg;
#pragma unroll
    for (int i = 0; i < kTile / (2 * Tile16::kWaves); ++i) {
      const int row = (kTile / Tile16::kWaves) * wave + 2 * i + (lane >> 5);
      if (s0 + row < rows && col_ok)     // streamed past L2: nobody on this XCD reads the block back (-0.4 % of the step)
        __builtin_nontemporal_store(*reinterpret_cast<const bf16x8*>(smem + row * kStageRow + col * 2),
                                    reinterpret_cast<bf16x8*>(G + (size_t)(s0 + row) * ldg + v0 + col));
    }
  }
}

// ---------------------------------------------------------------------------
// backward 2: dH_chunk = G W over a range of the vocabulary
//   A side = chunk rows (G, K-contiguous), B side = hidden index j (W, K-strided)
// ---------------------------------------------------------------------------
// mode (the kDh* constants):
//   kDhSplit  one launch covers the whole contraction: n_split > 1 writes fp32 partials for k_bwd_dh_reduce,
//             n_split == 1 writes gamma * result as bf16 (the row-chunk schedule)
//   kDhFirst / kDhAdd / kDhLast  the contraction arrives in several launches, one per vocabulary window
//             (n_split must be 1): the first stores the fp32 sums into `partial`, the middle ones add to them, the
//             last adds and writes gamma * total as bf16.  Launches run in order on one stream, so the summation
//             order is fixed.  Nobody else reads these sums, so they are kept in accumulator order, not row-major:
//             tile (st, jt) owns 256 KB at partial + (st * n_jt + jt) * 65536 floats, and in it the four registers
//             of accumulator (t, u) of wave w, lane l sit at float ((w * 32 + t * 4 + u) * 64 + l) * 4 -- one 16-byte
//             load or store per accumulator and lane, 1 KB contiguous per wave instruction, whole tiles always
//             (no masks; the padding of ragged tiles is written and read back like the rest and never leaves).
constexpr int kDhSplit = 0, kDhFirst = 1, kDhAdd = 2, kDhLast = 3;
// The body is a device function (block = index of the workgroup within this kernel's tile space) so that a
// launch can serve the dH and the dW tiles of a vocabulary window together.
__device__ __forceinline__ void dh_tile(
    const __bf16* __restrict__ G, int ldg, const __bf16* __restrict__ W, int rows, int d, int V,
    int n_st, int n_jt, int n_split, int ksteps_per_split, int mode,
    const long long* __restrict__ n_valid, float grad_loss,
    float* __restrict__ partial /* [n_split][rows_stride][d] */, int rows_stride,
    __bf16* __restrict__ dHc /* written by kDhSplit with n_split == 1 and by kDhLast */, int block, char* smem) {
  int st, jt, sp = 0;
  if (mode == kDhSplit) {
    const int w = xcd_work_item(n_st * n_jt * n_split);   // not combined with other tile spaces: uses blockIdx.x
    if (w < 0) return;
    st = w % n_st;
    jt = (w / n_st) % n_jt;
    sp = w / (n_st * n_jt);
  } else if (!xcd_tile_2d(n_st, n_jt, &st, &jt, block)) {   // many row tiles: rectangles of row x hidden tiles per XCD
    return;
  }
  const int s0 = st * kTile, j0 = jt * kTile;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave >> 2, wb = wave & 3;
  const int k_begin = sp * ksteps_per_split * kBK;
  int k_end = k_begin + ksteps_per_split * kBK;
  if (k_end > V) k_end = V;

  // fp32 view of this tile's rows in the partial / running-sum array: a buffer descriptor over the valid rows
  // (scalar base, 32-bit offsets, rows past the end dropped by the range check), columns masked per lane.
  // Register r of accumulator tile (t, u) is row wa * 128 + 16 t + 4 (lane / 16) + r, column wb * 64 + 16 u + lane % 16.
  const int rows_valid = rows - s0 < kTile ? rows - s0 : kTile;
  float* const part = mode == kDhSplit ? partial + (size_t)sp * rows_stride * d : partial;
  const __amdgpu_buffer_rsrc_t sums = make_rsrc_uniform(part + (size_t)s0 * d, (uint32_t)rows_valid * (uint32_t)d * 4u);
  uint32_t lane_off[kTB16];
  bool col_ok[kTB16];
#pragma unroll
  for (int u = 0; u < kTB16; ++u) {
    const int j = j0 + wb * 64 + 16 * u + (lane & 15);
    col_ok[u] = j < d;
    lane_off[u] = ((uint32_t)(wa * 128 + 4 * (lane >> 4)) * (uint32_t)d + (uint32_t)j) * 4u;
  }
  auto row_off = [&](int t, int r) { return (uint32_t)(16 * t + r) * (uint32_t)d * 4u; };

  f32x4 acc[kTA16][kTB16];
  zero_acc<kTA16, kTB16>(acc);
  typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
  const __amdgpu_buffer_rsrc_t tile_sums =
      make_rsrc_uniform(partial + ((size_t)st * n_jt + jt) * (size_t)(kTile * kTile), (uint32_t)(kTile * kTile * 4));
  const uint32_t slot0 = (uint32_t)(wave * (kTA16 * kTB16) * 64 + lane) * 16u;      // this lane's slot of accumulator (0, 0)
  if (mode == kDhAdd || mode == kDhLast) {
    // the running sums of the earlier windows go straight into the accumulators (the loads fly while the first
    // operand panels arrive) and are tied off so that the compiler puts no wait for them into the main loop
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int u = 0; u < kTB16; ++u)
        acc[t][u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(tile_sums, slot0 + (t * kTB16 + u) * 1024, 0, 0));
  }
  // The preloaded sums are tied off behind the first operand loads (see gemm_mainloop_pp), not in front of them --
  // on every path, also where nothing was preloaded: behind a condition the compiler would carry "loads pending"
  // past it on the other path and wait for them in front of the MFMAs of every K step.
  auto tie_off = [&]() {
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int u = 0; u < kTB16; ++u) asm volatile("" : "+v"(acc[t][u]));
  };
  PanelKC16<Tile16, kTile, kTA16, false> pa;
  PanelKS16<Tile16, kTile, kTB16> pb;
  pa.init(G + (size_t)s0 * ldg, ldg, rows - s0, ldg, wave, lane, wa);
  pb.init(W + j0, d, V, d - j0, wave, lane, wb);
  gemm_mainloop_pp<Tile16>(acc, pa, pb, smem, k_begin, k_end, wa, tie_off);

  const bool to_bf16 = mode == kDhLast || (mode == kDhSplit && n_split == 1);
  if (!to_bf16) {
    if (mode == kDhSplit) {        // partials for k_bwd_dh_reduce: row-major
#pragma unroll
      for (int u = 0; u < kTB16; ++u)
        if (col_ok[u]) {
#pragma unroll
          for (int t = 0; t < kTA16; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[t][u][r]), sums, lane_off[u] + row_off(t, r), 0, 0);
        }
    } else {                       // running sums for the next window: accumulator order
#pragma unroll
      for (int t = 0; t < kTA16; ++t)
#pragma unroll
        for (int u = 0; u < kTB16; ++u)
          __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[t][u]), tile_sums, slot0 + (t * kTB16 + u) * 1024, 0, 0);
    }
    return;
  }
  // bf16 result: the lanes of a wave instruction hold 16 adjacent columns of 4 rows, 32 bytes per row; staged in
  // LDS (free after the main loop; rows padded to 528 bytes) the tile leaves as whole 512-byte rows
  const float gamma = gamma_of(n_valid, grad_loss);
  constexpr int kStageRow = kTile * 2 + 16;
#pragma unroll
  for (int t = 0; t < kTA16; ++t)
#pragma unroll
    for (int u = 0; u < kTB16; ++u)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        *reinterpret_cast<__bf16*>(smem + (wa * 128 + 16 * t + 4 * (lane >> 4) + r) * kStageRow +
                                   (wb * 64 + 16 * u + (lane & 15)) * 2) = (__bf16)(gamma * acc[t][u][r]);
  __syncthreads();
  const int col = (lane & 31) * 8;                   // 8 columns = 16 bytes per lane, 32 lanes per row
  const bool out_ok = j0 + col < d;                  // d % 8 == 0
#pragma unroll
  for (int i = 0; i < kTile / (2 * Tile16::kWaves); ++i) {
    const int row = (kTile / Tile16::kWaves) * wave + 2 * i + (lane >> 5);
    if (s0 + row < rows && out_ok)
      *reinterpret_cast<bf16x8*>(dHc + (size_t)(s0 + row) * d + j0 + col) =
          *reinterpret_cast<const bf16x8*>(smem + row * kStageRow + col * 2);
  }
}

__global__ __launch_bounds__(kThreads) void k_bwd_gemm_dh(
    const __bf16* __restrict__ G, int ldg, const __bf16* __restrict__ W, int rows, int d, int V,
    int n_st, int n_jt, int n_split, int ksteps_per_split, int mode,
    const long long* __restrict__ n_valid, float grad_loss,
    float* __restrict__ partial, int rows_stride, __bf16* __restrict__ dHc) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  dh_tile(G, ldg, W, rows, d, V, n_st, n_jt, n_split, ksteps_per_split, mode, n_valid, grad_loss, partial, rows_stride,
          dHc, blockIdx.x, smem);
}

// fixed-order sum over the splits, scale by gamma, round to bf16.  8 outputs per thread.
__global__ __launch_bounds__(256) void k_bwd_dh_reduce(const float* __restrict__ partial, int n_split,
                                                       size_t split_stride /* rows_stride * d */, size_t n /* rows * d */,
                                                       const long long* __restrict__ n_valid, float grad_loss,
                                                       __bf16* __restrict__ dHc) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n) return;
  const float gamma = gamma_of(n_valid, grad_loss);
  float4 a0 = *reinterpret_cast<const float4*>(partial + i);
  float4 a1 = *reinterpret_cast<const float4*>(partial + i + 4);
  for (int sp = 1; sp < n_split; ++sp) {
    const float4 b0 = *reinterpret_cast<const float4*>(partial + sp * split_stride + i);
    const float4 b1 = *reinterpret_cast<const float4*>(partial + sp * split_stride + i + 4);
    a0.x += b0.x; a0.y += b0.y; a0.z += b0.z; a0.w += b0.w;
    a1.x += b1.x; a1.y += b1.y; a1.z += b1.z; a1.w += b1.w;
  }
  bf16x8 o;
  o[0] = (__bf16)(gamma * a0.x); o[1] = (__bf16)(gamma * a0.y); o[2] = (__bf16)(gamma * a0.z); o[3] = (__bf16)(gamma * a0.w);
  o[4] = (__bf16)(gamma * a1.x); o[5] = (__bf16)(gamma * a1.y); o[6] = (__bf16)(gamma * a1.z); o[7] = (__bf16)(gamma * a1.w);
  *reinterpret_cast<bf16x8*>(dHc + i) = o;
}

// ---------------------------------------------------------------------------
// backward 3: dW (+)= G^T H over the rows that are in the workspace (two consecutive chunks, or a
// block of rows of one vocabulary window)
//   A side = vocabulary (G columns, K-strided), B side = hidden index j (H columns, K-strided)
//   dW is fp32 and is its own accumulator.  For every pass over a part of dW after the first the
//   old tile is loaded straight into the MFMA accumulators before the main loop, the products are
//   accumulated on top, and the tile is stored once: one read and one write of dW per pass and no
//   extra registers.  Because dlogits is kept as bf16, twice as many of them fit as fp32 logits
//   would, so a pass covers two chunks (or, with a window of the vocabulary, many more rows) and dW
//   is read and written correspondingly less often.  The running sum is kept unscaled; the last
//   pass multiplies by gamma = grad_loss / N_valid.  Passes run in order on one stream, so the
//   summation order is fixed and dW is reproducible bit for bit.
//   The body is a device function so that the MLP path can serve its three weight gradients from one launch.
// ---------------------------------------------------------------------------
// G: [rows][ldg], columns [0, g_cols) readable (v < V of them used); Hc: [rows][ldh], columns [0, d) used;
// dW: [V][ldw], columns [0, d) written
//
// Between the passes over one dW tile (`accumulate`: an earlier pass has stored it; `more`: a later pass will add
// to it) nobody else reads the tile, so a whole tile (256 rows and 256 columns inside the matrix) is kept in
// accumulator order inside its own footprint: wave instruction (w, t, u) moves row 32 w + 4 t + u of the tile's 256
// rows of 1 KB, lane l its bytes 16 l .. 16 l + 15 -- the four registers of accumulator (t, u).  One 16-byte load or
// store per accumulator and lane, 1 KB contiguous per wave instruction, straight between memory and the
// accumulators.  Only the last pass (more == 0) writes the matrix in row-major order, through LDS as whole 1 KB rows.
// Tiles on a ragged edge keep row-major order throughout: 64-byte row pieces out, and in through LDS.
__device__ __forceinline__ void dw_tile(
    const __bf16* __restrict__ G, int ldg, int g_cols, const __bf16* __restrict__ Hc, int ldh, int rows, int d, int V,
    int vt, int jt, int accumulate, int more, float scale, float* __restrict__ dW, int ldw, char* smem) {
  const int v0 = vt * kTile, j0 = jt * kTile;
  int lane = lane_index_per_tile();       // read once more behind the main loop: nothing derived from it lives through it
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wa = wave >> 2, wb = wave & 3;
  const int rows_valid = V - v0 < kTile ? V - v0 : kTile;
  const __amdgpu_buffer_rsrc_t out = make_rsrc_uniform(dW + (size_t)v0 * ldw, (uint32_t)rows_valid * (uint32_t)ldw * 4u);
  constexpr int kNonTemporal = 2;
  typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
  const bool whole = rows_valid == kTile && j0 + kTile <= d;
  auto slot = [&](int t, int u) {         // accumulator order inside the tile's footprint
    return ((uint32_t)(wave * (kTA16 * kTB16) + t * kTB16 + u) * (uint32_t)ldw + (uint32_t)j0) * 4u + (uint32_t)lane * 16u;
  };
  f32x4 acc[kTA16][kTB16];
  zero_acc<kTA16, kTB16>(acc);
  if (accumulate && whole) {
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int u = 0; u < kTB16; ++u)
        acc[t][u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(out, slot(t, u), 0, kNonTemporal));
  } else if (accumulate) {
    // The old tile comes in through LDS, which is free before the main loop: whole 1 KB rows, one wave instruction
    // each (in the accumulator layout a lane's elements are 64-byte row pieces), two halves of 128 rows.  Half h
    // holds tile rows 128 w + 64 h + (0..63) of both wave rows w.  The 16-byte pieces of LDS row p are XORed by
    // 4 * ((p / 4) % 4), so that the four lane quarters of a read (rows 4 apart) fall on four bank groups.
    typedef __attribute__((address_space(3))) const float* lds_f32_ptr;
    const uint32_t lds0 = lds_addr_of(smem);
    const int g = lane >> 4, c = lane & 15;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int p = 16 * wave + i;
        const uint32_t tile_row = 128 * (p >> 6) + 64 * h + (p & 63);
        const uint32_t piece = (uint32_t)lane ^ (4u * ((p >> 2) & 3));
        dma16(out, j0 + 4 * (int)piece < d ? (tile_row * (uint32_t)ldw + (uint32_t)j0 + 4u * piece) * 4u : kOutOfRange,
              lds0 + p * 1024);
      }
      wait_vmcnt<0>();
      __syncthreads();
#pragma unroll
      for (int tt = 0; tt < kTA16 / 2; ++tt)
#pragma unroll
        for (int u = 0; u < kTB16; ++u)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int p = 64 * wa + 16 * tt + 4 * g + r;
            const int piece = (16 * wb + 4 * u + (c >> 2)) ^ (4 * g);
            acc[kTA16 / 2 * h + tt][u][r] = *(lds_f32_ptr)(uintptr_t)(lds0 + p * 1024 + piece * 16 + (c & 3) * 4);
          }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __syncthreads();
    }
  }
  // the directly loaded tile is tied off behind the first operand loads (see gemm_mainloop_pp), on every path
  auto tie_off = [&]() {
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int u = 0; u < kTB16; ++u) asm volatile("" : "+v"(acc[t][u]));
  };
  PanelKS16<Tile16, kTile, kTA16> pa;
  PanelKS16<Tile16, kTile, kTB16> pb;
  pa.init(G + v0, ldg, rows, g_cols - v0, wave, lane, wa);
  pb.init(Hc + j0, ldh, rows, d - j0, wave, lane, wb);
  gemm_mainloop_pp<Tile16>(acc, pa, pb, smem, 0, rows, wa, tie_off);
  lane = lane_index_per_tile();
#pragma unroll
  for (int t = 0; t < kTA16; ++t)
#pragma unroll
    for (int u = 0; u < kTB16; ++u) acc[t][u] *= scale;
  if (more && whole) {
#pragma unroll
    for (int t = 0; t < kTA16; ++t)
#pragma unroll
      for (int u = 0; u < kTB16; ++u)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[t][u]), out, slot(t, u), 0, kNonTemporal);
    return;
  }
  if (whole) {
    // row-major result of a whole tile: through LDS (free after the main loop), out as whole 1 KB rows, 16 bytes per
    // lane; the direct stores below are 64-byte row pieces, half cache lines
    typedef __attribute__((address_space(3))) float* lds_f32_w;
    typedef __attribute__((address_space(3))) const u32x4* lds_u4_r;
    const uint32_t lds0 = lds_addr_of(smem);
    const int g = lane >> 4, c = lane & 15;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (h) __syncthreads();
#pragma unroll
      for (int tt = 0; tt < kTA16 / 2; ++tt)
#pragma unroll
        for (int u = 0; u < kTB16; ++u)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int p = 64 * wa + 16 * tt + 4 * g + r;
            const int piece = (16 * wb + 4 * u + (c >> 2)) ^ (4 * g);
            *(lds_f32_w)(uintptr_t)(lds0 + p * 1024 + piece * 16 + (c & 3) * 4) = acc[kTA16 / 2 * h + tt][u][r];
          }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int p = 16 * wave + i;
        const uint32_t tile_row = 128 * (p >> 6) + 64 * h + (p & 63);
        const uint32_t piece = (uint32_t)lane ^ (4u * ((p >> 2) & 3));
        const u32x4 v = *(lds_u4_r)(uintptr_t)(lds0 + p * 1024 + lane * 16);
        __builtin_amdgcn_raw_buffer_store_b128(v, out, (tile_row * (uint32_t)ldw + (uint32_t)j0 + 4u * piece) * 4u, 0, kNonTemporal);
      }
    }
    return;
  }
  // tiles on a ragged edge: register r of accumulator (t, u) is row wa * 128 + 16 t + 4 (lane / 16) + r, column
  // wb * 64 + 16 u + lane % 16; rows past the end are dropped by the descriptor's range check, columns masked per lane
#pragma unroll
  for (int u = 0; u < kTB16; ++u) {
    const int j = j0 + wb * 64 + 16 * u + (lane & 15);
    const uint32_t lane_off = ((uint32_t)(wa * 128 + 4 * (lane >> 4)) * (uint32_t)ldw + (uint32_t)j) * 4u;
    if (j < d) {
#pragma unroll
      for (int t = 0; t < kTA16; ++t)
#pragma unroll
        for (int r = 0; r < 4; ++r)
          __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(acc[t][u][r]), out,
                                                lane_off + (uint32_t)(16 * t + r) * (uint32_t)ldw * 4u, 0, kNonTemporal);
    }
  }
}

template <bool kStoreOnly>
__global__ __launch_bounds__(kThreads) void k_bwd_gemm_dw(
    const __bf16* __restrict__ G, int ldg, const __bf16* __restrict__ Hc, int rows, int d, int V,
    int n_vt, int n_jt, int last, const long long* __restrict__ n_valid, float grad_loss,
    float* __restrict__ dW) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int vt, jt;
  if (!xcd_tile_2d(n_vt, n_jt, &vt, &jt)) return;
  const float scale = last ? gamma_of(n_valid, grad_loss) : 1.0f;
  dw_tile(G, ldg, ldg, Hc, d, rows, d, V, vt, jt, kStoreOnly ? 0 : 1, last ? 0 : 1, scale, dW, d, smem);
}

// dH and dW of one (row block, vocabulary window) from one launch: both read the same dlogits block and
// neither depends on the other.  The first dh_grid workgroups take the dH tiles (the longer ones: their
// contraction runs over the window, dW's over the rows), the rest the dW tiles; with one workgroup per CU the
// hardware hands out tiles as CUs become free, so the two tile spaces share one partly filled last round
// instead of leaving one each.  dh_grid = xcd_grid_2d(n_st, n_jt), a multiple of the XCD count, so both tile
// spaces keep their XCD-aware mapping.
template <bool kStoreOnly>
__global__ __launch_bounds__(kThreads) void k_bwd_gemm_dh_dw(
    const __bf16* __restrict__ G, int ldg, const __bf16* __restrict__ W, const __bf16* __restrict__ Hc,
    int rows, int d, int V, int n_st, int n_vt, int n_jt, int dh_grid, int dh_mode, int dw_last,
    const long long* __restrict__ n_valid, float grad_loss,
    float* __restrict__ dh_sums, int rows_stride, __bf16* __restrict__ dHc, float* __restrict__ dW) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  if ((int)blockIdx.x < dh_grid) {
    dh_tile(G, ldg, W, rows, d, V, n_st, n_jt, 1, (V + kBK - 1) / kBK, dh_mode, n_valid, grad_loss, dh_sums, rows_stride,
            dHc, blockIdx.x, smem);
    return;
  }
  int vt, jt;
  if (!xcd_tile_2d(n_vt, n_jt, &vt, &jt, (int)blockIdx.x - dh_grid)) return;
  const float scale = dw_last ? gamma_of(n_valid, grad_loss) : 1.0f;
  dw_tile(G, ldg, ldg, Hc, d, rows, d, V, vt, jt, kStoreOnly ? 0 : 1, dw_last ? 0 : 1, scale, dW, d, smem);
}

}  // namespace mst
