/*
 * mst_lmhead.h -- C ABI of the mini-sequence LM-head + cross-entropy library
 *                 (hand-written HIP for gfx950 / MI355X).
 *
 * The operation is the LM-head block of the Mini-Sequence Transformer paper:
 * Algorithm 2 (forward) and Algorithm 4 (backward with logit recomputation).
 * The token dimension S (the paper's N; batch folded in) is split into M
 * mini-sequences of C = ceil(S / M) rows.  For chunk i
 *
 *     logits_i = H_i W^T                          (Algorithm 2, line 4)
 *     loss    += sum of per-row NLL of chunk i    (Algorithm 2, line 6)
 *
 * and in the backward pass the chunk's logits are formed again and turned into
 *
 *     dlogits_i = (softmax(logits_i) - onehot(labels_i))        (Alg. 4, l. 5-6)
 *     dH_i      = dlogits_i W          * grad_loss / N_valid    (Alg. 4, l. 7, 9)
 *     dW       += dlogits_i^T H_i      * grad_loss / N_valid    (Alg. 4, l. 8, 10)
 *
 * so that only one C x V block of logits is alive at a time.  By the paper's
 * exactness claim (Section 3.1) the result equals the standard head
 * loss = crossentropy(H W^T, labels) of Theorem 4, for every M.
 *
 * Readings of the paper fixed by this interface:
 *   - the loss is the mean over all non-ignored tokens of the whole call
 *     (per-chunk sums, one division), which is the only reading of Algorithm 2
 *     line 7 that is independent of M when chunks hold different numbers of
 *     ignored labels;
 *   - W is stored [V, d] row-major (a bias-free linear layer d -> V, as in the
 *     paper's model listing), so logits = H W^T and dW is [V, d];
 *   - the upstream gradient of Algorithm 4 multiplies once, not once per chunk;
 *   - labels are already aligned with the rows of H (no causal shift here);
 *   - the ignore value (-100 in Algorithm 2, line 5) is an argument.
 *
 * Conventions
 *   - Every pointer named below is a DEVICE pointer owned by the caller, except
 *     where "host" is written.  The library allocates no device memory and
 *     keeps no state between calls (profiling events and the calling thread's
 *     backward-schedule override of mst_set_bwd_schedule aside).
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*); the
 *     calls return without waiting for the GPU.  They only launch kernels (no
 *     allocation, no memset, no synchronisation), so after one eager call in the
 *     process (which sets kernel attributes) they can be captured into a HIP
 *     graph and replayed; profiling must be off while capturing.
 *   - Return value: MST_OK (0) or a negative error code.  Argument errors are
 *     found on the host before anything is launched.  A label outside [0, V)
 *     that is not `ignore_index` is a data error found on the device: it never
 *     causes an out-of-range access; the forward call then writes NaN to *loss
 *     and -1 to *n_valid, and the backward call (given that -1, or counting the
 *     labels itself) fills dH and dW with NaN.
 *   - The device must be a whole MI355X (256 compute units behind one HIP
 *     device); a partitioned device is refused with MST_ERR_NO_DEVICE because the
 *     tile maps are laid out for 8 XCDs of 32 compute units.
 *   - Requirements: d % 8 == 0; H, W, dH, dW 16-byte aligned; lse 4-byte
 *     aligned; workspace 256-byte aligned; 1 <= M <= S; d < 2^22;
 *     V * d < 2^31; ceil(S/M) * (V rounded up to 8) < 2^30.
 *   - Arithmetic: bf16 operands, fp32 MFMA accumulation, fp32 log-sum-exp and
 *     softmax, dlogits = softmax - onehot rounded to bf16 (nearest even)
 *     before the two gradient GEMMs, grad_loss / N_valid applied in fp32 by
 *     their epilogues, dH rounded to bf16 (from fp32 sums), dW fp32.  What is
 *     accumulated across launches (dW over blocks of rows, dH over windows of
 *     the vocabulary or split partials) is summed in a fixed order without
 *     atomics: repeated calls give bit-identical dW and dH.
 *   - N_valid == 0: loss = 0, dH = 0, dW = 0.
 */
#ifndef MST_LMHEAD_H
#define MST_LMHEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int mst_status;

enum {
  MST_OK = 0,
  MST_ERR_NULL_POINTER = -1,   /* a required pointer is NULL                      */
  MST_ERR_BAD_SHAPE = -2,      /* S, d or V <= 0, d % 8 != 0, or a size limit hit  */
  MST_ERR_BAD_M = -3,          /* M < 1 or M > S                                  */
  MST_ERR_WORKSPACE = -4,      /* workspace NULL or smaller than required          */
  MST_ERR_ALIGNMENT = -5,      /* a pointer is not aligned as required             */
  MST_ERR_LAUNCH = -6,         /* the HIP runtime refused a launch                 */
  MST_ERR_NO_DEVICE = -7       /* no current device, or not a whole 256-CU gfx950  */
};

/* Human-readable text for a status code (host; static storage). */
const char* mst_strerror(mst_status status);

/* Library version string (host; static storage). */
const char* mst_version(void);

/*
 * Workspace sizes in bytes for the forward and the backward call (host-only,
 * launches nothing).  Either output pointer may be NULL.  The forward figure
 * is one (max, sum-exp) pair per row and 256-entry vocabulary tile for a group
 * of consecutive mini-sequences (all of them unless that would exceed half a
 * chunk of fp32 logits) plus 8 bytes per row: 33 MB at S = 8192, V = 128256.
 * The backward figure
 * is for the case that `lse` and `n_valid` from the forward call are supplied:
 * two bf16 dlogits chunks, 2 * ceil(S/M) * (V rounded up to 8) * 2 bytes, which
 * for V % 8 == 0 is exactly one chunk of fp32 logits, ceil(S/M) * V * 4.
 * Without `n_valid` the backward call counts the valid labels itself and needs
 * 512 bytes more; without `lse` it also runs the forward's log-sum-exp pass
 * first and needs bwd_bytes + 512 + fwd_bytes + 4 * S rounded up to 256.
 */
mst_status mst_workspace_bytes(int64_t S, int64_t d, int64_t V, int32_t M,
                               size_t* fwd_bytes, size_t* bwd_bytes);

/*
 * Chunk-count policy (host-only).  Section 3.4 of the paper keeps a constant
 * number of mini-sequences M = V / d for the LM head (32 for Llama3, 64 for
 * Gemma-2 in its rounding) and notes that splitting a short sequence only costs
 * time (its Appendix F measures an 11x slowdown at S = 1024, M = 32).  This
 * returns V / d rounded to the nearest integer, then lowered so that a chunk
 * never has fewer than 256 rows (one block tile of the GEMM kernels), and at
 * least 1.  It is advice: every M with 1 <= M <= S is accepted by the calls.
 * Returns 0 if S, d or V is not positive.
 */
int32_t mst_suggest_m(int64_t S, int64_t d, int64_t V);

/*
 * Next-token alignment of labels (optional helper; device, enqueued on `stream`).
 * Algorithm 2 takes hidden states X and labels L that are already aligned row
 * by row; the paper is silent on the causal shift that language-model training
 * applies before the head.  For B sequences of L positions each, folded into
 * S = B * L rows, this writes the label of row (b, t) as the token that
 * follows it:
 *
 *     labels_out[b * L + t] = labels_in[b * L + t + 1]     for t < L - 1
 *     labels_out[b * L + L - 1] = ignore_index             (nothing follows the last position)
 *
 * so that the unshifted H [B * L, d] and labels_out can be handed to the two
 * calls below.  Values of labels_in equal to ignore_index move with the shift.
 * labels_in and labels_out: int32 [B * L], 4-byte aligned, must not overlap.
 * Errors: MST_ERR_NULL_POINTER, MST_ERR_BAD_SHAPE (B or L not positive, or
 * B * L >= 2^40), MST_ERR_ALIGNMENT.
 */
mst_status mst_shift_labels(const int32_t* labels_in, int64_t B, int64_t L, int32_t ignore_index,
                            int32_t* labels_out, void* stream);

/*
 * Forward: mini-sequence LM-head loss (Algorithm 2).
 *   H        bf16 [S, d] row-major
 *   W        bf16 [V, d] row-major
 *   labels   int32 [S]; rows whose label equals ignore_index are skipped
 *   loss     out, fp32 scalar: mean NLL over the non-ignored rows
 *   lse      out, optional (may be NULL): fp32 [S], log-sum-exp of every row's
 *            logits; pass it to the backward call to save one GEMM pass
 *   n_valid  out, optional (may be NULL): int64 scalar, number of non-ignored rows
 *   workspace / workspace_bytes   scratch of at least the forward size above
 */
mst_status mst_lmhead_ce_fwd(const void* H, const void* W, const int32_t* labels,
                             int64_t S, int64_t d, int64_t V,
                             int32_t ignore_index, int32_t M,
                             void* workspace, size_t workspace_bytes,
                             float* loss, float* lse, int64_t* n_valid,
                             void* stream);

/*
 * The forward call for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, outputs and arithmetic as mst_lmhead_ce_fwd
 * (loss, lse and n_valid are bit-identical to its results), but the scratch
 * memory is a static device array inside the library, MST_STATIC_SCRATCH_BYTES
 * (32 MiB) per GPU the library runs on, held until the process ends.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine) and
 * only enqueues kernels on `stream`.
 *   - Limit: the (max, sum-exp) pairs of ONE mini-sequence plus 4 bytes per row of
 *     the call must fit, ceil(S/M) * (8 * ceil(V/256) + 4) + 4 * S + 1024 <=
 *     MST_STATIC_SCRATCH_BYTES; otherwise MST_ERR_WORKSPACE and nothing is
 *     launched (raise M, or use mst_lmhead_ce_fwd with a workspace).  Within the
 *     limit the pairs of as many consecutive mini-sequences as fit are merged by
 *     one launch; at S = 32768, V = 128256, M = 32 that is 8 of the 32.
 *   - Every call on a GPU uses that GPU's one array, which keeps the previous
 *     call's contents; nothing in it has to start at zero (every word a kernel
 *     reads has been written earlier in the same call).  Calls that overlap on
 *     one GPU (two streams, two threads) race on it: serialise them.
 *   - The first call on a device takes the array's device address (and, like the
 *     other calls, sets kernel attributes): make it outside stream capture; every
 *     later call only enqueues kernels and can be captured.
 *   - Other errors as for mst_lmhead_ce_fwd; MST_ERR_LAUNCH also if the array's
 *     device address cannot be obtained.
 */
#define MST_STATIC_SCRATCH_BYTES (32 * 1024 * 1024)
mst_status mst_lmhead_ce_fwd_static(const void* H, const void* W, const int32_t* labels,
                                    int64_t S, int64_t d, int64_t V,
                                    int32_t ignore_index, int32_t M,
                                    float* loss, float* lse, int64_t* n_valid,
                                    void* stream);

/*
 * Backward: mini-sequence LM-head gradients with recomputation (Algorithm 4).
 *   grad_loss  upstream d(objective)/d(loss) (the algorithm's "nabla loss"), host value
 *   lse        optional fp32 [S] from the forward call (NULL: recomputed here)
 *   n_valid    optional int64 scalar from the forward call on the same labels and
 *              ignore_index (NULL: recounted here, range check included); a supplied
 *              value is trusted, not re-checked; a negative one (the forward's report
 *              of a label outside [0, V)) makes dH and dW NaN
 *   dH         out, bf16 [S, d], fully overwritten (ignored rows are exactly 0)
 *   dW         out, fp32 [V, d], fully overwritten
 */
mst_status mst_lmhead_ce_bwd(const void* H, const void* W, const int32_t* labels,
                             int64_t S, int64_t d, int64_t V,
                             int32_t ignore_index, int32_t M,
                             float grad_loss, const float* lse, const int64_t* n_valid,
                             void* workspace, size_t workspace_bytes,
                             void* dH, float* dW,
                             void* stream);

/*
 * Order of the backward pass (Algorithm 4).  Both orders recompute every logit once, keep at most the
 * bytes mst_workspace_bytes reports (one mini-sequence of fp32 logits, (S/M) * V * 4) and give the same
 * dH and dW up to fp32 summation order; each is deterministic.
 *   MST_BWD_SCHEDULE_PAIRS   the loop over mini-sequences as printed, two per dW pass: the block of dlogits
 *                            alive at a time is 2 * ceil(S/M) rows by all of V; dW is read and rewritten
 *                            once per pair.
 *   MST_BWD_SCHEDULE_BLOCKS  the same bytes hold R rows by one window of the vocabulary (plus fp32 dH sums
 *                            of the R rows), R as large as fits: dW of a window accumulates over the row
 *                            blocks (no re-read at all when R covers S), dH of a row block over the windows.
 *   MST_BWD_SCHEDULE_BLOCKS_FUSED  the block order with the dH and the dW GEMM of each (row block, window)
 *                            in one launch: their tile spaces then share one partly filled last round of
 *                            workgroups instead of leaving one each (same arithmetic as BLOCKS, bit for bit).
 *   MST_BWD_SCHEDULE_AUTO    (default) PAIRS or BLOCKS_FUSED, whichever a host-side cost model (rounds of
 *                            workgroups plus fp32 gradient traffic) ranks faster for the shape.
 * mst_set_bwd_schedule: host; the override belongs to the CALLING THREAD (thread-local, AUTO in every new
 * thread) and takes effect at that thread's next backward call, so one caller's setting never changes the
 * summation order of another thread's call; MST_ERR_BAD_SHAPE for an unknown value.
 * mst_bwd_schedule_info_for: host, pure (no hidden state); fills info[0..7] = {schedule that would run
 * under the override `schedule`, rows per block, row blocks, vocabulary entries per window, windows, dH
 * split count, cost estimate of PAIRS in us, of the block order that would be chosen in us (0 if no block
 * shape fits)}.  mst_bwd_schedule_info: the same with the calling thread's current override.
 */
enum { MST_BWD_SCHEDULE_AUTO = 0, MST_BWD_SCHEDULE_PAIRS = 1, MST_BWD_SCHEDULE_BLOCKS = 2, MST_BWD_SCHEDULE_BLOCKS_FUSED = 3 };
mst_status mst_set_bwd_schedule(int32_t schedule);
mst_status mst_bwd_schedule_info(int64_t S, int64_t d, int64_t V, int32_t M, int64_t* info);
mst_status mst_bwd_schedule_info_for(int64_t S, int64_t d, int64_t V, int32_t M, int32_t schedule, int64_t* info);

/*
 * Workgroup -> tile map of the GEMM kernels (host-only test aid; the kernels call the same function).  A launch
 * over an n_slow x n_fast space of 256 x 256 tiles has mst_tile_grid(n_slow, n_fast) workgroups; workgroup b lands
 * on XCD b % 8, which owns a contiguous range of the slow coordinate and walks it in 4 x 8 rectangles of tiles:
 * order 0 (forward, dH, dW kernels) band by band of 4 slow tiles inside super-groups of 32 fast tiles, order 1
 * (dlogits kernel) group by group of 8 fast tiles.  mst_tile_of_workgroup writes the tile of workgroup `workgroup`
 * and returns 1, or returns 0 for a padding workgroup (it exits at once), or -1 for bad arguments.  Every tile is
 * the image of exactly one workgroup.
 */
int32_t mst_tile_grid(int32_t n_slow, int32_t n_fast);
int32_t mst_tile_of_workgroup(int32_t n_slow, int32_t n_fast, int32_t order, int32_t workgroup,
                              int32_t* slow, int32_t* fast);

/*
 * Matrix-core probe (measurement aid, not part of the path).  Enqueues a kernel in
 * which every wave of `blocks` workgroups of 512 threads issues iters * 16
 * v_mfma_f32_32x32x16_bf16 instructions on register-resident operands (no LDS, no
 * global loads), i.e. blocks * 8 * iters * 16 * 32768 flop in total.  Operands are
 * all zero when `scale` is 0 and pseudo-random of that magnitude otherwise; the
 * sustained rate depends on it because the chip is power limited.  `sink`: one
 * device float, never written in practice (it keeps the loop alive).  The caller
 * times the launch with events on `stream`.
 * Errors: MST_ERR_NULL_POINTER, MST_ERR_BAD_SHAPE (blocks or iters not in [1, 2^20]).
 */
mst_status mst_mfma_probe(int32_t blocks, int32_t iters, float scale, float* sink, void* stream);

/*
 * Per-kernel timing (host).  mst_profile_enable(every): 0 switches it off; n >= 1
 * brackets every n-th launch of each kernel kind of the two calls above (the
 * first, the n + 1st, ...) with HIP events on the caller's stream -- the events
 * themselves take a few microseconds each on the stream, so a caller that times
 * a whole step around them may prefer n > 1.  mst_profile_collect waits for the
 * recorded events, adds per kernel kind the elapsed milliseconds and the number
 * of launches they cover (their quotient is the average launch time) and, if
 * issued_per_kind is not NULL, the number of all launches of that kind while
 * timing was on, into the caller's arrays (each of length MST_PROFILE_KINDS,
 * indexed by the enum below), and clears the record.
 */
enum {
  MST_K_LABEL_SCAN = 0,  /* N_valid, label range check                         */
  MST_K_FWD_GEMM_LSE,    /* logits tile GEMM + running max / sum-exp epilogue   */
  MST_K_LSE_FINALIZE,    /* combine per-vocab-tile partials into lse, nll       */
  MST_K_LOSS_REDUCE,     /* fixed-order sum of nll / N_valid                    */
  MST_K_BWD_GEMM_DLOGITS,/* recomputed logits GEMM + softmax-minus-onehot       */
  MST_K_BWD_GEMM_DH,     /* dH_i = dlogits_i W (split over V)                   */
  MST_K_BWD_DH_REDUCE,   /* fixed-order sum of the dH split partials            */
  MST_K_BWD_GEMM_DW,     /* dW += dlogits_i^T H_i                               */
  MST_K_BWD_GEMM_DH_DW,  /* both of the above for one block, from one launch    */
  MST_PROFILE_KINDS
};
mst_status mst_profile_enable(int every);
mst_status mst_profile_collect(double* ms_per_kind, int64_t* launches_per_kind, int64_t* issued_per_kind);
const char* mst_profile_kind_name(int kind);

#ifdef __cplusplus
}
#endif
#endif /* MST_LMHEAD_H */
