/*
 * mst_mlp.h -- C ABI of the mini-sequence MLP library (hand-written HIP for
 *              gfx950 / MI355X).
 *
 * The operation is the MLP block of the Mini-Sequence Transformer paper:
 * Algorithm 1 (forward) and Algorithm 3 (backward with recomputation of the
 * intermediates).  The block is the Llama MLP of the paper's model listing
 * (Appendix C): three bias-free linear layers and SiLU,
 *
 *     O = ( silu(X Wg^T) * (X Wu^T) ) Wd^T            (Theorem 1)
 *
 * The token dimension S (the paper's N; batch folded in) is split into M
 * mini-sequences of C = ceil(S / M) rows (Algorithm 1, line 1).  For chunk i
 * the forward pass forms the C x I intermediate A_i = silu(X_i Wg^T) * (X_i Wu^T)
 * in the workspace, writes O_i = A_i Wd^T into rows i*C.. of O (Algorithm 1,
 * lines 3 and 5) and reuses the workspace for the next chunk, so only one
 * C x I intermediate is alive instead of S x I.  The backward pass recomputes
 * the chunk's gate and up projections and forms (Algorithm 3, lines 4-5)
 *
 *     dA_i  = dO_i Wd
 *     dG_i  = dA_i * U_i * silu'(G_i)        dU_i = dA_i * silu(G_i)
 *     dX_i  = dG_i Wg + dU_i Wu              (rows i*C.. of dX)
 *     dWg  += dG_i^T X_i     dWu += dU_i^T X_i     dWd += dO_i^T A_i
 *
 * By the paper's exactness claim (Section 3.1) the result does not depend on M.
 *
 * Readings of the paper fixed by this interface:
 *   - the activation acts on the gate branch only (the model listing's
 *     gate_proj / up_proj / down_proj / act_fn), although Theorem 1 prints it
 *     around the product;
 *   - weights are stored as the listing's Linear layers store them,
 *     [out_features, in_features] row-major: Wg, Wu [I, d], Wd [d, I];
 *   - "grad MLP" of Algorithm 3 is the exact derivative of the block above.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer owned by the caller, except where
 *     "host" is written.  The library allocates no device memory and keeps no
 *     state between calls (profiling events aside).
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*); the
 *     calls return without waiting for the GPU.
 *   - Return value: MST_OK (0) or a negative error code of mst_lmhead.h
 *     (MST_ERR_BAD_SHAPE also covers I).  Argument errors are found on the
 *     host before anything is launched.
 *   - Requirements: d % 8 == 0, I % 8 == 0; X, Wg, Wu, Wd, dO, O, dX, dWg,
 *     dWu, dWd 16-byte aligned; workspace 256-byte aligned;
 *     1 <= M <= S; d, I < 2^22; I * d < 2^31; ceil(S/M) * I < 2^30.
 *   - Arithmetic: bf16 operands, fp32 MFMA accumulation; silu, its derivative
 *     and the products in fp32 on the accumulators; A, dA, dG, dU rounded to
 *     bf16 (nearest even) before the GEMMs that consume them; O and dX
 *     rounded to bf16; the three weight gradients fp32, accumulated chunk by
 *     chunk in a fixed order without atomics (bit-identical across calls).
 */
#ifndef MST_MLP_H
#define MST_MLP_H

#include "mst_lmhead.h"

#ifdef __cplusplus
extern "C" {
#endif

/* host: "mst-mlp <version> (gfx950)" */
const char* mst_mlp_version(void);

/*
 * Bytes of workspace the two calls need (host, pure).
 *   fwd: one chunk of A, C * I bf16.
 *   bwd: three chunk-sized bf16 buffers (dA reused for dG, dU, A) = 3 * C * I * 2 bytes.
 * Either output pointer may be NULL.
 */
mst_status mst_mlp_workspace_bytes(int64_t S, int64_t d, int64_t I, int32_t M,
                                   size_t* fwd_bytes, size_t* bwd_bytes);

/*
 * Chunk policy of the paper's chunk-based variant (Section 3.3): a constant
 * chunk size equal to the hidden size, C = d, i.e. M = S / d to the nearest
 * integer and at least 1 (no split when S <= d).  Host, pure; 0 on bad shapes.
 */
int32_t mst_mlp_suggest_m(int64_t S, int64_t d, int64_t I);

/*
 * Forward (Algorithm 1).
 *   X  [S, d] bf16 row-major      block input
 *   Wg [I, d] bf16 row-major      gate projection
 *   Wu [I, d] bf16 row-major      up projection
 *   Wd [d, I] bf16 row-major      down projection
 *   O  [S, d] bf16 row-major      out, fully overwritten
 */
mst_status mst_mlp_fwd(const void* X, const void* Wg, const void* Wu, const void* Wd,
                       int64_t S, int64_t d, int64_t I, int32_t M,
                       void* workspace, size_t workspace_bytes,
                       void* O, void* stream);

/*
 * Backward (Algorithm 3).  Nothing is kept from the forward call: the gate and
 * up projections of every chunk are recomputed.
 *   dO  [S, d] bf16      upstream gradient of O
 *   dX  [S, d] bf16      out, fully overwritten
 *   dWg [I, d] fp32      out, fully overwritten (first chunk stores, later chunks accumulate)
 *   dWu [I, d] fp32      out
 *   dWd [d, I] fp32      out
 */
mst_status mst_mlp_bwd(const void* X, const void* Wg, const void* Wu, const void* Wd, const void* dO,
                       int64_t S, int64_t d, int64_t I, int32_t M,
                       void* workspace, size_t workspace_bytes,
                       void* dX, float* dWg, float* dWu, float* dWd, void* stream);

/*
 * Per-kernel timing (host), as in mst_lmhead.h: mst_mlp_profile_enable(every)
 * brackets every `every`-th launch of each kernel kind of the two calls above
 * with HIP events on the caller's stream (0 = off); collect adds, per kind, the
 * elapsed milliseconds, the number of launches they cover and (if the pointer
 * is not NULL) the number of all launches while timing was on (arrays of
 * length MST_MLP_PROFILE_KINDS) and clears the record.
 */
enum {
  MST_MLP_K_GATEUP = 0,   /* A_i = silu(X_i Wg^T) * (X_i Wu^T)                       */
  MST_MLP_K_DOWN,         /* O_i = A_i Wd^T                                          */
  MST_MLP_K_DA,           /* dA_i = dO_i Wd                                          */
  MST_MLP_K_GATEUP_BWD,   /* recomputed gate/up GEMM + dG_i, dU_i, A_i epilogue      */
  MST_MLP_K_DX,           /* dX_i = dG_i Wg + dU_i Wu                                */
  MST_MLP_K_DW,           /* dWg += dG_i^T X_i, dWu += dU_i^T X_i, dWd += dO_i^T A_i  */
  MST_MLP_PROFILE_KINDS
};
mst_status mst_mlp_profile_enable(int every);
mst_status mst_mlp_profile_collect(double* ms_per_kind, int64_t* launches_per_kind, int64_t* issued_per_kind);
const char* mst_mlp_profile_kind_name(int kind);

#ifdef __cplusplus
}
#endif
#endif /* MST_MLP_H */
