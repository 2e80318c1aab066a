"""CPU fp64 oracle for the LM-head + cross-entropy path.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the GPU kernels are measured against.  It is slow,
plain numpy in float64, shares no code with the HIP path and must never be
imported by the product package: only the tests, the smoke check and the
benchmark's CPU-baseline leg call it.

What it computes.  The mini-sequence LM-head (Algorithm 2 of the paper, and
Algorithm 4 for the backward pass) reaches, by the paper's own exactness claim
(Section 3.1, "Input Partition" and Appendix B's closing paragraph), the same
numbers as the standard head  loss = crossentropy(X W_out, L)  (Theorem 4).
So the oracle is that standard definition written out, with the full row of
logits per token and no chunking:

    z[s, v]  = sum_k H[s, k] * W[v, k]                       (W stored [V, d])
    lse[s]   = log sum_v exp z[s, v]
    loss     = (1 / N_valid) * sum_{s valid} (lse[s] - z[s, y_s])
    g[s, v]  = (exp(z[s, v] - lse[s]) - [v == y_s]) * grad_loss / N_valid   (0 on ignored rows)
    dH       = g  @ W          dW = g^T @ H

Rows are streamed in blocks only so that the S x V logits need not be held at
once; that is a memory convenience and does not change any per-row result.

`lmhead_ce_chunked` follows Algorithms 2 and 4 step by step (partition, per
chunk logits, per chunk loss, accumulate dW) and exists to show that the
definition is invariant to the number of mini-sequences M.

Readings of the paper taken here (the paper is silent or garbled on each):
  * the loss is the mean over ALL valid tokens (per-chunk sums, one division),
    not the mean of per-chunk means printed as line 7 of Algorithm 2, because
    only the former is "the exact same result" when chunks hold different
    numbers of ignored labels;
  * line 5 of Algorithm 2 (a label-range test whose two bounds coincide) is
    read as a no-op once labels are partitioned; it only fixes the ignore
    value -100;
  * the upstream gradient (lines 9-10 of Algorithm 4) multiplies once;
  * logits are recomputed, not passed in, in the backward pass;
  * N_valid == 0 returns loss 0 and zero gradients  -- convention only,
    PARITY UNPINNED for that case;
  * a label outside [0, V) that is not the ignore value raises ValueError.
"""
from __future__ import annotations

import numpy as np


def _check_labels(labels: np.ndarray, V: int, ignore_index: int) -> np.ndarray:
    labels = np.asarray(labels)
    valid = labels != ignore_index
    bad = valid & ((labels < 0) | (labels >= V))
    if bad.any():
        raise ValueError(f"label out of range [0,{V}) at row {int(np.flatnonzero(bad)[0])}")
    return valid


def logits_f64(H: np.ndarray, W: np.ndarray) -> np.ndarray:
    """z = H W^T in float64 (Algorithm 2, line 4)."""
    return np.asarray(H, dtype=np.float64) @ np.asarray(W, dtype=np.float64).T


def row_logsumexp(z: np.ndarray) -> np.ndarray:
    """lse[s] = log sum_v exp z[s, v], computed with the row maximum taken out."""
    m = z.max(axis=1)
    return m + np.log(np.exp(z - m[:, None]).sum(axis=1))


def lmhead_ce_forward(H, W, labels, ignore_index=-100, block_rows=256):
    """Loss of the standard LM head (Theorem 4's  crossentropyloss(XW, L)).

    Returns (loss, lse[S], nll[S], n_valid); nll is 0 on ignored rows.
    """
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    labels = np.asarray(labels)
    S, V = H.shape[0], W.shape[0]
    valid = _check_labels(labels, V, ignore_index)
    n_valid = int(valid.sum())
    lse = np.empty(S, dtype=np.float64)
    nll = np.zeros(S, dtype=np.float64)
    for r0 in range(0, S, block_rows):
        r1 = min(S, r0 + block_rows)
        z = logits_f64(H[r0:r1], W)
        lse[r0:r1] = row_logsumexp(z)
        rows = np.flatnonzero(valid[r0:r1])
        nll[r0 + rows] = lse[r0 + rows] - z[rows, labels[r0 + rows]]
    loss = float(nll.sum() / n_valid) if n_valid > 0 else 0.0
    return loss, lse, nll, n_valid


def dlogits_rows(z, lse, labels, valid, scale):
    """g = (softmax(z) - onehot(label)) * scale, zero on ignored rows
    (the cross-entropy backward of Algorithm 4, line 6)."""
    g = np.exp(z - lse[:, None])
    rows = np.flatnonzero(valid)
    g[rows, labels[rows]] -= 1.0
    g[~valid, :] = 0.0
    g *= scale
    return g


def lmhead_ce(H, W, labels, ignore_index=-100, grad_loss=1.0, block_rows=256):
    """Loss and full gradients of the standard LM head.

    Returns dict(loss, lse, n_valid, dH [S,d], dW [V,d]) in float64.
    """
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    labels = np.asarray(labels)
    S, d = H.shape
    V = W.shape[0]
    valid = _check_labels(labels, V, ignore_index)
    n_valid = int(valid.sum())
    dH = np.zeros((S, d), dtype=np.float64)
    dW = np.zeros((V, d), dtype=np.float64)
    lse = np.empty(S, dtype=np.float64)
    nll_sum = 0.0
    scale = grad_loss / n_valid if n_valid > 0 else 0.0
    for r0 in range(0, S, block_rows):
        r1 = min(S, r0 + block_rows)
        z = logits_f64(H[r0:r1], W)
        l = row_logsumexp(z)
        lse[r0:r1] = l
        rows = np.flatnonzero(valid[r0:r1])
        nll_sum += float((l[rows] - z[rows, labels[r0 + rows]]).sum())
        g = dlogits_rows(z, l, labels[r0:r1], valid[r0:r1], scale)
        dH[r0:r1] = g @ W                  # Algorithm 4, line 7
        dW += g.T @ H[r0:r1]               # Algorithm 4, line 8
    loss = nll_sum / n_valid if n_valid > 0 else 0.0
    return dict(loss=loss, lse=lse, n_valid=n_valid, dH=dH, dW=dW)


def lmhead_ce_grads_sampled(H, W, labels, lse, n_valid, rows, vocab_rows,
                            ignore_index=-100, grad_loss=1.0, block_rows=1024):
    """Exact dH on a subset of token rows and exact dW on a subset of vocab rows.

    `lse` must be the full-length output of `lmhead_ce_forward` on the same
    inputs.  dH[s,:] needs only row s of the logits; dW[v,:] needs only column
    v of dlogits, i.e. z[:, v] = H W[v]^T for all s.  Used at sizes where the
    full gradients would take the CPU too long.
    """
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    labels = np.asarray(labels)
    S = H.shape[0]
    valid = _check_labels(labels, W.shape[0], ignore_index)
    scale = grad_loss / n_valid if n_valid > 0 else 0.0
    rows = np.asarray(rows, dtype=np.int64)
    vocab_rows = np.asarray(vocab_rows, dtype=np.int64)
    # dH on the sampled token rows
    z = logits_f64(H[rows], W)
    g = dlogits_rows(z, lse[rows], labels[rows], valid[rows], scale)
    dH_rows = g @ W
    # dW on the sampled vocab rows
    Wv = W[vocab_rows]
    dW_rows = np.zeros((len(vocab_rows), H.shape[1]), dtype=np.float64)
    for r0 in range(0, S, block_rows):
        r1 = min(S, r0 + block_rows)
        zc = H[r0:r1] @ Wv.T                                  # [rows, len(vocab_rows)]
        gc = np.exp(zc - lse[r0:r1, None])
        gc -= (labels[r0:r1, None] == vocab_rows[None, :])
        gc[~valid[r0:r1], :] = 0.0
        gc *= scale
        dW_rows += gc.T @ H[r0:r1]
    return dH_rows, dW_rows


def lmhead_ce_chunked(H, W, labels, M, ignore_index=-100, grad_loss=1.0):
    """Algorithms 2 and 4 taken literally, chunk by chunk.

    Forward: partition X and L into M row blocks (lines 1-2), per block form
    logits_i = X_i W_out (line 4) and the block's summed NLL (line 6), then
    combine.  Backward: per block recompute logits_i (line 5 of Algorithm 4),
    dlogits_i (line 6), dX_i (line 7), and accumulate dW (line 8); the upstream
    gradient multiplies once.  Chunk length is ceil(S / M), last chunk shorter.
    """
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    labels = np.asarray(labels)
    S, d = H.shape
    V = W.shape[0]
    valid = _check_labels(labels, V, ignore_index)
    n_valid = int(valid.sum())
    C = -(-S // M)
    # forward
    nll_sum = 0.0
    for i in range(M):
        r0, r1 = i * C, min(S, (i + 1) * C)
        if r0 >= r1:
            break
        z = logits_f64(H[r0:r1], W)
        l = row_logsumexp(z)
        rows = np.flatnonzero(valid[r0:r1])
        nll_sum += float((l[rows] - z[rows, labels[r0 + rows]]).sum())
    loss = nll_sum / n_valid if n_valid > 0 else 0.0
    # backward with recomputation
    dH = np.zeros((S, d), dtype=np.float64)
    dW = np.zeros((V, d), dtype=np.float64)
    scale = grad_loss / n_valid if n_valid > 0 else 0.0
    for i in range(M):
        r0, r1 = i * C, min(S, (i + 1) * C)
        if r0 >= r1:
            break
        z = logits_f64(H[r0:r1], W)
        l = row_logsumexp(z)
        g = dlogits_rows(z, l, labels[r0:r1], valid[r0:r1], scale)
        dH[r0:r1] = g @ W
        dW += g.T @ H[r0:r1]
    return dict(loss=loss, n_valid=n_valid, dH=dH, dW=dW)


def shift_labels(labels, B: int, L: int, ignore_index: int = -100) -> np.ndarray:
    """Next-token alignment for B sequences of L positions folded into B * L rows: the label of position t
    is the entry at t + 1; the last position of every sequence has no successor and is ignored.  (The paper's
    Algorithm 2 takes aligned X and L and is silent on this step; this is the alignment language-model
    training applies before the head, written out as its definition.)"""
    labels = np.asarray(labels)
    if B <= 0 or L <= 0 or labels.shape != (B * L,):
        raise ValueError("labels must have B * L entries")
    out = np.full((B, L), ignore_index, dtype=labels.dtype)
    out[:, : L - 1] = labels.reshape(B, L)[:, 1:]
    return out.reshape(B * L)
