"""CPU fp64 oracle for the mini-sequence MLP path.  TEST INFRASTRUCTURE ONLY.

Yardstick for the GPU kernels of the MLP block: slow, plain numpy in float64,
no code shared with the HIP path, never imported by the product package (only
the tests, the smoke check and the benchmark's CPU-baseline leg call it).

What it computes.  The mini-sequence MLP (Algorithm 1 of the paper, Algorithm 3
for the backward pass) returns, by the paper's exactness claim (Section 3.1,
"Input Partition" / "Gradient Accumulation"), the same numbers as the standard
block of Theorem 1, the Llama MLP of the paper's model listing (three bias-free
linear layers and SiLU; Appendix C):

    G = X Wg^T        U = X Wu^T                 (Wg, Wu stored [I, d])
    A = silu(G) * U                              silu(g) = g / (1 + exp(-g))
    O = A Wd^T                                   (Wd stored [d, I])

and for an upstream gradient dO of O

    dA  = dO Wd
    dG  = dA * U * silu'(G)        silu'(g) = s (1 + g (1 - s)),  s = 1 / (1 + exp(-g))
    dU  = dA * silu(G)
    dX  = dG Wg + dU Wu
    dWg = dG^T X      dWu = dU^T X      dWd = dO^T A

So the oracle is that definition written out over all rows at once, with no
chunk parameter.  `mlp_chunked` follows Algorithms 1 and 3 step by step
(partition X and dO into M blocks of rows, run the block per mini-sequence,
concatenate the outputs, accumulate the three weight gradients) and exists to
show that the definition does not depend on M.

Readings of the paper taken here:
  * Theorem 1 prints the block as act((X Wg) * (X Wu)) Wd; the model listing
    (gate_proj, up_proj, down_proj, act_fn = SiLU) and the Llama architecture
    it describes apply the activation to the gate branch only:
    (silu(X Wg) * (X Wu)) Wd.  The listing's form is taken.
  * Algorithm 1 declares Wg, Wu in R^{d x I} and Wd in R^{I x d}; the listing's
    Linear layers store [out_features, in_features].  Storage here is the
    listing's: Wg, Wu [I, d], Wd [d, I]; no bias.
  * Algorithm 3 leaves "grad MLP" unspecified; it is the exact derivative of
    the block above (recomputation of G, U, A inside the backward pass changes
    no value).
"""
from __future__ import annotations

import numpy as np


def sigmoid(g: np.ndarray) -> np.ndarray:
    """1 / (1 + exp(-g)) evaluated without overflow for large |g|."""
    g = np.asarray(g, dtype=np.float64)
    e = np.exp(-np.abs(g))
    return np.where(g >= 0, 1.0 / (1.0 + e), e / (1.0 + e))


def silu(g: np.ndarray) -> np.ndarray:
    return np.asarray(g, dtype=np.float64) * sigmoid(g)


def silu_grad(g: np.ndarray) -> np.ndarray:
    s = sigmoid(g)
    return s * (1.0 + np.asarray(g, dtype=np.float64) * (1.0 - s))


def mlp_forward(X, Wg, Wu, Wd, return_intermediates: bool = False):
    """O = (silu(X Wg^T) * (X Wu^T)) Wd^T  (Theorem 1 / Algorithm 1, line 3, on all rows)."""
    X = np.asarray(X, dtype=np.float64)
    Wg = np.asarray(Wg, dtype=np.float64)
    Wu = np.asarray(Wu, dtype=np.float64)
    Wd = np.asarray(Wd, dtype=np.float64)
    if X.ndim != 2 or Wg.shape != Wu.shape or Wg.shape[1] != X.shape[1] or Wd.shape != Wg.shape[::-1]:
        raise ValueError("shapes: X [S,d], Wg/Wu [I,d], Wd [d,I]")
    G = X @ Wg.T
    U = X @ Wu.T
    A = silu(G) * U
    O = A @ Wd.T
    if return_intermediates:
        return O, G, U, A
    return O


def mlp(X, Wg, Wu, Wd, dO) -> dict:
    """Forward and backward of the standard block (the quantities Algorithm 3 returns)."""
    O, G, U, A = mlp_forward(X, Wg, Wu, Wd, return_intermediates=True)
    X = np.asarray(X, dtype=np.float64)
    Wg = np.asarray(Wg, dtype=np.float64)
    Wu = np.asarray(Wu, dtype=np.float64)
    Wd = np.asarray(Wd, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    if dO.shape != O.shape:
        raise ValueError("dO must have the shape of O")
    dA = dO @ Wd
    dG = dA * U * silu_grad(G)
    dU = dA * silu(G)
    return {
        "O": O,
        "dX": dG @ Wg + dU @ Wu,
        "dWg": dG.T @ X,
        "dWu": dU.T @ X,
        "dWd": dO.T @ A,
    }


def mlp_grads_sampled(X, Wg, Wu, Wd, dO, rows, inter_rows, hidden_rows) -> dict:
    """Exact values on samples, for sizes where the full result is too slow:
    O[rows, :], dX[rows, :], dWg[inter_rows, :], dWu[inter_rows, :] and the sub-block
    dWd[hidden_rows][:, inter_rows].

    O and dX of a token need only that token's row of X and dO.  Row i of dWg / dWu needs column i of
    dG / dU over all tokens, i.e. only rows i of Wg, Wu and column i of Wd.  Entry (j, i) of dWd needs
    column j of dO and column i of A, which again needs only rows i of Wg and Wu.
    """
    X = np.asarray(X, dtype=np.float64)
    Wg = np.asarray(Wg, dtype=np.float64)
    Wu = np.asarray(Wu, dtype=np.float64)
    Wd = np.asarray(Wd, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    rows = np.asarray(rows, dtype=np.int64)
    inter_rows = np.asarray(inter_rows, dtype=np.int64)
    hidden_rows = np.asarray(hidden_rows, dtype=np.int64)
    out = {}
    # O and dX on sampled tokens
    Xr, dOr = X[rows], dO[rows]
    G = Xr @ Wg.T
    U = Xr @ Wu.T
    out["O"] = (silu(G) * U) @ Wd.T
    dA = dOr @ Wd
    out["dX"] = (dA * U * silu_grad(G)) @ Wg + (dA * silu(G)) @ Wu
    # dWg, dWu on sampled intermediate indices, over all tokens
    Gi = X @ Wg[inter_rows].T
    Ui = X @ Wu[inter_rows].T
    dAi = dO @ Wd[:, inter_rows]
    out["dWg"] = (dAi * Ui * silu_grad(Gi)).T @ X
    out["dWu"] = (dAi * silu(Gi)).T @ X
    # dWd on sampled (hidden, intermediate) pairs
    out["dWd"] = dO[:, hidden_rows].T @ (silu(Gi) * Ui)
    return out


def mlp_chunked(X, Wg, Wu, Wd, dO, M: int) -> dict:
    """Algorithms 1 and 3 step by step: M mini-sequences of ceil(S / M) rows."""
    X = np.asarray(X, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    S = X.shape[0]
    if M < 1 or M > max(S, 1):
        raise ValueError("1 <= M <= S")
    C = -(-S // M)
    O_parts, dX_parts = [], []
    dWg = np.zeros(np.shape(Wg), dtype=np.float64)
    dWu = np.zeros(np.shape(Wu), dtype=np.float64)
    dWd = np.zeros(np.shape(Wd), dtype=np.float64)
    for i in range(M):
        r0, r1 = i * C, min(S, (i + 1) * C)
        if r0 >= r1:
            break
        r = mlp(X[r0:r1], Wg, Wu, Wd, dO[r0:r1])       # Alg. 1 line 3; Alg. 3 lines 4-5
        O_parts.append(r["O"])
        dX_parts.append(r["dX"])
        dWg += r["dWg"]
        dWu += r["dWu"]
        dWd += r["dWd"]
    return {"O": np.concatenate(O_parts), "dX": np.concatenate(dX_parts), "dWg": dWg, "dWu": dWu, "dWd": dWd}
