"""The pins must be able to fail: plausible mistakes are planted in a copy of the oracle (on the CPU)
and at least one closed-form / library / finite-difference pin has to notice each of them."""
import importlib.util
import math
import os

import numpy as np
import pytest

ORACLE_PATH = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "lmhead_ce_oracle.py")

MUTATIONS = {
    "dropped onehot": ("    g[rows, labels[rows]] -= 1.0\n", "    pass\n"),
    "wrong sign of onehot": ("    g[rows, labels[rows]] -= 1.0\n", "    g[rows, labels[rows]] += 1.0\n"),
    "ignored rows not zeroed": ("    g[~valid, :] = 0.0\n", "    pass\n"),
    "mean over all rows instead of valid rows": ("    scale = grad_loss / n_valid if n_valid > 0 else 0.0\n    for r0",
                                                  "    scale = grad_loss / S\n    for r0"),
    "transposed dW operand": ("        dW += g.T @ H[r0:r1]               # Algorithm 4, line 8\n",
                              "        dW += (H[r0:r1].T @ g).T * 0 + (g.T @ H[r0:r1])[::-1]\n"),
    "no max subtraction and natural log replaced": ("    return m + np.log(np.exp(z - m[:, None]).sum(axis=1))\n",
                                                    "    return m + np.log2(np.exp(z - m[:, None]).sum(axis=1))\n"),
    "dH uses W transposed wrongly": ("        dH[r0:r1] = g @ W                  # Algorithm 4, line 7\n",
                                     "        dH[r0:r1] = (g * 0.5) @ W\n"),
    "target logit taken from the wrong column": ("        nll_sum += float((l[rows] - z[rows, labels[r0 + rows]]).sum())\n        g = dlogits_rows",
                                                 "        nll_sum += float((l[rows] - z[rows, (labels[r0 + rows] + 1) % V]).sum())\n        g = dlogits_rows"),
    "grad_loss applied twice": ("    g *= scale\n    return g\n", "    g *= scale * scale\n    return g\n"),
}


def _load(source: str, name: str):
    spec = importlib.util.spec_from_loader(name, loader=None)
    mod = importlib.util.module_from_spec(spec)
    exec(compile(source, name, "exec"), mod.__dict__)
    return mod


def _pins_pass(orc) -> bool:
    """A compact subset of the pins in test_oracle_pins.py: returns False as soon as one fails."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    S, d, V = 14, 6, 9
    H = rng.standard_normal((S, d))
    W = rng.standard_normal((V, d)) * 0.7
    y = rng.integers(0, V, size=S).astype(np.int32)
    y[3] = -100
    y[8] = -100
    gl = 1.7
    try:
        r = orc.lmhead_ce(H, W, y, grad_loss=gl)
        # library routine with autograd
        Ht = torch.tensor(H, requires_grad=True)
        Wt = torch.tensor(W, requires_grad=True)
        loss = torch.nn.functional.cross_entropy(Ht @ Wt.T, torch.tensor(y, dtype=torch.long), ignore_index=-100)
        loss.backward(torch.tensor(gl, dtype=torch.float64))
        if abs(r["loss"] - float(loss)) > 1e-10:
            return False
        if np.abs(r["dH"] - Ht.grad.numpy()).max() > 1e-10 or np.abs(r["dW"] - Wt.grad.numpy()).max() > 1e-10:
            return False
        # closed form: W = 0
        r0 = orc.lmhead_ce(H, np.zeros_like(W), y)
        if abs(r0["loss"] - math.log(V)) > 1e-12 or np.abs(r0["dH"]).max() > 0:
            return False
        # invariant: columns of dW sum to zero; ignored rows have zero dH
        if np.abs(r["dW"].sum(axis=0)).max() > 1e-12 or np.abs(r["dH"][[3, 8]]).max() > 0:
            return False
        # forward-only entry agrees
        if abs(orc.lmhead_ce_forward(H, W, y)[0] - float(loss)) > 1e-10:
            return False
    except Exception:
        return False
    return True


def test_unmodified_oracle_passes_the_compact_pins():
    src = open(ORACLE_PATH).read()
    assert _pins_pass(_load(src, "oracle_copy"))


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name):
    src = open(ORACLE_PATH).read()
    old, new = MUTATIONS[name]
    assert src.count(old) >= 1, f"mutation target not found: {name}"
    mutated = src.replace(old, new, 1)
    assert mutated != src
    assert not _pins_pass(_load(mutated, "oracle_mutant")), f"pins did not notice: {name}"
