"""Planted mistakes in a copy of the MLP oracle (on the CPU) must be caught by the pins."""
import importlib.util
import os

import numpy as np
import pytest

ORACLE_PATH = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "mlp_oracle.py")

MUTATIONS = {
    "activation on the up branch instead of the gate": ("    A = silu(G) * U\n    O = A @ Wd.T\n", "    A = G * silu(U)\n    O = A @ Wd.T\n"),
    "activation applied to the product": ("    A = silu(G) * U\n    O = A @ Wd.T\n", "    A = silu(G * U)\n    O = A @ Wd.T\n"),
    "silu' without the g (1 - s) term": ("    return s * (1.0 + np.asarray(g, dtype=np.float64) * (1.0 - s))\n", "    return s\n"),
    "silu' with the wrong sign inside": ("    return s * (1.0 + np.asarray(g, dtype=np.float64) * (1.0 - s))\n",
                                         "    return s * (1.0 - np.asarray(g, dtype=np.float64) * (1.0 - s))\n"),
    "dX without the up branch": ('        "dX": dG @ Wg + dU @ Wu,\n', '        "dX": dG @ Wg,\n'),
    "dWd from dA instead of dO": ('        "dWd": dO.T @ A,\n', '        "dWd": (dO.T @ A) * 0 + (dA.T @ dO).T * 0 + dO.T @ (A * 0 + U),\n'),
    "gate and up gradients swapped": ('        "dWg": dG.T @ X,\n        "dWu": dU.T @ X,\n', '        "dWg": dU.T @ X,\n        "dWu": dG.T @ X,\n'),
    "dU uses the gate value instead of its activation": ("    dU = dA * silu(G)\n    return {", "    dU = dA * G\n    return {"),
    "dA through the transposed down projection": ("    dA = dO @ Wd\n    dG = dA * U * silu_grad(G)\n    dU = dA * silu(G)\n    return {",
                                                   "    dA = (dO @ Wd)[:, ::-1]\n    dG = dA * U * silu_grad(G)\n    dU = dA * silu(G)\n    return {"),
    "sigmoid of the wrong sign": ("    return np.where(g >= 0, 1.0 / (1.0 + e), e / (1.0 + e))\n", "    return np.where(g >= 0, e / (1.0 + e), 1.0 / (1.0 + e))\n"),
}


def _load(source: str, name: str):
    spec = importlib.util.spec_from_loader(name, loader=None)
    mod = importlib.util.module_from_spec(spec)
    exec(compile(source, name, "exec"), mod.__dict__)
    return mod


def _pins_pass(orc) -> bool:
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(21)
    S, d, I = 9, 5, 7
    X = rng.standard_normal((S, d))
    Wg = rng.standard_normal((I, d)) * 0.9
    Wu = rng.standard_normal((I, d)) * 0.9
    Wd = rng.standard_normal((d, I)) * 0.9
    dO = rng.standard_normal((S, d))
    sig1 = 0.7310585786300049
    try:
        r = orc.mlp(X, Wg, Wu, Wd, dO)
        t = [torch.tensor(a, requires_grad=True) for a in (X, Wg, Wu, Wd)]
        O = (torch.nn.functional.silu(t[0] @ t[1].T) * (t[0] @ t[2].T)) @ t[3].T
        O.backward(torch.tensor(dO))
        if np.abs(r["O"] - O.detach().numpy()).max() > 1e-11:
            return False
        for name, tt in zip(("dX", "dWg", "dWu", "dWd"), t):
            if np.abs(r[name] - tt.grad.numpy()).max() > 1e-10:
                return False
        s = orc.mlp([[1.0]], [[1.0]], [[2.0]], [[3.0]], [[1.0]])
        if abs(s["O"][0, 0] - 6.0 * sig1) > 1e-14 or abs(s["dWu"][0, 0] - 3.0 * sig1) > 1e-14:
            return False
        if orc.silu_grad(0.0) != 0.5:
            return False
    except Exception:
        return False
    return True


def test_unmodified_oracle_passes_the_compact_pins():
    assert _pins_pass(_load(open(ORACLE_PATH).read(), "mlp_oracle_copy"))


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistake_is_caught(name):
    old, new = MUTATIONS[name]
    src = open(ORACLE_PATH).read()
    assert src.count(old) >= 1, f"mutation target not found: {name}"
    mutated = src.replace(old, new, 1)
    assert not _pins_pass(_load(mutated, "mlp_oracle_mutant")), f"pins did not notice: {name}"
