"""Pins of the MLP oracle: what the mathematics fixes, checked without any GPU code.

Every check here is independent of the oracle's own formulas: textbook constants, closed forms, a library
routine with automatic differentiation, finite differences of the forward value, brute force in plain
Python floats, and invariants of the block (row independence, linearity, M-invariance)."""
import math

import numpy as np
import pytest

import mst_inputs as mi
from oracle import mlp_oracle as orc

SIG1 = 0.7310585786300049          # 1 / (1 + e^-1), the logistic function at 1


def _rand(seed=0, S=7, d=5, I=9):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((S, d)), rng.standard_normal((I, d)) * 0.8, rng.standard_normal((I, d)) * 0.8,
            rng.standard_normal((d, I)) * 0.8, rng.standard_normal((S, d)))


def test_scalar_block_textbook_values():
    # d = I = 1: O = silu(x wg) * (x wu) * wd with silu(1) = sigmoid(1)
    r = orc.mlp([[1.0]], [[1.0]], [[2.0]], [[3.0]], [[1.0]])
    assert r["O"][0, 0] == pytest.approx(SIG1 * 2.0 * 3.0, rel=1e-15)
    dsilu1 = SIG1 * (1.0 + (1.0 - SIG1))            # silu'(1) = s (1 + 1 (1 - s))
    # dA = 3; dG = 3 * U * silu'(1) = 3 * 2 * silu'(1); dU = 3 * silu(1)
    assert r["dWg"][0, 0] == pytest.approx(6.0 * dsilu1, rel=1e-15)
    assert r["dWu"][0, 0] == pytest.approx(3.0 * SIG1, rel=1e-15)
    assert r["dWd"][0, 0] == pytest.approx(SIG1 * 2.0, rel=1e-15)
    assert r["dX"][0, 0] == pytest.approx(6.0 * dsilu1 * 1.0 + 3.0 * SIG1 * 2.0, rel=1e-15)


def test_activation_special_values():
    assert orc.silu(0.0) == 0.0
    assert orc.silu_grad(0.0) == 0.5
    assert orc.silu(1.0) == pytest.approx(SIG1, rel=1e-15)
    assert orc.silu(-1.0) == pytest.approx(-(1.0 - SIG1), rel=1e-15)
    # far tails: silu(g) -> g and silu'(g) -> 1 for large g; both -> 0 for very negative g; no overflow
    assert orc.silu(800.0) == 800.0 and orc.silu_grad(800.0) == 1.0
    assert abs(orc.silu(-800.0)) < 1e-300 and abs(orc.silu_grad(-800.0)) < 1e-300
    # minimum of silu is at the root of 1 + g (1 - s) = 0, value about -0.27846
    g = np.linspace(-3, 0, 300001)
    assert orc.silu(g).min() == pytest.approx(-0.2784645427610738, abs=1e-10)


def test_zero_gate_weights_closed_form():
    X, Wg, Wu, Wd, dO = _rand(1)
    r = orc.mlp(X, np.zeros_like(Wg), Wu, Wd, dO)
    # G = 0 -> silu = 0, silu' = 1/2: the block outputs zero, only dWg is non-zero
    assert np.abs(r["O"]).max() == 0 and np.abs(r["dWu"]).max() == 0 and np.abs(r["dWd"]).max() == 0
    assert np.abs(r["dX"]).max() == 0
    expect = (0.5 * (dO @ Wd) * (X @ Wu.T)).T @ X
    assert np.allclose(r["dWg"], expect, rtol=1e-13, atol=1e-13)


def test_zero_up_weights_closed_form():
    X, Wg, Wu, Wd, dO = _rand(2)
    r = orc.mlp(X, Wg, np.zeros_like(Wu), Wd, dO)
    assert np.abs(r["O"]).max() == 0 and np.abs(r["dWg"]).max() == 0 and np.abs(r["dWd"]).max() == 0
    assert np.abs(r["dX"]).max() == 0
    G = X @ Wg.T
    expect = ((dO @ Wd) * (G / (1.0 + np.exp(-G)))).T @ X
    assert np.allclose(r["dWu"], expect, rtol=1e-13, atol=1e-13)


def test_saturated_gate_is_bilinear():
    # gate pre-activation = +40 everywhere: silu(40) = 40 to 1e-17 relative, so O = 40 * (X Wu^T) Wd^T
    S, d, I = 4, 3, 5
    rng = np.random.default_rng(3)
    X = np.abs(rng.standard_normal((S, d))) + 0.5
    Wu = rng.standard_normal((I, d))
    Wd = rng.standard_normal((d, I))
    Wg = np.tile(40.0 / X.sum(axis=1).mean() * np.ones((1, d)), (I, 1))
    X = X / X.sum(axis=1, keepdims=True) * X.sum(axis=1).mean()    # every row sums to the same value
    G = X @ Wg.T
    assert np.allclose(G, 40.0)
    O = orc.mlp_forward(X, Wg, Wu, Wd)
    assert np.allclose(O, 40.0 * (X @ Wu.T) @ Wd.T, rtol=1e-14)
    assert np.abs(orc.mlp_forward(X, -Wg, Wu, Wd)).max() < 1e-12    # gate = -40: block shuts


def test_library_routine_with_autograd():
    torch = pytest.importorskip("torch")
    X, Wg, Wu, Wd, dO = _rand(4, S=11, d=6, I=13)
    r = orc.mlp(X, Wg, Wu, Wd, dO)
    t = [torch.tensor(a, requires_grad=True) for a in (X, Wg, Wu, Wd)]
    O = (torch.nn.functional.silu(t[0] @ t[1].T) * (t[0] @ t[2].T)) @ t[3].T
    O.backward(torch.tensor(dO))
    assert np.abs(r["O"] - O.detach().numpy()).max() < 1e-12
    for name, tt in zip(("dX", "dWg", "dWu", "dWd"), t):
        assert np.abs(r[name] - tt.grad.numpy()).max() < 1e-11, name


def test_finite_differences_of_the_forward_value():
    X, Wg, Wu, Wd, dO = _rand(5, S=4, d=3, I=5)
    r = orc.mlp(X, Wg, Wu, Wd, dO)
    args = {"dX": 0, "dWg": 1, "dWu": 2, "dWd": 3}
    base = [X, Wg, Wu, Wd]
    f = lambda a: float((orc.mlp_forward(*a) * dO).sum())
    h = 1e-6
    rng = np.random.default_rng(6)
    for name, k in args.items():
        for _ in range(6):
            idx = tuple(rng.integers(0, n) for n in base[k].shape)
            ap = [b.copy() for b in base]
            am = [b.copy() for b in base]
            ap[k][idx] += h
            am[k][idx] -= h
            fd = (f(ap) - f(am)) / (2 * h)
            assert fd == pytest.approx(r[name][idx], rel=2e-6, abs=1e-8), (name, idx)


def test_brute_force_plain_python():
    X, Wg, Wu, Wd, dO = _rand(7, S=2, d=2, I=3)
    r = orc.mlp(X, Wg, Wu, Wd, dO)
    S, d = X.shape
    I = Wg.shape[0]
    for s in range(S):
        g = [sum(X[s, k] * Wg[i, k] for k in range(d)) for i in range(I)]
        u = [sum(X[s, k] * Wu[i, k] for k in range(d)) for i in range(I)]
        a = [g[i] / (1.0 + math.exp(-g[i])) * u[i] for i in range(I)]
        for j in range(d):
            assert sum(a[i] * Wd[j, i] for i in range(I)) == pytest.approx(r["O"][s, j], rel=1e-13, abs=1e-14)
    # dWd[j, i] = sum_s dO[s, j] A[s, i]
    for j in range(d):
        for i in range(I):
            tot = 0.0
            for s in range(S):
                gi = sum(X[s, k] * Wg[i, k] for k in range(d))
                ui = sum(X[s, k] * Wu[i, k] for k in range(d))
                tot += dO[s, j] * gi / (1.0 + math.exp(-gi)) * ui
            assert tot == pytest.approx(r["dWd"][j, i], rel=1e-13, abs=1e-14)


def test_rows_are_independent_and_weights_sum_over_rows():
    X, Wg, Wu, Wd, dO = _rand(8, S=9)
    r = orc.mlp(X, Wg, Wu, Wd, dO)
    perm = np.random.default_rng(9).permutation(9)
    p = orc.mlp(X[perm], Wg, Wu, Wd, dO[perm])
    assert np.allclose(p["O"], r["O"][perm], rtol=0, atol=1e-13)
    assert np.allclose(p["dX"], r["dX"][perm], rtol=0, atol=1e-13)
    for k in ("dWg", "dWu", "dWd"):
        assert np.allclose(p[k], r[k], rtol=1e-12, atol=1e-12)
    # a row with zero upstream gradient contributes nothing
    dO2 = dO.copy()
    dO2[4] = 0
    z = orc.mlp(X, Wg, Wu, Wd, dO2)
    drop = orc.mlp(np.delete(X, 4, 0), Wg, Wu, Wd, np.delete(dO, 4, 0))
    assert np.abs(z["dX"][4]).max() == 0
    for k in ("dWg", "dWu", "dWd"):
        assert np.allclose(z[k], drop[k], rtol=1e-12, atol=1e-12)


def test_linearity_in_up_down_and_upstream_gradient():
    X, Wg, Wu, Wd, dO = _rand(10)
    r = orc.mlp(X, Wg, Wu, Wd, dO)
    assert np.allclose(orc.mlp_forward(X, Wg, 2 * Wu, Wd), 2 * r["O"], rtol=1e-13)
    assert np.allclose(orc.mlp_forward(X, Wg, Wu, -3 * Wd), -3 * r["O"], rtol=1e-13)
    r2 = orc.mlp(X, Wg, Wu, Wd, 2.5 * dO)
    for k in ("dX", "dWg", "dWu", "dWd"):
        assert np.allclose(r2[k], 2.5 * r[k], rtol=1e-13)


@pytest.mark.parametrize("M", [1, 2, 3, 5, 7, 16])
def test_m_invariance_of_the_algorithms(M):
    X, Wg, Wu, Wd, dO = _rand(11, S=16, d=6, I=10)
    r = orc.mlp(X, Wg, Wu, Wd, dO)
    c = orc.mlp_chunked(X, Wg, Wu, Wd, dO, M)
    for k in r:
        assert np.allclose(c[k], r[k], rtol=1e-12, atol=1e-12), k


def test_sampled_equals_full():
    X, Wg, Wu, Wd, dO = _rand(12, S=20, d=7, I=12)
    r = orc.mlp(X, Wg, Wu, Wd, dO)
    rows, ir, hr = [0, 5, 19], [1, 11, 4], [6, 0]
    s = orc.mlp_grads_sampled(X, Wg, Wu, Wd, dO, rows, ir, hr)
    assert np.allclose(s["O"], r["O"][rows], rtol=1e-13, atol=1e-13)
    assert np.allclose(s["dX"], r["dX"][rows], rtol=1e-13, atol=1e-13)
    assert np.allclose(s["dWg"], r["dWg"][ir], rtol=1e-13, atol=1e-13)
    assert np.allclose(s["dWu"], r["dWu"][ir], rtol=1e-13, atol=1e-13)
    assert np.allclose(s["dWd"], r["dWd"][hr][:, ir], rtol=1e-13, atol=1e-13)


def test_shape_errors():
    X, Wg, Wu, Wd, dO = _rand(13)
    with pytest.raises(ValueError):
        orc.mlp_forward(X, Wg, Wu[:, :3], Wd)
    with pytest.raises(ValueError):
        orc.mlp_forward(X, Wg, Wu, Wd.T)
    with pytest.raises(ValueError):
        orc.mlp(X, Wg, Wu, Wd, dO[:3])
    with pytest.raises(ValueError):
        orc.mlp_chunked(X, Wg, Wu, Wd, dO, 0)


def test_tiny_configuration_statistics():
    """Gross generator / scaling mistakes: with X ~ N(0,1) and weights N(0, 0.02^2) the gate and up
    pre-activations of the tiny configuration are N(0, d * 0.02^2) = N(0, 0.32^2)."""
    inp = mi.make_mlp_inputs(1)
    X, Wg = inp.f64("X"), inp.f64("Wg")
    G = X @ Wg.T
    assert G.std() == pytest.approx(0.32, rel=0.05)
    O = orc.mlp_forward(X, Wg, inp.f64("Wu"), inp.f64("Wd"))
    assert O.shape == (512, 256) and np.isfinite(O).all()


def test_golden_tiny_configuration_values_are_reproduced():
    """Values written by tests/golden/make_golden_mlp.py (which calls only the oracle and the generator):
    a regression anchor that neither of the two drifted."""
    import json
    import os
    gold = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "mlp_cfg1_oracle.json")))
    inp = mi.make_mlp_inputs(1)
    for n, v in gold["bits_sum"].items():
        assert int(getattr(inp, n + "_bits").astype(np.uint64).sum()) == v, n
    r = orc.mlp(inp.f64("X"), inp.f64("Wg"), inp.f64("Wu"), inp.f64("Wd"), inp.f64("dO"))
    for k, lst in gold["samples"].items():
        for i, j, v in lst:
            assert r[k][i, j] == pytest.approx(v, rel=1e-12, abs=1e-15), (k, i, j)
    for k, v in gold["frobenius"].items():
        assert float(np.sqrt((r[k] ** 2).sum())) == pytest.approx(v, rel=1e-12)
