"""Pins for the CPU oracle: it is checked against things other than itself.

Closed forms, invariants, special cases that reduce to textbook formulas, a
library cross-entropy with autograd, finite differences and a brute-force
enumeration.  The paper prints no worked numeric example for the LM head, so
there is no printed value to pin against; the exactness claim of Section 3.1
(mini-sequence result == standard result) and Theorem 4's standard form
loss = crossentropyloss(XW, L) are what these tests hold the oracle to.
"""
import math

import numpy as np
import pytest

import mst_inputs as mi
from oracle import lmhead_ce_oracle as orc


def _small(S=24, d=16, V=40, seed=0, ignore_every=5, w_std=0.5):
    rng = np.random.default_rng(seed)
    H = mi.bf16_bits_to_f64(mi.f32_to_bf16_bits(rng.standard_normal((S, d)).astype(np.float32)))
    W = mi.bf16_bits_to_f64(mi.f32_to_bf16_bits((w_std * rng.standard_normal((V, d))).astype(np.float32)))
    y = rng.integers(0, V, size=S).astype(np.int32)
    if ignore_every:
        y[ignore_every - 1::ignore_every] = -100
    return H, W, y


# ---------------------------------------------------------------- closed forms
@pytest.mark.parametrize("V", [2, 7, 4096])
def test_zero_W_gives_lnV_and_closed_form_grads(V):
    """W = 0: every logit is 0, so loss = ln V, dH = 0 and
    dW[v] = (1/N) sum_s (1/V - [y_s = v]) h_s."""
    S, d = 12, 8
    rng = np.random.default_rng(1)
    H = rng.standard_normal((S, d))
    y = rng.integers(0, V, size=S).astype(np.int32)
    y[3] = -100
    r = orc.lmhead_ce(H, np.zeros((V, d)), y)
    assert r["n_valid"] == S - 1
    assert r["loss"] == pytest.approx(math.log(V), rel=1e-14)
    assert np.abs(r["dH"]).max() == 0.0
    valid = y != -100
    exp_dW = np.zeros((V, d))
    for s in range(S):
        if valid[s]:
            exp_dW += H[s][None, :] / V
            exp_dW[y[s]] -= H[s]
    exp_dW /= valid.sum()
    np.testing.assert_allclose(r["dW"], exp_dW, rtol=0, atol=1e-14)


def test_zero_H_gives_lnV_and_closed_form_dH():
    """H = 0: loss = ln V, dW = 0, dH[s] = (mean_v W[v] - W[y_s]) / N."""
    S, d, V = 10, 6, 33
    rng = np.random.default_rng(2)
    W = rng.standard_normal((V, d))
    y = rng.integers(0, V, size=S).astype(np.int32)
    y[0] = -100
    r = orc.lmhead_ce(np.zeros((S, d)), W, y)
    n = S - 1
    assert r["loss"] == pytest.approx(math.log(V), rel=1e-14)
    assert np.abs(r["dW"]).max() == 0.0
    exp = (W.mean(axis=0)[None, :] - W[np.where(y >= 0, y, 0)]) / n
    exp[0] = 0.0
    np.testing.assert_allclose(r["dH"], exp, rtol=0, atol=1e-14)


def test_binary_vocab_is_logistic_regression():
    """V = 2: loss per row = softplus(-(z_y - z_other)); gradient wrt the margin is -sigmoid(-margin)."""
    S, d = 9, 5
    rng = np.random.default_rng(3)
    H = rng.standard_normal((S, d))
    W = rng.standard_normal((2, d))
    y = rng.integers(0, 2, size=S).astype(np.int32)
    r = orc.lmhead_ce(H, W, y)
    z = H @ W.T
    margin = z[np.arange(S), y] - z[np.arange(S), 1 - y]
    exp_loss = np.mean(np.log1p(np.exp(-margin)))
    assert r["loss"] == pytest.approx(exp_loss, rel=1e-13)
    # d loss / d h_s = -sigmoid(-margin) * (W[y] - W[1-y]) / S
    sig = 1.0 / (1.0 + np.exp(margin))
    exp_dH = -(sig[:, None]) * (W[y] - W[1 - y]) / S
    np.testing.assert_allclose(r["dH"], exp_dH, rtol=1e-12, atol=1e-15)


def test_single_class_vocab_is_trivial():
    H = np.random.default_rng(4).standard_normal((5, 3))
    W = np.random.default_rng(5).standard_normal((1, 3))
    r = orc.lmhead_ce(H, W, np.zeros(5, dtype=np.int32))
    assert abs(r["loss"]) < 1e-15
    assert np.abs(r["dH"]).max() < 1e-15 and np.abs(r["dW"]).max() < 1e-15


# ------------------------------------------------------------------ invariants
def test_dlogits_rows_sum_to_zero_so_dW_columns_sum_to_zero():
    H, W, y = _small()
    r = orc.lmhead_ce(H, W, y)
    assert np.abs(r["dW"].sum(axis=0)).max() < 1e-15
    z = orc.logits_f64(H, W)
    lse = orc.row_logsumexp(z)
    g = orc.dlogits_rows(z, lse, y, y != -100, 1.0)
    assert np.abs(g.sum(axis=1)).max() < 1e-14


def test_logit_shift_and_vocab_permutation_invariance():
    H, W, y = _small(seed=7)
    base = orc.lmhead_ce(H, W, y)
    # adding the same vector c to every W row shifts every logit of row s by h_s.c
    c = np.random.default_rng(8).standard_normal(W.shape[1])
    shifted = orc.lmhead_ce(H, W + c[None, :], y)
    assert shifted["loss"] == pytest.approx(base["loss"], rel=1e-12)
    # relabel the vocabulary
    perm = np.random.default_rng(9).permutation(W.shape[0])
    inv = np.argsort(perm)
    y2 = np.where(y == -100, -100, inv[np.where(y >= 0, y, 0)]).astype(np.int32)
    permuted = orc.lmhead_ce(H, W[perm], y2)
    assert permuted["loss"] == pytest.approx(base["loss"], rel=1e-13)
    np.testing.assert_allclose(permuted["dW"], base["dW"][perm], atol=1e-15)
    np.testing.assert_allclose(permuted["dH"], base["dH"], atol=1e-15)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 7, 24, 32])
def test_mini_sequence_invariance(M):
    """Section 3.1 / Appendix B: chunked forward and backward give the standard result."""
    H, W, y = _small(S=24)
    if M > 24:
        M = 24
    base = orc.lmhead_ce(H, W, y, grad_loss=0.7)
    ch = orc.lmhead_ce_chunked(H, W, y, M, grad_loss=0.7)
    assert ch["loss"] == pytest.approx(base["loss"], rel=1e-13)
    np.testing.assert_allclose(ch["dH"], base["dH"], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(ch["dW"], base["dW"], rtol=1e-11, atol=1e-16)


def test_mean_of_chunk_means_differs_when_ignored_rows_are_uneven():
    """Why the global-mean reading is taken: the printed  sum(loss_i)/M  is not
    M-invariant once chunks hold different numbers of valid labels."""
    H, W, y = _small(S=24, ignore_every=0)
    y[:5] = -100                                  # all ignored rows in chunk 0
    base = orc.lmhead_ce_forward(H, W, y)[0]
    M, C = 2, 12
    means = []
    for i in range(M):
        sl = slice(i * C, (i + 1) * C)
        means.append(orc.lmhead_ce_forward(H[sl], W, y[sl])[0])
    assert abs(np.mean(means) - base) > 1e-4
    assert orc.lmhead_ce_chunked(H, W, y, 2)["loss"] == pytest.approx(base, rel=1e-13)


def test_ignored_rows_contribute_nothing():
    H, W, y = _small(seed=11)
    r = orc.lmhead_ce(H, W, y)
    ign = y == -100
    assert ign.any()
    assert np.abs(r["dH"][ign]).max() == 0.0
    keep = ~ign
    r2 = orc.lmhead_ce(H[keep], W, y[keep])
    assert r2["loss"] == pytest.approx(r["loss"], rel=1e-14)
    np.testing.assert_allclose(r2["dW"], r["dW"], atol=1e-16)
    np.testing.assert_allclose(r2["dH"], r["dH"][keep], atol=1e-16)
    # a different ignore value behaves the same way
    y3 = np.where(y == -100, -1, y).astype(np.int32)
    r3 = orc.lmhead_ce(H, W, y3, ignore_index=-1)
    assert r3["loss"] == r["loss"]


def test_grad_loss_scales_gradients_once():
    H, W, y = _small(seed=12)
    a = orc.lmhead_ce(H, W, y, grad_loss=1.0)
    b = orc.lmhead_ce(H, W, y, grad_loss=-2.5)
    np.testing.assert_allclose(b["dH"], -2.5 * a["dH"], rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(b["dW"], -2.5 * a["dW"], rtol=1e-12, atol=1e-16)
    assert b["loss"] == a["loss"]


def test_all_ignored_convention_and_label_range_error():
    H, W, y = _small()
    r = orc.lmhead_ce(H, W, np.full_like(y, -100))
    assert r["loss"] == 0.0 and r["n_valid"] == 0
    assert np.abs(r["dH"]).max() == 0.0 and np.abs(r["dW"]).max() == 0.0
    bad = y.copy()
    bad[0] = W.shape[0]
    with pytest.raises(ValueError):
        orc.lmhead_ce(H, W, bad)
    bad[0] = -1
    with pytest.raises(ValueError):
        orc.lmhead_ce_forward(H, W, bad)


def test_block_streaming_does_not_change_results():
    H, W, y = _small(S=37, ignore_every=6)
    a = orc.lmhead_ce(H, W, y, block_rows=37)
    b = orc.lmhead_ce(H, W, y, block_rows=5)
    assert a["loss"] == pytest.approx(b["loss"], rel=1e-14)
    np.testing.assert_allclose(a["dW"], b["dW"], atol=1e-16)
    np.testing.assert_array_equal(a["dH"], b["dH"])
    f = orc.lmhead_ce_forward(H, W, y, block_rows=4)
    assert f[0] == pytest.approx(a["loss"], rel=1e-14)
    np.testing.assert_allclose(f[1], a["lse"], rtol=1e-15)


# ---------------------------------------------------------- finite differences
def test_finite_differences_match_analytic_gradients():
    S, d, V = 6, 5, 11
    rng = np.random.default_rng(21)
    H = rng.standard_normal((S, d))
    W = rng.standard_normal((V, d))
    y = rng.integers(0, V, size=S).astype(np.int32)
    y[2] = -100
    gl = 1.3
    r = orc.lmhead_ce(H, W, y, grad_loss=gl)
    eps = 1e-6

    def loss(Hx, Wx):
        return orc.lmhead_ce_forward(Hx, Wx, y)[0]

    for (s, k) in [(0, 0), (1, 3), (2, 1), (5, 4), (3, 2)]:
        Hp, Hm = H.copy(), H.copy()
        Hp[s, k] += eps
        Hm[s, k] -= eps
        fd = gl * (loss(Hp, W) - loss(Hm, W)) / (2 * eps)
        assert r["dH"][s, k] == pytest.approx(fd, rel=1e-6, abs=1e-9)
    for (v, k) in [(0, 0), (int(y[0]), 1), (int(y[1]), 4), (10, 2), (7, 3)]:
        Wp, Wm = W.copy(), W.copy()
        Wp[v, k] += eps
        Wm[v, k] -= eps
        fd = gl * (loss(H, Wp) - loss(H, Wm)) / (2 * eps)
        assert r["dW"][v, k] == pytest.approx(fd, rel=1e-6, abs=1e-9)


# ----------------------------------------------------------- library routine
def test_matches_library_cross_entropy_with_autograd():
    """torch's CPU float64 log-softmax cross-entropy (mean over non-ignored
    rows, ignore_index=-100) and its autograd gradients: a stock routine that
    shares nothing with the oracle."""
    torch = pytest.importorskip("torch")
    H, W, y = _small(S=48, d=24, V=100, seed=31)
    gl = 0.37
    Ht = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    loss = torch.nn.functional.cross_entropy(Ht @ Wt.T, torch.tensor(y, dtype=torch.long), ignore_index=-100)
    loss.backward(torch.tensor(gl, dtype=torch.float64))
    r = orc.lmhead_ce(H, W, y, grad_loss=gl)
    assert r["loss"] == pytest.approx(float(loss), rel=1e-13)
    np.testing.assert_allclose(r["dH"], Ht.grad.numpy(), rtol=1e-11, atol=1e-16)
    np.testing.assert_allclose(r["dW"], Wt.grad.numpy(), rtol=1e-11, atol=1e-16)


def test_config1_matches_library_cross_entropy():
    torch = pytest.importorskip("torch")
    inp = mi.make_inputs(1)
    H, W = inp.H_f64(), inp.W_f64()
    Ht = torch.tensor(H, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    loss = torch.nn.functional.cross_entropy(Ht @ Wt.T, torch.tensor(inp.labels, dtype=torch.long), ignore_index=-100)
    loss.backward()
    r = orc.lmhead_ce(H, W, inp.labels)
    assert r["n_valid"] == 480
    assert r["loss"] == pytest.approx(float(loss), rel=1e-13)
    np.testing.assert_allclose(r["dH"], Ht.grad.numpy(), rtol=1e-10, atol=1e-18)
    np.testing.assert_allclose(r["dW"], Wt.grad.numpy(), rtol=1e-10, atol=1e-18)
    # statistical sanity: logits of a row are ~N(0, (0.02 |h|)^2)  =>  loss ~ ln V + sigma^2/2
    assert r["loss"] == pytest.approx(math.log(4096) + 0.5 * (0.02 ** 2) * 256, rel=1e-2)


# ------------------------------------------------------------------ brute force
def test_brute_force_enumeration():
    """Literal evaluation of the definition with Python floats and math.fsum."""
    S, d, V = 4, 3, 8
    rng = np.random.default_rng(41)
    H = rng.standard_normal((S, d))
    W = rng.standard_normal((V, d))
    y = np.array([3, -100, 0, 7], dtype=np.int32)
    gl = 2.0
    n = 3
    loss_terms = []
    dH = [[0.0] * d for _ in range(S)]
    dW = [[0.0] * d for _ in range(V)]
    for s in range(S):
        if y[s] == -100:
            continue
        z = [math.fsum(H[s, k] * W[v, k] for k in range(d)) for v in range(V)]
        denom = math.fsum(math.exp(zv) for zv in z)
        loss_terms.append(math.log(denom) - z[y[s]])
        for v in range(V):
            g = (math.exp(z[v]) / denom - (1.0 if v == y[s] else 0.0)) * gl / n
            for k in range(d):
                dH[s][k] += g * W[v, k]
                dW[v][k] += g * H[s, k]
    r = orc.lmhead_ce(H, W, y, grad_loss=gl)
    assert r["loss"] == pytest.approx(math.fsum(loss_terms) / n, rel=1e-14)
    np.testing.assert_allclose(r["dH"], np.array(dH), rtol=1e-12, atol=1e-16)
    np.testing.assert_allclose(r["dW"], np.array(dW), rtol=1e-12, atol=1e-16)


def test_large_logits_do_not_overflow():
    H = np.array([[1000.0, 0.0]])
    W = np.array([[1.0, 0.0], [0.5, 0.0], [-1.0, 0.0]])
    r = orc.lmhead_ce(H, W, np.array([1], dtype=np.int32))
    # lse = 1000 + log(1 + e^-500 + e^-2000) = 1000 ; nll = 1000 - 500
    assert r["loss"] == pytest.approx(500.0, rel=1e-15)
    assert np.isfinite(r["dW"]).all()


# ------------------------------------------------------------------ sampled mode
def test_sampled_gradients_equal_full_gradients():
    H, W, y = _small(S=64, d=16, V=96, seed=51, ignore_every=7)
    full = orc.lmhead_ce(H, W, y, grad_loss=1.5)
    loss, lse, nll, n_valid = orc.lmhead_ce_forward(H, W, y)
    rows = np.array([0, 6, 13, 63])
    vrows = np.array([0, int(y[0]), 50, 95])
    dH_r, dW_r = orc.lmhead_ce_grads_sampled(H, W, y, lse, n_valid, rows, vrows, grad_loss=1.5, block_rows=10)
    np.testing.assert_allclose(dH_r, full["dH"][rows], rtol=1e-12, atol=1e-17)
    np.testing.assert_allclose(dW_r, full["dW"][vrows], rtol=1e-12, atol=1e-17)


# ------------------------------------------------------------------ stored values
def test_golden_config1_values_are_reproduced():
    """Values written by tests/golden/make_golden.py (which calls only the
    oracle) guard against silent drift of the oracle or the input generator."""
    import json
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "cfg1_oracle.json")
    with open(path) as f:
        gold = json.load(f)
    inp = mi.make_inputs(1)
    r = orc.lmhead_ce(inp.H_f64(), inp.W_f64(), inp.labels)
    assert r["n_valid"] == gold["n_valid"]
    assert r["loss"] == pytest.approx(gold["loss"], rel=1e-13)
    for (s, k, val) in gold["dH_samples"]:
        assert r["dH"][s, k] == pytest.approx(val, rel=1e-11, abs=1e-20)
    for (v, k, val) in gold["dW_samples"]:
        assert r["dW"][v, k] == pytest.approx(val, rel=1e-11, abs=1e-20)
    assert int(inp.H_bits.astype(np.uint64).sum()) == gold["H_bits_sum"]
    assert int(inp.W_bits.astype(np.uint64).sum()) == gold["W_bits_sum"]
    assert int(inp.labels.astype(np.int64).sum()) == gold["labels_sum"]


def test_shift_labels_matches_the_sliced_next_token_loss():
    """Library cross-check of the alignment helper: the loss over unshifted hidden states with shifted labels
    equals the usual next-token loss that slices logits[:, :-1] against labels[:, 1:]."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(31)
    B, L, d, V = 3, 7, 5, 11
    H = rng.standard_normal((B * L, d))
    W = rng.standard_normal((V, d))
    tok = rng.integers(0, V, size=B * L).astype(np.int32)
    tok[[4, 9]] = -100                                   # masked positions move with the shift
    y = orc.shift_labels(tok, B, L)
    assert list(y.reshape(B, L)[:, -1]) == [-100] * B
    assert (y.reshape(B, L)[:, :-1] == tok.reshape(B, L)[:, 1:]).all()
    loss = orc.lmhead_ce_forward(H, W, y)[0]
    logits = torch.tensor(H @ W.T).reshape(B, L, V)
    ref = torch.nn.functional.cross_entropy(logits[:, :-1].reshape(-1, V),
                                            torch.tensor(tok.reshape(B, L)[:, 1:].reshape(-1), dtype=torch.long),
                                            ignore_index=-100)
    assert loss == pytest.approx(float(ref), rel=1e-12)
    # degenerate: sequences of one position have no successor at all
    assert (orc.shift_labels(np.arange(4, dtype=np.int32), 4, 1) == -100).all()
    with pytest.raises(ValueError):
        orc.shift_labels(tok, B, L + 1)


def test_sampled_gradients_reject_out_of_range_labels_like_the_full_oracle():
    rng = np.random.default_rng(5)
    H, W = rng.standard_normal((6, 4)), rng.standard_normal((5, 4))
    y = np.array([0, 1, 7, -100, 2, 4])       # 7 is outside [0, 5)
    with pytest.raises(ValueError):
        orc.lmhead_ce(H, W, y)
    with pytest.raises(ValueError):
        orc.lmhead_ce_grads_sampled(H, W, y, np.zeros(6), 5, [0], [0])
