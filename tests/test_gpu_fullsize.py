"""Full-size GPU parity at the benchmark configurations, in the launch configuration bench.py times
(same M, same workspace sizes).  The oracle computes the loss and the log-sum-exp of every row
exactly (one streamed fp64 forward pass), exact dH on a stratified sample of token rows (at least one
in every 256-row tile, so every row block, row tile and XCD rectangle of the launch is hit) and exact
dW on a stratified sample of vocabulary rows (at least one in every 256-entry vocabulary tile, so every
vocabulary window and the ragged last tile are hit); properties that hold at any size cover the rest:
columns of dW sum to ~0, ignored rows of dH are exactly 0, loss, lse, dW and dH are bit-identical across runs.

What the tolerances can and cannot see.  Against max|reference| over the tensor (the stated bar) the
softmax part of the gradients is invisible at configurations 2 and 3: with logit sigma = 0.08 the softmax is
nearly uniform and its whole contribution is a few 1e-3 of max|dH| and 1e-4 of max|dW|, below the 2e-2
allowed.  Two checks make it visible.  (1) Vocabulary rows that are never a label are pure softmax
(dW[v,:] = gamma * sum_s p_sv h_s): their error is taken relative to that row's OWN max|reference|.
dlogits is rounded to bf16 (8 significant bits: half an ulp is 2^-9 to 2^-8 of each term, signs random over the
S terms of a sum), so element errors are about 3e-3 / sqrt(3) of the typical element and the row maximum of the
error stays near 2e-3 to 4e-3 of the row's max|reference| (observed: 0.7e-3 to 3.6e-3); the bound asserted is 1e-2.  (2) One extra full-size run of
the Llama3 shape with W scaled so that logit sigma = 3: the softmax part is then O(1) of both gradients and
the stated tolerance sees it.  For both, the expected values with the softmax term dropped on purpose
(-onehot only) must FAIL the same comparison; that is asserted too."""
import time

import numpy as np
import pytest

import mst_inputs as mi
from oracle import lmhead_ce_oracle as orc

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-3
GRAD_TOL = 2e-2
PURE_SOFTMAX_ROW_TOL = 1e-2     # never-labelled vocabulary rows, relative to the row's own max|ref| (see above)
TILE = 256                      # rows / vocabulary entries per block tile of the GEMM kernels


def stratified(n, tile, rng, extra=()):
    """One random index in every `tile`-sized range of [0, n), plus the first and last index of every 8th range
    and the last range's end, plus `extra`."""
    starts = np.arange(0, n, tile)
    ends = np.minimum(starts + tile, n)
    picks = starts + (rng.random(len(starts)) * (ends - starts)).astype(np.int64)
    edges = np.concatenate([starts[::8], ends[::8] - 1, [n - 1]])
    extra = np.asarray([e for e in extra if 0 <= e < n], dtype=np.int64)
    return np.unique(np.concatenate([picks, edges, extra]).astype(np.int64))


def onehot_only_reference(inp, n_valid, rows, vrows, grad_loss=1.0):
    """The expected values with a mistake planted on purpose: the softmax term of dlogits dropped, i.e.
    g = -onehot * grad_loss / N_valid.  Used to show that a comparison would notice a kernel that did this."""
    W64 = inp.W_f64()
    gamma = grad_loss / n_valid
    y = inp.labels
    valid = y != inp.ignore_index
    dH = np.zeros((len(rows), inp.cfg.d))
    ok = valid[rows]
    dH[ok] = -gamma * W64[y[rows][ok]]
    dW = np.zeros((len(vrows), inp.cfg.d))
    for i, v in enumerate(vrows):
        hit = np.flatnonzero(valid & (y == v))
        if len(hit):
            dW[i] = -gamma * inp.H_f64(hit).sum(axis=0)
    return dH, dW


def grad_checks(dH_s, dW_s, dH_ref, dW_ref, never_label):
    """The comparisons of this file as numbers: (dH error, dW error) of max|ref| over the sample, and the worst
    never-labelled vocabulary row's error relative to its own max|ref| (0 if there is none)."""
    eH = np.abs(dH_s - dH_ref).max() / np.abs(dH_ref).max()
    eW = np.abs(dW_s - dW_ref).max() / np.abs(dW_ref).max()
    e_rows = 0.0
    if never_label.any():
        num = np.abs(dW_s[never_label] - dW_ref[never_label]).max(axis=1)
        den = np.abs(dW_ref[never_label]).max(axis=1)
        e_rows = float((num / den).max())
    return float(eH), float(eW), e_rows


def run_and_check(cfg, tag, expect_softmax_visible_globally):
    import torch
    import paper_2407_15892_amd as mst
    from tests.gpu_harness import DeviceRun, bf16_tensor_to_f64

    t0 = time.time()
    inp = mi.make_inputs(cfg)
    run = DeviceRun(inp)
    cap = cfg.C * cfg.V * 4
    assert run.fwd_bytes <= cap and run.bwd_bytes <= cap, "workspace exceeds one fp32 logits chunk"
    loss, lse, nv = run.forward()
    dH, dW = run.backward()
    dW_first = dW.clone()
    dH_first = dH.clone()
    print(f"{tag}: inputs+gpu {time.time() - t0:.1f}s", flush=True)

    # --- oracle: exact loss and lse for all rows, gradients on stratified samples
    t0 = time.time()
    W64 = inp.W_f64()
    H64 = inp.H_f64()
    ref_loss, ref_lse, ref_nll, ref_nv = orc.lmhead_ce_forward(H64, W64, inp.labels, inp.ignore_index, block_rows=1024)
    sched = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
    rng = np.random.default_rng(1000 + cfg.index)
    R, Vw = sched["rows_per_block"], sched["vocab_per_window"]
    ignored = np.flatnonzero(inp.labels == inp.ignore_index)
    rows = stratified(cfg.S, TILE, rng, extra=list(ignored[:3]) + [cfg.C - 1, cfg.C] +
                      [b for k in range(1, sched["row_blocks"]) for b in (k * R - 1, k * R)])
    valid_labels = inp.labels[inp.labels != inp.ignore_index]
    counts = np.bincount(valid_labels, minlength=cfg.V)
    hot = int(counts.argmax())
    vrows = stratified(cfg.V, TILE, rng, extra=[hot, 255, 256] + list(valid_labels[:6]) +
                       [b for k in range(1, sched["windows"]) for b in (k * Vw - 1, k * Vw)])
    never_label = counts[vrows] == 0
    assert len(rows) >= -(-cfg.S // TILE) and len(vrows) >= -(-cfg.V // TILE)
    assert never_label.sum() >= 10 and (~never_label).sum() >= 5, "the sample needs both kinds of vocabulary rows"
    dH_ref, dW_ref = orc.lmhead_ce_grads_sampled(H64, W64, inp.labels, ref_lse, ref_nv, rows, vrows,
                                                 inp.ignore_index, block_rows=4096)
    dH_mut, dW_mut = onehot_only_reference(inp, ref_nv, rows, vrows)
    print(f"{tag}: oracle {time.time() - t0:.1f}s; {len(rows)} token rows, {len(vrows)} vocabulary rows "
          f"({int(never_label.sum())} never a label)", flush=True)

    assert nv == ref_nv == inp.n_valid
    assert abs(loss - ref_loss) <= LOSS_RTOL * abs(ref_loss), (loss, ref_loss)
    assert np.abs(lse - ref_lse).max() <= 2e-3 * np.abs(ref_lse).max()

    def sample(dH_t, dW_t):
        return (bf16_tensor_to_f64(dH_t[torch.from_numpy(rows).cuda()]),
                dW_t[torch.from_numpy(vrows).cuda()].cpu().numpy().astype(np.float64))

    dH_s, dW_s = sample(dH, dW)
    # every scale below comes from the oracle alone
    eH, eW, e_rows = grad_checks(dH_s, dW_s, dH_ref, dW_ref, never_label)
    print(f"{tag}: loss {loss:.6f} ref {ref_loss:.6f}; dH err {eH:.2e}, dW err {eW:.2e} of max|ref| over the sample; "
          f"never-labelled vocabulary rows: worst error {e_rows:.2e} of the row's own max|ref|", flush=True)
    assert eH <= GRAD_TOL and eW <= GRAD_TOL
    assert e_rows <= PURE_SOFTMAX_ROW_TOL
    # the same comparisons must reject expected values whose softmax term was dropped
    num = np.abs(dW_s[never_label] - dW_mut[never_label]).max(axis=1)
    m_rows = float((num / np.abs(dW_ref[never_label]).max(axis=1)).max())
    print(f"{tag}: against -onehot-only expected values the never-labelled rows are off by {m_rows:.2e} of their own max|ref|",
          flush=True)
    assert m_rows > 10 * PURE_SOFTMAX_ROW_TOL, "the never-labelled-row check cannot see a dropped softmax term"
    if expect_softmax_visible_globally:
        gH, gW, _ = grad_checks(dH_s, dW_s, dH_mut, dW_mut, never_label)
        print(f"{tag}: sharp softmax: -onehot-only expected values are off by dH {gH:.2e}, dW {gW:.2e} of max|ref|", flush=True)
        assert gH > 5 * GRAD_TOL and gW > 5 * GRAD_TOL, "the stated tolerance cannot see a dropped softmax term here"

    # --- properties at full size
    ign = torch.from_numpy(inp.labels == inp.ignore_index).cuda()
    assert float(dH[ign].float().abs().max()) == 0.0
    assert torch.isfinite(dW).all() and torch.isfinite(dH.float()).all()
    col_sums = dW.double().sum(dim=0).abs().max().item()
    # rows of bf16 dlogits sum to zero within 2^-8 relative steps; bound by mean|H| * 2^-7 per unit grad_loss
    assert col_sums <= 2.0 ** -7 * max(cfg.h_std, 1e-3), col_sums
    # bit-identical loss, lse, dW and dH on a second run
    loss2, lse2, _ = run.forward()
    dH2, dW2 = run.backward()
    assert loss2 == loss and np.array_equal(lse2, lse)
    assert torch.equal(dW_first.view(torch.int32), dW2.view(torch.int32))
    assert torch.equal(dH_first.view(torch.int16), dH2.view(torch.int16))

    # --- the other order of the backward pass against the same references
    other = mst.BWD_SCHEDULE_BLOCKS if sched["schedule"] == mst.BWD_SCHEDULE_PAIRS else mst.BWD_SCHEDULE_PAIRS
    try:
        mst.mst_set_bwd_schedule(other)
        forced = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
        print(f"{tag}: default schedule {sched}, also run {forced}", flush=True)
        if forced["schedule"] == other:
            dH_o, dW_o = run.backward()
            oH, oW, o_rows = grad_checks(*sample(dH_o, dW_o), dH_ref, dW_ref, never_label)
            assert oH <= GRAD_TOL and oW <= GRAD_TOL and o_rows <= PURE_SOFTMAX_ROW_TOL, (oH, oW, o_rows)
            assert float(dH_o[ign].float().abs().max()) == 0.0
            assert torch.isfinite(dW_o).all() and torch.isfinite(dH_o.float()).all()
            # both orders form the same products; only the fp32 summation order differs
            assert float((dW_o - dW_first).abs().max()) <= 1e-3 * float(dW_first.abs().max())
    finally:
        mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_AUTO)


@pytest.mark.parametrize("cfg_index", [2, 3, 4, 5])
def test_fullsize_config_matches_oracle_on_samples(cfg_index):
    run_and_check(mi.CONFIGS[cfg_index], f"cfg {cfg_index}", expect_softmax_visible_globally=False)


def test_fullsize_llama3_shape_with_a_sharp_softmax():
    """Configuration 2's shape and launch configuration with W scaled to logit sigma = w_std * |h| = 0.75 * 4 = 3
    (same generator, its own seed index): rows then have a few dominant classes and the softmax term is as large
    as the onehot term in dH and dW, so the stated tolerance itself sees it."""
    cfg = mi.custom_config(8192, 4096, 128256, 8, index=12, h_std=4.0 / 64.0, w_std=0.75, label_dist="uniform",
                           ignore_frac=0.01, name="llama3-8b-sharp-softmax")
    run_and_check(cfg, "sharp", expect_softmax_visible_globally=True)
