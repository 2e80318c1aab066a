"""GPU parity: the HIP path, called through the C ABI, against the CPU fp64 oracle
on the same seeded inputs.  Tolerances are the ones the task states: loss relative
error <= 1e-3; dH and dW max-abs error <= 2e-2 * max|reference|; dW bit-identical
across repeated runs; integer outputs exact."""
import numpy as np
import pytest

import mst_inputs as mi
from oracle import lmhead_ce_oracle as orc

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-3
GRAD_TOL = 2e-2


def _harness():
    from tests.gpu_harness import DeviceRun, bf16_tensor_to_f64
    return DeviceRun, bf16_tensor_to_f64


def _check_full(inp, M=None, grad_loss=1.0, use_lse=True, use_nv=True, scale_floor=1e-30):
    DeviceRun, bf2f = _harness()
    ref = orc.lmhead_ce(inp.H_f64(), inp.W_f64(), inp.labels, inp.ignore_index, grad_loss=grad_loss)
    run = DeviceRun(inp, M=M)
    loss, lse, nv = run.forward()
    assert nv == ref["n_valid"]
    if ref["n_valid"] > 0:
        assert abs(loss - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"]), (loss, ref["loss"])
    else:
        assert loss == 0.0
    np.testing.assert_allclose(lse, ref["lse"], rtol=0, atol=2e-3 * max(1.0, np.abs(ref["lse"]).max()))
    dH, dW = run.backward(grad_loss=grad_loss, use_lse=use_lse, use_nv=use_nv and use_lse)
    dH = bf2f(dH)
    dW = dW.cpu().numpy().astype(np.float64)
    assert np.isfinite(dH).all() and np.isfinite(dW).all()
    sH = max(np.abs(ref["dH"]).max(), scale_floor)
    sW = max(np.abs(ref["dW"]).max(), scale_floor)
    eH = np.abs(dH - ref["dH"]).max() / sH
    eW = np.abs(dW - ref["dW"]).max() / sW
    assert eH <= GRAD_TOL, f"dH max-abs error {eH:.3e} of max|ref|"
    assert eW <= GRAD_TOL, f"dW max-abs error {eW:.3e} of max|ref|"
    ign = inp.labels == inp.ignore_index
    if ign.any():
        assert np.abs(dH[ign]).max() == 0.0
    return run, ref, (loss, eH, eW)


def test_config1_tiny_matches_oracle():
    run, ref, errs = _check_full(mi.make_inputs(1))
    print("cfg1 loss, dH err, dW err:", errs)


def test_config1_without_saved_lse_and_with_grad_loss():
    _check_full(mi.make_inputs(1), grad_loss=-0.75, use_lse=False)


def test_config1_with_lse_but_recounted_n_valid():
    _check_full(mi.make_inputs(1), grad_loss=2.0, use_lse=True, use_nv=False)


@pytest.mark.parametrize("M", [3, 5])
def test_odd_number_of_chunks_leaves_a_lone_last_chunk(M):
    """The backward pairs chunks for the dW pass; an odd count ends with a single-chunk pass."""
    cfg = mi.custom_config(650, 128, 900, M, index=310 + M, w_std=0.2)
    _check_full(mi.make_inputs(cfg))


@pytest.mark.parametrize("S,d,V,M", [
    (300, 136, 520, 3),      # ragged in every dimension; last chunk shorter; d not a multiple of 64
    (777, 264, 1000, 2),     # several row tiles per chunk, ragged tails
    (64, 8, 40, 64),         # one row per chunk, minimal d
    (515, 72, 3000, 5),      # S not divisible by M
    (33, 16, 7, 1),          # tiny vocabulary, V < 8
])
def test_ragged_shapes_match_oracle(S, d, V, M):
    cfg = mi.custom_config(S, d, V, M, index=200 + S, w_std=0.3, ignore_frac=0.1)
    _check_full(mi.make_inputs(cfg), grad_loss=1.25)


@pytest.mark.parametrize("M", [1, 2, 4, 8, 512])
def test_mini_sequence_invariance_on_gpu(M):
    """Same inputs, different M: loss, dH and dW agree with the oracle (which has no M) each time."""
    _check_full(mi.make_inputs(1), M=M)


@pytest.mark.parametrize("S,d,V,M", [
    (1177, 288, 3165, 29), (257, 480, 255, 1), (889, 160, 9, 10), (255, 232, 255, 1), (255, 424, 257, 19),
    (257, 448, 1, 1), (2788, 496, 257, 30), (1, 352, 1349, 1), (1452, 88, 255, 1), (7, 200, 2, 5),
    (256, 504, 2304, 39), (1, 472, 2, 1), (257, 8, 1, 34), (1, 24, 7906, 1),
])
def test_seeded_random_shapes_match_oracle(schedule, S, d, V, M):
    """Shapes drawn once from a seeded generator (tile edges at 255 / 256 / 257, single rows, one- and two-class
    vocabularies, d from 8 to 504, M up to 39): loss, lse, dH and dW against the oracle under the automatic choice of the
    backward order and again with the block order forced wherever a block shape exists."""
    import paper_2407_15892_amd as mst
    cfg = mi.custom_config(S, d, V, M, index=500 + (S * 7 + V) % 97, w_std=0.25, ignore_frac=0.08 if S > 20 else 0.0,
                           label_dist="zipf" if V > 50 else "uniform")
    inp = mi.make_inputs(cfg)
    # V = 1: the exact gradients are zero (softmax = 1 = onehot); fp32 may leave exp(rounding residue) - 1 = one ulp,
    # so the scale of the comparison gets a floor there instead of max|ref| = 0
    floor = 1e-6 if V == 1 else 1e-30
    _check_full(inp, grad_loss=0.9, scale_floor=floor)
    schedule(mst.BWD_SCHEDULE_BLOCKS_FUSED)
    _check_full(inp, grad_loss=0.9, use_lse=False, scale_floor=floor)


@pytest.mark.parametrize("S,d,V,M", [
    (512, 8192, 1024, 2),        # d of 32 column tiles: K of the forward twice that of the benchmark shapes
    (2, 32768, 16, 1),           # two rows, a very long contraction
    (8, 64, 1000003, 1),         # a million classes for a handful of rows: 3907 vocabulary tiles, ragged last one
    (1000003, 8, 8, 7),          # a million rows, smallest legal d: 3907 row tiles, chunks of 142858 rows
    (70000, 8, 1024, 35000),     # two rows per mini-sequence
])
def test_extreme_aspect_ratios_match_oracle(schedule, S, d, V, M):
    """Shapes far from the benchmark's, each dimension in turn much larger than the others: loss, lse, dH and dW against
    the oracle under the automatic backward order and with the pair order forced."""
    import paper_2407_15892_amd as mst
    cfg = mi.custom_config(S, d, V, M, index=800 + (S + V) % 83, w_std=0.05, ignore_frac=0.1 if S > 20 else 0.0,
                           label_dist="zipf" if V > 50 else "uniform")
    inp = mi.make_inputs(cfg)
    _check_full(inp)
    schedule(mst.BWD_SCHEDULE_PAIRS)
    _check_full(inp, use_lse=False)


def test_confidently_predicted_labels():
    """The regime of a trained model: for most rows the label is the class with the largest logit and the softmax is
    sharp (logit sigma about 9), so p_label is close to 1, the per-row loss is small and p - 1 is a small difference.
    Loss, lse, dH and dW against the oracle at the usual tolerances."""
    cfg = mi.custom_config(900, 128, 3000, 3, index=450, w_std=0.8, ignore_frac=0.05)
    inp = mi.make_inputs(cfg)
    z = orc.logits_f64(inp.H_f64(), inp.W_f64())
    rng = np.random.default_rng(450)
    take = (rng.random(cfg.S) < 0.8) & (inp.labels != inp.ignore_index)
    inp.labels[take] = z.argmax(axis=1)[take].astype(np.int32)
    run, ref, (loss, eH, eW) = _check_full(inp, grad_loss=1.0)
    p_label = np.exp(z[take, inp.labels[take]] - ref["lse"][take])
    print(f"confident labels: loss {loss:.4f}, median p_label {np.median(p_label):.4f}, dH err {eH:.2e}, dW err {eW:.2e}")
    assert np.median(p_label) > 0.7
    _check_full(inp, grad_loss=1.0, use_lse=False)


def test_huge_logits_do_not_overflow():
    """Logits of several hundred in magnitude (sigma about 70): the maximum is taken out before every exponential, in
    the per-tile partials, in their merge and in dlogits, so nothing overflows and the one-hot-like softmax comes out."""
    cfg = mi.custom_config(520, 64, 1100, 2, index=451, h_std=3.0, w_std=3.0, ignore_frac=0.05)
    inp = mi.make_inputs(cfg)
    run, ref, (loss, eH, eW) = _check_full(inp)
    assert np.abs(ref["lse"]).max() > 150.0
    print(f"huge logits: loss {loss:.3f}, max |lse| {np.abs(ref['lse']).max():.1f}, dH err {eH:.2e}, dW err {eW:.2e}")


def test_forward_is_bit_identical_for_every_number_of_mini_sequences():
    """The forward stores no logits, so its row tiles ignore mini-sequence boundaries and every row's arithmetic is
    the same whatever M is: lse and loss agree bit for bit between M = 1, ragged M, one row per mini-sequence, and
    several merge groups (the static-scratch entry point shortens the groups; M = 37 with V = 70000 also splits them
    in the workspace entry point)."""
    import torch
    DeviceRun, _ = _harness()
    inp = mi.make_inputs(mi.custom_config(1111, 72, 70000, 1, index=440, w_std=0.3, ignore_frac=0.07, label_dist="zipf"))
    ref = None
    for M in (1, 2, 7, 37, 300, 1111):
        run = DeviceRun(inp, M=M)
        loss, lse, nv = run.forward()
        bits = (np.float32(loss).view(np.uint32), lse.astype(np.float32).view(np.uint32), nv)
        if ref is None:
            ref = bits
            ref_o = orc.lmhead_ce_forward(inp.H_f64(), inp.W_f64(), inp.labels, inp.ignore_index)
            assert nv == ref_o[3] and abs(loss - ref_o[0]) <= LOSS_RTOL * abs(ref_o[0])
        else:
            assert bits[0] == ref[0] and np.array_equal(bits[1], ref[1]) and bits[2] == ref[2], f"M = {M}"


def test_dW_and_dH_bit_identical_across_runs():
    DeviceRun, _ = _harness()
    import torch
    inp = mi.make_inputs(mi.custom_config(1200, 512, 5000, 5, index=301, label_dist="zipf"))
    run = DeviceRun(inp)
    run.forward()
    dH0, dW0 = run.backward()
    dH0, dW0 = dH0.clone(), dW0.clone()
    for _ in range(3):
        run.forward()
        dH1, dW1 = run.backward()
        assert torch.equal(dW0.view(torch.int32), dW1.view(torch.int32))
        assert torch.equal(dH0.view(torch.int16), dH1.view(torch.int16))


def test_all_rows_ignored():
    DeviceRun, bf2f = _harness()
    inp = mi.make_inputs(mi.custom_config(260, 64, 300, 2, index=302))
    inp.labels[:] = inp.ignore_index
    run = DeviceRun(inp)
    loss, lse, nv = run.forward()
    assert nv == 0 and loss == 0.0
    dH, dW = run.backward()
    assert float(dH.float().abs().max()) == 0.0 and float(dW.abs().max()) == 0.0


def test_zero_W_gives_ln_V():
    """Closed form that needs no oracle: W = 0 => loss = ln V exactly in fp32 terms."""
    DeviceRun, bf2f = _harness()
    inp = mi.make_inputs(mi.custom_config(400, 128, 1000, 2, index=303))
    inp.W_bits[:] = 0
    run = DeviceRun(inp)
    loss, lse, nv = run.forward()
    assert abs(loss - np.log(1000.0)) < 1e-5
    dH, dW = run.backward()
    assert float(dH.float().abs().max()) == 0.0
    # columns of dW sum to zero because rows of dlogits sum to zero; on the GPU dlogits is
    # rounded to bf16 (relative step 2^-8), so each row's sum is off by at most about
    # 2 * 2^-9 and the column sums by that times mean|H| (= 0.8 here)
    assert float(dW.double().sum(dim=0).abs().max()) < 2.0 ** -8


def test_out_of_range_label_is_reported_not_dereferenced():
    DeviceRun, _ = _harness()
    inp = mi.make_inputs(mi.custom_config(256, 64, 500, 2, index=304))
    inp.labels[5] = 500
    inp.labels[9] = -3
    run = DeviceRun(inp)
    loss, lse, nv = run.forward()
    assert np.isnan(loss) and nv == -1
    # the backward call must not fault and must not hand back plausible numbers: whether it counts the labels
    # itself (with or without the saved lse) or is given the forward's -1, dH and dW are NaN throughout
    import torch
    for kw in (dict(use_nv=False), dict(use_lse=False, use_nv=False), dict(use_nv=True)):
        dH, dW = run.backward(poison="zero", **kw)
        assert torch.isnan(dH.float()).all() and torch.isnan(dW).all(), kw


def test_workspace_is_not_overrun():
    """Sentinel bytes beyond the declared workspace stay untouched."""
    DeviceRun, _ = _harness()
    inp = mi.make_inputs(mi.custom_config(700, 264, 1500, 3, index=305))
    run = DeviceRun(inp, pad_workspace=4096)
    run.forward()
    assert bool((run.last_ws[run.fwd_bytes:] == 0xA5).all())
    run.backward()
    assert run.bwd_bytes_used == run.bwd_bytes
    assert bool((run.last_ws[run.bwd_bytes:] == 0xA5).all())
    run.backward(use_lse=False)
    assert bool((run.last_ws[run.bwd_bytes_used:] == 0xA5).all())


def test_argument_errors_are_synchronous():
    import torch
    import paper_2407_15892_amd as mst
    DeviceRun, _ = _harness()
    inp = mi.make_inputs(mi.custom_config(64, 16, 40, 2, index=306))
    run = DeviceRun(inp)
    loss = torch.zeros(1, device="cuda")
    small = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(mst.MstError) as e:
        mst.mst_lmhead_ce_fwd(run.H, run.W, run.labels, -100, 2, small, loss)
    assert e.value.status == -4
    ws = torch.zeros(run.fwd_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(mst.MstError) as e:
        mst.mst_lmhead_ce_fwd(run.H, run.W, run.labels, -100, 65, ws, loss)
    assert e.value.status == -3
    buf = torch.zeros(64 * 16 + 8, dtype=torch.bfloat16, device="cuda")
    H_misaligned = buf[1:1 + 64 * 16].view(64, 16)          # 2 bytes off a 16-byte boundary
    with pytest.raises(mst.MstError) as e:
        mst.mst_lmhead_ce_fwd(H_misaligned, run.W, run.labels, -100, 2, ws, loss)
    assert e.value.status == -5


def test_zero_upstream_gradient_gives_zero_gradients():
    DeviceRun, _ = _harness()
    inp = mi.make_inputs(mi.custom_config(300, 64, 700, 2, index=320))
    run = DeviceRun(inp)
    run.forward()
    dH, dW = run.backward(grad_loss=0.0)
    assert float(dH.float().abs().max()) == 0.0 and float(dW.abs().max()) == 0.0


def test_ignore_value_inside_the_vocabulary_range():
    """ignore_index = 0: rows labelled 0 are skipped, class 0 still takes part in every softmax."""
    inp = mi.make_inputs(mi.custom_config(400, 64, 300, 3, index=321, ignore_frac=0.0))
    inp.labels[::7] = 0
    inp.ignore_index = 0
    _check_full(inp)


def test_labels_on_tile_boundaries():
    """Labels at the first / last column of vocabulary tiles and of the 16-wide accumulator groups."""
    inp = mi.make_inputs(mi.custom_config(512, 128, 1000, 2, index=322, ignore_frac=0.0))
    special = np.array([0, 15, 16, 31, 32, 127, 128, 255, 256, 511, 512, 767, 768, 999], dtype=np.int32)
    inp.labels[:] = special[np.arange(512) % len(special)]
    _check_full(inp)


def test_many_row_tiles_per_chunk():
    """Long chunks (thousands of rows, dozens of row tiles) against a small head."""
    cfg = mi.custom_config(20000, 64, 520, 3, index=323, w_std=0.3, label_dist="zipf")
    _check_full(mi.make_inputs(cfg))


@pytest.mark.parametrize("S,d,V,M", [
    (600, 136, 23000, 1),     # 3 x 90 tiles per chunk, ragged rows, K and vocabulary
    (1300, 128, 14000, 1),    # 6 x 55 tiles, K of two steps
    (257, 264, 66000, 1),     # 2 x 258 tiles: the second row tile holds one row
])
def test_more_tiles_than_compute_units(S, d, V, M):
    """More than 256 tiles per launch (several rounds of workgroups, partly filled last round), ragged rows, K and
    vocabulary; labels land in every part of a tile."""
    cfg = mi.custom_config(S, d, V, M, index=330 + M + d, w_std=0.3, ignore_frac=0.05, label_dist="zipf")
    _check_full(mi.make_inputs(cfg), grad_loss=0.5)


def test_repeated_calls_reuse_the_same_buffers():
    """Back-to-back calls on one stream with the same workspace (as bench.py does) stay correct."""
    import torch
    import paper_2407_15892_amd as mst
    DeviceRun, bf2f = _harness()
    inp = mi.make_inputs(mi.custom_config(700, 136, 900, 4, index=324, w_std=0.2))
    ref = orc.lmhead_ce(inp.H_f64(), inp.W_f64(), inp.labels)
    run = DeviceRun(inp)
    ws = torch.empty(max(run.fwd_bytes, run.bwd_bytes), dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, device="cuda")
    lse = torch.empty(run.S, device="cuda")
    nv = torch.zeros(1, dtype=torch.int64, device="cuda")
    dH = torch.empty((run.S, run.d), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((run.V, run.d), dtype=torch.float32, device="cuda")
    for _ in range(3):
        mst.mst_lmhead_ce_fwd(run.H, run.W, run.labels, -100, 4, ws, loss, lse, nv)
        mst.mst_lmhead_ce_bwd(run.H, run.W, run.labels, -100, 4, 1.0, lse, nv, ws, dH, dW)
    torch.cuda.synchronize()
    assert abs(float(loss) - ref["loss"]) <= LOSS_RTOL * abs(ref["loss"])
    assert np.abs(dW.cpu().numpy() - ref["dW"]).max() <= GRAD_TOL * np.abs(ref["dW"]).max()
    assert np.abs(bf2f(dH) - ref["dH"]).max() <= GRAD_TOL * np.abs(ref["dH"]).max()


@pytest.mark.parametrize("B,L", [(1, 1), (4, 1), (1, 257), (3, 1000), (64, 513), (2, 100003)])
def test_shift_labels_is_bit_exact(B, L):
    import torch
    import paper_2407_15892_amd as mst
    rng = np.random.default_rng(B * 1000 + L)
    tok = rng.integers(0, 128256, size=B * L).astype(np.int32)
    tok[rng.integers(0, B * L, size=max(1, B * L // 50))] = -100
    ref = orc.shift_labels(tok, B, L)
    t_in = torch.from_numpy(tok).cuda()
    t_out = torch.full((B * L + 8,), 12345, dtype=torch.int32, device="cuda")     # guard elements after the end
    mst.mst_shift_labels(t_in, B, L, -100, t_out)
    torch.cuda.synchronize()
    got = t_out.cpu().numpy()
    assert np.array_equal(got[: B * L], ref)
    assert (got[B * L:] == 12345).all()


def test_shifted_labels_feed_the_forward_pass():
    import torch
    import paper_2407_15892_amd as mst
    DeviceRun, _ = _harness()
    B, L = 4, 75
    inp = mi.make_inputs(mi.custom_config(B * L, 64, 520, 3, index=77, ignore_frac=0.1))
    shifted = orc.shift_labels(inp.labels, B, L)
    ref_loss = orc.lmhead_ce_forward(inp.H_f64(), inp.W_f64(), shifted)[0]
    run = DeviceRun(inp)
    out = torch.empty_like(run.labels)
    mst.mst_shift_labels(run.labels, B, L, inp.ignore_index, out)
    run.labels = out
    loss, _, nv = run.forward()
    assert nv == int((shifted != -100).sum())
    assert abs(loss - ref_loss) <= LOSS_RTOL * abs(ref_loss)


# ---- the two orders of the backward pass

@pytest.fixture
def schedule():
    """Forces a backward schedule for one test and restores the default afterwards."""
    import paper_2407_15892_amd as mst

    def force(which):
        mst.mst_set_bwd_schedule(which)
    yield force
    mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_AUTO)


@pytest.mark.parametrize("S,d,V,M,blocks,windows", [
    (1024, 128, 3000, 8, 2, 4),     # two row blocks of 512 rows, four windows of 768, ragged last window (V = 11.7 tiles)
    (1000, 136, 2900, 4, 1, 4),     # one ragged row block, d not a multiple of 64
    (1400, 72, 5000, 12, 2, 7),     # ragged second row block (768 + 632 rows), seven windows
    (1800, 136, 2900, 12, 4, 3),    # four row blocks: dW stored, accumulated twice, accumulated and scaled
    (600, 64, 70000, 1, 1, 2),      # wide windows, V not a multiple of 8
    (9000, 64, 600, 2, 2, 2),       # two row blocks of more than 4096 rows each (long contraction in the dW pass that reads dW back)
    (13001, 72, 601, 2, 2, 2),      # row blocks of 6656 and 6345 rows: the read-back pass is long enough for the tile body
                                    # that stages the old dW tile through LDS; ragged d (72) and a last vocabulary tile of 89 rows
    (26000, 264, 520, 2, 3, 2),     # three such row blocks (8704, 8704, 8592): stored, staged + accumulated, staged + scaled;
                                    # second column tile 8 wide, last vocabulary tile 8 rows
])
@pytest.mark.parametrize("fused", [False, True])
def test_block_schedule_matches_oracle(schedule, S, d, V, M, blocks, windows, fused):
    """Row blocks x vocabulary windows: dW accumulates over row blocks, dH over windows; with `fused` the dH and the
    dW GEMM of a block come from one launch."""
    import paper_2407_15892_amd as mst
    which = mst.BWD_SCHEDULE_BLOCKS_FUSED if fused else mst.BWD_SCHEDULE_BLOCKS
    schedule(which)
    info = mst.mst_bwd_schedule_info(S, d, V, M)
    assert info["schedule"] == which and info["windows"] >= 2, info
    if not fused:       # the fused variant may prefer another block shape; the expectations are for separate launches
        assert info["row_blocks"] == blocks and info["windows"] == windows, info
    cfg = mi.custom_config(S, d, V, M, index=400 + S % 97, w_std=0.3, ignore_frac=0.1, label_dist="zipf")
    _check_full(mi.make_inputs(cfg), grad_loss=0.8)
    _check_full(mi.make_inputs(cfg), grad_loss=0.8, use_lse=False)


@pytest.mark.parametrize("which", ["pairs_one_chunk", "blocks"])
def test_dlogits_block_left_in_the_workspace_matches_oracle(schedule, which):
    """The only direct look at the bf16 dlogits block (Algorithm 4 line 6): after a backward call the start of the
    workspace still holds the block written last -- with one mini-sequence and the printed loop that is all rows x all
    of V (leading dimension V rounded up to 8), with the block order the last row block x the last vocabulary window
    (leading dimension = entries per window).  It is compared element by element with the oracle's UNSCALED
    softmax - onehot: the kernel rounds to bf16 (8 significant bits, nearest even: half an ulp is between 2^-9 and
    2^-8 of the value, for the label entry p - 1 too), and its fp32 logits and log-sum-exp add a relative 1e-4 at most."""
    import torch
    import paper_2407_15892_amd as mst
    DeviceRun, bf2f = _harness()
    if which == "pairs_one_chunk":
        S, d, V, M = 700, 136, 3003, 1
        schedule(mst.BWD_SCHEDULE_PAIRS)
    else:
        S, d, V, M = 1800, 136, 2900, 12
        schedule(mst.BWD_SCHEDULE_BLOCKS)
    info = mst.mst_bwd_schedule_info(S, d, V, M)
    inp = mi.make_inputs(mi.custom_config(S, d, V, M, index=430, w_std=0.3, ignore_frac=0.1, label_dist="zipf"))
    run = DeviceRun(inp, M=M)
    run.forward()
    run.backward(grad_loss=0.7)          # the block is unscaled: grad_loss must not show in it
    if which == "pairs_one_chunk":
        assert info["schedule"] == mst.BWD_SCHEDULE_PAIRS
        r0, rows, v0, cols, ld = 0, S, 0, V, (V + 7) // 8 * 8
    else:
        assert info["schedule"] == mst.BWD_SCHEDULE_BLOCKS and info["windows"] >= 2 and info["row_blocks"] >= 2, info
        R, Vw = info["rows_per_block"], info["vocab_per_window"]
        r0 = (info["row_blocks"] - 1) * R
        rows = S - r0
        v0 = (info["windows"] - 1) * Vw
        cols, ld = V - v0, Vw
    G = bf2f(run.last_ws[: rows * ld * 2].view(torch.bfloat16).view(rows, ld))
    H64, W64 = inp.H_f64(), inp.W_f64()
    z = orc.logits_f64(H64[r0:r0 + rows], W64)
    lse = orc.row_logsumexp(z)
    y = inp.labels[r0:r0 + rows]
    valid = y != inp.ignore_index
    g_ref = orc.dlogits_rows(z, lse, y, valid, 1.0)[:, v0:v0 + cols]
    err = np.abs(G[:, :cols] - g_ref)
    bound = (2.0 ** -8 + 1e-4) * np.abs(g_ref) + 1e-30
    worst = float((err / bound).max())
    print(f"dlogits block {which}: {rows} x {cols}, worst error / bound = {worst:.3f}; "
          f"label entries in block: {int((valid & (y >= v0) & (y < v0 + cols)).sum())}")
    assert worst <= 1.0
    assert np.all(G[~valid] == 0.0), "ignored rows must be exactly zero"
    assert np.all(G[:, cols:ld if which == 'pairs_one_chunk' else min(ld, (cols + 255) // 256 * 256)] == 0.0), \
        "padding columns must be zero"
    in_block = valid & (y >= v0) & (y < v0 + cols)
    assert in_block.sum() > 10
    lab = G[np.flatnonzero(in_block), (y - v0)[in_block]]
    assert np.all(lab < 0.0) and np.all(lab >= -1.0) and lab.mean() < -0.9, "label entries are p - 1"


def test_pair_schedule_with_long_pairs(schedule):
    """Two pairs of mini-sequences of 9000 rows each: the second pair's dW pass adds to the stored sums over a long
    contraction (141 K steps)."""
    import paper_2407_15892_amd as mst
    schedule(mst.BWD_SCHEDULE_PAIRS)
    cfg = mi.custom_config(18000, 64, 600, 4, index=431, w_std=0.3, ignore_frac=0.05, label_dist="zipf")
    assert mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)["schedule"] == mst.BWD_SCHEDULE_PAIRS
    _check_full(mi.make_inputs(cfg), grad_loss=1.25)


def test_block_and_pair_schedules_agree_and_repeat_bit_for_bit(schedule):
    DeviceRun, bf2f = _harness()
    import torch
    import paper_2407_15892_amd as mst
    inp = mi.make_inputs(mi.custom_config(1024, 256, 6000, 4, index=411, w_std=0.3, ignore_frac=0.05))
    out = {}
    for which in (mst.BWD_SCHEDULE_PAIRS, mst.BWD_SCHEDULE_BLOCKS):
        schedule(which)
        assert mst.mst_bwd_schedule_info(1024, 256, 6000, 4)["schedule"] == which
        run = DeviceRun(inp)
        run.forward()
        dH0, dW0 = run.backward()
        dH0, dW0 = dH0.clone(), dW0.clone()
        for _ in range(2):
            dH1, dW1 = run.backward()
            assert torch.equal(dW0.view(torch.int32), dW1.view(torch.int32))
            assert torch.equal(dH0.view(torch.int16), dH1.view(torch.int16))
        out[which] = (bf2f(dH0), dW0.cpu().numpy().astype(np.float64))
    # the combined dH + dW launch runs the same tiles as the two separate launches: identical bits
    schedule(mst.BWD_SCHEDULE_BLOCKS_FUSED)
    assert mst.mst_bwd_schedule_info(1024, 256, 6000, 4)["schedule"] == mst.BWD_SCHEDULE_BLOCKS_FUSED
    run = DeviceRun(inp)
    run.forward()
    dHf, dWf = run.backward()
    dHb, dWb = out[mst.BWD_SCHEDULE_BLOCKS]
    assert np.array_equal(bf2f(dHf), dHb) and np.array_equal(dWf.cpu().numpy().astype(np.float64), dWb)
    (hA, wA), (hB, wB) = out[mst.BWD_SCHEDULE_PAIRS], out[mst.BWD_SCHEDULE_BLOCKS]
    # same products, different fp32 summation order (and one more bf16 rounding point for neither)
    assert np.abs(hA - hB).max() <= 2.0 ** -7 * np.abs(hA).max()
    assert np.abs(wA - wB).max() <= 1e-4 * np.abs(wA).max()


def test_block_schedule_does_not_overrun_the_workspace(schedule):
    import paper_2407_15892_amd as mst
    DeviceRun, _ = _harness()
    schedule(mst.BWD_SCHEDULE_BLOCKS)
    inp = mi.make_inputs(mi.custom_config(1024, 128, 3000, 8, index=412))
    run = DeviceRun(inp, pad_workspace=4096)
    run.forward()
    run.backward()
    tail = run.last_ws[-4096:]
    assert bool((tail == 0xA5).all())


def test_forward_and_backward_replay_from_a_hip_graph(schedule):
    """The calls allocate nothing, never synchronise and only enqueue kernels, so a caller can capture them into a
    HIP graph.  Every replay (with eager work and synchronisation in between) must reproduce the eager results bit for
    bit, for both orders of the backward pass."""
    import torch
    import paper_2407_15892_amd as mst
    from tests.gpu_harness import to_device_bf16
    inp = mi.make_inputs(mi.custom_config(1024, 256, 6000, 4, index=431, w_std=0.3, ignore_frac=0.05))
    S, d, V, M = 1024, 256, 6000, 4
    H, W = to_device_bf16(inp.H_bits), to_device_bf16(inp.W_bits)
    labels = torch.from_numpy(inp.labels).cuda()
    fwd_bytes, bwd_bytes = mst.mst_workspace_bytes(S, d, V, M)
    ws = torch.empty(max(fwd_bytes, bwd_bytes), dtype=torch.uint8, device="cuda")
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lse = torch.empty(S, dtype=torch.float32, device="cuda")
    nv = torch.zeros(1, dtype=torch.int64, device="cuda")
    dH = torch.empty((S, d), dtype=torch.bfloat16, device="cuda")
    dW = torch.empty((V, d), dtype=torch.float32, device="cuda")

    def step():
        mst.mst_lmhead_ce_fwd(H, W, labels, inp.ignore_index, M, ws, loss, lse, nv)
        mst.mst_lmhead_ce_bwd(H, W, labels, inp.ignore_index, M, 1.0, lse, nv, ws, dH, dW)

    for which in (mst.BWD_SCHEDULE_PAIRS, mst.BWD_SCHEDULE_BLOCKS_FUSED):
        schedule(which)
        step()                                   # eager reference (also the first call's one-time kernel attributes)
        torch.cuda.synchronize()
        ref = (loss.clone(), lse.clone(), dH.clone(), dW.clone())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        for _ in range(3):
            loss.fill_(float("nan")); lse.fill_(float("nan")); dW.fill_(float("nan"))
            dH.view(torch.int16).fill_(0x7FC0)
            ws.fill_(0xA5)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(loss.view(torch.int32), ref[0].view(torch.int32))
            assert torch.equal(lse.view(torch.int32), ref[1].view(torch.int32))
            assert torch.equal(dH.view(torch.int16), ref[2].view(torch.int16))
            assert torch.equal(dW.view(torch.int32), ref[3].view(torch.int32))
        del graph


def test_two_callers_on_two_streams_do_not_disturb_each_other():
    """Two unrelated problems, each with its own buffers and workspace, enqueued alternately on two side streams of the
    default priority with no synchronisation between them: every output of both equals, bit for bit, what the same
    calls give one after the other on the default stream.  The calls keep their state (label counts, gamma, log-sum-exp
    partials, running dH sums) in the caller's workspace, so nothing is shared between them."""
    import torch
    import paper_2407_15892_amd as mst

    def problem(S, d, V, M, index):
        inp = mi.make_inputs(mi.custom_config(S, d, V, M, index=index, w_std=0.2, ignore_frac=0.1, label_dist="zipf"))
        DeviceRun, _ = _harness()
        run = DeviceRun(inp)
        fb, bb = mst.mst_workspace_bytes(S, d, V, M)
        out = dict(ws=torch.empty(max(fb, bb), dtype=torch.uint8, device="cuda"),
                   loss=torch.zeros(1, dtype=torch.float32, device="cuda"),
                   lse=torch.zeros(S, dtype=torch.float32, device="cuda"),
                   nv=torch.zeros(1, dtype=torch.int64, device="cuda"),
                   dH=torch.zeros((S, d), dtype=torch.bfloat16, device="cuda"),
                   dW=torch.zeros((V, d), dtype=torch.float32, device="cuda"))
        return run, out

    def fwd(run, o, stream):
        mst.mst_lmhead_ce_fwd(run.H, run.W, run.labels, run.inp.ignore_index, run.M, o["ws"], o["loss"], o["lse"],
                              o["nv"], stream)

    def bwd(run, o, stream):
        mst.mst_lmhead_ce_bwd(run.H, run.W, run.labels, run.inp.ignore_index, run.M, 0.7, o["lse"], o["nv"], o["ws"],
                              o["dH"], o["dW"], stream)

    def snapshot(o):
        return [o[k].clone().view(torch.uint8).cpu() for k in ("loss", "lse", "nv", "dH", "dW")]

    a, oa = problem(1500, 256, 3000, 6, 611)
    b, ob = problem(900, 136, 5000, 3, 612)
    for run, o in ((a, oa), (b, ob)):
        fwd(run, o, None)
        bwd(run, o, None)
    torch.cuda.synchronize()
    want_a, want_b = snapshot(oa), snapshot(ob)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        for o in (oa, ob):
            for k in ("loss", "lse", "dH", "dW"):
                o[k].fill_(float("nan"))
        torch.cuda.synchronize()
        fwd(a, oa, sa)
        fwd(b, ob, sb)
        bwd(b, ob, sb)
        bwd(a, oa, sa)
        torch.cuda.synchronize()
        for got, want in zip(snapshot(oa) + snapshot(ob), want_a + want_b):
            assert torch.equal(got, want), f"replay {rep}: outputs differ between concurrent and serial calls"


def test_kernel_timing_covers_every_nth_launch_of_each_kind():
    """mst_profile_enable(n) brackets the first, the n + 1st, ... launch of each kernel kind; collect returns the time of
    those launches, how many they were, and how many launches of the kind there were in all."""
    import torch
    import paper_2407_15892_amd as mst
    DeviceRun, _ = _harness()
    inp = mi.make_inputs(mi.custom_config(1500, 256, 3000, 6, index=640, w_std=0.2, ignore_frac=0.1, label_dist="zipf"))
    run = DeviceRun(inp)
    counts = {}
    for every in (1, 3):
        mst.mst_profile_enable(every)
        try:
            for _ in range(2):
                run.forward()
                run.backward()
            torch.cuda.synchronize()
            got = mst.mst_profile_collect()
        finally:
            mst.mst_profile_enable(0)
        counts[every] = got
        for kind, (ms, timed, issued) in got.items():
            assert timed == -(-issued // every), (kind, every, timed, issued)
            assert (ms > 0.0) == (timed > 0), (kind, ms, timed)
    assert {k: v[2] for k, v in counts[1].items()} == {k: v[2] for k, v in counts[3].items()}
    assert counts[1]["fwd_gemm_lse"][2] == 2 and counts[1]["bwd_gemm_dlogits"][2] >= 2
    assert all(v == (0.0, 0, 0) for v in mst.mst_profile_collect().values()), "collect clears the record"
