"""GPU parity of the MLP path: the HIP kernels, called through the C ABI, against the CPU fp64 oracle on
the same seeded inputs, element by element.  Tolerance: max-abs error <= 2e-2 * max|reference| for O, dX and
the three weight gradients (the bar the LM-head gradients are held to; the arithmetic is the same bf16
operand / fp32 accumulate / bf16 intermediate scheme); weight gradients bit-identical across runs."""
import numpy as np
import pytest

import mst_inputs as mi
from oracle import mlp_oracle as orc

pytestmark = pytest.mark.gpu

TOL = 2e-2
NAMES = ("O", "dX", "dWg", "dWu", "dWd")


def _harness():
    from tests.mlp_gpu_harness import MlpDeviceRun, f64
    return MlpDeviceRun, f64


def _reference(inp):
    return orc.mlp(inp.f64("X"), inp.f64("Wg"), inp.f64("Wu"), inp.f64("Wd"), inp.f64("dO"))


def _run_all(inp, M=None, pad=0):
    MlpDeviceRun, f64 = _harness()
    run = MlpDeviceRun(inp, M=M, pad_workspace=pad)
    O = run.forward()
    ws_f = run.last_ws
    dX, dWg, dWu, dWd = run.backward()
    got = {"O": f64(O), "dX": f64(dX), "dWg": f64(dWg), "dWu": f64(dWu), "dWd": f64(dWd)}
    return run, got, ws_f


def _check(inp, M=None):
    ref = _reference(inp)
    run, got, _ = _run_all(inp, M=M)
    errs = {}
    for k in NAMES:
        assert np.isfinite(got[k]).all(), f"{k}: not every element was written"
        scale = max(np.abs(ref[k]).max(), 1e-30)
        errs[k] = float(np.abs(got[k] - ref[k]).max() / scale)
        assert errs[k] <= TOL, f"{k}: max-abs error {errs[k]:.3e} of max|ref|"
    return run, got, ref, errs


def test_tiny_configuration_matches_oracle():
    _, _, _, errs = _check(mi.make_mlp_inputs(1))
    print("mlp cfg1 errors / max|ref|:", {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("S,d,I,M", [
    (300, 136, 200, 3),      # nothing a multiple of a tile; last chunk of 100 rows; I % 128 = 72
    (257, 64, 136, 1),       # one row into the second row tile; I % 16 == 8
    (64, 8, 8, 2),           # smallest legal d and I
    (1100, 264, 520, 2),     # several row tiles, several 128-wide and 256-wide tiles of I, ragged everywhere
    (520, 512, 1160, 5),     # d of two tiles; chunks of 104 rows
    (7, 16, 24, 7),          # one row per chunk
])
def test_ragged_shapes_match_oracle(S, d, I, M):
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(S, d, I, M, index=200 + S % 97, w_std=0.05))
    _check(inp)


@pytest.mark.parametrize("S,d,I,M", [
    (57, 656, 1680, 4), (526, 704, 1944, 3), (1920, 320, 584, 1), (513, 144, 1776, 10), (255, 672, 920, 5),
    (1151, 1008, 1184, 4), (2232, 1032, 512, 6), (7, 936, 1984, 5), (1498, 832, 416, 11), (512, 960, 512, 1),
    (257, 704, 1632, 7), (1, 8, 2048, 1),
])
def test_seeded_random_shapes_match_oracle(S, d, I, M):
    """Shapes drawn once from a seeded generator (S around the 255 / 256 / 257 / 512 / 513 tile edges and single rows,
    d from 8 to 1032, I from 416 to 2048, M up to 11, so that d spans several tiles of the dX and weight-gradient
    launches and the chunks are ragged): all five outputs against the oracle."""
    w_std = (0.02, 0.05, 0.3)[(S + I) % 3]
    _check(mi.make_mlp_inputs(mi.custom_mlp_config(S, d, I, M, index=300 + (S * 5 + I) % 89, w_std=w_std)))


def test_large_activations_saturate_without_nan():
    # gate pre-activations with |g| up to ~60: exp2 overflows inside the logistic function and must give 0, not NaN
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(256, 128, 256, 2, index=301, x_std=4.0, w_std=0.4))
    _check(inp)


@pytest.mark.parametrize("M", [1, 2, 4, 16])
def test_result_does_not_depend_on_m(M):
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(512, 128, 384, 1, index=302, w_std=0.05))
    _, base, _ = _run_all(inp, M=1)
    _, got, _ = _run_all(inp, M=M)
    # a token's O and dX rows never see the partition: bit-identical
    assert np.array_equal(got["O"], base["O"])
    assert np.array_equal(got["dX"], base["dX"])
    # weight gradients: same terms, different grouping of the fp32 sums
    for k in ("dWg", "dWu", "dWd"):
        scale = np.abs(base[k]).max()
        assert np.abs(got[k] - base[k]).max() <= 1e-5 * scale, k


def test_weight_gradients_are_bit_identical_across_runs():
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(700, 256, 640, 3, index=303, w_std=0.05))
    _, a, _ = _run_all(inp)
    _, b, _ = _run_all(inp)
    for k in NAMES:
        assert np.array_equal(a[k], b[k]), k


def test_zero_upstream_gradient_gives_zero_gradients():
    import torch
    MlpDeviceRun, f64 = _harness()
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(300, 64, 136, 2, index=304))
    run = MlpDeviceRun(inp)
    dX, dWg, dWu, dWd = run.backward(dO=torch.zeros_like(run.dO))
    for t in (dX, dWg, dWu, dWd):
        assert np.abs(f64(t)).max() == 0.0


def test_zero_gate_weights_closed_form():
    # Wg = 0: O = 0, dX = 0, dWu = 0, dWd = 0; dWg = (0.5 * dA * U)^T X  (silu'(0) = 1/2)
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(260, 64, 136, 2, index=305, w_std=0.1))
    inp.Wg_bits[:] = 0
    _, got, ref, _ = _check(inp)
    assert np.abs(got["O"]).max() == 0 and np.abs(got["dX"]).max() == 0
    assert np.abs(got["dWu"]).max() == 0 and np.abs(got["dWd"]).max() == 0
    assert np.abs(ref["dWg"]).max() > 0


def test_workspace_is_respected():
    MlpDeviceRun, _ = _harness()
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(300, 136, 200, 3, index=306))
    run = MlpDeviceRun(inp, pad_workspace=4096)
    run.forward()
    assert (run.last_ws[run.fwd_bytes:].cpu().numpy() == 0xA5).all(), "forward wrote past its declared workspace"
    run.backward()
    assert (run.last_ws[run.bwd_bytes:].cpu().numpy() == 0xA5).all(), "backward wrote past its declared workspace"
    assert run.fwd_bytes == -(-inp.cfg.C * inp.cfg.I * 2 // 256) * 256 or run.fwd_bytes == inp.cfg.C * inp.cfg.I * 2


def test_argument_errors_on_the_device_box():
    import torch
    MlpDeviceRun, _ = _harness()
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(64, 16, 40, 2, index=307))
    run = MlpDeviceRun(inp)
    O = torch.empty((64, 16), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(run.fwd_bytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(run.mst.MstError) as e:
        run.mst.mst_mlp_fwd(run.X, run.Wg, run.Wu, run.Wd, run.M, ws[: run.fwd_bytes - 256], O)
    assert e.value.status == -4
    with pytest.raises(run.mst.MstError) as e:
        run.mst.mst_mlp_fwd(run.X, run.Wg, run.Wu, run.Wd, 0, ws, O)
    assert e.value.status == -3


def test_repeated_calls_reuse_the_workspace():
    MlpDeviceRun, f64 = _harness()
    inp = mi.make_mlp_inputs(mi.custom_mlp_config(300, 136, 200, 3, index=308))
    ref = _reference(inp)
    run = MlpDeviceRun(inp)
    for _ in range(3):
        O = f64(run.forward())
        assert np.abs(O - ref["O"]).max() <= TOL * np.abs(ref["O"]).max()
        dX = f64(run.backward()[0])
        assert np.abs(dX - ref["dX"]).max() <= TOL * np.abs(ref["dX"]).max()
