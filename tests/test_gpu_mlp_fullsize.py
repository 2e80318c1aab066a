"""Full-size GPU parity of the MLP path at the Llama-shaped configurations, in the launch configuration
bench.py times (same M, same workspace sizes).  The oracle computes exact O and dX on a seeded sample of
token rows, exact rows of dWg and dWu on a seeded sample of intermediate indices and the exact sub-block of
dWd on sampled (hidden, intermediate) pairs; properties that hold at any size cover the rest: every element
finite and written, weight gradients bit-identical across runs."""
import time

import numpy as np
import pytest

import mst_inputs as mi
from oracle import mlp_oracle as orc

pytestmark = pytest.mark.gpu

TOL = 2e-2


@pytest.mark.parametrize("cfg_index", [2, 3, 4])
def test_fullsize_mlp_configuration_matches_oracle_on_samples(cfg_index):
    import torch
    from tests.mlp_gpu_harness import MlpDeviceRun, f64

    cfg = mi.MLP_CONFIGS[cfg_index]
    t0 = time.time()
    inp = mi.make_mlp_inputs(cfg)
    run = MlpDeviceRun(inp)
    assert run.fwd_bytes == cfg.C * cfg.I * 2 and run.bwd_bytes == 3 * cfg.C * cfg.I * 2
    O = run.forward()
    dX, dWg, dWu, dWd = run.backward()
    first = [t.clone() for t in (dWg, dWu, dWd)]
    print(f"mlp cfg {cfg_index}: inputs+gpu {time.time() - t0:.1f}s", flush=True)

    t0 = time.time()
    rng = np.random.default_rng(2000 + cfg_index)
    rows = np.unique(np.concatenate([[0, cfg.S - 1, cfg.C - 1, cfg.C % cfg.S, 255, 256], rng.integers(0, cfg.S, 26)]))
    irows = np.unique(np.concatenate([[0, cfg.I - 1, 127, 128, 255, 256], rng.integers(0, cfg.I, 18)]))
    hrows = np.unique(np.concatenate([[0, cfg.d - 1, 255, 256], rng.integers(0, cfg.d, 12)]))
    ref = orc.mlp_grads_sampled(inp.f64("X"), inp.f64("Wg"), inp.f64("Wu"), inp.f64("Wd"), inp.f64("dO"),
                                rows, irows, hrows)
    print(f"mlp cfg {cfg_index}: oracle {time.time() - t0:.1f}s", flush=True)

    tr, ti, th = (torch.from_numpy(a).cuda() for a in (rows, irows, hrows))
    got = {
        "O": f64(O[tr]), "dX": f64(dX[tr]), "dWg": f64(dWg[ti]), "dWu": f64(dWu[ti]),
        "dWd": f64(dWd[th][:, ti]),
    }
    full_max = {"O": float(O.float().abs().max()), "dX": float(dX.float().abs().max()),
                "dWg": float(dWg.abs().max()), "dWu": float(dWu.abs().max()), "dWd": float(dWd.abs().max())}
    errs = {}
    for k in got:
        assert got[k].shape == ref[k].shape, k
        # the sampled reference itself sets the scale (stricter than the maximum over the whole tensor)
        errs[k] = float(np.abs(got[k] - ref[k]).max() / np.abs(ref[k]).max())
        assert np.abs(ref[k]).max() <= 1.5 * full_max[k] + 1e-30, k
    print(f"mlp cfg {cfg_index}: max-abs error / max|ref| on samples:", {k: f"{v:.2e}" for k, v in errs.items()}, flush=True)
    for k, v in errs.items():
        assert v <= TOL, (k, v)

    for t in (O, dX):
        assert torch.isfinite(t.float()).all()
    for t in (dWg, dWu, dWd):
        assert torch.isfinite(t).all()
    run.forward()
    again = run.backward()[1:]
    for a, b in zip(first, again):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
