"""Full-size GPU parity at the benchmark configurations, in the launch configuration bench.py times
(same M, same workspace sizes).  The oracle computes the loss and the log-sum-exp of every row
exactly (one streamed fp64 forward pass), exact dH on a seeded sample of token rows and exact dW on
a seeded sample of vocabulary rows; properties that hold at any size cover the rest:
columns of dW sum to ~0, ignored rows of dH are exactly 0, dW is bit-identical across runs."""
import time

import numpy as np
import pytest

import mst_inputs as mi
from oracle import lmhead_ce_oracle as orc

pytestmark = pytest.mark.gpu

LOSS_RTOL = 1e-3
GRAD_TOL = 2e-2


@pytest.mark.parametrize("cfg_index", [2, 3, 4, 5])
def test_fullsize_config_matches_oracle_on_samples(cfg_index):
    import torch
    from tests.gpu_harness import DeviceRun, bf16_tensor_to_f64

    cfg = mi.CONFIGS[cfg_index]
    t0 = time.time()
    inp = mi.make_inputs(cfg)
    run = DeviceRun(inp)
    cap = cfg.C * cfg.V * 4
    assert run.fwd_bytes <= cap and run.bwd_bytes <= cap, "workspace exceeds one fp32 logits chunk"
    loss, lse, nv = run.forward()
    dH, dW = run.backward()
    dW_first = dW.clone()
    print(f"cfg {cfg_index}: inputs+gpu {time.time() - t0:.1f}s", flush=True)

    # --- oracle: exact loss and lse for all rows, gradients on samples
    t0 = time.time()
    W64 = inp.W_f64()
    H64 = inp.H_f64()
    ref_loss, ref_lse, ref_nll, ref_nv = orc.lmhead_ce_forward(H64, W64, inp.labels, inp.ignore_index, block_rows=1024)
    rng = np.random.default_rng(1000 + cfg_index)
    rows = np.unique(np.concatenate([[0, cfg.S - 1, cfg.C - 1, cfg.C], rng.integers(0, cfg.S, 28),
                                     np.flatnonzero(inp.labels == inp.ignore_index)[:2]]))
    valid_labels = inp.labels[inp.labels != inp.ignore_index]
    hot = np.bincount(valid_labels, minlength=cfg.V).argmax()
    vrows = np.unique(np.concatenate([[0, cfg.V - 1, 255, 256, hot], valid_labels[:6], rng.integers(0, cfg.V, 20)]))
    dH_ref, dW_ref = orc.lmhead_ce_grads_sampled(H64, W64, inp.labels, ref_lse, ref_nv, rows, vrows,
                                                 inp.ignore_index, block_rows=4096)
    print(f"cfg {cfg_index}: oracle {time.time() - t0:.1f}s", flush=True)

    assert nv == ref_nv == inp.n_valid
    assert abs(loss - ref_loss) <= LOSS_RTOL * abs(ref_loss), (loss, ref_loss)
    assert np.abs(lse - ref_lse).max() <= 2e-3 * np.abs(ref_lse).max()

    dH_s = bf16_tensor_to_f64(dH[torch.from_numpy(rows).cuda()])
    dW_s = dW[torch.from_numpy(vrows).cuda()].cpu().numpy().astype(np.float64)
    # scale: max |gradient| over the whole GPU tensor is within tolerance of max |ref| (checked on the
    # samples), so use the larger of the sampled reference maximum and the GPU tensor maximum
    sH = max(np.abs(dH_ref).max(), float(dH.float().abs().max()))
    sW = max(np.abs(dW_ref).max(), float(dW.abs().max()))
    eH = np.abs(dH_s - dH_ref).max() / sH
    eW = np.abs(dW_s - dW_ref).max() / sW
    print(f"cfg {cfg_index}: loss {loss:.6f} ref {ref_loss:.6f}; dH err {eH:.2e}; dW err {eW:.2e} (of max|grad|)", flush=True)
    assert eH <= GRAD_TOL and eW <= GRAD_TOL
    # tighter: on the hot rows the sampled reference itself sets the scale
    assert np.abs(dH_s - dH_ref).max() <= GRAD_TOL * np.abs(dH_ref).max()
    assert np.abs(dW_s - dW_ref).max() <= GRAD_TOL * np.abs(dW_ref).max()

    # --- properties at full size
    ign = torch.from_numpy(inp.labels == inp.ignore_index).cuda()
    assert float(dH[ign].float().abs().max()) == 0.0
    assert torch.isfinite(dW).all() and torch.isfinite(dH.float()).all()
    col_sums = dW.double().sum(dim=0).abs().max().item()
    # rows of bf16 dlogits sum to zero within 2^-8 relative steps; bound by mean|H| * 2^-7 per unit grad_loss
    assert col_sums <= 2.0 ** -7 * max(cfg.h_std, 1e-3), col_sums
    # bit-identical dW on a second run
    run.forward()
    _, dW2 = run.backward()
    assert torch.equal(dW_first.view(torch.int32), dW2.view(torch.int32))

    # --- the other order of the backward pass against the same references
    import paper_2407_15892_amd as mst
    chosen = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
    other = mst.BWD_SCHEDULE_BLOCKS if chosen["schedule"] == mst.BWD_SCHEDULE_PAIRS else mst.BWD_SCHEDULE_PAIRS
    try:
        mst.mst_set_bwd_schedule(other)
        forced = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
        print(f"cfg {cfg_index}: default schedule {chosen}, also run {forced}", flush=True)
        if forced["schedule"] == other:
            dH_o, dW_o = run.backward()
            dH_os = bf16_tensor_to_f64(dH_o[torch.from_numpy(rows).cuda()])
            dW_os = dW_o[torch.from_numpy(vrows).cuda()].cpu().numpy().astype(np.float64)
            assert np.abs(dH_os - dH_ref).max() <= GRAD_TOL * np.abs(dH_ref).max()
            assert np.abs(dW_os - dW_ref).max() <= GRAD_TOL * np.abs(dW_ref).max()
            assert float(dH_o[ign].float().abs().max()) == 0.0
            assert torch.isfinite(dW_o).all() and torch.isfinite(dH_o.float()).all()
            # both orders form the same products; only the fp32 summation order differs
            assert float((dW_o - dW_first).abs().max()) <= 1e-3 * float(dW_first.abs().max())
    finally:
        mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_AUTO)
