"""The forward entry point that allocates nothing (static device scratch inside the library), called through the
C ABI and compared with the ordinary forward entry point on the same inputs: loss, lse and n_valid must be
bit-identical (same kernels, same per-row arithmetic; only where the scratch lives differs).  Two calls in a row,
the second on a smaller input, so that what the first call left in the shared array cannot leak into the second."""
import ctypes

import numpy as np
import pytest

import mst_inputs as mi
from oracle import lmhead_ce_oracle as orc

pytestmark = pytest.mark.gpu


def _both(lib, torch, inp, M):
    """(loss, lse, n_valid) of the workspace entry point and of the static one, as numpy bit patterns."""
    import paper_2407_15892_amd as mst
    S, d, V = inp.cfg.S, inp.cfg.d, inp.cfg.V
    H = mi.to_device_bf16(inp.H_bits)
    W = mi.to_device_bf16(inp.W_bits)
    y = torch.from_numpy(inp.labels).cuda()
    fwd_bytes, _ = mst.mst_workspace_bytes(S, d, V, M)
    ws = torch.full((fwd_bytes,), 0x5A, dtype=torch.uint8, device="cuda")
    out = []
    for static in (False, True):
        loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((S,), float("nan"), dtype=torch.float32, device="cuda")
        nv = torch.full((1,), -7, dtype=torch.int64, device="cuda")
        stream = torch.cuda.current_stream().cuda_stream or None
        if static:
            rc = lib.mst_lmhead_ce_fwd_static(H.data_ptr(), W.data_ptr(), y.data_ptr(), S, d, V, inp.ignore_index, M,
                                              loss.data_ptr(), lse.data_ptr(), nv.data_ptr(), stream)
        else:
            rc = lib.mst_lmhead_ce_fwd(H.data_ptr(), W.data_ptr(), y.data_ptr(), S, d, V, inp.ignore_index, M,
                                       ws.data_ptr(), fwd_bytes, loss.data_ptr(), lse.data_ptr(), nv.data_ptr(), stream)
        assert rc == 0, (static, rc)
        torch.cuda.synchronize()
        out.append((loss.cpu().numpy().view(np.uint32), lse.cpu().numpy().view(np.uint32), int(nv.item()),
                    float(loss.item()), lse.cpu().numpy().astype(np.float64)))
    return out


def test_static_scratch_forward_matches_the_workspace_forward_twice():
    import torch
    import paper_2407_15892_amd as mst
    lib = mst.load_library()
    # first call: several mini-sequences per merge group and more than one group inside the 32 MiB array
    # (C = 1100 rows x 137 vocabulary tiles x 8 B = 1.2 MB per mini-sequence, 30 of them), ragged rows and vocabulary;
    # second call: a smaller problem whose every shape differs
    cases = [(mi.custom_config(33000, 128, 35000, 30, index=340, w_std=0.3, ignore_frac=0.03, label_dist="zipf"), 30),
             (mi.custom_config(700, 136, 900, 4, index=341, w_std=0.2, ignore_frac=0.1), 4)]
    for cfg, M in cases:
        inp = mi.make_inputs(cfg)
        (l0, lse0, nv0, _, _), (l1, lse1, nv1, loss1, lse1_f) = _both(lib, torch, inp, M)
        print(f"static forward S={cfg.S} V={cfg.V} M={M}: loss {loss1:.6f}, n_valid {nv1}", flush=True)
        assert nv0 == nv1 == inp.n_valid
        assert np.array_equal(l0, l1), "loss differs between the two entry points"
        assert np.array_equal(lse0, lse1), "lse differs between the two entry points"
        # and against the oracle, at the forward's bar
        ref_loss, ref_lse, _, ref_nv = orc.lmhead_ce_forward(inp.H_f64(), inp.W_f64(), inp.labels, inp.ignore_index)
        assert ref_nv == nv1
        assert abs(loss1 - ref_loss) <= 1e-3 * abs(ref_loss)
        assert np.abs(lse1_f - ref_lse).max() <= 2e-3 * max(1.0, np.abs(ref_lse).max())


def test_static_scratch_forward_replays_from_a_hip_graph():
    """The audience of this entry point: code under HIP graph capture.  After one eager call on the device (which takes
    the array's address and sets kernel attributes) the call is captured and every replay reproduces the eager bits."""
    import torch
    import paper_2407_15892_amd as mst
    inp = mi.make_inputs(mi.custom_config(900, 136, 5000, 3, index=342, w_std=0.3, ignore_frac=0.05))
    H, W = mi.to_device_bf16(inp.H_bits), mi.to_device_bf16(inp.W_bits)
    y = torch.from_numpy(inp.labels).cuda()
    loss = torch.zeros(1, dtype=torch.float32, device="cuda")
    lse = torch.empty(inp.cfg.S, dtype=torch.float32, device="cuda")
    nv = torch.zeros(1, dtype=torch.int64, device="cuda")

    def call():
        mst.mst_lmhead_ce_fwd_static(H, W, y, inp.ignore_index, inp.cfg.M, loss, lse, nv)

    call()
    torch.cuda.synchronize()
    ref = (loss.clone(), lse.clone(), nv.clone())
    assert int(ref[2]) == inp.n_valid
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for _ in range(3):
        loss.fill_(float("nan")); lse.fill_(float("nan")); nv.fill_(-5)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(loss.view(torch.int32), ref[0].view(torch.int32))
        assert torch.equal(lse.view(torch.int32), ref[1].view(torch.int32))
        assert int(nv) == int(ref[2])
    del graph
