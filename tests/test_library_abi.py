"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares, and
its host-only logic (workspace sizing, chunk arithmetic limits, argument validation) behaves.
No kernel is launched here."""
import ctypes
import os
import re

import pytest

import mst_inputs as mi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mst():
    import paper_2407_15892_amd as m
    if not os.path.exists(m.binding.LIB_PATH):
        from paper_2407_15892_amd.build import build
        build()
    m.load_library()
    return m


def test_every_declared_symbol_is_exported(mst):
    text = open(os.path.join(ROOT, "include", "mst_lmhead.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(mst_[a-z_]+)\s*\(", text))
    assert {"mst_lmhead_ce_fwd", "mst_lmhead_ce_bwd", "mst_workspace_bytes", "mst_strerror"} <= names
    lib = mst.load_library()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"
    assert "gfx950" in mst.mst_version()


def test_workspace_stays_below_one_fp32_logits_chunk(mst):
    for cfg in mi.CONFIGS.values():
        f, b = mst.mst_workspace_bytes(cfg.S, cfg.d, cfg.V, cfg.M)
        cap = cfg.C * cfg.V * 4
        assert 0 < f <= cap and 0 < b <= cap, (cfg.name, f, b, cap)
        assert b == cap          # two bf16 dlogits chunks fill exactly one fp32 logits chunk
        # never a function of the full S x V logits
        assert b < cfg.S * cfg.V * 2 or cfg.M == 1


def test_workspace_scales_with_chunk_not_with_sequence(mst):
    _, b1 = mst.mst_workspace_bytes(8192, 4096, 128256, 8)
    _, b2 = mst.mst_workspace_bytes(32768, 4096, 128256, 32)   # same chunk length, 4x the sequence
    assert b1 == b2
    _, b3 = mst.mst_workspace_bytes(8192, 4096, 128256, 16)    # half the chunk
    assert b3 * 2 == b1


def test_shape_and_m_validation(mst):
    st = mst.binding.mst_workspace_bytes_status
    assert st(8, 16, 32, 1) == 0
    assert st(0, 16, 32, 1) == -2
    assert st(8, 0, 32, 1) == -2
    assert st(8, 16, 0, 1) == -2
    assert st(8, 12, 32, 1) == -2          # d % 8 != 0
    assert st(8, 16, 32, 0) == -3
    assert st(8, 16, 32, 9) == -3          # M > S
    assert st(8, 1 << 16, 1 << 16, 1) == -2   # V * d >= 2^31
    assert st(1 << 20, 8, 1 << 15, 1) == -2   # one chunk's dlogits >= 2^31 elements
    for code in (0, -1, -2, -3, -4, -5, -6, -7):
        assert isinstance(mst.mst_strerror(code), str) and mst.mst_strerror(code)


def test_null_and_workspace_errors_come_before_any_launch(mst):
    lib = mst.load_library()
    S, d, V, M = 64, 16, 40, 2
    f, b = mst.mst_workspace_bytes(S, d, V, M)
    fake = 0x1000   # never dereferenced: validation fails first
    # NULL H
    assert lib.mst_lmhead_ce_fwd(None, fake, fake, S, d, V, -100, M, fake, f, fake, None, None, None) == -1
    # NULL loss
    assert lib.mst_lmhead_ce_fwd(fake, fake, fake, S, d, V, -100, M, fake, f, None, None, None, None) == -1
    # workspace too small / NULL
    assert lib.mst_lmhead_ce_fwd(fake, fake, fake, S, d, V, -100, M, fake, f - 1, fake, None, None, None) == -4
    assert lib.mst_lmhead_ce_fwd(fake, fake, fake, S, d, V, -100, M, None, f, fake, None, None, None) == -4
    # misaligned H
    assert lib.mst_lmhead_ce_fwd(fake + 2, fake, fake, S, d, V, -100, M, fake, f, fake, None, None, None) == -5
    # backward: NULL dW, small workspace (with and without lse)
    assert lib.mst_lmhead_ce_bwd(fake, fake, fake, S, d, V, -100, M, 1.0, fake, fake, fake, b, fake, None, None) == -1
    assert lib.mst_lmhead_ce_bwd(fake, fake, fake, S, d, V, -100, M, 1.0, fake, fake, fake, b - 1, fake, fake, None) == -4
    assert lib.mst_lmhead_ce_bwd(fake, fake, fake, S, d, V, -100, M, 1.0, fake, None, fake, b, fake, fake, None) == -4
    assert lib.mst_lmhead_ce_bwd(fake, fake, fake, S, d, V, -100, M, 1.0, None, None, fake, b + 512, fake, fake, None) == -4


def test_profile_kind_names(mst):
    lib = mst.load_library()
    names = [lib.mst_profile_kind_name(i).decode() for i in range(mst.binding.PROFILE_KINDS)]
    assert names[1] == "fwd_gemm_lse" and names[-1] == "bwd_gemm_dh_dw" and len(set(names)) == len(names)


def test_chunk_count_policy(mst):
    """Section 3.4: M = V / d for the LM head; never chunks shorter than one 256-row tile."""
    assert mst.mst_suggest_m(32768, 4096, 128256) == 31      # 31.3 -> 31 (the paper rounds this to 32)
    assert mst.mst_suggest_m(131072, 3584, 256000) == 71     # 71.4 -> 71 (the paper quotes 64)
    assert mst.mst_suggest_m(8192, 4096, 128256) == 31
    assert mst.mst_suggest_m(1024, 4096, 128256) == 4        # the 11x-slowdown case: keep 256-row chunks
    assert mst.mst_suggest_m(100, 4096, 128256) == 1         # short sequence: do not split
    assert mst.mst_suggest_m(8192, 4096, 1000) == 1
    assert mst.mst_suggest_m(0, 4096, 1000) == 0
    for S, d, V in [(8192, 4096, 128256), (777, 264, 1000), (64, 8, 40)]:
        M = mst.mst_suggest_m(S, d, V)
        assert 1 <= M <= S and mst.binding.mst_workspace_bytes_status(S, d, V, M) == 0


def test_shift_labels_argument_errors(mst):
    lib = mst.load_library()
    fake = 0x1000
    assert lib.mst_shift_labels(None, 2, 3, -100, fake, None) == -1
    assert lib.mst_shift_labels(fake, 2, 3, -100, None, None) == -1
    assert lib.mst_shift_labels(fake, 0, 3, -100, fake, None) == -2
    assert lib.mst_shift_labels(fake, 2, 0, -100, fake, None) == -2
    assert lib.mst_shift_labels(fake, 1 << 30, 1 << 30, -100, fake, None) == -2
    assert lib.mst_shift_labels(fake + 2, 2, 3, -100, fake, None) == -5


def test_mfma_probe_argument_errors(mst):
    lib = mst.load_library()
    fake = 0x1000
    assert lib.mst_mfma_probe(0, 10, 1.0, fake, None) == -2
    assert lib.mst_mfma_probe(8, 0, 1.0, fake, None) == -2
    assert lib.mst_mfma_probe(8, (1 << 20) + 1, 1.0, fake, None) == -2
    assert lib.mst_mfma_probe(8, 10, 1.0, None, None) == -1


def test_backward_schedule_choice_and_block_shapes(mst):
    """Host-only: which order of the backward pass the cost model picks, and that a block shape always fits the
    bytes mst_workspace_bytes reports."""
    try:
        for cfg in mi.CONFIGS.values():
            _, cap = mst.mst_workspace_bytes(cfg.S, cfg.d, cfg.V, cfg.M)
            mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_AUTO)
            auto = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
            mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_PAIRS)
            pairs = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
            assert pairs["schedule"] == mst.BWD_SCHEDULE_PAIRS
            assert pairs["rows_per_block"] == 2 * cfg.C and pairs["windows"] == 1 and pairs["vocab_per_window"] == cfg.V
            mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_BLOCKS)
            blocks = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
            assert blocks["schedule"] in (mst.BWD_SCHEDULE_BLOCKS, mst.BWD_SCHEDULE_PAIRS)   # never fused unless asked
            mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_BLOCKS_FUSED)
            fused = mst.mst_bwd_schedule_info(cfg.S, cfg.d, cfg.V, cfg.M)
            assert fused["schedule"] in (mst.BWD_SCHEDULE_BLOCKS_FUSED, mst.BWD_SCHEDULE_PAIRS)
            if blocks["schedule"] == mst.BWD_SCHEDULE_BLOCKS:
                R, Vw = blocks["rows_per_block"], blocks["vocab_per_window"]
                assert R % 256 == 0 and Vw % 256 == 0 and blocks["windows"] >= 2
                assert blocks["row_blocks"] == -(-cfg.S // R) and blocks["windows"] == -(-cfg.V // Vw)
                # dlogits of the block (bf16) and the fp32 dH sums of its rows fit the same bytes
                assert R * Vw * 2 + R * cfg.d * 4 + 256 <= cap, (cfg.name, blocks, cap)
            # the automatic choice is the cheaper estimate
            if 0 < auto["est_blocks_us"] < auto["est_pairs_us"]:
                assert auto["schedule"] in (mst.BWD_SCHEDULE_BLOCKS, mst.BWD_SCHEDULE_BLOCKS_FUSED), (cfg.name, auto)
            else:
                assert auto["schedule"] == mst.BWD_SCHEDULE_PAIRS, (cfg.name, auto)
        # large vocabulary, short chunks: blocks; tiny problems: pairs
        mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_AUTO)
        # where blocks win, the automatic choice lets dH and dW share a launch
        assert mst.mst_bwd_schedule_info(8192, 4096, 128256, 8)["schedule"] == mst.BWD_SCHEDULE_BLOCKS_FUSED
        assert mst.mst_bwd_schedule_info(16384, 3584, 256000, 16)["schedule"] == mst.BWD_SCHEDULE_BLOCKS_FUSED
        assert mst.mst_bwd_schedule_info(512, 256, 4096, 4)["schedule"] == mst.BWD_SCHEDULE_PAIRS
        with pytest.raises(mst.MstError):
            mst.mst_set_bwd_schedule(7)
    finally:
        mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_AUTO)


def test_block_shapes_fit_and_cover_for_random_shapes(mst):
    """Host-only property test of the block schedule's shapes: whenever one is offered it covers S x V with whole
    tiles, fits the reported workspace bytes together with the fp32 dH sums, and keeps 32-bit offsets in range."""
    import random
    rng = random.Random(20240715)
    offered = 0
    try:
        mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_BLOCKS)
        for _ in range(400):
            d = 8 * rng.randint(1, 1024)
            V = rng.randint(1, 300000)
            S = rng.randint(1, 200000)
            M = rng.randint(1, min(S, 256))
            if mst.binding.mst_workspace_bytes_status(S, d, V, M) != 0:
                continue
            _, cap = mst.mst_workspace_bytes(S, d, V, M)
            info = mst.mst_bwd_schedule_info(S, d, V, M)
            C = -(-S // M)
            if info["schedule"] == mst.BWD_SCHEDULE_PAIRS:
                assert info["rows_per_block"] == 2 * C and info["windows"] == 1
                continue
            assert info["schedule"] == mst.BWD_SCHEDULE_BLOCKS
            offered += 1
            R, Vw = info["rows_per_block"], info["vocab_per_window"]
            assert R >= 256 and R % 256 == 0 and Vw >= 256 and Vw % 256 == 0
            assert info["windows"] >= 2 and (info["windows"] - 1) * Vw < V <= info["windows"] * Vw
            assert (info["row_blocks"] - 1) * R < S <= info["row_blocks"] * R
            # bf16 dlogits of the block + fp32 dH sums of its rows, kept as whole 256-column tiles
            assert R * Vw * 2 + 256 + R * (-(-d // 256) * 256) * 4 <= cap, (S, d, V, M, info, cap)
            assert R * Vw < 2 ** 30 and R * d < 2 ** 30
        assert offered > 50
    finally:
        mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_AUTO)


def test_profile_kind_count_matches_the_library(mst):
    """mst_profile_collect fills MST_PROFILE_KINDS entries: the binding's array length has to be that number."""
    lib = mst.load_library()
    names = []
    while lib.mst_profile_kind_name(len(names)).decode() != "?":
        names.append(lib.mst_profile_kind_name(len(names)).decode())
    assert len(names) == mst.binding.PROFILE_KINDS, names
    header = open(os.path.join(os.path.dirname(__file__), "..", "include", "mst_lmhead.h")).read()
    enum = header[header.index("MST_K_LABEL_SCAN = 0"):header.index("MST_PROFILE_KINDS\n")]
    assert enum.count("MST_K_") == len(names)


def test_schedule_override_is_per_thread_and_the_pure_query_ignores_it(mst):
    """The override set by one thread is invisible to another thread's calls, and mst_bwd_schedule_info_for answers
    for an explicit override without reading or changing any state."""
    import threading
    shape = (8192, 4096, 128256, 8)
    seen = {}
    try:
        mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_PAIRS)
        assert mst.mst_bwd_schedule_info(*shape)["schedule"] == mst.BWD_SCHEDULE_PAIRS

        def other():
            seen["fresh_thread"] = mst.mst_bwd_schedule_info(*shape)["schedule"]
            mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_BLOCKS)
            seen["after_own_set"] = mst.mst_bwd_schedule_info(*shape)["schedule"]

        th = threading.Thread(target=other)
        th.start()
        th.join()
        assert seen["fresh_thread"] == mst.BWD_SCHEDULE_BLOCKS_FUSED    # AUTO's choice for this shape
        assert seen["after_own_set"] == mst.BWD_SCHEDULE_BLOCKS
        assert mst.mst_bwd_schedule_info(*shape)["schedule"] == mst.BWD_SCHEDULE_PAIRS   # this thread's is untouched
        for forced, want in ((mst.BWD_SCHEDULE_AUTO, mst.BWD_SCHEDULE_BLOCKS_FUSED), (mst.BWD_SCHEDULE_PAIRS, mst.BWD_SCHEDULE_PAIRS),
                             (mst.BWD_SCHEDULE_BLOCKS, mst.BWD_SCHEDULE_BLOCKS),
                             (mst.BWD_SCHEDULE_BLOCKS_FUSED, mst.BWD_SCHEDULE_BLOCKS_FUSED)):
            assert mst.mst_bwd_schedule_info(*shape, schedule=forced)["schedule"] == want
        assert mst.mst_bwd_schedule_info(*shape)["schedule"] == mst.BWD_SCHEDULE_PAIRS
        info = (ctypes.c_int64 * 8)()
        assert mst.load_library().mst_bwd_schedule_info_for(*shape, 9, info) == -2
        assert mst.load_library().mst_bwd_schedule_info_for(*shape, 0, None) == -1
    finally:
        mst.mst_set_bwd_schedule(mst.BWD_SCHEDULE_AUTO)


def test_static_scratch_forward_rejects_what_does_not_fit(mst):
    """A call whose per-row scratch alone exceeds the static array: refused on the host, nothing launched."""
    lib = mst.load_library()
    S, d, V, M = 8_400_000, 8, 8, 8400     # 4 bytes per row = 33.6 MB > 32 MiB
    assert 4 * S > mst.binding.STATIC_SCRATCH_BYTES
    fake = 0x10000
    assert mst.binding.mst_workspace_bytes_status(S, d, V, M) == 0          # the shape itself is accepted
    rc = lib.mst_lmhead_ce_fwd_static(fake, fake, fake, S, d, V, -100, M, fake, None, None, None)
    assert rc == -4 and "workspace" in mst.mst_strerror(rc)


def test_workgroup_to_tile_map_is_a_bijection(mst):
    """The GEMM kernels' XCD-aware map from the linear workgroup id to a tile (the same function, called on the
    host): every tile of the space is hit by exactly one workgroup, padding workgroups report themselves, each XCD
    (workgroup id mod 8) owns a contiguous range of the slow coordinate, and the 32 workgroups that are resident
    on an XCD at a time read at most 12 distinct operand panels."""
    lib = mst.load_library()
    lib.mst_tile_grid.restype = ctypes.c_int32
    lib.mst_tile_of_workgroup.restype = ctypes.c_int32
    s, f = ctypes.c_int32(), ctypes.c_int32()
    shapes = [(1, 1), (3, 5), (8, 4), (9, 33), (63, 32), (501, 4), (16, 16), (63, 16), (125, 64), (32, 16), (7, 100)]
    for n_slow, n_fast, order in [sh + (o,) for sh in shapes for o in (0, 1)]:
        grid = lib.mst_tile_grid(n_slow, n_fast)
        assert grid == 8 * -(-n_slow // 8) * n_fast
        seen = {}
        per_xcd = {x: [] for x in range(8)}
        for b in range(grid):
            rc = lib.mst_tile_of_workgroup(n_slow, n_fast, order, b, ctypes.byref(s), ctypes.byref(f))
            assert rc in (0, 1)
            if rc == 0:
                per_xcd[b % 8].append(None)                         # a padding workgroup still takes a slot of its round
            if rc == 1:
                assert 0 <= s.value < n_slow and 0 <= f.value < n_fast
                assert (s.value, f.value) not in seen, (n_slow, n_fast, b)
                seen[(s.value, f.value)] = b
                per_xcd[b % 8].append((s.value, f.value))
        assert len(seen) == n_slow * n_fast
        spx = -(-n_slow // 8)
        for x, tiles in per_xcd.items():
            assert all(x * spx <= t[0] < (x + 1) * spx for t in tiles if t)
            for r0 in range(0, len(tiles), 32):                     # one round of resident workgroups
                rnd = [t for t in tiles[r0:r0 + 32] if t]
                panels = len({t[0] for t in rnd}) + len({t[1] for t in rnd})
                if spx >= 4 and n_fast >= 8:
                    assert panels <= 13, (n_slow, n_fast, x, r0, panels)
    assert lib.mst_tile_of_workgroup(4, 4, 0, -1, ctypes.byref(s), ctypes.byref(f)) == -1
    assert lib.mst_tile_of_workgroup(4, 4, 0, 10 ** 6, ctypes.byref(s), ctypes.byref(f)) == -1
    assert lib.mst_tile_of_workgroup(4, 4, 2, 0, ctypes.byref(s), ctypes.byref(f)) == -1
    assert lib.mst_tile_grid(0, 4) == -1
