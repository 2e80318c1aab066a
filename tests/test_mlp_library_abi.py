"""CPU-side checks of the MLP C-ABI library: it loads, exports every symbol its header declares, and its
host-only logic (workspace sizing, chunk policy, argument validation) behaves.  No kernel is launched here."""
import os
import re

import pytest

import mst_inputs as mi

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def mst():
    import paper_2407_15892_amd as m
    if not os.path.exists(m.mlp_binding.MLP_LIB_PATH) or not os.path.exists(m.binding.LIB_PATH):
        from paper_2407_15892_amd.build import build
        build()
    m.load_mlp_library()
    return m


def test_every_declared_symbol_is_exported(mst):
    text = open(os.path.join(ROOT, "include", "mst_mlp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(mst_mlp_[a-z_]+)\s*\(", text))
    assert {"mst_mlp_fwd", "mst_mlp_bwd", "mst_mlp_workspace_bytes", "mst_mlp_suggest_m"} <= names
    lib = mst.load_mlp_library()
    for n in sorted(names):
        assert hasattr(lib, n), f"{n} is declared in the header but not exported"
    assert "gfx950" in mst.mst_mlp_version()
    kinds = [lib.mst_mlp_profile_kind_name(i).decode() for i in range(mst.mlp_binding.MLP_PROFILE_KINDS)]
    assert kinds == ["gateup", "down", "da", "gateup_bwd", "dx", "dw"]
    assert lib.mst_mlp_profile_kind_name(mst.mlp_binding.MLP_PROFILE_KINDS).decode() == "?"


def test_workspace_is_chunk_sized(mst):
    for cfg in mi.MLP_CONFIGS.values():
        f, b = mst.mst_mlp_workspace_bytes(cfg.S, cfg.d, cfg.I, cfg.M)
        assert f == cfg.C * cfg.I * 2, cfg.name          # one chunk of the bf16 intermediate
        assert b == 3 * f, cfg.name                      # dA/dG, dU, A
        # the standard block would hold S x I; the chunked one holds 1/M of it
        assert f * cfg.M == cfg.S * cfg.I * 2
    _, b1 = mst.mst_mlp_workspace_bytes(8192, 4096, 14336, 2)
    _, b2 = mst.mst_mlp_workspace_bytes(32768, 4096, 14336, 8)    # same chunk, 4x the sequence
    assert b1 == b2


def test_chunk_policy_constant_chunk_equal_to_hidden_size(mst):
    sm = mst.mst_mlp_suggest_m
    assert sm(8192, 4096, 14336) == 2
    assert sm(32768, 4096, 14336) == 8
    assert sm(16384, 4096, 11008) == 4
    assert sm(1024, 4096, 14336) == 1      # sequence shorter than the chunk: no split
    assert sm(4096, 4096, 14336) == 1
    assert sm(10000, 4096, 14336) == 2     # nearest integer
    assert sm(0, 4096, 14336) == 0 and sm(8, 0, 8) == 0
    for cfg in mi.MLP_CONFIGS.values():
        assert sm(cfg.S, cfg.d, cfg.I) == cfg.M, cfg.name


def test_shape_and_m_validation(mst):
    st = mst.mlp_binding.mst_mlp_workspace_bytes_status
    assert st(8, 16, 32, 1) == 0
    assert st(0, 16, 32, 1) == -2
    assert st(8, 0, 32, 1) == -2
    assert st(8, 16, 0, 1) == -2
    assert st(8, 12, 32, 1) == -2            # d % 8 != 0
    assert st(8, 16, 36, 1) == -2            # I % 8 != 0
    assert st(8, 16, 32, 0) == -3
    assert st(8, 16, 32, 9) == -3            # M > S
    assert st(8, 1 << 16, 1 << 16, 1) == -2  # I * d >= 2^31
    assert st(1 << 20, 8, 1 << 15, 1) == -2  # one chunk of the intermediate >= 2^30 elements


def test_null_workspace_and_alignment_errors_come_before_any_launch(mst):
    lib = mst.load_mlp_library()
    S, d, I, M = 64, 16, 40, 2
    f, b = mst.mst_mlp_workspace_bytes(S, d, I, M)
    fake = 0x1000    # never dereferenced: validation fails first
    assert lib.mst_mlp_fwd(None, fake, fake, fake, S, d, I, M, fake, f, fake, None) == -1
    assert lib.mst_mlp_fwd(fake, fake, fake, fake, S, d, I, M, fake, f, None, None) == -1
    assert lib.mst_mlp_fwd(fake, fake, fake, fake, S, d, I, M, fake, f - 1, fake, None) == -4
    assert lib.mst_mlp_fwd(fake, fake, fake, fake, S, d, I, M, None, f, fake, None) == -4
    assert lib.mst_mlp_fwd(fake + 8, fake, fake, fake, S, d, I, M, fake, f, fake, None) == -5
    assert lib.mst_mlp_fwd(fake, fake, fake, fake, S, d, I, M, fake + 16, f, fake, None) == -5
    assert lib.mst_mlp_bwd(fake, fake, fake, fake, None, S, d, I, M, fake, b, fake, fake, fake, fake, None) == -1
    assert lib.mst_mlp_bwd(fake, fake, fake, fake, fake, S, d, I, M, fake, b, fake, fake, fake, None, None) == -1
    assert lib.mst_mlp_bwd(fake, fake, fake, fake, fake, S, d, I, M, fake, b - 1, fake, fake, fake, fake, None) == -4
    assert lib.mst_mlp_bwd(fake, fake, fake, fake, fake, S, d, I, M, fake, b, fake, fake + 2, fake, fake, None) == -5
    assert lib.mst_mlp_bwd(fake, fake, fake, fake, fake, S, d, I, 0, fake, b, fake, fake, fake, fake, None) == -3
