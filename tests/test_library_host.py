"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, and its host-only helpers agree with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import slim_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "slim.h")


@pytest.fixture(scope="module")
def binding():
    from paper_2405_14917_amd import binding as b
    if not os.path.exists(b.LIB_PATH):
        from paper_2405_14917_amd import build
        build.build(verbose=False)
    return b


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slim_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(binding):
    lib = binding.load()
    names = _declared_symbols()
    assert len(names) >= 17
    for name in names:
        assert hasattr(lib, name), "libslim.so does not export %s" % name
    assert sorted(binding.EXPORTS) == names


def test_default_tau_is_the_oracle_grid_bit_for_bit(binding):
    tau = binding.default_tau()
    ref = orc.tau_grid(0.1, 50)
    assert tau.shape == ref.shape == (100,)
    assert np.array_equal(tau.view(np.uint64), ref.view(np.uint64))


def test_default_params_and_mode_constants(binding):
    lib = binding.load()
    p = binding.SlimParams(7, 7, 7, 7)
    lib.slim_default_params(ctypes.byref(p))
    assert (p.sqc_weight_mode, p.mask_scope, p.q1_mode, p.sal_mode) == (0, 0, 0, 0)
    # the header's mode values are an interface shared with the oracle's switches
    text = open(HEADER).read()
    for name, val in (("SLIM_WEIGHT_MASK_MEAN", orc.WEIGHT_MASK_MEAN), ("SLIM_WEIGHT_UNIFORM", orc.WEIGHT_UNIFORM),
                      ("SLIM_WEIGHT_ELEMENT", orc.WEIGHT_ELEMENT), ("SLIM_Q1_SIGN", orc.Q1_SIGN),
                      ("SLIM_Q1_AFFINE", orc.Q1_AFFINE), ("SLIM_SCOPE_BLOCK", orc.SCOPE_BLOCK),
                      ("SLIM_SCOPE_ROW", orc.SCOPE_ROW), ("SLIM_SAL_HINV_DIAG", orc.SAL_HINV_DIAG),
                      ("SLIM_SAL_CHOL_DIAG", orc.SAL_CHOL_DIAG)):
        assert re.search(r"\b%s\s*=\s*%d\b" % (name, val), text), name


def test_null_context_is_rejected_without_a_gpu(binding):
    lib = binding.load()
    assert lib.slim_destroy(None) == binding.ERR_INVALID_ARG
    assert lib.slim_profile_enable(None, 1) == binding.ERR_INVALID_ARG
    assert lib.slim_workspace_bytes(None) == 0
    assert lib.slim_last_error(None) == b"null context"
    nt = ctypes.c_int64(0)
    assert lib.slim_hessian_accumulate(None, None, 0, 8, 8, 8, None, 8, ctypes.byref(nt)) == binding.ERR_INVALID_ARG


def test_missing_library_fails_loudly(binding, monkeypatch, tmp_path):
    """There is no CPU fallback: without the built library the binding raises instead of computing anything."""
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libslim.so"))
    with pytest.raises(FileNotFoundError):
        binding.load()
    with pytest.raises(FileNotFoundError):
        binding.default_tau()


def test_the_product_never_imports_the_oracle():
    """The oracle is test infrastructure: nothing in the package refers to it."""
    pkg = os.path.join(ROOT, "paper_2405_14917_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f), errors="ignore").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), f
                assert "slim_oracle" not in text, f


def test_workspace_query_is_host_only_and_follows_the_entry_points(binding):
    """slim_workspace_query needs no GPU; for the benchmark shapes the inverse (two m x m fp64 matrices), the bit
    allocation (three n x m and two n x t_s fp64 matrices) or the partial tiles of the Gram matrix dominate."""
    q = binding.workspace_query
    assert q(0, 0, 0) == 0
    m = 4096
    assert q(0, m, 0) >= 2 * 8 * m * m                        # the inverse alone
    assert q(0, m, 0, t_c=131072, num_cus=256) >= q(0, m, 0)   # plus the Gram matrix's partial tiles
    n, beta, ts = 4096, 128, 2048
    sba = 3 * 8 * n * m + 2 * 8 * m * ts + 2 * 8 * n * ts
    assert q(n, m, beta, t_s=ts) >= sba
    assert q(n, m, beta) >= 8 * n * m + 8 * n * 512           # the sweep: working copy of W and a window of errors
    full = q(n, m, beta, 131072, ts, 16, 256)
    assert full == max(q(0, m, 0, t_c=131072, num_cus=256), q(n, m, beta, t_s=ts), q(n, m, beta, t_x=16, num_cus=256))
    # a small Gram matrix is split into more token ranges: the requirement is not monotone in m
    assert q(0, 256, 0, t_c=1 << 20, num_cus=256) > 0


def test_bench_inverse_work_formulas_add_up():
    """The per-site flop counts that bench.py rates the inverse's products with share out (2/3) m^3 (the factorisation
    and the triangular inverse, triangles counted once) without gaps or double counting; the diagonal blocks' own
    work (64^3 each, inside the diagonal kernel) is what is left."""
    import bench
    from paper_2405_14917_amd import synth
    for name in ("C2", "C3", "C4", "C5"):
        cfg = synth.CONFIGS[name]
        m = cfg.m
        sites = ("inv_panel_dgemm", "inv_window_dgemm", "inv_group_next_dgemm", "inv_syrk_dgemm", "inv_trtri_dgemm",
                 "inv_trtri_rows_dgemm", "inv_trtri_terms_dgemm")
        total = 0.0
        for s in sites:
            bound, peak, work = bench.algorithmic_work(s, cfg, 1)
            assert bound == "mfma" and work > 0.0
            total += work
        whole = 2.0 * m ** 3 / 3.0
        # the diagonal kernel's share is about (m / 64) * 64^3 flops: a few parts in ten thousand at these sizes
        assert 0.97 * whole < total < 1.03 * whole, (name, total / whole)
