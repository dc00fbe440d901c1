"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, derives the same sizes as the oracle, and rejects bad calls before
launching anything."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import draft_attention as oa
from paper_2505_14708_amd import binding as da
from paper_2505_14708_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.skipif(not os.path.exists(da.LIB_PATH), reason="library not built")

FAKE = 0x10000  # a non-NULL, 16-byte aligned value that is never dereferenced on the error paths


def _exported(path):
    """Dynamic symbols a shared library defines."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], capture_output=True, text=True, check=True).stdout
    return {line.split()[-1] for line in out.splitlines() if line.strip()}


def test_every_declared_symbol_is_exported():
    """include/ holds da.h alone; the product library exports what it declares, and none of the bench's
    measuring sticks (they live in a library of their own)."""
    header = open(os.path.join(ROOT, "include", "da.h")).read()
    declared = set(re.findall(r"\b(da_[a-z0-9_]+)\s*\(", header))
    assert declared == set(da.EXPORTS)
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["da.h"]
    L = da.lib()
    for name in declared:
        assert getattr(L, name) is not None
    c_names = {n for n in _exported(da.LIB_PATH) if n.startswith("da_")}
    assert c_names == declared, c_names ^ declared


def test_probe_library_is_separate():
    from paper_2505_14708_amd import probe
    if not os.path.exists(probe.LIB_PATH):
        pytest.skip("probe library not built")
    header = open(os.path.join(ROOT, "paper_2505_14708_amd", "csrc", "probe", "da_probe.h")).read()
    declared = set(re.findall(r"\b(da_[a-z0-9_]+)\s*\(", header))
    assert declared == set(probe.EXPORTS)
    assert {n for n in _exported(probe.LIB_PATH) if n.startswith("da_")} == declared


def test_struct_layout_matches_header():
    assert ctypes.sizeof(da.da_problem) == 56 and da.da_problem.sparsity.offset == 40 and da.da_problem.pool.offset == 48
    assert ctypes.sizeof(da.da_dims) == 40 and da.da_dims.n.offset == 24
    assert ctypes.sizeof(da.da_global_dims) == 32 and da.da_global_dims.select_ws.offset == 16


def test_derive_matches_oracle_on_all_configs():
    for w in W.CONFIGS.values():
        dims = da.da_derive(da.problem_of(w))
        ref = oa.derive_dims(w.T, w.fh, w.fw, w.ph, w.pw, w.sparsity)
        got = dict(gh=dims.gh, gw=dims.gw, g=dims.g, block=dims.block, n=dims.n, n_pad=dims.n_pad, k=dims.k)
        assert got == ref, w.name


def test_derive_k_rule():
    for (T, fh, fw, s) in [(33, 45, 80, 0.9), (5, 17, 23, 0.0), (5, 17, 23, 0.3), (7, 8, 8, 0.99), (3, 16, 16, 0.51)]:
        p = da.problem(1, 1, T, fh, fw, 128, sparsity=s)
        assert da.da_derive(p).k == oa.derive_dims(T, fh, fw, 8, 8, s)["k"]
    p = da.problem(1, 1, 4, 16, 16, 128, keep_blocks=5)
    assert da.da_derive(p).k == 5
    p = da.problem(1, 1, 4, 16, 16, 128, keep_blocks=500)
    assert da.da_derive(p).k == 16


def test_derive_k_rule_against_integer_arithmetic():
    """Sparsities given in whole per cent: k = g - floor(s g) computed in integers is what both the library and the
    oracle must return, for every g a frame grid can give up to 5000 and beyond (the product s*g in doubles lands a
    hair under an integer for many of these pairs: that is what the rule's epsilon is for)."""
    rng = np.random.default_rng(11)
    gs = list(range(1, 600)) + [int(x) for x in rng.integers(600, 200000, 1500)]
    for g in gs:
        # a grid with exactly g blocks: T = g frames of one 8x8 patch
        for a in (0, 1, 10, 25, 30, 33, 50, 55, 70, 75, 80, 90, 95, 99):
            want = max(1, g - (a * g) // 100)
            s = a / 100.0
            assert oa.derive_dims(g, 8, 8, 8, 8, s)["k"] == want, (g, a)
            assert da.da_derive(da.problem(1, 1, g, 8, 8, 128, sparsity=s)).k == want, (g, a)
            if g <= 40000:
                assert oa.global_budget(g, s) == max(1, g * g - (a * g * g) // 100), (g, a)
                assert da.da_global_sizes(da.problem(1, 1, g, 8, 8, 128, sparsity=s)).budget == oa.global_budget(g, s)


def test_derive_matches_oracle_on_random_problems():
    rng = np.random.default_rng(12)
    for _ in range(3000):
        T, fh, fw = int(rng.integers(1, 70)), int(rng.integers(1, 100)), int(rng.integers(1, 100))
        ph, pw = int(rng.integers(1, 17)), int(rng.integers(1, 17))
        s = float(rng.choice([0.0, 0.1, 0.3, 0.5, 0.75, 0.9, 0.99, rng.uniform(0, 0.999)]))
        keep = int(rng.integers(0, 3)) * int(rng.integers(1, 50))
        dims = da.da_derive(da.problem(1, 3, T, fh, fw, 64, ph=ph, pw=pw, sparsity=s, keep_blocks=keep))
        got = dict(gh=dims.gh, gw=dims.gw, g=dims.g, block=dims.block, n=dims.n, n_pad=dims.n_pad, k=dims.k)
        assert got == oa.derive_dims(T, fh, fw, ph, pw, s, keep), (T, fh, fw, ph, pw, s, keep)


def _status(fn, *args):
    with pytest.raises(da.DaError) as e:
        fn(*args)
    return e.value.status


def test_bad_problems_are_rejected():
    bad = [da.problem(0, 1, 1, 8, 8, 128), da.problem(1, 1, 1, 8, 8, 0), da.problem(1, 1, 1, 8, 8, 128, ph=0),
           da.problem(1, 1, 1, 8, 8, 128, sparsity=1.0), da.problem(1, 1, 1, 8, 8, 128, sparsity=-0.1),
           da.problem(1, 1, 1, 8, 8, 128, sparsity=float("nan")), da.problem(1, 1, 1, 8, 8, 128, dtype=7),
           da.problem(1, 1, 1, 8, 8, 128, keep_blocks=-1), da.problem(1, 1, 1, 8, 8, 128, pool=2), da.problem(1, 1, 100000, 4000, 4000, 128)]
    for p in bad:
        assert _status(da.da_derive, p) == -2
        assert _status(da.da_workspace_size, p) == -2
        assert _status(da.da_permute, p, FAKE, FAKE, da.DA_REORDER_ROWS, 0) == -2


def test_null_alignment_mode_and_support_checks():
    p = da.problem_of(W.CONFIGS["480p"])
    assert _status(da.da_permute, p, None, FAKE, da.DA_REORDER_ROWS, 0) == -1
    assert _status(da.da_permute, p, FAKE, FAKE + 4, da.DA_REORDER_ROWS, 0) == -5
    assert _status(da.da_permute, p, FAKE, FAKE, 9, 0) == -2
    assert _status(da.da_draft_map, p, FAKE, None, FAKE, FAKE, None, None, 0) == -1
    assert _status(da.da_draft_map, p, FAKE, FAKE, None, FAKE, None, None, 0) == -1
    assert _status(da.da_select_blocks, p, None, FAKE, None, 0) == -1
    assert _status(da.da_select_blocks, p, FAKE, FAKE + 2, None, 0) == -5
    assert _status(da.da_sparse_attn, p, FAKE, FAKE, FAKE, None, FAKE, None, 0) == -1
    # unsupported shapes for the attention kernels: window of neither 64 nor 128 slots (bf16) or not 64 (f32),
    # head dim, dtype/d pair
    for q in (da.problem(1, 1, 2, 16, 16, 128, ph=4, pw=8), da.problem(1, 1, 2, 16, 16, 96),
              da.problem(1, 1, 2, 16, 16, 64, ph=8, pw=16, dtype=da.DA_F32),
              da.problem(1, 1, 2, 16, 16, 64, dtype=da.DA_BF16), da.problem(1, 1, 2, 16, 16, 256, dtype=da.DA_F32)):
        assert _status(da.da_sparse_attn, q, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0) == -3
    # da_sparse_attn_ex: the same checks, plus its two extras
    assert _status(da.da_sparse_attn_ex, p, FAKE, FAKE, FAKE, None, FAKE, None, 0, None, 0) == -1
    assert _status(da.da_sparse_attn_ex, p, FAKE, FAKE, FAKE, FAKE, FAKE, None, 2, None, 0) == -2
    assert _status(da.da_sparse_attn_ex, p, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, FAKE + 4, 0) == -5
    f = da.problem_of(W.CONFIGS["tiny_fp32"])
    assert _status(da.da_sparse_attn_ex, f, FAKE, FAKE, FAKE, FAKE, FAKE, None, 1, None, 0) == -3   # f32: no in-place order
    assert _status(da.da_sparse_attn_ex, f, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0, FAKE, 0) == -3   # f32: no tile counts
    assert da.lib().da_wait_failures(None) == -1
    # bf16 attention keeps per-workgroup block lists in LDS: more than ~7000 blocks with nothing dropped do not fit
    q = da.problem(1, 1, 8000, 8, 8, 128)
    assert _status(da.da_sparse_attn, q, FAKE, FAKE, FAKE, FAKE, FAKE, None, 0) == -3
    # rows that are not a whole number of 16-byte chunks
    q = da.problem(1, 1, 2, 16, 16, 12)
    assert _status(da.da_permute, q, FAKE, FAKE, da.DA_REORDER_ROWS, 0) == -3
    assert _status(da.da_draft_map, q, FAKE, FAKE, FAKE, FAKE, None, None, 0) == -3


def test_forward_workspace_checks():
    p = da.problem_of(W.CONFIGS["tiny_fp32"])
    need = da.da_workspace_size(p)
    assert need > 4 * 512 * 64 * 4 * 2
    L = da.lib()
    args = [ctypes.byref(p)] + [ctypes.c_void_p(FAKE)] * 4 + [None, ctypes.c_void_p(FAKE)]
    assert L.da_forward(*args, ctypes.c_size_t(need - 1), None) == -4
    assert L.da_forward(*args[:-1], ctypes.c_void_p(FAKE + 16), ctypes.c_size_t(need), None) == -5
    assert L.da_forward(*args[:-1], None, ctypes.c_size_t(need), None) == -1
    # the workspace of the headline configuration is a few GB, far below one GPU's HBM
    big = da.da_workspace_size(da.problem_of(W.CONFIGS["720p_hunyuan"]))
    assert 1.5e9 < big < 6.0e9


def test_global_sizes_match_oracle_and_checks():
    for w in list(W.CONFIGS.values()) + list(W.EXTRA_CONFIGS.values()):
        p = da.problem_of(w)
        g = da.da_derive(p).g
        sz = da.da_global_sizes(p)
        assert sz.budget == oa.global_budget(g, w.sparsity), w.name
        assert sz.budget + g <= sz.cap < sz.budget + g + 4 and sz.cap % 4 == 0
        assert sz.forward_ws > sz.select_ws > 0
    p = da.problem(1, 1, 12, 8, 8, 128, keep_blocks=5)
    assert da.da_global_sizes(p).budget == oa.global_budget(12, keep_blocks=5) == 60
    assert _status(da.da_global_sizes, da.problem(1, 1, 1, 8, 8, 128, sparsity=1.0)) == -2
    # offsets of a head's lists are int32
    assert _status(da.da_global_sizes, da.problem(1, 1, 60000, 8, 8, 128, sparsity=0.1)) == -2
    p = da.problem_of(W.CONFIGS["480p"])
    sz = da.da_global_sizes(p)
    L = da.lib()
    V = ctypes.c_void_p
    assert L.da_select_blocks_global(ctypes.byref(p), V(FAKE), V(FAKE), V(FAKE), None, V(FAKE),
                                     ctypes.c_size_t(sz.select_ws - 1), None) == -4
    assert L.da_select_blocks_global(ctypes.byref(p), V(FAKE), None, V(FAKE), None, V(FAKE),
                                     ctypes.c_size_t(sz.select_ws), None) == -1
    assert L.da_select_blocks_global(ctypes.byref(p), V(FAKE), V(FAKE), V(FAKE), None, V(FAKE + 16),
                                     ctypes.c_size_t(sz.select_ws), None) == -5
    assert _status(da.da_sparse_attn_lists, p, FAKE, FAKE, FAKE, None, FAKE, sz.cap, FAKE, None, 0) == -1
    assert _status(da.da_sparse_attn_lists, p, FAKE, FAKE, FAKE, FAKE, FAKE, 0, FAKE, None, 0) == -2
    assert _status(da.da_sparse_attn_lists, p, FAKE, FAKE, FAKE, FAKE, FAKE, 6, FAKE, None, 0) == -2   # not a multiple of 4
    args = [ctypes.byref(p)] + [V(FAKE)] * 4
    assert L.da_forward_global(*args, None, None, V(FAKE), ctypes.c_size_t(sz.forward_ws - 1), None) == -4
    assert L.da_forward_global(*args, V(FAKE), None, V(FAKE), ctypes.c_size_t(sz.forward_ws), None) == -1   # one of the two


def test_forward_ex_layout_checks():
    p = da.problem_of(W.CONFIGS["480p"])
    need = da.da_workspace_size(p)
    L = da.lib()
    V = ctypes.c_void_p

    def call(lin, lout, reordered):
        li = ctypes.byref(lin) if lin is not None else None
        lo = ctypes.byref(lout) if lout is not None else None
        return L.da_forward_ex(ctypes.byref(p), li, lo, reordered, V(FAKE), V(FAKE), V(FAKE), V(FAKE), None, V(FAKE + 16),
                               ctypes.c_size_t(need), None)
    d = 128
    good = da.da_layout(10 ** 9, d, 3 * 24 * d)
    assert call(good, good, 0) == -5                                   # gets as far as the workspace alignment check
    assert call(good, good, 2) == -2                                   # reordered is 0 or 1
    assert call(da.da_layout(10 ** 9, d, d - 8), None, 0) == -2        # rows overlap
    assert call(da.da_layout(10 ** 9, d + 4, 3 * d), None, 0) == -5    # not a multiple of 16 bytes
    assert call(None, da.da_layout(0, d, d), 1) == -2
    assert ctypes.sizeof(da.da_layout) == 24


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """Without the built library every call raises: nothing in the package computes on the CPU instead, and the
    package never imports the oracle."""
    monkeypatch.setattr(da, "_lib", None)
    monkeypatch.setattr(da, "LIB_PATH", str(tmp_path / "libdraftattn.so"))
    with pytest.raises(RuntimeError, match="not built"):
        da.da_derive(da.problem_of(W.CONFIGS["tiny_fp32"]))
    pkg = os.path.join(ROOT, "paper_2505_14708_amd")
    for name in os.listdir(pkg):
        if name.endswith(".py"):
            src = open(os.path.join(pkg, name)).read()
            assert "import oracle" not in src and "from oracle" not in src, name


def test_status_strings():
    assert da.status_string(0) == "ok"
    for s in range(-6, 0):
        assert da.status_string(s) not in ("ok", "unknown status")
    assert da.status_string(-99) == "unknown status"
