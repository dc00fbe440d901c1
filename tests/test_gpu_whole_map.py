"""GPU parity of the whole-map form of the guided sparsity (Section 3.2.2: the threshold is the
ceil(r g^2)-th largest score of a head's map): the selector bit for bit, the attention on lists of
any length and the whole path within the output tolerances, all through the C ABI."""
import numpy as np
import pytest

from oracle import draft_attention as oa
from paper_2505_14708_amd import binding as da
from paper_2505_14708_amd import workloads as W
from gpu_util import HeadRef, TOL, empty, output_error, say, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

SMALL = {
    "tiny_fp32": W.CONFIGS["tiny_fp32"],
    "bf16_480p_T3": W.CONFIGS["480p"].with_(name="bf16_480p_T3", H=2, T=3, sparsity=0.75),
    "f32_ragged": W.Workload("f32_ragged", B=2, H=1, d=64, T=2, fh=20, fw=12, sparsity=0.4, dtype=W.F32, seed=3),
    "bf16_B2_T5": W.Workload("bf16_B2_T5", B=2, H=2, d=128, T=5, fh=16, fw=24, sparsity=0.6, seed=7),
    "bf16_8x16_ragged": W.Workload("bf16_8x16_ragged", B=1, H=1, d=128, T=3, fh=30, fw=52, ph=8, pw=16, sparsity=0.5,
                                   seed=6),
}


@pytest.fixture(scope="module")
def torch_mod():
    import torch
    assert torch.cuda.is_available()
    return torch


@pytest.fixture(scope="module")
def cases():
    out = {}
    for name, w in SMALL.items():
        Q, K, V = W.make_qkv(w)
        refs = {(b, h): HeadRef(w, Q[b, h], K[b, h], V[b, h]) for b in range(w.B) for h in range(w.H)}
        out[name] = (w, Q, K, V, refs)
    return out


def _select(torch, p, L):
    """da_select_blocks_global on host scores L [B,H,g,g] -> (row_ptr, cols, mask) as numpy, and the sizes."""
    sz = da.da_global_sizes(p)
    B, H, g = L.shape[0], L.shape[1], L.shape[2]
    row_ptr = torch.full((B, H, g + 1), -1, dtype=torch.int32, device="cuda")
    cols = torch.full((B, H, sz.cap), -1, dtype=torch.int32, device="cuda")
    mask = torch.full((B, H, g, g), 9, dtype=torch.uint8, device="cuda")
    ws = torch.empty(sz.select_ws, dtype=torch.uint8, device="cuda")
    da.da_select_blocks_global(p, torch.from_numpy(np.ascontiguousarray(L)).cuda(), row_ptr, cols, ws, mask)
    torch.cuda.synchronize()
    return row_ptr.cpu().numpy(), cols.cpu().numpy(), mask.cpu().numpy(), sz


def _check_against_oracle(rp, cl, mk, L, budget):
    want_rp, want_cols, want_mask = oa.select_blocks_global(L, budget)
    assert np.array_equal(rp, want_rp)
    assert np.array_equal(cl[:want_rp[-1]], want_cols)
    assert (cl[want_rp[-1]:] == -1).all()               # nothing written past the lists
    assert np.array_equal(mk, want_mask)


@pytest.mark.parametrize("name", list(SMALL))
def test_select_global_on_oracle_logits(torch_mod, cases, name):
    w, Q, K, V, refs = cases[name]
    say(f"select_global {name}")
    p = da.problem_of(w)
    g = da.da_derive(p).g
    L = np.stack([np.stack([refs[(b, h)].logits for h in range(w.H)]) for b in range(w.B)])
    rp, cl, mk, sz = _select(torch_mod, p, L)
    assert sz.budget == oa.global_budget(g, w.sparsity) and sz.cap >= sz.budget + g and sz.cap % 4 == 0
    for (b, h) in refs:
        _check_against_oracle(rp[b, h], cl[b, h], mk[b, h], L[b, h], sz.budget)


def test_select_global_planted(torch_mod):
    """Maps with many equal scores (also at the threshold), rows under the threshold, signed zeros, infinities;
    budgets from one entry to the whole map; g across several chunks of the histogram pass and ragged tails, and
    across the row lengths that the fill kernel treats differently (up to 1024, 2048, 4096 columns, and beyond)."""
    torch = torch_mod
    rng = np.random.default_rng(11)
    for (g, k) in [(7, 1), (7, 7), (64, 5), (65, 33), (200, 37), (1000, 100), (1980, 198), (2500, 20), (4200, 9)]:
        say(f"select_global planted g={g} k={k}")
        L = np.stack([rng.normal(size=(g, g)).astype(np.float32) for _ in range(3)])[None]
        L[0, 0] = np.round(L[0, 0] * 2) / 2             # head 0: duplicates everywhere, ties at the threshold
        L[0, 1, 0, :] = 0.0
        L[0, 1, 1, ::2] = 0.0; L[0, 1, 1, 1::2] = -0.0
        L[0, 1, 2, :] = -50.0                           # a row far under the threshold: keeps column 0
        L[0, 1, 3, :] = -50.0; L[0, 1, 3, g // 2] = -49.0   # ... keeps its best column
        L[0, 1, 4, : g // 2] = -np.inf
        L[0, 1, min(5, g - 1), -1] = np.inf
        L[0, 2, :, :] = 1.5                             # head 2: all equal, the budget runs out in row-major order
        p = da.problem(1, 3, g, 8, 8, 128, keep_blocks=k)
        rp, cl, mk, sz = _select(torch, p, L)
        assert sz.budget == k * g
        for h in range(3):
            _check_against_oracle(rp[0, h], cl[0, h], mk[0, h], L[0, h], sz.budget)
    # a budget given by the ratio, one entry, and the whole map
    for (g, s) in [(50, 0.9996), (50, 0.0), (33, 0.37)]:
        L = rng.normal(size=(1, 1, g, g)).astype(np.float32)
        p = da.problem(1, 1, g, 8, 8, 128, sparsity=s)
        rp, cl, mk, sz = _select(torch, p, L)
        assert sz.budget == oa.global_budget(g, s)
        _check_against_oracle(rp[0, 0], cl[0, 0], mk[0, 0], L[0, 0], sz.budget)


def _lists_to_dev(torch, refs, w, g, cap, sel):
    rp = np.zeros((w.B, w.H, g + 1), np.int32)
    cl = np.full((w.B, w.H, cap), -1, np.int32)
    for (b, h) in refs:
        r, c, _ = sel[(b, h)]
        rp[b, h] = r
        cl[b, h, :len(c)] = c
    return torch.from_numpy(rp).cuda(), torch.from_numpy(cl).cuda()


@pytest.mark.parametrize("name", list(SMALL))
def test_sparse_attn_lists_stage(torch_mod, cases, name):
    torch = torch_mod
    w, Q, K, V, refs = cases[name]
    say(f"sparse_attn_lists {name}")
    p = da.problem_of(w)
    dims = da.da_derive(p)
    sz = da.da_global_sizes(p)
    sel = {key: oa.select_blocks_global(ref.logits, sz.budget) for key, ref in refs.items()}
    row_ptr, cols = _lists_to_dev(torch, refs, w, dims.g, sz.cap, sel)
    Qp = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    Kp = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    Vt = empty((w.B, w.H, dims.g, w.d, dims.block), w.dtype)
    da.da_permute(p, to_dev(Q, w.dtype), Qp, da.DA_REORDER_ROWS)
    da.da_permute(p, to_dev(K, w.dtype), Kp, da.DA_REORDER_ROWS)
    da.da_permute(p, to_dev(V, w.dtype), Vt, da.v_layout(w.dtype))
    Op = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    lse = torch.empty((w.B, w.H, dims.n_pad), dtype=torch.float32, device="cuda")
    da.da_sparse_attn_lists(p, Qp, Kp, Vt, row_ptr, cols, sz.cap, Op, lse)
    torch.cuda.synchronize()
    got = to_host_f64(Op, w.dtype)
    assert np.isfinite(got).all()
    tol_max, tol_mean = TOL[w.dtype]
    for (b, h), ref in refs.items():
        r, c, _ = sel[(b, h)]
        lens = np.diff(r)
        want, want_lse = ref.attention(idx=oa.lists_of(r, c), want_lse=True)
        real = ref.perm >= 0
        emax, emean = output_error(got[b, h][real], want[real])
        say(f"  {name} head {(b, h)}: lists of {lens.min()}..{lens.max()} blocks, max-abs {emax:.3e} mean-abs {emean:.3e}")
        assert emax <= tol_max and emean <= tol_mean
        lerr = np.abs(lse.cpu().numpy()[b, h][real] - want_lse[real]).max()
        assert lerr < (2e-2 if w.dtype == W.BF16 else 1e-4)


@pytest.mark.parametrize("name", ["bf16_B2_T5", "f32_ragged"])
def test_sparse_attn_lists_empty_and_unsorted_rows(torch_mod, cases, name):
    """Lists a caller made by hand: some query blocks attend nothing (their rows come out as zeros, in both storage
    types), the others hold their blocks in any order.  The tolerance is the stated one, on every head's output as a
    whole and, the maximum, on every block."""
    torch = torch_mod
    w, Q, K, V, refs = cases[name]
    say(f"sparse_attn_lists with empty rows, {name}")
    p = da.problem_of(w)
    dims = da.da_derive(p)
    g = dims.g
    rng = np.random.default_rng(12)
    lists = {}
    for key in refs:
        rows = []
        for i in range(g):
            n = 0 if i % 7 == 3 else int(rng.integers(1, min(12, g + 1)))
            rows.append(rng.choice(g, size=n, replace=False).astype(np.int64))
        lists[key] = rows
    cap = (max(sum(len(r) for r in rows) for rows in lists.values()) + 3) // 4 * 4
    sel = {key: (np.concatenate([[0], np.cumsum([len(r) for r in rows])]), np.concatenate(rows), None)
           for key, rows in lists.items()}
    row_ptr, cols = _lists_to_dev(torch, refs, w, g, cap, sel)
    Qp = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    Kp = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    Vt = empty((w.B, w.H, dims.g, w.d, dims.block), w.dtype)
    da.da_permute(p, to_dev(Q, w.dtype), Qp, da.DA_REORDER_ROWS)
    da.da_permute(p, to_dev(K, w.dtype), Kp, da.DA_REORDER_ROWS)
    da.da_permute(p, to_dev(V, w.dtype), Vt, da.v_layout(w.dtype))
    Op = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    Op.fill_(7.0)
    lse = torch.empty((w.B, w.H, dims.n_pad), dtype=torch.float32, device="cuda")
    da.da_sparse_attn_lists(p, Qp, Kp, Vt, row_ptr, cols, cap, Op, lse)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Op.float()).all())
    got = to_host_f64(Op, w.dtype)
    tol_max, tol_mean = TOL[w.dtype]
    for (b, h), ref in refs.items():
        full = [i for i in range(g) if len(lists[(b, h)][i])]
        want = ref.attention(rows=full, idx=lists[(b, h)])
        live = np.zeros(dims.n_pad, bool)
        for i in range(g):
            sl = slice(i * dims.block, i * dims.block + ref.valid[i])
            if len(lists[(b, h)][i]) == 0:
                assert (got[b, h][sl] == 0.0).all(), i
            else:
                live[sl] = True
                emax, _ = output_error(got[b, h][sl], want[sl])
                assert emax <= tol_max, (i, emax)
        emax, emean = output_error(got[b, h][live], want[live])
        say(f"  {name} head {(b, h)}: max-abs {emax:.3e} mean-abs {emean:.3e}")
        assert emean <= tol_mean, emean


def test_sparse_attn_lists_equals_fixed_k(torch_mod, cases):
    """Lists that all hold k entries: the result of da_sparse_attn on the [g, k] table (to rounding: the walk
    over the tiles may take another order)."""
    torch = torch_mod
    w, Q, K, V, refs = cases["bf16_B2_T5"]
    say("sparse_attn_lists with k per row")
    p = da.problem_of(w)
    dims = da.da_derive(p)
    g, k = dims.g, dims.k
    idx_np = np.stack([np.stack([refs[(b, h)].idx for h in range(w.H)]) for b in range(w.B)]).astype(np.int32)
    cap = (g * k + 3) // 4 * 4
    cl = np.zeros((w.B, w.H, cap), np.int32)
    cl[:, :, :g * k] = idx_np.reshape(w.B, w.H, g * k)
    rp = np.broadcast_to(np.arange(g + 1, dtype=np.int32) * k, (w.B, w.H, g + 1)).copy()
    Qp = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    Kp = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    Vt = empty((w.B, w.H, dims.g, w.d, dims.block), w.dtype)
    da.da_permute(p, to_dev(Q, w.dtype), Qp, da.DA_REORDER_ROWS)
    da.da_permute(p, to_dev(K, w.dtype), Kp, da.DA_REORDER_ROWS)
    da.da_permute(p, to_dev(V, w.dtype), Vt, da.v_layout(w.dtype))
    O1 = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    O2 = empty((w.B, w.H, dims.n_pad, w.d), w.dtype)
    da.da_sparse_attn(p, Qp, Kp, Vt, torch.from_numpy(idx_np).cuda(), O1, None)
    da.da_sparse_attn_lists(p, Qp, Kp, Vt, torch.from_numpy(rp).cuda(), torch.from_numpy(cl).cuda(), cap, O2, None)
    torch.cuda.synchronize()
    real = refs[(0, 0)].perm >= 0
    emax, emean = output_error(to_host_f64(O1, w.dtype)[:, :, real], to_host_f64(O2, w.dtype)[:, :, real])
    say(f"  lists vs table: max-abs {emax:.3e} mean-abs {emean:.3e}")
    assert emax <= 2e-2 and emean <= 2e-4


@pytest.mark.parametrize("name", list(SMALL))
def test_forward_global_end_to_end(torch_mod, cases, name):
    torch = torch_mod
    w, Q, K, V, refs = cases[name]
    say(f"forward_global {name}")
    p = da.problem_of(w)
    dims = da.da_derive(p)
    sz = da.da_global_sizes(p)
    ws = torch.empty(sz.forward_ws, dtype=torch.uint8, device="cuda")
    O = empty((w.B, w.H, dims.n, w.d), w.dtype)
    row_ptr = torch.full((w.B, w.H, dims.g + 1), -1, dtype=torch.int32, device="cuda")
    cols = torch.full((w.B, w.H, sz.cap), -1, dtype=torch.int32, device="cuda")
    dQ, dK, dV = (to_dev(x, w.dtype) for x in (Q, K, V))
    da.da_forward_global(p, dQ, dK, dV, O, ws, row_ptr, cols)
    torch.cuda.synchronize()
    got = to_host_f64(O, w.dtype)
    tol_max, tol_mean = TOL[w.dtype]
    for (b, h), ref in refs.items():
        r, c, _ = oa.select_blocks_global(ref.logits, sz.budget)
        assert np.array_equal(row_ptr.cpu().numpy()[b, h], r)
        assert np.array_equal(cols.cpu().numpy()[b, h][:r[-1]], c)
        want = oa.restore(ref.attention(idx=oa.lists_of(r, c)), ref.inv)
        emax, emean = output_error(got[b, h], want)
        say(f"  {name} head {(b, h)}: max-abs {emax:.3e} mean-abs {emean:.3e}")
        assert emax <= tol_max and emean <= tol_mean
    # without the list outputs: the same bits
    O2 = torch.empty_like(O)
    da.da_forward_global(p, dQ, dK, dV, O2, ws)
    torch.cuda.synchronize()
    as_int = torch.int16 if w.dtype == W.BF16 else torch.int32
    assert torch.equal(O.view(as_int), O2.view(as_int))
