"""GPU parity at the benchmark configurations, at their real sizes and head counts, in the launch
configuration bench.py times (one da_forward on the full problem).

For every configuration, on all of its heads:
  * the kept-block lists of EVERY head are compared bit for bit with the oracle's;
  * the whole output is checked to be finite on the device, and no wave of the attention kernel may have
    given up a wait (da_wait_failures);
  * on every head at least 16 query blocks (first/last frame, interior, every edge-block class) are compared
    element by element with the oracle: a query block's output depends only on its own list, so a sampled
    block is an exact check of that block;
  * one head's output is compared with the oracle in full.
The headline configuration runs a second time with Q scaled by 2^-5 (exact in bf16 and in every float32 step of
the draft, so the lists stay the same bit for bit): the scores of a row are then so close together that the kernel's
drop rule leaves nothing out and every tile takes the full path (exponentials, V loads, second product)."""
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from oracle import draft_attention as oa
from paper_2505_14708_amd import binding as da
from paper_2505_14708_amd import workloads as W
from gpu_util import HeadRef, TOL, empty, output_error, say, stratified_rows, to_dev, to_host_f64

pytestmark = pytest.mark.gpu

#        id                 config          Q scale   head compared in full
PLAN = [("480p", "480p", 1.0, 5),
        ("720p_hunyuan", "720p_hunyuan", 1.0, 11),
        ("720p_hunyuan_no_drop", "720p_hunyuan", 2.0 ** -5, 17),
        ("720p_wan", "720p_wan", 1.0, 39),
        ("long", "long", 1.0, 23),
        # the paper's own window and frame shape: 8x16 patches (128-token blocks), 48x80 latents
        ("768p_8x16", "768p_8x16", 1.0, 20)]


def _scaled(Q, scale, dtype):
    """Stored Q times a power of two (exact in either storage type)."""
    if scale == 1.0:
        return Q
    return W.to_storage(W.storage_to_f64(Q, dtype) * scale, dtype)


def sample_rows(ref, at_least=16, seed=0):
    """Query blocks covering first/last frame, interior and every edge-block class, at least `at_least` of them."""
    rows = set(stratified_rows(ref, per_class=4, seed=seed))
    rng = np.random.default_rng(1000 + seed)
    g = ref.dims["g"]
    while len(rows) < min(at_least, g):
        rows.add(int(rng.integers(0, g)))
    return sorted(rows)


def block_errors(ref, got, want, rows, block):
    worst = (0.0, 0.0)
    for r in rows:
        slots = np.arange(r * block, r * block + ref.valid[r])
        emax, emean = output_error(got[ref.perm[slots]], want[slots])
        worst = (max(worst[0], emax), max(worst[1], emean))
    return worst


@pytest.mark.parametrize("case,name,q_scale,full_head", PLAN, ids=[p[0] for p in PLAN])
def test_full_config(case, name, q_scale, full_head):
    import torch
    w = W.CONFIGS[name] if name in W.CONFIGS else W.EXTRA_CONFIGS[name]
    t0 = time.time()
    say(f"{case}: generating {w.H} heads, N={w.N}")
    Q, K, V = W.make_qkv(w, threads=8)
    Q = _scaled(Q, q_scale, w.dtype)
    say(f"{case}: generated in {time.time() - t0:.1f}s; running da_forward")
    p = da.problem_of(w)
    dims = da.da_derive(p)
    ws = torch.empty(da.da_workspace_size(p), dtype=torch.uint8, device="cuda")
    O = empty((w.B, w.H, dims.n, w.d), w.dtype)
    O.fill_(float("nan"))                               # a row the kernel did not write would show
    idx = torch.empty((w.B, w.H, dims.g, dims.k), dtype=torch.int32, device="cuda")
    dQ, dK, dV = (to_dev(x, w.dtype) for x in (Q, K, V))
    failures_before = da.da_wait_failures()
    da.da_forward(p, dQ, dK, dV, O, ws, idx)
    torch.cuda.synchronize()
    assert da.da_wait_failures() == failures_before, "a wave of the attention kernel gave up waiting for a tile"
    finite = bool(torch.isfinite(O).all())
    say(f"{case}: GPU done; g={dims.g} k={dims.k}; whole output finite: {finite}")
    assert finite
    hidx = idx.cpu().numpy()
    del ws, dQ, dK, dV
    torch.cuda.empty_cache()
    tol_max, tol_mean = TOL[w.dtype]

    # every head: lists bit for bit, >= 16 sampled query blocks element by element
    def check_head(h):
        ref = HeadRef(w, Q[0, h], K[0, h], V[0, h])
        same = np.array_equal(hidx[0, h], ref.idx)
        if not same:
            return h, False, ref.near_ties(), (0.0, 0.0), 0
        rows = sample_rows(ref, 16, seed=h)
        want = ref.attention(rows=rows)
        got = to_host_f64(O[0, h], w.dtype)
        return h, True, 0, block_errors(ref, got, want, rows, dims.block), len(rows)

    t1 = time.time()
    worst = (0.0, 0.0)
    with ThreadPoolExecutor(8) as ex:
        for h, same, ties, err, nrows in ex.map(check_head, range(w.H)):
            say(f"{case} head {h}: lists {'match' if same else 'DIFFER'}; {nrows} sampled query blocks, "
                f"max-abs {err[0]:.3e} mean-abs {err[1]:.3e} ({time.time() - t1:.0f}s)")
            assert same, f"head {h}: near-ties in float64: {ties}"
            assert err[0] <= tol_max and err[1] <= tol_mean, (h, err)
            worst = (max(worst[0], err[0]), max(worst[1], err[1]))
    say(f"{case}: all {w.H} heads' lists match; sampled blocks worst max-abs {worst[0]:.3e} mean-abs {worst[1]:.3e}")

    # one head in full, in stretches of query blocks (a progress line after each)
    h = full_head
    ref = HeadRef(w, Q[0, h], K[0, h], V[0, h])
    got = to_host_f64(O[0, h], w.dtype)
    emax, esum, cnt = 0.0, 0.0, 0
    t1 = time.time()
    step = max(1, dims.g // 6)
    for r0 in range(0, dims.g, step):
        rows = list(range(r0, min(dims.g, r0 + step)))
        want = ref.attention(rows=rows)
        for r in rows:
            slots = np.arange(r * dims.block, r * dims.block + ref.valid[r])
            diff = np.abs(got[ref.perm[slots]] - want[slots])
            emax, esum, cnt = max(emax, float(diff.max())), esum + float(diff.sum()), cnt + diff.size
        say(f"{case} head {h} in full: query blocks < {rows[-1] + 1} of {dims.g} ({time.time() - t1:.0f}s)")
    assert cnt == w.N * w.d
    say(f"{case} head {h} in full: max-abs {emax:.3e} mean-abs {esum / cnt:.3e}")
    assert emax <= tol_max and esum / cnt <= tol_mean
    del O
    torch.cuda.empty_cache()


@pytest.mark.parametrize("q_scale", [1.0, 2.0 ** -5], ids=["as_generated", "nothing_dropped"])
def test_dense_layer_full_size(q_scale):
    """A dense layer (sparsity 0) at the headline shape, two heads: da_forward ranks nothing, every workgroup walks all
    1980 key tiles, and the result is full attention (Definition 3.1).  Sampled query tokens of every block class are
    compared with the oracle's full attention row by row (a row of full attention depends on nothing but its query);
    the whole output must be finite.  With Q scaled by 2^-5 the drop rule leaves nothing out."""
    import torch
    w = W.CONFIGS["720p_hunyuan"].with_(name="720p_hunyuan_dense", H=2, sparsity=0.0)
    say(f"dense layer: generating {w.H} heads, N={w.N}")
    Q, K, V = W.make_qkv(w, threads=8)
    Q = _scaled(Q, q_scale, w.dtype)
    p = da.problem_of(w)
    dims = da.da_derive(p)
    assert dims.k == dims.g
    ws = torch.empty(da.da_workspace_size(p), dtype=torch.uint8, device="cuda")
    O = empty((w.B, w.H, dims.n, w.d), w.dtype)
    O.fill_(float("nan"))
    failures_before = da.da_wait_failures()
    da.da_forward(p, *(to_dev(x, w.dtype) for x in (Q, K, V)), O, ws)
    torch.cuda.synchronize()
    assert da.da_wait_failures() == failures_before
    assert bool(torch.isfinite(O).all())
    tol_max, tol_mean = TOL[w.dtype]
    for h in range(w.H):
        ref = HeadRef(w, Q[0, h], K[0, h], V[0, h])
        blocks = sample_rows(ref, 16, seed=h)
        tokens = np.concatenate([ref.perm[b * dims.block + np.arange(0, ref.valid[b], 5)] for b in blocks])
        q64, k64, v64 = (oa.widen_f64(x[0, h], w.dtype) for x in (Q, K, V))
        want = oa.full_attention(q64[tokens], k64, v64)
        got = to_host_f64(O[0, h], w.dtype)[tokens]
        emax, emean = output_error(got, want)
        say(f"dense layer head {h}: {len(tokens)} query tokens of {len(blocks)} blocks, max-abs {emax:.3e} mean-abs {emean:.3e}")
        assert emax <= tol_max and emean <= tol_mean


@pytest.mark.parametrize("name,heads,check", [("720p_hunyuan", [0, 7, 16, 23], [0, 23]), ("768p_8x16", [3, 20], [20])],
                         ids=["720p_hunyuan", "768p_8x16"])
def test_full_config_whole_map(name, heads, check):
    """The same with the whole-map selection (Section 3.2.2): one threshold per head, lists of any length."""
    import torch
    w = W.CONFIGS[name] if name in W.CONFIGS else W.EXTRA_CONFIGS[name]
    say(f"{name} whole map: generating {len(heads)} heads")
    Q, K, V = W.make_qkv(w, heads=heads, threads=8)
    wg = w.with_(H=len(heads))
    p = da.problem_of(wg)
    dims = da.da_derive(p)
    sz = da.da_global_sizes(p)
    ws = torch.empty(sz.forward_ws, dtype=torch.uint8, device="cuda")
    O = empty((1, len(heads), dims.n, w.d), w.dtype)
    row_ptr = torch.empty((1, len(heads), dims.g + 1), dtype=torch.int32, device="cuda")
    cols = torch.empty((1, len(heads), sz.cap), dtype=torch.int32, device="cuda")
    dQ, dK, dV = (to_dev(x, w.dtype) for x in (Q, K, V))
    da.da_forward_global(p, dQ, dK, dV, O, ws, row_ptr, cols)
    torch.cuda.synchronize()
    hrp, hcols = row_ptr.cpu().numpy(), cols.cpu().numpy()
    say(f"{name} whole map: GPU done; g={dims.g} budget={sz.budget}")
    # structure of every head's lists: offsets ascend, every row holds something, the budget is met
    lens = np.diff(hrp, axis=-1)
    assert (hrp[..., 0] == 0).all() and (lens >= 1).all() and (lens <= dims.g).all()
    assert (hrp[..., -1] >= sz.budget).all() and (hrp[..., -1] <= sz.cap).all()
    tol_max, tol_mean = TOL[w.dtype]
    for h in check:
        i = heads.index(h)
        ref = HeadRef(w, Q[0, i], K[0, i], V[0, i])
        r, c, _ = oa.select_blocks_global(ref.logits, sz.budget)
        same = np.array_equal(hrp[0, i], r) and np.array_equal(hcols[0, i][:r[-1]], c)
        say(f"{name} head {h}: lists {'match' if same else 'DIFFER'}; {lens[0, i].min()}..{lens[0, i].max()} blocks a row, "
            f"{int((np.diff(r) == 1).sum())} rows of one")
        assert same
        lists = oa.lists_of(r, c)
        rows = sorted(set(stratified_rows(ref, per_class=2, seed=h)) |
                      {int(np.argmax(np.diff(r))), int(np.argmin(np.diff(r)))})      # the longest and a shortest list too
        want = ref.attention(rows=rows, idx=lists)
        got = to_host_f64(O[0, i], w.dtype)
        worst = (0.0, 0.0)
        for q in rows:
            slots = np.arange(q * dims.block, q * dims.block + ref.valid[q])
            emax, emean = output_error(got[ref.perm[slots]], want[slots])
            worst = (max(worst[0], emax), max(worst[1], emean))
        say(f"{name} head {h}: {len(rows)} sampled query blocks, worst max-abs {worst[0]:.3e} mean-abs {worst[1]:.3e}")
        assert worst[0] <= tol_max and worst[1] <= tol_mean
    del ws, O, dQ, dK, dV
    torch.cuda.empty_cache()


def test_many_blocks_ascending_walk():
    """A problem whose union lists are too long for the balanced walk's extra arrays (the kernel
    then walks in ascending order): 3000 one-patch frames, 800 key blocks kept per query block."""
    import torch
    w = W.Workload("many_blocks", B=1, H=1, d=128, T=3000, fh=8, fw=8, sparsity=0.0, seed=11)
    say("many_blocks: generating")
    Q, K, V = W.make_qkv(w)
    p = da.problem(w.B, w.H, w.T, w.fh, w.fw, w.d, keep_blocks=800)
    dims = da.da_derive(p)
    assert dims.g == 3000 and dims.k == 800
    ws = torch.empty(da.da_workspace_size(p), dtype=torch.uint8, device="cuda")
    O = empty((1, 1, dims.n, w.d), w.dtype)
    idx = torch.empty((1, 1, dims.g, dims.k), dtype=torch.int32, device="cuda")
    da.da_forward(p, *(to_dev(x, w.dtype) for x in (Q, K, V)), O, ws, idx)
    torch.cuda.synchronize()
    say("many_blocks: GPU done")
    ref = HeadRef(w, Q[0, 0], K[0, 0], V[0, 0], keep_blocks=800)
    assert np.array_equal(idx.cpu().numpy()[0, 0], ref.idx)
    rows = [0, 1, 2, 3, 1499, 2996, 2997, 2998, 2999]
    want = ref.attention(rows=rows)
    got = to_host_f64(O[0, 0], w.dtype)
    for r in rows:
        slots = np.arange(r * 64, (r + 1) * 64)
        emax, emean = output_error(got[ref.perm[slots]], want[slots])
        assert emax <= 2e-2 and emean <= 2e-3, (r, emax, emean)
