"""The entry point that allocates nothing (da_select_blocks_global_static: its scratch is a buffer built into the
library) against the entry point it is a variant of (da_select_blocks_global, scratch from the caller), bit for bit,
through the C ABI: two calls in a row, the second on a smaller problem, so that what the first call left in the
shared buffer would show."""
import numpy as np
import pytest

from oracle import draft_attention as oa
from paper_2505_14708_amd import binding as da

pytestmark = pytest.mark.gpu


def _both(torch, p, L):
    """row_ptr, cols, mask from the two entry points on host scores L [B,H,g,g]."""
    sz = da.da_global_sizes(p)
    B, H, g = L.shape[:3]
    scores = torch.from_numpy(np.ascontiguousarray(L)).cuda()
    out = []
    for static in (False, True):
        row_ptr = torch.full((B, H, g + 1), -1, dtype=torch.int32, device="cuda")
        cols = torch.full((B, H, sz.cap), -1, dtype=torch.int32, device="cuda")
        mask = torch.full((B, H, g, g), 9, dtype=torch.uint8, device="cuda")
        if static:
            da.da_select_blocks_global_static(p, scores, row_ptr, cols, mask)
        else:
            ws = torch.empty(sz.select_ws, dtype=torch.uint8, device="cuda")
            da.da_select_blocks_global(p, scores, row_ptr, cols, ws, mask)
        torch.cuda.synchronize()
        out.append((row_ptr.cpu().numpy(), cols.cpu().numpy(), mask.cpu().numpy()))
    return out, sz


def _scores(rng, B, H, g, ties):
    L = rng.normal(size=(B, H, g, g)).astype(np.float32)
    if ties:                                             # many equal scores around the threshold, and rows under it
        L = np.round(L * 2.0) / 2.0
        L[:, :, ::5, :] -= 6.0
    return L


def test_static_scratch_matches_caller_scratch():
    import torch
    assert torch.cuda.is_available()
    rng = np.random.default_rng(21)
    # (frames of one 8x8 patch each -> g, heads, sparsity, ties): large first, then a smaller one, then one with ties
    for (g, H, s, ties) in [(700, 3, 0.9, False), (130, 2, 0.75, True), (257, 1, 0.5, True)]:
        print(f"[gpu-test] static scratch: g={g} H={H} sparsity={s}", flush=True)
        p = da.problem(1, H, g, 8, 8, 128, sparsity=s)
        L = _scores(rng, 1, H, g, ties)
        (a, b), sz = _both(torch, p, L)
        assert sz.select_ws <= da.DA_STATIC_SCRATCH_BYTES
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
        # and both are the oracle's selection
        for h in range(H):
            rp, cl, mk = oa.select_blocks_global(L[0, h], sz.budget)
            assert np.array_equal(b[0][0, h], rp) and np.array_equal(b[1][0, h][:rp[-1]], cl) and np.array_equal(b[2][0, h], mk)


def test_static_scratch_rejects_problems_beyond_its_size():
    """No launch, a clear status: the headline map with 40 heads needs more than the built-in buffer holds."""
    p = da.problem(1, 40, 33, 45, 80, 128, sparsity=0.9)
    assert da.da_global_sizes(p).select_ws > da.DA_STATIC_SCRATCH_BYTES
    with pytest.raises(da.DaError) as e:
        da.da_select_blocks_global_static(p, 0x10000, 0x10000, 0x10000, None, 0)
    assert e.value.status == -7 and "scratch" in str(e.value)
