"""GPU parity of the whole path on a seeded spread of small shapes the fixed cases do not reach: very few frames or
blocks, frames narrower or lower than a patch, one kept block, every block kept, both windows, both storage types.
Lists bit for bit, outputs within the stated tolerances, element by element against the oracle."""
import numpy as np
import pytest

from oracle import draft_attention as oa
from paper_2505_14708_amd import binding as da
from paper_2505_14708_amd import workloads as W
from gpu_util import TOL, empty, output_error, say, to_dev, to_host_f64

pytestmark = pytest.mark.gpu


def _shapes():
    rng = np.random.default_rng(2024)
    out = [  # hand-picked corners first: (B, H, T, fh, fw, ph, pw, dtype, sparsity)
        (1, 1, 1, 8, 8, 8, 8, W.BF16, 0.0),            # one block in all
        (1, 1, 1, 3, 5, 8, 8, W.BF16, 0.0),            # one partial block
        (1, 2, 2, 8, 9, 8, 8, W.BF16, 0.5),            # a column of one-token-wide blocks
        (1, 1, 3, 9, 8, 8, 8, W.BF16, 0.9),            # a row of one-token-high blocks; one block kept
        (2, 1, 7, 16, 8, 8, 8, W.BF16, 0.3),           # seven frames: one group of four and a tail of three
        (1, 1, 9, 8, 16, 8, 16, W.BF16, 0.4),          # 128-token blocks, odd frame count
        (1, 1, 2, 17, 33, 8, 16, W.BF16, 0.0),         # 128-token blocks, ragged both ways, everything kept
        (1, 1, 1, 8, 8, 8, 8, W.F32, 0.0),
        (1, 2, 3, 9, 17, 8, 8, W.F32, 0.6),
    ]
    for _ in range(9):
        bf16 = rng.random() < 0.7
        wide = bf16 and rng.random() < 0.3
        out.append((int(rng.integers(1, 3)), int(rng.integers(1, 3)), int(rng.integers(1, 11)), int(rng.integers(1, 28)),
                    int(rng.integers(1, 40)), 8, 16 if wide else 8, W.BF16 if bf16 else W.F32,
                    float(rng.choice([0.0, 0.25, 0.5, 0.8, 0.95]))))
    return out


@pytest.mark.parametrize("shape", _shapes(), ids=lambda s: "B%dH%dT%d_%dx%d_p%dx%d_%s_s%g" % (s[0], s[1], s[2], s[3], s[4], s[5], s[6], "bf16" if s[7] == W.BF16 else "f32", s[8]))
def test_forward_on_odd_shapes(shape):
    import torch
    B, H, T, fh, fw, ph, pw, dtype, sparsity = shape
    d = 128 if dtype == W.BF16 else 64
    w = W.Workload("shape", B=B, H=H, d=d, T=T, fh=fh, fw=fw, ph=ph, pw=pw, sparsity=sparsity, dtype=dtype, seed=T * 1000 + fh * 37 + fw)
    say(f"odd shape {shape}")
    Q, K, V = W.make_qkv(w)
    p = da.problem_of(w)
    dims = da.da_derive(p)
    ws = torch.empty(da.da_workspace_size(p), dtype=torch.uint8, device="cuda")
    O = empty((B, H, dims.n, d), dtype)
    O.fill_(float("nan"))
    idx = torch.full((B, H, dims.g, dims.k), -1, dtype=torch.int32, device="cuda")
    da.da_forward(p, *(to_dev(x, dtype) for x in (Q, K, V)), O, ws, idx)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(O).all())
    got = to_host_f64(O, dtype)
    hidx = idx.cpu().numpy()
    tol_max, tol_mean = TOL[dtype]
    for b in range(B):
        for h in range(H):
            ref = oa.forward_head(Q[b, h], K[b, h], V[b, h], dtype, T, fh, fw, ph, pw, sparsity)
            assert np.array_equal(hidx[b, h], ref["idx"]), (b, h)
            emax, emean = output_error(got[b, h], ref["O"])
            assert emax <= tol_max and emean <= tol_mean, (b, h, emax, emean)
