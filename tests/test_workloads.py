"""The seeded input generator: determinism, shapes, storage formats."""
import numpy as np

from paper_2505_14708_amd import workloads as W


def test_configs_match_the_benchmark_list():
    c = W.CONFIGS
    assert (c["tiny_fp32"].N, c["480p"].N, c["720p_hunyuan"].N, c["720p_wan"].N, c["long"].N) == \
        (512, 32760, 118800, 75600, 234000)
    assert c["tiny_fp32"].dtype == W.F32 and c["tiny_fp32"].d == 64 and c["tiny_fp32"].H == 2
    assert all(c[n].d == 128 and c[n].dtype == W.BF16 for n in ("480p", "720p_hunyuan", "720p_wan", "long"))
    assert c["720p_wan"].H == 40 and c["long"].drift and not c["480p"].drift


def test_heads_are_independent_and_reproducible():
    w = W.CONFIGS["480p"].with_(T=2, H=3)
    Q, K, V = W.make_qkv(w)
    assert Q.shape == (1, 3, w.N, 128) and Q.dtype == np.uint16
    Q1, K1, V1 = W.make_qkv(w, heads=[2])
    assert np.array_equal(Q1[0, 0], Q[0, 2]) and np.array_equal(V1[0, 0], V[0, 2])
    assert not np.array_equal(Q[0, 0], Q[0, 1])
    assert not np.array_equal(Q, K)                       # independent noise on Q and K


def test_field_statistics():
    w = W.CONFIGS["480p"].with_(T=3)
    q, k, v = (W.storage_to_f64(x, w.dtype) for x in W.make_head(w, 0, 0))
    assert abs(v.mean()) < 0.01 and abs(v.std() - 1.0) < 0.01
    assert 1.6 < q.std() < 2.4                           # 8 unit modes (variance 4) + 0.09 noise
    assert abs((q - k).std() - 0.3 * np.sqrt(2)) < 0.02   # the smooth part is shared


def test_bf16_rounding_is_nearest_even():
    x = np.float32([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38])
    bits = W.f32_to_bf16_bits(x)
    # 1 + 2^-8 is a tie -> even (1.0); 1 + 3*2^-8 is a tie -> even (1 + 2^-6)
    assert list(W.bf16_bits_to_f32(bits)[:4]) == [1.0, 1.0, 1.015625, -2.5]
    y = W.bf16_bits_to_f32(bits)
    assert np.array_equal(W.f32_to_bf16_bits(y), bits)   # idempotent
