"""The synthetic workloads have the sizes stated for them (closed forms worked by hand)."""
import numpy as np
import pytest

import oracle
from paper_2506_19225_amd import workloads as wl


@pytest.mark.parametrize("name,n,c,s_total,l_mix,pairs", [
    ("config0", 576, 4, 64, 352, 80160),
    ("config1", 16640, 64, 2048, 4096, None),
    ("config2", 131328, 256, 16384, 23808, None),
    ("config3", 164096, 640, 10240, 18176, None),
])
def test_fixed_chunk_workload_sizes(name, n, c, s_total, l_mix, pairs):
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    assert lay.n_tokens == n and lay.n_chunks == c and lay.sparse_offsets[-1] == s_total
    assert len(lay.sparse_idx) == s_total
    clen = lay.chunk_len(0)
    assert w.n_prefix + w.k * clen + (c - w.k) * w.kept_per_chunk == l_mix
    for cc in (0, c // 2, c - 1):
        kept = lay.kept(cc)
        assert (np.diff(kept) > 0).all()
        assert kept[0] >= lay.chunk_bounds[cc] and kept[-1] < lay.chunk_bounds[cc + 1]
    if not w.kept_random:
        assert lay.kept(1)[0] == lay.chunk_bounds[1]          # kept tokens start at the chunk start
    if pairs is not None:
        assert oracle.allowed_pair_count(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets) == pairs
    flops = 4 * w.head_dim * w.n_q_heads * oracle.allowed_pair_count(
        lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets)
    want = {"config0": 41.04e6, "config1": 0.3275e12, "config2": 16.30e12, "config3": 12.91e12}[name]
    assert abs(flops / want - 1) < 2e-3


def test_bf16_rounding_helpers():
    x = np.array([1.0, 1.00390625, 1.005859375, -3.14159, 1e-3, 0.0], np.float32)
    r = wl.round_to_bf16(x)
    assert r[0] == 1.0
    assert r[1] == 1.0                 # 1 + 2^-8 is a tie: rounds to even mantissa
    assert r[2] == 1.0078125           # 1 + 1.5 * 2^-8 rounds up to 1 + 2^-7
    assert np.array_equal(wl.from_bf16_bits(wl.to_bf16_bits(r)), r)
    assert (np.abs(r - x) <= np.abs(x) * 2.0 ** -8).all()


def test_generators_are_deterministic_and_in_storage_precision():
    w = wl.WORKLOADS["config0"]
    lay = wl.make_layout(w)
    a = wl.make_qkv(w, lay)
    b = wl.make_qkv(w, lay)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert a[0].shape == (2, 576, 64) and a[1].shape == (1, 576, 64) and a[0].dtype == np.float32
    w1 = wl.tiny_workload("bf16", 4, 2, 16, T=2, B=1, k=1, seed=9)
    lay1 = wl.random_layout(np.random.default_rng(1), 2, 3, 2, 5)
    q, k, v = wl.make_qkv(w1, lay1)
    assert np.array_equal(wl.round_to_bf16(q), q) and np.array_equal(wl.round_to_bf16(k), k)
    assert abs(float(q.std()) - 1.0) < 0.1
