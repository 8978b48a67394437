"""Pins of the pre-filling oracle: hand-written mask, closed forms, library special cases
(torch CPU scaled_dot_product_attention), invariants and brute force on tiny inputs.
The paper prints no worked numeric example for this step, so none of these is a paper value."""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2506_19225_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_layout():
    return wl.layout_from_lists(2, [3, 4, 2], [np.array([2]), np.array([5, 7]), np.array([9])])


def rand_qkv(rng, hq, hkv, n, d, scale=1.0):
    q = (rng.standard_normal((hq, n, d)) * scale).astype(np.float32)
    k = (rng.standard_normal((hkv, n, d)) * scale).astype(np.float32)
    v = rng.standard_normal((hkv, n, d)).astype(np.float32)
    return q, k, v


def sdpa_causal(q, k, v):
    """Dense causal GQA attention by the library routine (float64)."""
    grp = q.shape[0] // k.shape[0]
    tq = torch.from_numpy(q.astype(np.float64))[None]
    tk = torch.from_numpy(k.astype(np.float64)).repeat_interleave(grp, dim=0)[None]
    tv = torch.from_numpy(v.astype(np.float64)).repeat_interleave(grp, dim=0)[None]
    return torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].numpy()


def test_mask_matches_hand_written_fixture():
    want = np.loadtxt(os.path.join(GOLDEN, "prefill_mask_small.txt"), comments="#").astype(bool)
    lay = small_layout()
    got = oracle.allowed_mask(np.arange(lay.n_tokens), lay.n_prefix, lay.chunk_bounds, lay.sparse_idx)
    assert got.shape == want.shape
    assert np.array_equal(got, want)
    assert got.sum() == 50 == oracle.allowed_pair_count(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets)


def test_pair_census_closed_form():
    w = wl.WORKLOADS["config0"]
    lay = wl.make_layout(w)
    m = oracle.allowed_mask(np.arange(lay.n_tokens), lay.n_prefix, lay.chunk_bounds, lay.sparse_idx)
    assert m.sum() == 80160      # 2080 + 16448 + 18496 + 20544 + 22592, worked by hand
    assert oracle.allowed_pair_count(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets) == 80160
    rng = np.random.default_rng(5)
    for _ in range(10):
        lay = wl.random_layout(rng, int(rng.integers(0, 6)), int(rng.integers(1, 6)), 1, 9)
        m = oracle.allowed_mask(np.arange(lay.n_tokens), lay.n_prefix, lay.chunk_bounds, lay.sparse_idx)
        assert m.sum() == oracle.allowed_pair_count(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets)


def test_mask_is_causal_and_contains_diagonal():
    rng = np.random.default_rng(6)
    lay = wl.random_layout(rng, 3, 5, 2, 8)
    m = oracle.allowed_mask(np.arange(lay.n_tokens), lay.n_prefix, lay.chunk_bounds, lay.sparse_idx)
    assert not np.triu(m, 1).any()
    assert np.diag(m).all()
    assert m[:, :lay.n_prefix][lay.n_prefix:].all()       # every visual token sees the whole prefix


@pytest.mark.parametrize("hq,hkv", [(2, 1), (4, 2), (6, 2)])
def test_single_chunk_is_dense_causal(hq, hkv):
    rng = np.random.default_rng(10 + hq)
    n, d = 37, 16
    q, k, v = rand_qkv(rng, hq, hkv, n, d)
    lay = wl.layout_from_lists(0, [n], [np.zeros(0, np.int32)])
    want = sdpa_causal(q, k, v)
    got = oracle.prefill_def(q, k, v, 0, lay.chunk_bounds, lay.sparse_idx)
    assert np.abs(got - want).max() < 1e-12
    got = oracle.prefill_blk(q, k, v, 0, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    assert np.abs(got - want).max() < 1e-12


def test_keeping_every_token_is_dense_causal_for_any_chunking():
    rng = np.random.default_rng(11)
    lens = [5, 1, 9, 4, 7]
    p = 3
    n = p + sum(lens)
    q, k, v = rand_qkv(rng, 4, 2, n, 8)
    kept, s = [], p
    for ln in lens:
        kept.append(np.arange(s, s + ln))
        s += ln
    lay = wl.layout_from_lists(p, lens, kept)
    want = sdpa_causal(q, k, v)
    for got in (oracle.prefill_def(q, k, v, p, lay.chunk_bounds, lay.sparse_idx),
                oracle.prefill_blk(q, k, v, p, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)):
        assert np.abs(got - want).max() < 1e-12


def test_no_kept_no_prefix_is_block_diagonal():
    rng = np.random.default_rng(12)
    lens = [6, 3, 8]
    n = sum(lens)
    q, k, v = rand_qkv(rng, 2, 1, n, 8)
    lay = wl.layout_from_lists(0, lens, [np.zeros(0, np.int32)] * 3)
    got = oracle.prefill_def(q, k, v, 0, lay.chunk_bounds, lay.sparse_idx)
    s = 0
    for ln in lens:
        want = sdpa_causal(q[:, s:s + ln], k[:, s:s + ln], v[:, s:s + ln])
        assert np.abs(got[:, s:s + ln] - want).max() < 1e-12
        s += ln


def test_prefix_rows_are_plain_causal_attention_over_the_prefix():
    rng = np.random.default_rng(13)
    lay = wl.random_layout(rng, 7, 3, 3, 6)
    q, k, v = rand_qkv(rng, 2, 2, lay.n_tokens, 8)
    got = oracle.prefill_def(q, k, v, 7, lay.chunk_bounds, lay.sparse_idx, rows=np.arange(7))
    want = sdpa_causal(q[:, :7], k[:, :7], v[:, :7])
    assert np.abs(got - want).max() < 1e-12


def test_brute_force_scalar_loops():
    """Independent scalar evaluation: python sets for A(i), math.exp, explicit sums."""
    rng = np.random.default_rng(14)
    lay = wl.random_layout(rng, 2, 3, 2, 5)
    n, d, hq, hkv = lay.n_tokens, 4, 4, 2
    q, k, v = rand_qkv(rng, hq, hkv, n, d)
    got = oracle.prefill_def(q, k, v, 2, lay.chunk_bounds, lay.sparse_idx)
    got2 = oracle.prefill_blk(q, k, v, 2, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    bounds = [int(x) for x in lay.chunk_bounds]
    for h in range(hq):
        g = h // (hq // hkv)
        for i in range(n):
            if i < 2:
                allowed = set(range(i + 1))
            else:
                c = max(cc for cc in range(lay.n_chunks) if bounds[cc] <= i)
                allowed = set(range(2)) | set(range(bounds[c], i + 1))
                for cc in range(c):
                    allowed |= set(int(x) for x in lay.kept(cc))
            logit = {j: sum(float(q[h, i, t]) * float(k[g, j, t]) for t in range(d)) / math.sqrt(d)
                     for j in allowed}
            z = sum(math.exp(x) for x in logit.values())
            for t in range(d):
                o = sum(math.exp(logit[j]) / z * float(v[g, j, t]) for j in allowed)
                assert abs(o - got[h, i, t]) < 1e-12
                assert abs(o - got2[h, i, t]) < 1e-12


def test_blk_equals_def_on_random_layouts_and_row_subsets():
    rng = np.random.default_rng(15)
    for trial in range(6):
        p = int(rng.integers(0, 5))
        lay = wl.random_layout(rng, p, int(rng.integers(1, 6)), 1, 12)
        q, k, v = rand_qkv(rng, 4, 2, lay.n_tokens, 8)
        a, la = oracle.prefill_def(q, k, v, p, lay.chunk_bounds, lay.sparse_idx, return_lse=True)
        b, lb = oracle.prefill_blk(q, k, v, p, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx,
                                   return_lse=True)
        assert np.abs(a - b).max() < 1e-12 and np.abs(la - lb).max() < 1e-12
        rows = rng.permutation(lay.n_tokens)[: max(1, lay.n_tokens // 2)]
        c = oracle.prefill_blk(q, k, v, p, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx,
                               rows=rows, heads=[3, 0])
        assert np.abs(c[0] - a[3][rows]).max() < 1e-12
        assert np.abs(c[1] - a[0][rows]).max() < 1e-12


def test_probabilities_sum_to_one_and_vanish_outside_the_allowed_set():
    rng = np.random.default_rng(16)
    lay = wl.random_layout(rng, 3, 4, 2, 7)
    q, k, v = rand_qkv(rng, 2, 1, lay.n_tokens, 8, scale=3.0)
    _, probs = oracle.prefill_def(q, k, v, 3, lay.chunk_bounds, lay.sparse_idx, return_probs=True)
    m = oracle.allowed_mask(np.arange(lay.n_tokens), 3, lay.chunk_bounds, lay.sparse_idx)
    assert np.abs(probs.sum(axis=-1) - 1.0).max() < 1e-12
    assert (probs[:, ~m] == 0.0).all()
    assert (probs[:, m] > 0.0).all()


def test_value_probes_constant_indicator_and_mass():
    rng = np.random.default_rng(17)
    lay = wl.random_layout(rng, 2, 4, 2, 7)
    n = lay.n_tokens
    q, k, _ = rand_qkv(rng, 2, 1, n, 8)
    args = (2, lay.chunk_bounds, lay.sparse_idx)
    const = np.full((1, n, 8), 0.37, np.float32)
    assert np.abs(oracle.prefill_def(q, k, const, *args) - np.float64(np.float32(0.37))).max() < 1e-14
    m = oracle.allowed_mask(np.arange(n), *args)
    _, probs = oracle.prefill_def(q, k, const, *args, return_probs=True)
    i = n - 1                                        # a row that has disallowed earlier keys
    assert (~m[i, :i]).any()
    ind = np.zeros((1, n, 8), np.float32)
    ind[0, ~m[i], :] = 1.0
    assert (oracle.prefill_def(q, k, ind, *args, rows=[i]) == 0.0).all()      # mask leak detector
    sel = np.zeros(n, bool)
    sel[lay.kept(0)] = True
    ind = np.zeros((1, n, 8), np.float32)
    ind[0, sel, :] = 1.0
    mass = oracle.prefill_def(q, k, ind, *args, rows=[i])
    assert np.abs(mass[:, 0, 0] - probs[:, i, sel].sum(axis=-1)).max() < 1e-14


def test_locality_of_a_non_kept_token():
    """Changing K/V of a token that is not kept changes only later rows of its own chunk."""
    rng = np.random.default_rng(18)
    lens = [6, 7, 5]
    kept = [np.array([2, 4]), np.array([8, 12]), np.array([15])]
    lay = wl.layout_from_lists(2, lens, kept)
    q, k, v = rand_qkv(rng, 2, 1, lay.n_tokens, 8)
    base = oracle.prefill_def(q, k, v, 2, lay.chunk_bounds, lay.sparse_idx)
    j = 10                                              # in chunk 1 = [8, 15), not kept
    k2, v2 = k.copy(), v.copy()
    k2[:, j] += 1.0
    v2[:, j] -= 2.0
    pert = oracle.prefill_def(q, k2, v2, 2, lay.chunk_bounds, lay.sparse_idx)
    changed = np.abs(pert - base).max(axis=(0, 2)) > 0
    assert changed[10:15].all()
    assert not changed[:10].any() and not changed[15:].any()
    # a kept token of the same chunk does reach later chunks
    k3 = k.copy()
    k3[:, 12] += 1.0
    pert = oracle.prefill_def(q, k3, v, 2, lay.chunk_bounds, lay.sparse_idx)
    changed = np.abs(pert - base).max(axis=(0, 2)) > 0
    assert changed[12:].all() and not changed[:12].any()


def test_gqa_head_map():
    """Query head h reads KV head h // (Hq/Hkv): zero V on all KV heads but one."""
    rng = np.random.default_rng(19)
    lay = wl.random_layout(rng, 1, 2, 3, 5)
    q, k, v = rand_qkv(rng, 6, 3, lay.n_tokens, 4)
    v[0] = 0.0
    v[2] = 0.0
    out = oracle.prefill_def(q, k, v, 1, lay.chunk_bounds, lay.sparse_idx)
    assert (out[[0, 1, 4, 5]] == 0).all() and (np.abs(out[[2, 3]]).max(axis=(1, 2)) > 0).all()


def test_explicit_scale_and_shift_invariance():
    rng = np.random.default_rng(20)
    lay = wl.random_layout(rng, 2, 3, 3, 6)
    q, k, v = rand_qkv(rng, 2, 1, lay.n_tokens, 16)
    a = oracle.prefill_def(q, k, v, 2, lay.chunk_bounds, lay.sparse_idx)                  # 1/sqrt(16)
    b = oracle.prefill_def(2.0 * q, k, v, 2, lay.chunk_bounds, lay.sparse_idx, scale=0.125)
    assert np.abs(a - b).max() < 1e-12
    # adding one vector u to every key shifts all logits of a row by q.u: softmax unchanged
    u = rng.standard_normal(16)
    c = oracle.prefill_def(q, k.astype(np.float64) + u, v, 2, lay.chunk_bounds, lay.sparse_idx)
    assert np.abs(a - c).max() < 1e-12


def test_config0_def_and_blk_agree():
    w = wl.WORKLOADS["config0"]
    lay = wl.make_layout(w)
    q, k, v = wl.make_qkv(w, lay)
    a = oracle.prefill_def(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_idx)
    b = oracle.prefill_blk(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    assert np.abs(a - b).max() < 1e-12


# ------------------------------------------------------------------ sliding chunk window
def test_window_mask_matches_hand_written_fixture():
    want = np.loadtxt(os.path.join(GOLDEN, "prefill_mask_window_small.txt"), comments="#").astype(bool)
    lay = small_layout()
    got = oracle.allowed_mask(np.arange(lay.n_tokens), lay.n_prefix, lay.chunk_bounds, lay.sparse_idx, window=2)
    assert np.array_equal(got, want)
    assert got.sum() == 60 == oracle.allowed_pair_count(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets,
                                                        lay.sparse_idx, window=2)


def test_window_mask_against_set_enumeration():
    """The vectorised mask against plain Python sets built token by token from the definition."""
    rng = np.random.default_rng(61)
    for _ in range(25):
        lay = wl.random_layout(rng, int(rng.integers(0, 5)), int(rng.integers(1, 6)), 1, 9)
        window = int(rng.integers(0, 14))
        b, p = [int(x) for x in lay.chunk_bounds], lay.n_prefix
        kept_by_chunk = [set(int(t) for t in lay.sparse_idx[lay.sparse_offsets[c]:lay.sparse_offsets[c + 1]])
                         for c in range(lay.n_chunks)]
        want = np.zeros((lay.n_tokens, lay.n_tokens), dtype=bool)
        for i in range(lay.n_tokens):
            if i < p:
                allowed = set(range(i + 1))
            else:
                c = max(cc for cc in range(lay.n_chunks) if b[cc] <= i)
                allowed = set(range(p))
                for cc in range(c):
                    allowed |= kept_by_chunk[cc]
                allowed |= set(range(max(p, b[c] - window), i + 1))
            want[i, sorted(allowed)] = True
        got = oracle.allowed_mask(np.arange(lay.n_tokens), p, lay.chunk_bounds, lay.sparse_idx, window=window)
        assert np.array_equal(got, want)
        assert got.sum() == oracle.allowed_pair_count(p, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx,
                                                      window=window)
        if window == 0:
            assert np.array_equal(got, oracle.allowed_mask(np.arange(lay.n_tokens), p, lay.chunk_bounds,
                                                           lay.sparse_idx))


def test_window_covering_everything_is_dense_causal():
    rng = np.random.default_rng(62)
    lay = wl.random_layout(rng, 3, 5, 2, 9)
    n = lay.n_tokens
    q, k, v = rand_qkv(rng, 4, 2, n, 16)
    want = sdpa_causal(q, k, v)
    got = oracle.prefill_def(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_idx, window=n)
    blk = oracle.prefill_blk(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx, window=n)
    assert np.abs(got - want).max() < 1e-12
    assert np.abs(blk - want).max() < 1e-12


def test_window_without_history_is_banded_attention():
    """No prefix, nothing kept: token i of chunk c sees exactly [b_c - window, i]; compared with
    a row-by-row evaluation that shares nothing with the oracle's matrix code."""
    rng = np.random.default_rng(63)
    lens, window, d = [5, 7, 4, 6], 3, 8
    lay = wl.layout_from_lists(0, lens, [np.zeros(0, np.int32)] * len(lens))
    n = lay.n_tokens
    q, k, v = rand_qkv(rng, 2, 1, n, d)
    got = oracle.prefill_blk(q, k, v, 0, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx, window=window)
    starts = np.cumsum([0] + lens)
    for h in range(2):
        for i in range(n):
            c = int(np.searchsorted(starts, i, side="right") - 1)
            lo = max(0, int(starts[c]) - window)
            w_ = [math.exp(float(np.dot(q[h, i].astype(np.float64), k[0, j].astype(np.float64))) / math.sqrt(d))
                  for j in range(lo, i + 1)]
            o = sum(wj * v[0, j].astype(np.float64) for wj, j in zip(w_, range(lo, i + 1))) / sum(w_)
            assert np.abs(got[h, i] - o).max() < 1e-12


def test_window_def_and_blk_agree():
    rng = np.random.default_rng(64)
    for _ in range(6):
        lay = wl.random_layout(rng, int(rng.integers(0, 4)), int(rng.integers(2, 6)), 2, 12)
        window = int(rng.integers(1, 10))
        q, k, v = rand_qkv(rng, 4, 2, lay.n_tokens, 8)
        a, la = oracle.prefill_def(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_idx, return_lse=True,
                                   window=window)
        b, lb = oracle.prefill_blk(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx,
                                   return_lse=True, window=window)
        assert np.abs(a - b).max() < 1e-12 and np.abs(la - lb).max() < 1e-12
