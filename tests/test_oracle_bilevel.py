"""Pins of the bi-level decoding oracle: hand-written index fixture, exhaustive enumeration,
brute force, closed forms, library special cases and algebraic identities.  The paper prints
no worked numeric example for these steps, so none of these is a paper value."""
import itertools
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


def lay_args(lay):
    return lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx


# ----------------------------------------------------------------------------- scores / top-k
def test_score_is_mean_logit_by_brute_force():
    rng = np.random.default_rng(30)
    lay = wl.random_layout(rng, 3, 4, 1, 6)
    hq, hkv, d, t, bsz = 6, 2, 5, 3, 2
    qd = rng.standard_normal((bsz, t, hq, d)).astype(np.float32)
    k = rng.standard_normal((hkv, lay.n_tokens, d)).astype(np.float32)
    got = oracle.chunk_scores(qd, k, lay.chunk_bounds)
    for b in range(bsz):
        for c in range(lay.n_chunks):
            vals = []
            for tt in range(t):
                for h in range(hq):
                    g = h // (hq // hkv)
                    for j in range(lay.chunk_bounds[c], lay.chunk_bounds[c + 1]):
                        vals.append(sum(float(qd[b, tt, h, x]) * float(k[g, j, x]) for x in range(d))
                                    / math.sqrt(d))
            assert abs(sum(vals) / len(vals) - got[b, c]) < 1e-13


def test_mass_score_by_brute_force():
    """Attention-mass score against scalar loops with math.exp (nothing shared with the matrix code)."""
    rng = np.random.default_rng(35)
    lay = wl.random_layout(rng, 2, 4, 1, 6)
    hq, hkv, d, t, bsz = 4, 2, 5, 3, 2
    qd = rng.standard_normal((bsz, t, hq, d)).astype(np.float32)
    k = rng.standard_normal((hkv, lay.n_tokens, d)).astype(np.float32)
    got = oracle.chunk_scores_mass(qd, k, lay.n_prefix, lay.chunk_bounds)
    want = np.zeros_like(got)
    for b in range(bsz):
        for tt in range(t):
            for h in range(hq):
                g = h // (hq // hkv)
                e = [math.exp(sum(float(qd[b, tt, h, x]) * float(k[g, j, x]) for x in range(d)) / math.sqrt(d))
                     for j in range(lay.n_tokens)]
                z = sum(e)
                for c in range(lay.n_chunks):
                    want[b, c] += sum(e[lay.chunk_bounds[c]:lay.chunk_bounds[c + 1]]) / z
    want /= t * hq
    assert np.abs(got - want).max() < 1e-14


def test_mass_score_closed_forms():
    rng = np.random.default_rng(36)
    lay = wl.random_layout(rng, 5, 6, 1, 9)
    n = lay.n_tokens
    lens = np.diff(lay.chunk_bounds)
    qd = rng.standard_normal((2, 3, 4, 8)).astype(np.float32)
    # identical keys everywhere: the attention is uniform, a chunk's mass is its share of the tokens
    k = np.broadcast_to(rng.standard_normal((2, 1, 8)).astype(np.float32), (2, n, 8)).copy()
    got = oracle.chunk_scores_mass(qd, k, lay.n_prefix, lay.chunk_bounds)
    assert np.abs(got - lens[None, :] / n).max() < 1e-14
    # the scores of a query and its mean prefix mass add up to one
    k = rng.standard_normal((2, n, 8)).astype(np.float32)
    got = oracle.chunk_scores_mass(qd, k, lay.n_prefix, lay.chunk_bounds)
    no_prefix = oracle.chunk_scores_mass(qd, k[:, lay.n_prefix:], 0, lay.chunk_bounds - lay.n_prefix)
    assert (got >= 0).all() and (got.sum(axis=1) < 1).all()
    assert np.abs(no_prefix.sum(axis=1) - 1).max() < 1e-14
    # scale 0: uniform again, whatever the keys
    got = oracle.chunk_scores_mass(qd, k, lay.n_prefix, lay.chunk_bounds, scale=0.0)
    assert np.abs(got - lens[None, :] / n).max() < 1e-14
    # one key far above the others takes all the mass for its chunk
    c, qd1 = 3, np.ones((1, 1, 2, 8), np.float32)
    k1 = np.zeros((2, n, 8), np.float32)
    k1[:, lay.chunk_bounds[c] + 1] = 40.0
    got = oracle.chunk_scores_mass(qd1, k1, lay.n_prefix, lay.chunk_bounds)
    assert abs(got[0, c] - 1) < 1e-12 and np.abs(np.delete(got[0], c)).max() < 1e-12


def test_mass_score_small_logits_follow_the_mean_logit_score():
    """For small logits exp(s) ~ 1 + s: mass_c ~ len_c/N * (1 + mean logit of c - mean logit overall),
    i.e. per token the mass score orders chunks like the mean-logit score."""
    rng = np.random.default_rng(37)
    lay = wl.layout_from_lists(0, [6] * 5, [np.zeros(0, np.int32)] * 5)
    qd = (rng.standard_normal((1, 2, 4, 8)) * 0.01).astype(np.float32)
    k = (rng.standard_normal((2, 30, 8)) * 0.01).astype(np.float32)
    mass = oracle.chunk_scores_mass(qd, k, 0, lay.chunk_bounds)
    # first-order expansion evaluated with the explicit logit matrix
    grp = 2
    first = np.zeros(5)
    for t in range(2):
        for h in range(4):
            s = (qd[0, t, h].astype(np.float64) @ k[h // grp].astype(np.float64).T) / math.sqrt(8)
            first += np.array([(1 + s[6 * c:6 * c + 6] - s.mean()).sum() / 30 for c in range(5)])
    first /= 8
    assert np.abs(mass - first).max() < 1e-7


def test_topk_exhaustive_enumeration():
    rng = np.random.default_rng(31)
    for trial in range(40):
        c_n = int(rng.integers(1, 11))
        k = int(rng.integers(0, c_n + 2))
        # few distinct values => many ties
        s = rng.integers(0, 4, size=(1, c_n)).astype(np.float64) if trial % 2 else rng.standard_normal((1, c_n))
        idx, mask = oracle.select_topk(s, k)
        kk = min(k, c_n)
        assert idx.shape == (1, kk) and mask.sum() == kk
        best_sum = max(sum(s[0, list(sub)]) for sub in itertools.combinations(range(c_n), kk))
        assert abs(sum(s[0, idx[0]]) - best_sum) < 1e-12
        # among all maximisers the chosen set is the lexicographically smallest one
        maximisers = [sub for sub in itertools.combinations(range(c_n), kk)
                      if abs(sum(s[0, list(sub)]) - best_sum) < 1e-12]
        assert tuple(sorted(idx[0])) == min(maximisers)
        assert set(np.nonzero(mask[0])[0]) == set(idx[0])
        # order: score descending, ties ascending id
        for a, b in zip(idx[0][:-1], idx[0][1:]):
            assert (s[0, a] > s[0, b]) or (s[0, a] == s[0, b] and a < b)


def test_topk_duplicated_chunks_pick_lower_index():
    rng = np.random.default_rng(32)
    d, ln = 8, 5
    blk = rng.standard_normal((2, ln, d)).astype(np.float32)
    other = (rng.standard_normal((2, ln, d)) - 5.0).astype(np.float32)
    k = np.concatenate([other, blk, other, blk, blk], axis=1)          # chunks 1, 3, 4 identical
    lay = wl.layout_from_lists(0, [ln] * 5, [np.zeros(0, np.int32)] * 5)
    qd = np.abs(rng.standard_normal((1, 2, 4, d))).astype(np.float32)
    s = oracle.chunk_scores(qd, k, lay.chunk_bounds)
    assert s[0, 1] == s[0, 3] == s[0, 4]
    if s[0, 1] > s[0, 0]:
        idx, mask = oracle.select_topk(s, 2)
        assert list(idx[0]) == [1, 3] and list(mask[0]) == [0, 1, 0, 1, 0]


def test_topk_edge_cases_and_scale_invariance():
    s = np.array([[0.3, -1.0, 2.0, 0.3]])
    idx, mask = oracle.select_topk(s, 0)
    assert idx.shape == (1, 0) and mask.sum() == 0
    idx, mask = oracle.select_topk(s, 9)
    assert list(idx[0]) == [2, 0, 3, 1] and mask.all()
    idx, _ = oracle.select_topk(s, 2)
    assert list(idx[0]) == [2, 0]
    rng = np.random.default_rng(33)
    lay = wl.random_layout(rng, 0, 9, 2, 6)
    qd = rng.standard_normal((3, 2, 4, 8)).astype(np.float32)
    k = rng.standard_normal((2, lay.n_tokens, 8)).astype(np.float32)
    a = oracle.select_topk(oracle.chunk_scores(qd, k, lay.chunk_bounds), 4)
    b = oracle.select_topk(oracle.chunk_scores(8.0 * qd, k, lay.chunk_bounds), 4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_planted_chunks_are_recalled_by_query_zero():
    w = wl.WORKLOADS["config4"]
    lay = wl.make_layout(w)
    assert lay.n_tokens == 65792 and lay.chunk_bounds[0] == 256
    lens = np.diff(lay.chunk_bounds)
    assert lens.min() >= 1 and lens.max() <= 1024 and (lens[:-1] % 64 == 0).all()
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    planted = wl.planted_chunks(w, lay)
    s = oracle.chunk_scores(qd, k, lay.chunk_bounds)
    idx, _ = oracle.select_topk(s, len(planted))
    assert set(idx[0]) == set(planted)                    # query 0 carries the signal
    assert set(idx[1]) != set(planted)                    # the other queries are controls


# ----------------------------------------------------------------------------- gather
def test_mixed_index_matches_hand_written_fixture():
    lay = small_layout()
    with open(os.path.join(GOLDEN, "mixed_index_small.txt")) as f:
        lines = [ln for ln in f if ln.strip() and not ln.startswith("#")]
    assert len(lines) == 6
    for ln in lines:
        bits, ids = ln.split(":")
        mask = [int(ch) for ch in bits.strip()]
        want = [int(x) for x in ids.split()]
        got = oracle.mixed_source_index(mask, *lay_args(lay))
        assert list(got) == want


def test_gather_properties():
    rng = np.random.default_rng(34)
    lay = wl.random_layout(rng, 3, 6, 1, 9)
    n = lay.n_tokens
    k = rng.integers(0, 2 ** 16, size=(2, n, 4)).astype(np.uint16)       # arbitrary bit patterns
    v = rng.integers(0, 2 ** 16, size=(2, n, 4)).astype(np.uint16)
    masks = rng.integers(0, 2, size=(5, lay.n_chunks)).astype(np.uint8)
    masks[0] = 0
    masks[1] = 1
    kmix, vmix, lens, src = oracle.gather_bilevel(k, v, masks, *lay_args(lay), l_cap=n + 3)
    lens_c = np.diff(lay.chunk_bounds)
    s_c = np.diff(lay.sparse_offsets)
    for b in range(5):
        want_len = lay.n_prefix + int(np.where(masks[b] == 1, lens_c, s_c).sum())
        assert lens[b] == want_len
        ids = src[b, :lens[b]]
        assert (np.diff(ids) > 0).all()
        assert np.array_equal(kmix[b, :, :lens[b]], k[:, ids])
        assert np.array_equal(vmix[b, :, :lens[b]], v[:, ids])
        assert (src[b, lens[b]:] == -1).all() and (kmix[b, :, lens[b]:] == 0).all()
    assert lens[0] == lay.n_prefix + lay.sparse_offsets[-1]                  # k = 0
    assert lens[1] == n and np.array_equal(kmix[1, :, :n], k)                # k >= C


# ----------------------------------------------------------------------------- decode
def sdpa_full(qd_b, k, v):
    """Non-causal GQA attention of T query tokens over all keys, by the library routine."""
    grp = qd_b.shape[1] // k.shape[0]
    tq = torch.from_numpy(qd_b.astype(np.float64)).permute(1, 0, 2)[None]          # [1,Hq,T,D]
    tk = torch.from_numpy(k.astype(np.float64)).repeat_interleave(grp, dim=0)[None]
    tv = torch.from_numpy(v.astype(np.float64)).repeat_interleave(grp, dim=0)[None]
    o = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0]            # [Hq,T,D]
    return o.permute(1, 0, 2).numpy()


def test_all_dense_equals_full_kv_decode():
    rng = np.random.default_rng(35)
    lens = [4, 6, 3, 5]
    kept, s = [], 2
    for ln in lens:
        kept.append(np.arange(s, s + ln))
        s += ln
    lay = wl.layout_from_lists(2, lens, kept)
    n = lay.n_tokens
    qd = rng.standard_normal((2, 3, 4, 8)).astype(np.float32)
    k = rng.standard_normal((2, n, 8)).astype(np.float32)
    v = rng.standard_normal((2, n, 8)).astype(np.float32)
    for mask in (np.ones((2, 4), np.uint8), np.zeros((2, 4), np.uint8)):      # k = C; sparse = all
        kmix, vmix, ml, _ = oracle.gather_bilevel(k, v, mask, *lay_args(lay))
        assert (ml == n).all()
        got = oracle.decode_mixed(qd, kmix, vmix, ml)
        for b in range(2):
            assert np.abs(got[b] - sdpa_full(qd[b], k, v)).max() < 1e-12


def test_decode_of_T_tokens_is_T_single_token_decodes_and_ignores_padding():
    rng = np.random.default_rng(36)
    lay = wl.random_layout(rng, 2, 4, 2, 6)
    n = lay.n_tokens
    qd = rng.standard_normal((2, 4, 4, 8)).astype(np.float32)
    k = rng.standard_normal((2, n, 8)).astype(np.float32)
    v = rng.standard_normal((2, n, 8)).astype(np.float32)
    mask = np.array([[1, 0, 0, 1], [0, 0, 1, 0]], np.uint8)
    kmix, vmix, ml, _ = oracle.gather_bilevel(k, v, mask, *lay_args(lay), l_cap=n + 5)
    kmix[:, :, ml.max():] = 1e30          # garbage beyond mix_len must not matter
    full = oracle.decode_mixed(qd, kmix, vmix, ml)
    for t in range(4):
        one = oracle.decode_mixed(qd[:, t:t + 1], kmix, vmix, ml)
        assert np.abs(one[:, 0] - full[:, t]).max() < 1e-13
    const = np.full_like(vmix, 0.25)
    assert np.abs(oracle.decode_mixed(qd, kmix, const, ml) - 0.25).max() < 1e-14


def test_decode_equals_prefill_row_with_the_same_visible_set():
    """A query token placed as a new last chunk sees prefix + kept sets + itself in pre-filling;
    with its own key pushed to a logit of -800 its weight is exactly zero, so the pre-filling
    row must equal the decode over the all-sparse mixed set."""
    rng = np.random.default_rng(37)
    lay = wl.random_layout(rng, 3, 4, 2, 6, allow_empty_kept=False)
    n, d = lay.n_tokens, 8
    k = rng.standard_normal((1, n + 1, d)).astype(np.float64)
    v = rng.standard_normal((1, n + 1, d)).astype(np.float64)
    q = rng.standard_normal((2, n + 1, d)).astype(np.float64)
    lens = list(np.diff(lay.chunk_bounds)) + [1]
    kept = [lay.kept(c) for c in range(lay.n_chunks)] + [np.zeros(0, np.int32)]
    lay2 = wl.layout_from_lists(3, lens, kept)
    out = np.zeros((2, d))
    for h in range(2):
        kk = k.copy()
        kk[0, n] = -800.0 * math.sqrt(d) * q[h, n] / (q[h, n] @ q[h, n])
        out[h] = oracle.prefill_def(q, kk, v, 3, lay2.chunk_bounds, lay2.sparse_idx, rows=[n])[h, 0]
    kmix, vmix, ml, _ = oracle.gather_bilevel(k[:, :n], v[:, :n], np.zeros((1, lay.n_chunks), np.uint8),
                                              *lay_args(lay))
    qd = q[:, n][None, None]                                   # [1, 1, Hq, D]
    dec = oracle.decode_mixed(qd, kmix, vmix, ml)[0, 0]
    assert np.abs(dec - out).max() < 1e-12


def test_lse_merge_identity():
    """Attention over a union equals the log-sum-exp merge of attention over the parts."""
    rng = np.random.default_rng(38)
    qd = (3.0 * rng.standard_normal((1, 2, 2, 8))).astype(np.float32)
    kmix = rng.standard_normal((1, 1, 20, 8)).astype(np.float32)
    vmix = rng.standard_normal((1, 1, 20, 8)).astype(np.float32)
    o, l = oracle.decode_lse(qd, kmix, vmix, [20])
    oa, la = oracle.decode_lse(qd, kmix[:, :, :7], vmix[:, :, :7], [7])
    ob, lb = oracle.decode_lse(qd, kmix[:, :, 7:], vmix[:, :, 7:], [13])
    m = np.maximum(la, lb)
    wa, wb = np.exp(la - m), np.exp(lb - m)
    merged = (oa * wa[..., None] + ob * wb[..., None]) / (wa + wb)[..., None]
    assert np.abs(merged - o).max() < 1e-12
    assert np.abs(m + np.log(wa + wb) - l).max() < 1e-12
    # LSE against its definition
    s = (qd[0, 0, 1].astype(np.float64) @ kmix[0, 0].astype(np.float64).T) / math.sqrt(8)
    assert abs(math.log(sum(math.exp(x) for x in s)) - l[0, 0, 1]) < 1e-12


# --------------------------------------------------------------------------------- pooled sparse KVs
def _pool_fixture():
    rows = {}
    for ln in open(os.path.join(GOLDEN, "pooled_kv_small.txt")):
        if ln.startswith("#") or not ln.strip():
            continue
        i, vals = ln.split(":")
        rows[int(i)] = [float(x) for x in vals.split()]
    return rows


def test_pooled_kv_hand_worked_fixture():
    rows = _pool_fixture()
    bounds, soff = [1, 5, 12, 14], [0, 2, 5, 7]
    k = np.stack([np.arange(14.0), 10.0 * np.arange(14.0)], axis=1)[None]        # [1, 14, 2]
    ksp, vsp = oracle.pool_sparse_kv(k, -k, bounds, soff)
    assert ksp.shape == (1, 7, 2)
    for i, want in rows.items():
        assert np.array_equal(ksp[0, i], np.array(want)), i
    assert np.array_equal(vsp, -ksp)


def test_pool_groups_partition_the_chunk():
    for length in range(1, 40):
        for count in range(1, length + 1):
            g = oracle.pool_groups(length, count)
            assert len(g) == count and g[0][0] == 0 and g[-1][1] == length
            sizes = [hi - lo for lo, hi in g]
            assert all(g[i][1] == g[i + 1][0] for i in range(count - 1))
            assert min(sizes) >= 1 and max(sizes) - min(sizes) <= 1              # as even as it gets
            if length % count == 0:
                assert set(sizes) == {length // count}                            # plain average pooling


def test_pooled_kv_special_cases_and_brute_force():
    rng = np.random.default_rng(81)
    lay = wl.random_layout(rng, 3, 6, 1, 23, allow_empty_kept=False)
    n, hkv, d = lay.n_tokens, 2, 4
    k = rng.standard_normal((hkv, n, d))
    v = rng.standard_normal((hkv, n, d))
    b, off = lay.chunk_bounds, lay.sparse_offsets
    ksp, vsp = oracle.pool_sparse_kv(k, v, b, off)
    # brute force with python loops over tokens (nothing shared with the slicing code)
    for c in range(lay.n_chunks):
        ln, cnt = int(b[c + 1] - b[c]), int(off[c + 1] - off[c])
        for m in range(cnt):
            # membership by the group bounds: j in [floor(m*ln/cnt), floor((m+1)*ln/cnt))
            toks = [int(b[c]) + j for j in range(ln) if (m * ln) // cnt <= j < ((m + 1) * ln) // cnt]
            for g in range(hkv):
                for e in range(d):
                    want = sum(k[g, t, e] for t in toks) / len(toks)
                    assert abs(ksp[g, off[c] + m, e] - want) < 1e-12
                    want = sum(v[g, t, e] for t in toks) / len(toks)
                    assert abs(vsp[g, off[c] + m, e] - want) < 1e-12
    # as many sparse rows as dense rows: pooling is the identity
    full_off = np.concatenate([[0], np.cumsum(np.diff(b))])
    ksp, vsp = oracle.pool_sparse_kv(k, v, b, full_off)
    assert np.array_equal(ksp, k[:, lay.n_prefix:]) and np.array_equal(vsp, v[:, lay.n_prefix:])
    # one sparse row per chunk: the chunk mean (the summary the mean-logit score is built on)
    one_off = np.arange(lay.n_chunks + 1)
    ksp, _ = oracle.pool_sparse_kv(k, v, b, one_off)
    for c in range(lay.n_chunks):
        assert np.allclose(ksp[:, c], k[:, b[c]:b[c + 1]].mean(axis=1), rtol=0, atol=1e-12)
    # constant rows stay constant; pooling is linear
    kc = np.broadcast_to(np.array([1.0, -2.0, 0.5, 4.0]), (hkv, n, d))
    ksp, _ = oracle.pool_sparse_kv(kc, kc, b, off)
    assert np.array_equal(ksp, np.broadcast_to(kc[0, 0], ksp.shape))
    a1, _ = oracle.pool_sparse_kv(k, v, b, off)
    a2, _ = oracle.pool_sparse_kv(v, k, b, off)
    a3, _ = oracle.pool_sparse_kv(2.0 * k - 3.0 * v, k, b, off)
    assert np.allclose(a3, 2.0 * a1 - 3.0 * a2, rtol=0, atol=1e-12)


def test_pooled_gather_structure():
    rng = np.random.default_rng(82)
    lay = wl.random_layout(rng, 2, 5, 2, 9, allow_empty_kept=False)
    n, hkv, d = lay.n_tokens, 1, 3
    k = rng.standard_normal((hkv, n, d))
    v = rng.standard_normal((hkv, n, d))
    b, off = lay.chunk_bounds, lay.sparse_offsets
    ksp, vsp = oracle.pool_sparse_kv(k, v, b, off)
    masks = np.array([[0] * 5, [1] * 5, [1, 0, 0, 1, 0]], dtype=np.uint8)
    kmix, vmix, lens, src = oracle.gather_bilevel_pooled(k, v, ksp, vsp, masks, lay.n_prefix, b, off)
    assert lens[0] == lay.n_prefix + off[-1] and lens[1] == n
    assert np.array_equal(kmix[1, :, :n], k) and np.array_equal(src[1, :n], np.arange(n))     # all dense: the cache itself
    assert np.array_equal(kmix[0, :, lay.n_prefix:lens[0]], ksp)                              # all sparse: prefix + pooled rows
    assert np.array_equal(src[0, lay.n_prefix:lens[0]], -1 - np.arange(off[-1]))
    # mixed: same lengths and the same dense rows as the index-selection gather for the same mask
    _, _, lens_sel, src_sel = oracle.gather_bilevel(k, v, masks, lay.n_prefix, b, off, lay.sparse_idx)
    assert np.array_equal(lens, lens_sel)
    s2 = src[2, :lens[2]]
    dense_rows = s2 >= 0
    assert np.array_equal(s2[dense_rows], src_sel[2, :lens[2]][dense_rows])
    assert np.array_equal(vmix[2][:, :lens[2]][:, dense_rows], v[:, s2[dense_rows]])
    assert np.array_equal(vmix[2][:, :lens[2]][:, ~dense_rows], vsp[:, -1 - s2[~dense_rows]])
