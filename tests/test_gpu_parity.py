"""GPU parity: every C-ABI call against the float64 oracle on the same seeded inputs.
Integer outputs and gathered KV are compared bit for bit; attention outputs within the stated
tolerances (gpu_util)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_19225_amd import vxl, workloads as wl

from gpu_util import (assert_close, desc_of, gpu_decode, gpu_gather, gpu_prefill, gpu_score_topk,
                      make_layout)

pytestmark = pytest.mark.gpu


def lay_args(lay):
    return lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx


def oracle_prefill(q, k, v, lay, **kw):
    return oracle.prefill_blk(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx, **kw)


# --------------------------------------------------------------------------------- prefill
def test_prefill_config0_fp32():
    w = wl.WORKLOADS["config0"]
    lay = wl.make_layout(w)
    q, k, v = wl.make_qkv(w, lay)
    got, lse = gpu_prefill(w, lay, q, k, v, want_lse=True)
    want, wlse = oracle_prefill(q, k, v, lay, return_lse=True)
    assert_close(got, want, "f32", what="config0 prefill")
    assert np.abs(lse - wlse).max() < 1e-4


TINY_CASES = [
    # (dtype, Hq, Hkv, D, P, n_chunks, len_lo, len_hi, seed)
    ("f32", 2, 1, 64, 0, 3, 1, 40, 100),
    ("f32", 4, 2, 128, 5, 4, 3, 70, 101),
    ("bf16", 4, 2, 128, 0, 3, 1, 50, 102),
    ("bf16", 6, 2, 64, 7, 5, 2, 90, 103),
    ("bf16", 7, 1, 128, 70, 4, 60, 200, 104),
    ("bf16", 2, 2, 128, 129, 3, 127, 300, 105),
    # several 256-row bands per chunk, the last ragged, 7 and 12 query heads per KV head
    ("bf16", 14, 2, 128, 33, 3, 257, 600, 106),
    ("bf16", 12, 1, 64, 10, 2, 100, 400, 107),
]


@pytest.mark.parametrize("case", TINY_CASES, ids=lambda c: f"{c[0]}-h{c[1]}-d{c[3]}-p{c[4]}-s{c[8]}")
@pytest.mark.parametrize("qb", [0, 1])
def test_prefill_ragged_layouts(case, qb):
    dtype, hq, hkv, d, p, nc, lo, hi, seed = case
    if dtype == "f32" and qb != 0:
        pytest.skip("kernel instances only exist for the matrix-core path")
    rng = np.random.default_rng(seed)
    lay = wl.random_layout(rng, p, nc, lo, hi)
    w = wl.tiny_workload(dtype, hq, hkv, d, T=2, B=1, k=1, seed=seed)
    q, k, v = wl.make_qkv(w, lay)
    vxl.debug_prefill_variant(qb)
    try:
        got, lse = gpu_prefill(w, lay, q, k, v, want_lse=True)
    finally:
        vxl.debug_prefill_variant(0)
    want, wlse = oracle_prefill(q, k, v, lay, return_lse=True)
    assert_close(got, want, dtype, what=f"ragged prefill {case}")
    assert np.abs(lse - wlse).max() < (1e-4 if dtype == "f32" else 2e-2)


def test_prefill_edge_layouts_bf16():
    """No prefix and no kept tokens (block diagonal); everything kept (dense causal); one chunk;
    prefix only."""
    w = wl.tiny_workload("bf16", 4, 2, 128, T=1, B=1, k=1, seed=7, value_scale=0.5)
    lens = [65, 130, 64]
    empty = [np.zeros(0, np.int32)] * 3
    full, s = [], 3
    for ln in lens:
        full.append(np.arange(s, s + ln))
        s += ln
    for lay in (wl.layout_from_lists(0, lens, empty),
                wl.layout_from_lists(3, lens, full),
                wl.layout_from_lists(0, [200], [np.zeros(0, np.int32)]),
                wl.layout_from_lists(150, [], [])):
        q, k, v = wl.make_qkv(w, lay)
        got = gpu_prefill(w, lay, q, k, v)
        assert_close(got, oracle_prefill(q, k, v, lay), "bf16", what="edge layout")


@pytest.mark.parametrize("qb", [0, 1])
def test_prefill_medium_bf16_sharp_softmax(qb):
    """Several 256-token chunks at GQA 14/2, with logits of std ~3 so that the running maximum
    moves and the rescaling path is exercised."""
    w = wl.tiny_workload("bf16", 14, 2, 128, T=4, B=1, k=2, seed=21, value_scale=1.0)
    lens = [256, 256, 320, 192, 256]
    kept, s = [], 256
    for ln in lens:
        kept.append(wl.strided_kept(s, ln, ln // 8))
        s += ln
    lay = wl.layout_from_lists(256, lens, kept)
    q, k, v = wl.make_qkv(w, lay)
    q = wl.round_to_bf16(q * np.float32(3.0))        # q.k/sqrt(128) then has std 3
    vxl.debug_prefill_variant(qb)
    try:
        got, lse = gpu_prefill(w, lay, q, k, v, want_lse=True)
    finally:
        vxl.debug_prefill_variant(0)
    want, wlse = oracle_prefill(q, k, v, lay, return_lse=True)
    assert_close(got, want, "bf16", what="medium sharp prefill")
    assert np.abs(lse - wlse).max() < 2e-2


def test_prefill_matrix_core_kernel_agrees_with_vector_kernel_on_device():
    w = wl.tiny_workload("bf16", 8, 2, 128, T=1, B=1, k=1, seed=31, value_scale=0.3)
    rng = np.random.default_rng(31)
    lay = wl.random_layout(rng, 33, 6, 30, 260)
    q, k, v = wl.make_qkv(w, lay)
    a = gpu_prefill(w, lay, q, k, v)
    vxl.debug_force_simple(True)
    try:
        b = gpu_prefill(w, lay, q, k, v)
    finally:
        vxl.debug_force_simple(False)
    want = oracle_prefill(q, k, v, lay)
    assert_close(a, want, "bf16", what="mfma")
    assert_close(b, want, "bf16", what="simple")


_CONFIG1_ORACLE = {}


def config1_oracle(window=0):
    """config1 in full -- every row of every head -- from the oracle, computed once per window."""
    if window not in _CONFIG1_ORACLE:
        w = wl.WORKLOADS["config1"]
        lay = wl.make_layout(w)
        q, k, v = wl.make_qkv(w, lay)
        _CONFIG1_ORACLE[window] = (w, lay, q, k, v, oracle_prefill(q, k, v, lay, window=window))
    return _CONFIG1_ORACLE[window]


@pytest.mark.parametrize("qb", [0, 1])
def test_prefill_config1_all_rows(qb):
    w, lay, q, k, v, want = config1_oracle()
    vxl.debug_prefill_variant(qb)
    try:
        got = gpu_prefill(w, lay, q, k, v)
    finally:
        vxl.debug_prefill_variant(0)
    assert_close(got, want, "bf16", what="config1 prefill, all rows")


def test_prefill_locality_and_determinism_bit_exact():
    """Changing K/V of a token that is not kept changes only later rows of its own chunk, bit
    for bit; two runs on the same inputs are bit-identical."""
    w = wl.tiny_workload("bf16", 4, 2, 128, T=1, B=1, k=1, seed=41, value_scale=0.3)
    lens = [100, 140, 90]
    kept = [np.array([40, 41, 99]), np.array([140, 200]), np.array([281])]
    lay = wl.layout_from_lists(40, lens, kept)
    q, k, v = wl.make_qkv(w, lay)
    base = gpu_prefill(w, lay, q, k, v)
    again = gpu_prefill(w, lay, q, k, v)
    assert np.array_equal(base, again)
    j = 170                                            # chunk 1 = [140, 280), not kept
    k2, v2 = k.copy(), v.copy()
    k2[:, j] = wl.round_to_bf16(k2[:, j] + 1.0)
    v2[:, j] = wl.round_to_bf16(v2[:, j] - 2.0)
    pert = gpu_prefill(w, lay, q, k2, v2)
    changed = (pert != base).any(axis=(0, 2))
    assert changed[170:280].any()
    assert not changed[:170].any() and not changed[280:].any()


# --------------------------------------------------------------------------------- sliding chunk window
WINDOW_CASES = [
    # (dtype, Hq, Hkv, D, P, n_chunks, len_lo, len_hi, window, seed)
    ("f32", 2, 1, 64, 3, 4, 5, 60, 7, 110),
    ("bf16", 4, 2, 128, 0, 4, 20, 90, 33, 111),
    ("bf16", 6, 2, 64, 9, 5, 30, 150, 64, 112),
    ("bf16", 4, 1, 128, 70, 4, 100, 300, 130, 113),        # look-back longer than two key tiles
    ("bf16", 2, 2, 128, 5, 6, 40, 200, 100000, 114),       # window covers everything: dense causal
]


@pytest.mark.parametrize("case", WINDOW_CASES, ids=lambda c: f"{c[0]}-d{c[3]}-p{c[4]}-w{c[8]}")
@pytest.mark.parametrize("qb", [0, 1])
def test_prefill_sliding_window(case, qb):
    dtype, hq, hkv, d, p, nc, lo, hi, window, seed = case
    if dtype == "f32" and qb != 0:
        pytest.skip("kernel variants only exist for the matrix-core path")
    rng = np.random.default_rng(seed)
    lay = wl.random_layout(rng, p, nc, lo, hi)
    w = wl.tiny_workload(dtype, hq, hkv, d, T=1, B=1, k=1, seed=seed)
    q, k, v = wl.make_qkv(w, lay)
    gl = make_layout(lay, window=window)
    assert gl.pair_count() == oracle.allowed_pair_count(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets,
                                                        lay.sparse_idx, window=window)
    vxl.debug_prefill_variant(qb)
    try:
        got, lse = gpu_prefill(w, lay, q, k, v, want_lse=True, gl=gl)
    finally:
        vxl.debug_prefill_variant(0)
    want, wlse = oracle_prefill(q, k, v, lay, return_lse=True, window=window)
    assert_close(got, want, dtype, what=f"windowed prefill {case}")
    assert np.abs(lse - wlse).max() < (1e-4 if dtype == "f32" else 2e-2)
    if dtype == "bf16" and qb == 0:                       # the vector kernel walks the same sets on its own
        vxl.debug_force_simple(True)
        try:
            alt = gpu_prefill(w, lay, q, k, v, gl=gl)
        finally:
            vxl.debug_force_simple(False)
        assert_close(alt, want, dtype, what=f"windowed prefill, vector kernel {case}")


def test_prefill_window_config1_all_rows():
    """config1 with a look-back of one frame group (64 tokens): full size, every row."""
    w, lay, q, k, v, want = config1_oracle(window=64)
    got = gpu_prefill(w, lay, q, k, v, gl=make_layout(lay, window=64))
    assert_close(got, want, "bf16", what="config1 windowed prefill, all rows")


def test_prefill_two_workgroups_per_unit_instance_is_reproducible():
    """The instance of the streaming kernel that runs as two independent 4-wave workgroups per
    compute unit walks the same tiles in the same order as the default one, so on config1 with a
    look-back window it must give the default's bits, run after run."""
    w = wl.WORKLOADS["config1"]
    lay = wl.make_layout(w)
    q, k, v = wl.make_qkv(w, lay)
    gl = make_layout(lay, window=64)
    ref = gpu_prefill(w, lay, q, k, v, gl=gl)
    vxl.debug_prefill_variant(1)
    try:
        runs = [gpu_prefill(w, lay, q, k, v, gl=gl) for _ in range(3)]
    finally:
        vxl.debug_prefill_variant(0)
    for r in runs:
        assert np.array_equal(r, ref)


# --------------------------------------------------------------------------------- score / top-k
def check_topk_order(idx, want_idx, scores, want_s, tol=None):
    """topk_idx lists the selected chunks best first.  Position i must hold the oracle's chunk
    wherever that chunk's float64 score is separated from both neighbours in the oracle's order
    by more than twice the score tolerance (closer than that, fp32 scores may order them either
    way); and the device's order is always the (score descending, id ascending) order of the
    device's own scores."""
    tol = (2e-5 * np.abs(want_s).max() + 1e-7) if tol is None else tol
    for b in range(idx.shape[0]):
        key = [(-scores[b, c], c) for c in idx[b]]
        assert key == sorted(key)
        sw = want_s[b, want_idx[b]]
        for i in range(idx.shape[1]):
            left_ok = i == 0 or sw[i - 1] - sw[i] > 2 * tol
            right_ok = i + 1 == idx.shape[1] or sw[i] - sw[i + 1] > 2 * tol
            if left_ok and right_ok:
                assert idx[b, i] == want_idx[b, i], (b, i, idx[b], want_idx[b])


def check_topk(w, lay, qd, k, top_k):
    idx, mask, scores = gpu_score_topk(w, lay, qd, k, top_k)
    want_s = oracle.chunk_scores(qd, k, lay.chunk_bounds)
    assert np.abs(scores - want_s).max() <= 2e-5 * np.abs(want_s).max() + 1e-7
    want_idx, want_mask = oracle.select_topk(want_s, top_k)
    kk = min(top_k, lay.n_chunks)
    # the decision is only defined when the rank-k margin exceeds the fp32 score error
    srt = np.sort(want_s, axis=1)[:, ::-1]
    if 0 < kk < lay.n_chunks:
        margin = (srt[:, kk - 1] - srt[:, kk]).min()
        assert margin > 1e-6 * np.abs(want_s).max(), "degenerate seed: rank-k margin too small"
    assert np.array_equal(mask, want_mask)
    assert np.array_equal(np.sort(idx, axis=1), np.sort(want_idx, axis=1))
    check_topk_order(idx, want_idx, scores, want_s)
    return idx, mask


def test_score_topk_config0_and_config1():
    for name in ("config0", "config1"):
        w = wl.WORKLOADS[name]
        lay = wl.make_layout(w)
        _, k, _ = wl.make_qkv(w, lay, with_q=False)
        qd = wl.make_decode_queries(w)
        for top_k in (0, 1, w.k, lay.n_chunks, lay.n_chunks + 5):
            check_topk(w, lay, qd, k, top_k)


def test_score_topk_ragged_and_ties():
    rng = np.random.default_rng(51)
    for dtype, d in (("f32", 64), ("bf16", 128)):
        w = wl.tiny_workload(dtype, 6, 2, d, T=3, B=3, k=2, seed=51)
        lay = wl.random_layout(rng, 5, 13, 1, 300)
        _, k, _ = wl.make_qkv(w, lay, with_q=False)
        qd = wl.make_decode_queries(w)
        for top_k in (1, 4, 13):
            check_topk(w, lay, qd, k, top_k)
    # exact ties: chunks 1, 3, 4 hold identical keys -> identical scores -> lower ids win
    w = wl.tiny_workload("bf16", 4, 2, 128, T=2, B=1, k=2, seed=52)
    ln = 70
    lay = wl.layout_from_lists(3, [ln] * 5, [np.zeros(0, np.int32)] * 5)
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = np.abs(wl.make_decode_queries(w))
    blk = np.abs(k[:, 3 + ln:3 + 2 * ln]).copy()
    for c in (1, 3, 4):
        k[:, 3 + c * ln:3 + (c + 1) * ln] = blk
    for c in (0, 2):
        k[:, 3 + c * ln:3 + (c + 1) * ln] = -np.abs(k[:, 3 + c * ln:3 + (c + 1) * ln])
    idx, mask, scores = gpu_score_topk(w, lay, qd, k, 2)
    assert scores[0, 1] == scores[0, 3] == scores[0, 4]
    assert list(idx[0]) == [1, 3] and list(mask[0]) == [0, 1, 0, 1, 0]


# --------------------------------------------------------------------------------- gather
def check_gather(w, lay, k, v, masks, l_cap):
    kmix, vmix, mix_len, src = gpu_gather(w, lay, k, v, masks, l_cap)
    wk, wv, wlen, wsrc = oracle.gather_bilevel(k, v, masks, *lay_args(lay), l_cap=l_cap)
    assert np.array_equal(mix_len.cpu().numpy(), wlen)
    hk, hv, hsrc = vxl.to_host(kmix), vxl.to_host(vmix), src.cpu().numpy()
    for b in range(masks.shape[0]):
        n = wlen[b]
        assert np.array_equal(hsrc[b, :n], wsrc[b, :n])
        assert np.array_equal(hk[b, :, :n], wk[b, :, :n])          # bit-exact (exact upcast)
        assert np.array_equal(hv[b, :, :n], wv[b, :, :n])
        assert (hk[b, :, n:] == 7.0).all() and (hsrc[b, n:] == -5).all()   # rows beyond untouched
    return kmix, vmix, mix_len


def test_gather_bit_exact():
    rng = np.random.default_rng(61)
    for name in ("config0", "config1"):
        w = wl.WORKLOADS[name]
        lay = wl.make_layout(w)
        _, k, v = wl.make_qkv(w, lay, with_q=False)
        masks = np.zeros((3, lay.n_chunks), np.uint8)
        masks[1] = 1
        masks[2, rng.choice(lay.n_chunks, size=w.k, replace=False)] = 1
        check_gather(w, lay, k, v, masks, lay.n_tokens)
    w = wl.tiny_workload("bf16", 4, 2, 64, T=1, B=4, k=2, seed=62)
    lay = wl.random_layout(rng, 9, 300, 1, 20)                       # more chunks than one scan pass
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    masks = rng.integers(0, 2, size=(4, lay.n_chunks)).astype(np.uint8)
    check_gather(w, lay, k, v, masks, lay.n_tokens + 11)


def test_gather_overflow_is_reported_not_truncated():
    """A mask that selects more rows than the mixed buffers hold: mix_len = -(rows needed), no row
    of that query is written (Kmix, Vmix, src_idx keep their sentinels); the other queries of the
    call are gathered as usual; decode reads the negative length as an empty set."""
    rng = np.random.default_rng(63)
    w = wl.tiny_workload("bf16", 4, 2, 128, T=2, B=3, k=1, seed=63)
    lay = wl.random_layout(rng, 6, 9, 20, 60)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    gl = make_layout(lay)
    l_cap = gl.mixed_kv_capacity(1)                       # room for one dense chunk
    masks = np.zeros((3, lay.n_chunks), np.uint8)
    masks[0, int(np.argmax(np.diff(lay.chunk_bounds)))] = 1        # fits exactly or with room
    masks[1, :] = 1                                        # every chunk dense: does not fit
    kmix, vmix, mix_len, src = gpu_gather(w, lay, k, v, masks, l_cap, gl=gl)
    _, _, wlen, wsrc = oracle.gather_bilevel(k, v, masks[[0, 2]], *lay_args(lay))
    lens = mix_len.cpu().numpy()
    assert lay.n_tokens > l_cap
    assert list(lens) == [wlen[0], -lay.n_tokens, wlen[1]]
    hk, hv, hsrc = vxl.to_host(kmix), vxl.to_host(vmix), src.cpu().numpy()
    assert (hk[1] == 7.0).all() and (hv[1] == 7.0).all() and (hsrc[1] == -5).all()
    for b, ob in ((0, 0), (2, 1)):
        n = wlen[ob]
        assert np.array_equal(hsrc[b, :n], wsrc[ob, :n]) and (hsrc[b, n:] == -5).all()
        assert np.array_equal(hk[b, :, :n], k[:, wsrc[ob, :n]])
    qd = wl.make_decode_queries(w)
    got, lse = gpu_decode(w, qd, kmix, vmix, mix_len, want_lse=True)
    assert (got[1] == 0).all() and np.isneginf(lse[1]).all()
    wk, wv, _, _ = oracle.gather_bilevel(k, v, masks[[0, 2]], *lay_args(lay), l_cap=l_cap)
    want = oracle.decode_mixed(qd[[0, 2]], wk, wv, wlen)
    assert_close(got[[0, 2]], want, "bf16", head_axis=2, what="decode beside an overflowed query")


# --------------------------------------------------------------------------------- decode
@pytest.mark.parametrize("dtype,t_q", [("f32", 2), ("bf16", 1), ("bf16", 8), ("bf16", 40)])
def test_decode_empty_mixed_set(dtype, t_q):
    """mix_len = 0 (no prefix, nothing kept, nothing dense) beside a non-empty query: the empty
    one gives O = 0 and LSE = -inf on every decode kernel, the other is unaffected."""
    rng = np.random.default_rng(70 + t_q)
    d, hq, hkv, l_cap = 128, 14, 2, 300
    w = wl.tiny_workload(dtype, hq, hkv, d, T=t_q, B=2, k=1, seed=70 + t_q)
    rnd = lambda *shape: (rng.standard_normal(shape).astype(np.float32) * np.float32(0.5))
    kmix, vmix, qd = rnd(2, hkv, l_cap, d), rnd(2, hkv, l_cap, d), rnd(2, t_q, hq, d)
    if dtype == "bf16":
        kmix, vmix, qd = (wl.round_to_bf16(x) for x in (kmix, vmix, qd))
    mix_len = np.array([0, 217], dtype=np.int32)
    got, lse = gpu_decode(w, qd, vxl.to_device(kmix, dtype), vxl.to_device(vmix, dtype),
                          torch.from_numpy(mix_len).cuda(), want_lse=True)
    assert (got[0] == 0).all() and np.isneginf(lse[0]).all()
    want, wlse = oracle.decode_lse(qd[1:], kmix[1:], vmix[1:], mix_len[1:])
    assert_close(got[1:], want, dtype, head_axis=2, what=f"decode beside an empty set T={t_q}")
    assert np.abs(lse[1:] - wlse).max() < (1e-4 if dtype == "f32" else 2e-2)


def test_decode_config0_fp32_and_tiny_bf16():
    rng = np.random.default_rng(71)
    w = wl.WORKLOADS["config0"]
    lay = wl.make_layout(w)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    _, mask = oracle.select_topk(oracle.chunk_scores(qd, k, lay.chunk_bounds), w.k)
    kmix, vmix, mix_len = check_gather(w, lay, k, v, mask, 400)
    got, lse = gpu_decode(w, qd, kmix, vmix, mix_len, want_lse=True)
    wk, wv, wlen, _ = oracle.gather_bilevel(k, v, mask, *lay_args(lay), l_cap=400)
    want, wlse = oracle.decode_lse(qd, wk, wv, wlen)
    assert_close(got, want, "f32", head_axis=2, what="config0 decode")
    assert np.abs(lse - wlse).max() < 1e-4
    # stacked rows 7 (wave kernel), 35 (split kernel), 280 and 210 (ring kernel, both head dims)
    for t_q, bsz, d in ((1, 2, 128), (5, 3, 64), (40, 1, 128), (30, 2, 64)):
        w = wl.tiny_workload("bf16", 14, 2, d, T=t_q, B=bsz, k=2, seed=72 + t_q)
        lay = wl.random_layout(rng, 17, 9, 5, 120)
        _, k, v = wl.make_qkv(w, lay, with_q=False)
        qd = wl.make_decode_queries(w)
        masks = rng.integers(0, 2, size=(bsz, lay.n_chunks)).astype(np.uint8)
        kmix, vmix, mix_len = check_gather(w, lay, k, v, masks, lay.n_tokens)
        got, lse = gpu_decode(w, qd, kmix, vmix, mix_len, want_lse=True)
        wk, wv, wlen, _ = oracle.gather_bilevel(k, v, masks, *lay_args(lay), l_cap=lay.n_tokens)
        want, wlse = oracle.decode_lse(qd, wk, wv, wlen)
        assert_close(got, want, "bf16", head_axis=2, what=f"tiny decode T={t_q}")
        assert np.abs(lse - wlse).max() < 2e-2


def run_bilevel_chain(w, lay, k, v, qd, top_k):
    """score -> gather -> decode entirely on the device, no host round trip in between."""
    gl = make_layout(lay)
    desc = desc_of(w)
    dk, dv, dqd = (vxl.to_device(x, w.dtype) for x in (k, v, qd))
    bsz, t = qd.shape[0], qd.shape[1]
    kk = min(top_k, lay.n_chunks)
    idx = torch.zeros((bsz, max(kk, 1)), dtype=torch.int32, device="cuda")
    mask = torch.zeros((bsz, lay.n_chunks), dtype=torch.uint8, device="cuda")
    l_cap = gl.mixed_kv_capacity(top_k)
    kmix = torch.zeros((bsz, w.n_kv_heads, l_cap, w.head_dim), dtype=dk.dtype, device="cuda")
    vmix = torch.zeros_like(kmix)
    mix_len = torch.zeros((bsz,), dtype=torch.int32, device="cuda")
    out = torch.zeros_like(dqd)
    ws1 = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_TOPK, gl, desc, bsz, t))
    ws3 = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, bsz, t, l_cap))
    vxl.chunk_score_topk(gl, desc, dqd, dk, top_k, idx, mask, workspace=ws1)
    vxl.gather_bilevel_kv(gl, desc, dk, dv, mask, kmix, vmix, mix_len)
    vxl.bilevel_decode(desc, dqd, kmix, vmix, mix_len, out, None, ws3)
    torch.cuda.synchronize()
    return vxl.to_host(out), mask.cpu().numpy(), mix_len.cpu().numpy(), l_cap


@pytest.mark.parametrize("name", ["config0", "config1"])
def test_bilevel_chain(name):
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    got, mask, mix_len, l_cap = run_bilevel_chain(w, lay, k, v, qd, w.k)
    s = oracle.chunk_scores(qd, k, lay.chunk_bounds)
    _, wmask = oracle.select_topk(s, w.k)
    assert np.array_equal(mask, wmask)
    wk, wv, wlen, _ = oracle.gather_bilevel(k, v, wmask, *lay_args(lay), l_cap=l_cap)
    assert np.array_equal(mix_len, wlen)
    assert wlen[0] == {"config0": 352, "config1": 4096}[name]
    want = oracle.decode_mixed(qd, wk, wv, wlen)
    assert_close(got, want, w.dtype, head_axis=2, what=f"{name} chain decode")


def test_all_dense_decode_equals_prefill_free_full_attention():
    """Sparse set = whole chunk and k = C: the mixed KV is the full KV cache."""
    w = wl.tiny_workload("bf16", 14, 2, 128, T=3, B=2, k=4, seed=81, value_scale=0.4)
    lens = [70, 64, 130, 33]
    kept, s = [], 10
    for ln in lens:
        kept.append(np.arange(s, s + ln))
        s += ln
    lay = wl.layout_from_lists(10, lens, kept)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    got, mask, mix_len, l_cap = run_bilevel_chain(w, lay, k, v, qd, 4)
    assert mask.all() and (mix_len == lay.n_tokens).all() and l_cap == lay.n_tokens
    full_k = np.broadcast_to(k[None], (2,) + k.shape)
    full_v = np.broadcast_to(v[None], (2,) + v.shape)
    want = oracle.decode_mixed(qd, full_k, full_v, [lay.n_tokens] * 2)
    assert_close(got, want, "bf16", head_axis=2, what="all-dense decode")


# --------------------------------------------------------------------------------- streams and graphs
def _whole_path(w, lay, gl, desc, dq, dk, dv, dqd, bufs):
    out, idx, mask, kmix, vmix, mix_len, od, ws = bufs
    vxl.chunk_prefill(gl, desc, dq, dk, dv, out, None, ws[0])
    vxl.chunk_score_topk(gl, desc, dqd, dk, w.k, idx, mask, workspace=ws[1])
    vxl.gather_bilevel_kv(gl, desc, dk, dv, mask, kmix, vmix, mix_len)
    vxl.bilevel_decode(desc, dqd, kmix, vmix, mix_len, od, None, ws[2])


def test_whole_path_on_a_side_stream_and_in_a_replayed_graph():
    """The four calls never allocate or synchronise, so they run on any stream and can be captured
    into a HIP graph.  Every replay (with eager work and synchronisations in between, and with
    the persistent kernel's work queue reset inside the graph) must reproduce the eager result
    bit for bit."""
    w = wl.tiny_workload("bf16", 14, 2, 128, T=8, B=2, k=2, seed=95, value_scale=0.4)
    rng = np.random.default_rng(95)
    lay = wl.random_layout(rng, 40, 7, 60, 400)
    q, k, v = wl.make_qkv(w, lay)
    qd = wl.make_decode_queries(w)
    gl = make_layout(lay)
    desc = desc_of(w)
    dq, dk, dv, dqd = (vxl.to_device(x, w.dtype) for x in (q, k, v, qd))
    l_cap = gl.mixed_kv_capacity(w.k)

    def buffers():
        return (torch.full_like(dq, float("nan")),
                torch.zeros((w.B, w.k), dtype=torch.int32, device="cuda"),
                torch.zeros((w.B, lay.n_chunks), dtype=torch.uint8, device="cuda"),
                torch.zeros((w.B, w.n_kv_heads, l_cap, w.head_dim), dtype=dk.dtype, device="cuda"),
                torch.zeros((w.B, w.n_kv_heads, l_cap, w.head_dim), dtype=dk.dtype, device="cuda"),
                torch.zeros((w.B,), dtype=torch.int32, device="cuda"),
                torch.full_like(dqd, float("nan")),
                [vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc)),
                 vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_TOPK, gl, desc, w.B, w.T)),
                 vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, w.B, w.T, l_cap))])

    eager = buffers()
    _whole_path(w, lay, gl, desc, dq, dk, dv, dqd, eager)
    torch.cuda.synchronize()
    want = oracle_prefill(q, k, v, lay)
    assert_close(vxl.to_host(eager[0]), want, "bf16", what="eager prefill")

    side = torch.cuda.Stream()
    on_side = buffers()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _whole_path(w, lay, gl, desc, dq, dk, dv, dqd, on_side)
    side.synchronize()
    for a, b in zip(eager[:7], on_side[:7]):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))

    captured = buffers()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _whole_path(w, lay, gl, desc, dq, dk, dv, dqd, captured)
    for rep in range(3):
        for t in (captured[0], captured[6]):
            t.fill_(float("nan"))                          # eager work between the replays
        captured[4].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(eager[:7], captured[:7]):
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), f"replay {rep} differs"


def test_whole_path_from_several_host_threads_sharing_one_layout():
    """The library keeps no per-call state outside the caller's buffers: four host threads, each with
    its own stream, workspaces and outputs but the SAME layout handle and inputs, run the whole path
    concurrently (ctypes releases the interpreter lock during a call) and must each reproduce the
    single-threaded result bit for bit, call after call."""
    import threading
    w = wl.tiny_workload("bf16", 14, 2, 128, T=8, B=2, k=2, seed=96, value_scale=0.4)
    rng = np.random.default_rng(96)
    lay = wl.random_layout(rng, 40, 7, 60, 400)
    q, k, v = wl.make_qkv(w, lay)
    qd = wl.make_decode_queries(w)
    gl = make_layout(lay)
    desc = desc_of(w)
    dq, dk, dv, dqd = (vxl.to_device(x, w.dtype) for x in (q, k, v, qd))
    l_cap = gl.mixed_kv_capacity(w.k)

    def buffers():
        return (torch.full_like(dq, float("nan")),
                torch.zeros((w.B, w.k), dtype=torch.int32, device="cuda"),
                torch.zeros((w.B, lay.n_chunks), dtype=torch.uint8, device="cuda"),
                torch.zeros((w.B, w.n_kv_heads, l_cap, w.head_dim), dtype=dk.dtype, device="cuda"),
                torch.zeros((w.B, w.n_kv_heads, l_cap, w.head_dim), dtype=dk.dtype, device="cuda"),
                torch.zeros((w.B,), dtype=torch.int32, device="cuda"),
                torch.full_like(dqd, float("nan")),
                [vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc)),
                 vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_TOPK, gl, desc, w.B, w.T)),
                 vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, w.B, w.T, l_cap))])

    eager = buffers()
    _whole_path(w, lay, gl, desc, dq, dk, dv, dqd, eager)
    torch.cuda.synchronize()
    n_threads, n_rounds = 4, 8
    per_thread = [buffers() for _ in range(n_threads)]
    streams = [torch.cuda.Stream() for _ in range(n_threads)]
    torch.cuda.synchronize()
    failures = []

    def worker(i):
        try:
            with torch.cuda.stream(streams[i]):
                for rnd in range(n_rounds):
                    per_thread[i][0].fill_(float("nan"))
                    per_thread[i][6].fill_(float("nan"))
                    _whole_path(w, lay, gl, desc, dq, dk, dv, dqd, per_thread[i])
                    streams[i].synchronize()
                    for a, b in zip(eager[:7], per_thread[i][:7]):
                        if not torch.equal(a.view(torch.uint8), b.view(torch.uint8)):
                            failures.append((i, rnd))
        except Exception as err:                                    # noqa: BLE001 -- reported below
            failures.append((i, repr(err)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not failures, failures


@pytest.mark.parametrize("d,lens", [(128, [40001, 711]), (64, [40001]), (64, [711])],
                         ids=["d128-long+short", "d64-long", "d64-short"])
def test_decode_step_mode_more_splits_than_the_merge_prefetches(d, lens):
    """One KV head and a long mixed-set capacity: 105 (two queries) or 157 (one query) key splits,
    more than the merge kernel requests up front (64 at D = 128, 128 at D = 64), so it goes on
    into its loop; a short set leaves most splits empty (weight 0, LSE -inf) and ends in a ragged
    tile."""
    rng = np.random.default_rng(500 + d + len(lens) + lens[0])
    hq, hkv, l_cap, bsz = 4, 1, 40037, len(lens)
    w = wl.tiny_workload("bf16", hq, hkv, d, T=1, B=bsz, k=1, seed=500 + d)
    kmix = wl.round_to_bf16(rng.standard_normal((bsz, hkv, l_cap, d)).astype(np.float32) * np.float32(0.5))
    vmix = wl.round_to_bf16(rng.standard_normal((bsz, hkv, l_cap, d)).astype(np.float32) * np.float32(0.5))
    qd = wl.round_to_bf16(rng.standard_normal((bsz, 1, hq, d)).astype(np.float32) * np.float32(0.5))
    mix_len = np.array(lens, dtype=np.int32)
    got, lse = gpu_decode(w, qd, vxl.to_device(kmix, "bf16"), vxl.to_device(vmix, "bf16"),
                          torch.from_numpy(mix_len).cuda(), want_lse=True)
    want, wlse = oracle.decode_lse(qd, kmix, vmix, mix_len)
    assert_close(got, want, "bf16", head_axis=2, what=f"long single-head step decode d={d}")
    assert np.abs(lse - wlse).max() < 2e-2


@pytest.mark.parametrize("t_q,d,lens", [(1, 128, [1000, 37, 4096]), (4, 64, [33, 2047]), (1, 64, [1, 64]),
                                        (10, 128, [500, 1]), (40, 128, [777]), (30, 64, [1500, 90])],
                         ids=lambda x: str(x))
def test_decode_never_uses_rows_past_the_mixed_length(t_q, d, lens):
    """Rows of the mixed buffers at and past mix_len[b] are NaN (what an uninitialised buffer may
    hold): no kernel form (step, 128-row, 256-row ring) may let them reach O or LSE, also where
    the length falls inside a tile, at a tile border and in a wave's first tile."""
    rng = np.random.default_rng(900 + t_q + d)
    hq, hkv, l_cap, bsz = 14, 2, 4096, len(lens)
    w = wl.tiny_workload("bf16", hq, hkv, d, T=t_q, B=bsz, k=1, seed=900 + d)
    kmix = wl.round_to_bf16(rng.standard_normal((bsz, hkv, l_cap, d)).astype(np.float32) * np.float32(0.5))
    vmix = wl.round_to_bf16(rng.standard_normal((bsz, hkv, l_cap, d)).astype(np.float32) * np.float32(0.5))
    qd = wl.round_to_bf16(rng.standard_normal((bsz, t_q, hq, d)).astype(np.float32) * np.float32(0.5))
    mix_len = np.array(lens, dtype=np.int32)
    dk, dv = vxl.to_device(kmix, "bf16"), vxl.to_device(vmix, "bf16")
    for b, n in enumerate(lens):
        dk[b, :, n:] = float("nan")
        dv[b, :, n:] = float("nan")
    got, lse = gpu_decode(w, qd, dk, dv, torch.from_numpy(mix_len).cuda(), want_lse=True)
    assert np.isfinite(got).all() and np.isfinite(lse).all()
    want, wlse = oracle.decode_lse(qd, kmix, vmix, mix_len)
    assert_close(got, want, "bf16", head_axis=2, what=f"decode with NaN rows past the length, T={t_q} d={d}")
    assert np.abs(lse - wlse).max() < 2e-2


@pytest.fixture
def step_waves(request):
    """Both forms of the step-mode kernel: 0 = the default (4 double-buffered waves), 8 = the
    single-buffered 8-wave form."""
    vxl.debug_decode_step_waves(request.param)
    yield request.param
    vxl.debug_decode_step_waves(0)


@pytest.mark.parametrize("step_waves", [0, 8], indirect=True)
@pytest.mark.parametrize("name,t_q", [("config1", 1), ("config1", 4), ("config2", 1)])
def test_decode_step_mode_many_splits(name, t_q, step_waves):
    """Step mode (at most 32 stacked rows) at the mixed-set sizes of config1 / config2: many key
    splits, a workspace that starts with arbitrary bytes, repeated calls on one workspace, and
    replays of a captured graph with eager calls in between."""
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)[:, :t_q].copy()
    _, mask = oracle.select_topk(oracle.chunk_scores(qd, k, lay.chunk_bounds), w.k)
    gl = make_layout(lay)
    l_cap = gl.mixed_kv_capacity(w.k)
    kmix, vmix, mix_len, _ = gpu_gather(w, lay, k, v, mask, l_cap, gl=gl)
    wk, wv, wlen, _ = oracle.gather_bilevel(k, v, mask, *lay_args(lay), l_cap=l_cap)
    want, wlse = oracle.decode_lse(qd, wk, wv, wlen)
    desc = desc_of(w)
    dqd = vxl.to_device(qd, w.dtype)
    nbytes = vxl.workspace_bytes(vxl.OP_DECODE, None, desc, qd.shape[0], t_q, l_cap)
    ws = torch.randint(0, 256, (nbytes,), dtype=torch.uint8, device="cuda")        # arbitrary initial bytes
    outs = []
    for _ in range(3):
        out = torch.full_like(dqd, float("nan"))
        lse = torch.full(dqd.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
        vxl.bilevel_decode(desc, dqd, kmix, vmix, mix_len, out, lse, ws)
        torch.cuda.synchronize()
        assert_close(vxl.to_host(out), want, w.dtype, head_axis=2, what=f"{name} step decode T={t_q}")
        assert np.abs(vxl.to_host(lse) - wlse).max() < 2e-2
        outs.append(out.clone())
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])          # deterministic
    # captured once, replayed three times with eager work in between
    side = torch.cuda.Stream()
    out = torch.zeros_like(dqd)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        vxl.bilevel_decode(desc, dqd, kmix, vmix, mix_len, out, None, ws, stream=side)      # warm-up on the stream
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            vxl.bilevel_decode(desc, dqd, kmix, vmix, mix_len, out, None, ws, stream=side)
    torch.cuda.synchronize()
    for _ in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, outs[0])
        vxl.bilevel_decode(desc, dqd, kmix, vmix, mix_len, out, None, ws)           # an eager call between replays
        torch.cuda.synchronize()
        assert torch.equal(out, outs[0])
