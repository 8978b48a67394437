"""GPU parity of the softmax attention-mass relevance score (vxl_chunk_score_topk_mass) against
the float64 oracle.  Scores are compared numerically; the selection is compared bit for bit with
a full sort of the device's own fp32 scores (both sides decide in fp32) and, wherever the rank-k
margin of the oracle's scores exceeds the score tolerance, with the oracle's selection."""
import numpy as np
import pytest

import oracle
from paper_2506_19225_amd import vxl, workloads as wl

from gpu_util import check_selection_valid, full_sort_selection, gpu_score_topk_mass

pytestmark = pytest.mark.gpu

RTOL = 1e-4       # fp32 exponentials and sums of up to ~10^5 terms against float64


def check_mass(w, lay, qd, k, top_k, scale=0.0, rtol=RTOL):
    idx, mask, scores = gpu_score_topk_mass(w, lay, qd, k, top_k, scale=scale)
    want = oracle.chunk_scores_mass(qd, k, lay.n_prefix, lay.chunk_bounds, scale=scale or None)
    tol = rtol * np.abs(want).max()
    assert np.isfinite(scores).all()
    assert np.abs(scores - want).max() <= tol, (np.abs(scores - want).max(), tol)
    assert (scores.sum(axis=1) <= 1.0 + 1e-4).all()          # the prefix holds the rest of the mass
    # the device's selection is the full-sort selection of its own scores, bit for bit
    own_idx, own_mask = full_sort_selection(scores, top_k)
    assert np.array_equal(idx, own_idx) and np.array_equal(mask, own_mask)
    # and a valid selection for the oracle's scores: nothing clearly better is left out
    check_selection_valid(idx, mask, want, oracle.select_topk(want, top_k)[1], top_k, tol)
    return idx, mask, scores


def test_mass_config0_fp32():
    w = wl.WORKLOADS["config0"]
    lay = wl.make_layout(w)
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    for top_k in (0, 1, w.k, lay.n_chunks + 3):
        check_mass(w, lay, qd, k, top_k, rtol=2e-5)


@pytest.mark.parametrize("dtype,d", [("f32", 64), ("f32", 128), ("bf16", 64), ("bf16", 128)])
def test_mass_ragged_layouts(dtype, d):
    rng = np.random.default_rng(71 + d)
    # odd chunk lengths, a short prefix, 9 stacked rows per KV head (not a multiple of 32)
    w = wl.tiny_workload(dtype, 6, 2, d, T=3, B=3, k=2, seed=71)
    lay = wl.random_layout(rng, 5, 13, 1, 300)
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    for top_k in (1, 4, 13):
        check_mass(w, lay, qd, k, top_k)
    # no prefix, one chunk longer than a piece (several items per chunk), 224 stacked rows (two
    # row tiles), a custom scale
    w = wl.tiny_workload(dtype, 14, 2, d, T=32, B=2, k=2, seed=72, value_scale=0.5)
    lay = wl.layout_from_lists(0, [2500, 77, 1024, 1025, 64], [np.zeros(0, np.int32)] * 5)
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    check_mass(w, lay, qd, k, 2, scale=0.2)


def test_mass_exact_ties_go_to_the_lower_chunk():
    w = wl.tiny_workload("bf16", 4, 2, 128, T=2, B=1, k=2, seed=73, value_scale=0.3)
    ln = 70
    lay = wl.layout_from_lists(3, [ln] * 5, [np.zeros(0, np.int32)] * 5)
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = np.abs(wl.make_decode_queries(w))
    blk = np.abs(k[:, 3 + ln:3 + 2 * ln]).copy()
    for c in (1, 3, 4):
        k[:, 3 + c * ln:3 + (c + 1) * ln] = blk
    for c in (0, 2):
        k[:, 3 + c * ln:3 + (c + 1) * ln] = -np.abs(k[:, 3 + c * ln:3 + (c + 1) * ln])
    idx, mask, scores = gpu_score_topk_mass(w, lay, qd, k, 2)
    assert scores[0, 1] == scores[0, 3] == scores[0, 4]
    assert list(idx[0]) == [1, 3] and list(mask[0]) == [0, 1, 0, 1, 0]


def test_mass_config1_and_sharp_queries():
    w = wl.WORKLOADS["config1"]
    lay = wl.make_layout(w)
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    check_mass(w, lay, qd, k, w.k)
    # sharp softmax: queries scaled so that the logits have a standard deviation of about 3
    qs = wl.round_to_bf16(qd * np.float32(np.sqrt(128.0) * 3.0 * np.sqrt(128.0)))
    check_mass(w, lay, qs, k, w.k)


def test_mass_matrix_core_kernel_agrees_with_vector_kernel_on_device():
    rng = np.random.default_rng(74)
    w = wl.tiny_workload("bf16", 14, 2, 128, T=5, B=2, k=3, seed=74)
    lay = wl.random_layout(rng, 40, 9, 30, 700)
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    _, mask_a, sc_a = gpu_score_topk_mass(w, lay, qd, k, 3)
    vxl.debug_force_simple(True)
    try:
        _, mask_b, sc_b = gpu_score_topk_mass(w, lay, qd, k, 3)
    finally:
        vxl.debug_force_simple(False)
    assert np.abs(sc_a - sc_b).max() <= 2e-5 * np.abs(sc_b).max()
    assert np.array_equal(mask_a, mask_b)


@pytest.mark.parametrize("name", ["config2", "config4"])
def test_mass_full_size(name):
    """Full-size layouts (131,328 tokens with T = 64; variable chunks with 8 queries)."""
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    _, k, _ = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    check_mass(w, lay, qd, k, w.k)
