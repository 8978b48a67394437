"""Gather-free decode (vxl_bilevel_decode_inplace): the split-KV kernels read the dense rows of the
selected chunks from K / V and the sparse rows of the others in place, through a per-query row
map.  The oracle is the decode over the oracle's gathered mixed set (index selection or pooled
sparse KVs); the lengths are compared exactly, and the result also against gather + decode on the
device."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_19225_amd import vxl, workloads as wl

from gpu_util import (assert_close, desc_of, gpu_decode, gpu_decode_inplace as inplace, gpu_gather, kept_rows,
                      make_layout, storage_round)

pytestmark = pytest.mark.gpu


def lay_args(lay):
    return lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx


def check_case(w, lay, k, v, qd, masks, mode, l_cap=None, tol_lse=2e-2):
    gl = make_layout(lay)
    dk, dv = vxl.to_device(k, w.dtype), vxl.to_device(v, w.dtype)
    l_cap = lay.n_tokens if l_cap is None else l_cap
    if mode == "kept_in_place":
        sparse = None
        wk, wv, wlen, _ = oracle.gather_bilevel(k, v, masks, *lay_args(lay), l_cap=l_cap)
    elif mode == "kept_compacted":
        sparse = (vxl.to_device(kept_rows(k, lay), w.dtype), vxl.to_device(kept_rows(v, lay), w.dtype))
        wk, wv, wlen, _ = oracle.gather_bilevel(k, v, masks, *lay_args(lay), l_cap=l_cap)
    else:
        desc = desc_of(w)
        s_total = max(int(lay.sparse_offsets[-1]), 1)
        ksp = torch.empty((w.n_kv_heads, s_total, w.head_dim), dtype=dk.dtype, device="cuda")
        vsp = torch.empty_like(ksp)
        vxl.pool_sparse_kv(gl, desc, dk, dv, ksp, vsp)
        torch.cuda.synchronize()
        sparse = (ksp, vsp)
        # (the oracle pools for itself: its inputs never come from the device)
        ok, ov = oracle.pool_sparse_kv(k, v, lay.chunk_bounds, lay.sparse_offsets)
        wk, wv, wlen, _ = oracle.gather_bilevel_pooled(k, v, storage_round(w, ok), storage_round(w, ov), masks,
                                                       lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, l_cap=l_cap)
    got, lse, lens = inplace(w, lay, qd, dk, dv, masks, l_cap, sparse, gl=gl)
    assert np.array_equal(lens, wlen)
    want, wlse = oracle.decode_lse(qd, wk, wv, wlen)
    assert_close(got, want, w.dtype, head_axis=2, what=f"in-place decode ({mode}, T={qd.shape[1]})")
    assert np.abs(lse - wlse).max() < (1e-4 if w.dtype == "f32" else tol_lse)
    return got


MODES = ["kept_in_place", "kept_compacted", "pooled"]


@pytest.mark.parametrize("mode", MODES)
def test_inplace_config0_fp32(mode):
    w = wl.WORKLOADS["config0"]
    lay = wl.make_layout(w)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    _, mask = oracle.select_topk(oracle.chunk_scores(qd, k, lay.chunk_bounds), w.k)
    check_case(w, lay, k, v, qd, mask, mode, l_cap=400)


@pytest.mark.parametrize("mode", MODES)
@pytest.mark.parametrize("t_q,bsz,d", [(1, 2, 128), (4, 1, 64), (5, 3, 64), (18, 2, 128), (40, 1, 128), (30, 2, 64)],
                         ids=lambda x: str(x))
def test_inplace_ragged_bf16(mode, t_q, bsz, d):
    """Stacked rows 14 and 56 (step kernel: <= 32 rows... 14, 28), 70 and 252 (128-row kernel, one
    and two row tiles), 560 (five row tiles) and 420; ragged chunks, some without kept rows, random
    selections including none and all."""
    rng = np.random.default_rng(1000 + 7 * t_q + d)
    w = wl.tiny_workload("bf16", 14, 2, d, T=t_q, B=bsz, k=2, seed=1000 + t_q, value_scale=0.5)
    lay = wl.random_layout(rng, 17, 11, 1, 150)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    masks = rng.integers(0, 2, size=(bsz, lay.n_chunks)).astype(np.uint8)
    masks[0] = 0
    if bsz > 1:
        masks[1] = 1
    got = check_case(w, lay, k, v, qd, masks, mode)
    if mode == "kept_in_place":                      # and against gather + decode on the device
        kmix, vmix, mix_len, _ = gpu_gather(w, lay, k, v, masks, lay.n_tokens)
        ref = gpu_decode(w, qd, kmix, vmix, mix_len)
        assert_close(got, ref, "bf16", head_axis=2, what="in-place vs gathered decode")


def test_inplace_map_survives_a_change_of_query_token_count():
    """The question in one call (40 tokens, which builds the row map), then one token per call with
    map_ready on the same workspace: the map's place does not depend on n_q_tokens."""
    rng = np.random.default_rng(4040)
    w = wl.tiny_workload("bf16", 14, 2, 128, T=40, B=2, k=2, seed=4040, value_scale=0.5)
    lay = wl.random_layout(rng, 17, 11, 1, 150)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    masks = rng.integers(0, 2, size=(2, lay.n_chunks)).astype(np.uint8)
    gl, desc, l_cap = make_layout(lay), desc_of(w), lay.n_tokens
    dk, dv, dqd = (vxl.to_device(x, "bf16") for x in (k, v, qd))
    dm = torch.from_numpy(masks).cuda()
    ws = vxl.alloc_workspace(max(vxl.workspace_bytes(vxl.OP_DECODE_INPLACE, gl, desc, 2, t, l_cap) for t in (40, 1)))
    out = torch.full_like(dqd, float("nan"))
    vxl.bilevel_decode_inplace(gl, desc, dqd, dk, dv, None, None, dm, l_cap, out, None, None, ws)
    wk, wv, wlen, _ = oracle.gather_bilevel(k, v, masks, *lay_args(lay), l_cap=l_cap)
    want, _ = oracle.decode_lse(qd, wk, wv, wlen)
    torch.cuda.synchronize()
    assert_close(vxl.to_host(out), want, "bf16", head_axis=2, what="in-place decode, the question")
    for t in (0, 17, 39):                                           # single tokens, the map reused
        one = dqd[:, t:t + 1].contiguous()
        out1 = torch.full_like(one, float("nan"))
        vxl.bilevel_decode_inplace(gl, desc, one, dk, dv, None, None, dm, l_cap, out1, None, None, ws, map_ready=True)
        torch.cuda.synchronize()
        assert_close(vxl.to_host(out1), want[:, t:t + 1], "bf16", head_axis=2, what=f"in-place decode, token {t} on the reused map")


def test_inplace_decode_in_a_replayed_graph():
    """Both forms of the call (building the row map, and reusing it) captured into one HIP graph on a
    side stream; every replay, with eager calls and synchronisations in between, reproduces the
    eager result bit for bit."""
    rng = np.random.default_rng(4141)
    w = wl.tiny_workload("bf16", 14, 2, 128, T=3, B=2, k=2, seed=4141, value_scale=0.5)
    lay = wl.random_layout(rng, 33, 9, 20, 300)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    masks = rng.integers(0, 2, size=(2, lay.n_chunks)).astype(np.uint8)
    gl, desc, l_cap = make_layout(lay), desc_of(w), lay.n_tokens
    dk, dv, dqd = (vxl.to_device(x, "bf16") for x in (k, v, qd))
    dm = torch.from_numpy(masks).cuda()
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE_INPLACE, gl, desc, 2, 3, l_cap))
    eager = torch.full_like(dqd, float("nan"))
    vxl.bilevel_decode_inplace(gl, desc, dqd, dk, dv, None, None, dm, l_cap, eager, None, None, ws)
    torch.cuda.synchronize()
    out_a, out_b = torch.zeros_like(dqd), torch.zeros_like(dqd)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        vxl.bilevel_decode_inplace(gl, desc, dqd, dk, dv, None, None, dm, l_cap, out_a, None, None, ws)      # warm-up on the stream
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            vxl.bilevel_decode_inplace(gl, desc, dqd, dk, dv, None, None, dm, l_cap, out_a, None, None, ws)
            vxl.bilevel_decode_inplace(gl, desc, dqd, dk, dv, None, None, dm, l_cap, out_b, None, None, ws, map_ready=True)
    for rep in range(3):
        out_a.zero_()
        out_b.zero_()
        ws.zero_()                                                  # the map is rebuilt inside the graph
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out_a.view(torch.uint8), eager.view(torch.uint8)), f"replay {rep}: map-building call differs"
        assert torch.equal(out_b.view(torch.uint8), eager.view(torch.uint8)), f"replay {rep}: map-reusing call differs"
        vxl.bilevel_decode_inplace(gl, desc, dqd, dk, dv, None, None, dm, l_cap, out_a, None, None, ws)      # eager work in between
        torch.cuda.synchronize()
    wk, wv, wlen, _ = oracle.gather_bilevel(k, v, masks, *lay_args(lay), l_cap=l_cap)
    assert_close(vxl.to_host(eager), oracle.decode_mixed(qd, wk, wv, wlen), "bf16", head_axis=2, what="in-place decode (graph test)")


def test_inplace_overflow_and_empty():
    """A selection that does not fit the row map is reported (negative length, O = 0, LSE = -inf);
    a layout without prefix and kept rows with nothing selected is an empty set."""
    rng = np.random.default_rng(1100)
    w = wl.tiny_workload("bf16", 4, 2, 128, T=2, B=2, k=1, seed=1100)
    lay = wl.random_layout(rng, 6, 9, 20, 60)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    gl = make_layout(lay)
    l_cap = gl.mixed_kv_capacity(1)
    masks = np.zeros((2, lay.n_chunks), np.uint8)
    masks[1] = 1
    dk, dv = vxl.to_device(k, "bf16"), vxl.to_device(v, "bf16")
    got, lse, lens = inplace(w, lay, qd, dk, dv, masks, l_cap, gl=gl)
    assert lens[1] == -lay.n_tokens and (got[1] == 0).all() and np.isneginf(lse[1]).all()
    wk, wv, wlen, _ = oracle.gather_bilevel(k, v, masks[:1], *lay_args(lay), l_cap=l_cap)
    assert lens[0] == wlen[0]
    assert_close(got[:1], oracle.decode_mixed(qd[:1], wk, wv, wlen), "bf16", head_axis=2, what="beside an overflow")
    lay0 = wl.layout_from_lists(0, [40, 50], [np.zeros(0, np.int32)] * 2)
    _, k0, v0 = wl.make_qkv(w, lay0, with_q=False)
    got, lse, lens = inplace(w, lay0, qd, vxl.to_device(k0, "bf16"), vxl.to_device(v0, "bf16"),
                             np.array([[0, 0], [0, 1]], np.uint8), 64)
    assert lens[0] == 0 and (got[0] == 0).all() and np.isneginf(lse[0]).all() and lens[1] == 50


def test_inplace_token_major_storage():
    """K and V stored token-major [N, Hkv, D], as a projection writes them."""
    rng = np.random.default_rng(1200)
    w = wl.tiny_workload("bf16", 8, 2, 128, T=3, B=2, k=2, seed=1200, value_scale=0.5)
    lay = wl.random_layout(rng, 9, 8, 10, 90)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    masks = rng.integers(0, 2, size=(2, lay.n_chunks)).astype(np.uint8)
    gl = make_layout(lay)
    desc = vxl.make_desc(w.n_q_heads, w.n_kv_heads, w.head_dim, "bf16", token_major=True)
    dk = vxl.to_device(np.ascontiguousarray(k.transpose(1, 0, 2)), "bf16")
    dv = vxl.to_device(np.ascontiguousarray(v.transpose(1, 0, 2)), "bf16")
    for sparse in (None, (vxl.to_device(kept_rows(k, lay), "bf16"), vxl.to_device(kept_rows(v, lay), "bf16"))):
        got, lse, lens = inplace(w, lay, qd, dk, dv, masks, lay.n_tokens, sparse, gl=gl, desc=desc)
        wk, wv, wlen, _ = oracle.gather_bilevel(k, v, masks, *lay_args(lay), l_cap=lay.n_tokens)
        assert np.array_equal(lens, wlen)
        assert_close(got, oracle.decode_mixed(qd, wk, wv, wlen), "bf16", head_axis=2, what="token-major in-place decode")


@pytest.mark.parametrize("name,t_q,mode", [("config1", 1, "kept_in_place"), ("config1", 32, "kept_compacted"),
                                           ("config2", 1, "kept_compacted"), ("config2", 4, "kept_in_place"),
                                           ("config2", 64, "pooled"), ("config4", 1, "kept_compacted"),
                                           ("config4", 32, "kept_in_place")])
def test_inplace_full_size(name, t_q, mode):
    """The workloads at full size: step mode and batched, the oracle's own selection."""
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)[:, :t_q].copy()
    _, masks = oracle.select_topk(oracle.chunk_scores(wl.make_decode_queries(w), k, lay.chunk_bounds), w.k)
    gl = make_layout(lay)
    check_case(w, lay, k, v, qd, masks, mode, l_cap=gl.mixed_kv_capacity(w.k))


def test_inplace_maximum_chunk_count():
    rng = np.random.default_rng(1300)
    c_n = vxl.MAX_CHUNKS
    lens = rng.integers(1, 4, size=c_n)
    kept, s = [], 5
    for ln in lens:
        kept.append(np.array([s], dtype=np.int64) if ln >= 2 else np.zeros(0, np.int64))
        s += int(ln)
    lay = wl.layout_from_lists(5, [int(x) for x in lens], kept)
    w = wl.tiny_workload("bf16", 4, 2, 64, T=2, B=2, k=100, seed=1300, value_scale=0.5)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    masks = (rng.random((2, c_n)) < 0.1).astype(np.uint8)
    for mode in ("kept_in_place", "pooled"):
        check_case(w, lay, k, v, qd, masks, mode)
