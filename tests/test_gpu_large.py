"""GPU parity at the full sizes of workloads config2, config3 (three of its 28 layers, one resident at a time;
the 28-layer resident run is tests/test_gpu_config3_stack.py) and
config4, in the launch configuration bench.py uses.  The oracle evaluates sampled rows one
chunk at a time (all rows of a few chunks, first and last row of a spread of chunks); integer
outputs and the gathered KV are compared in full, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_19225_amd import vxl, workloads as wl

from gpu_util import assert_close, desc_of, make_layout

pytestmark = pytest.mark.gpu


def lay_args(lay):
    return lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx


def sampled_rows(lay, full_chunks, edge_step):
    rows = set(range(0, lay.n_prefix, max(1, lay.n_prefix // 8))) | {lay.n_prefix - 1}
    for c in full_chunks:
        rows |= set(range(int(lay.chunk_bounds[c]), int(lay.chunk_bounds[c + 1])))
    for c in range(0, lay.n_chunks, edge_step):
        rows.add(int(lay.chunk_bounds[c]))
        rows.add(int(lay.chunk_bounds[c + 1]) - 1)
    rows.discard(-1)
    return np.array(sorted(rows), dtype=np.int64)


def prefill_and_check(w, lay, layer, full_chunks, edge_step, gl=None):
    q, k, v = wl.make_qkv(w, lay, layer=layer)
    gl = gl or make_layout(lay)
    desc = desc_of(w)
    dq, dk, dv = (vxl.to_device(x, w.dtype) for x in (q, k, v))
    out = torch.full_like(dq, float("nan"))
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
    vxl.chunk_prefill(gl, desc, dq, dk, dv, out, None, ws)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(out).all())
    rows = sampled_rows(lay, full_chunks, edge_step)
    got = vxl.to_host(out[:, torch.from_numpy(rows).cuda()])
    want = oracle.prefill_blk(q, k, v, *lay_args(lay), rows=rows)
    assert_close(got, want, w.dtype, what=f"{w.name} layer {layer} prefill ({len(rows)} sampled rows)")
    del dq, out
    return k, v, dk, dv, gl


def chain_and_check(w, lay, gl, k, v, dk, dv, qd, top_k, mask_from=None):
    """score/top-k (unless a mask is handed in) -> gather -> decode on the device; full
    comparison of mask, mix_len, gathered KV and the decode output."""
    desc = desc_of(w)
    dqd = vxl.to_device(qd, w.dtype)
    bsz, t, c_n = qd.shape[0], qd.shape[1], lay.n_chunks
    kk = min(top_k, c_n)
    l_cap = gl.mixed_kv_capacity(top_k)
    mask = torch.zeros((bsz, c_n), dtype=torch.uint8, device="cuda")
    if mask_from is None:
        idx = torch.zeros((bsz, max(kk, 1)), dtype=torch.int32, device="cuda")
        scores = torch.zeros((bsz, c_n), dtype=torch.float32, device="cuda")
        ws1 = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_TOPK, gl, desc, bsz, t))
        vxl.chunk_score_topk(gl, desc, dqd, dk, top_k, idx, mask, scores, workspace=ws1)
        want_s = oracle.chunk_scores(qd, k, lay.chunk_bounds)
        _, want_mask = oracle.select_topk(want_s, top_k)
        if 0 < kk < c_n:                                   # the decision must be well separated
            srt = np.sort(want_s, axis=1)[:, ::-1]
            assert (srt[:, kk - 1] - srt[:, kk]).min() > 1e-6 * np.abs(want_s).max()
        torch.cuda.synchronize()
        assert np.abs(scores.cpu().numpy() - want_s).max() <= 2e-5 * np.abs(want_s).max() + 1e-7
        assert np.array_equal(mask.cpu().numpy(), want_mask)
    else:
        mask.copy_(torch.from_numpy(mask_from))
        want_mask = mask_from
    kmix = torch.full((bsz, w.n_kv_heads, l_cap, w.head_dim), 7.0, dtype=dk.dtype, device="cuda")
    vmix = torch.full_like(kmix, 7.0)
    mix_len = torch.zeros((bsz,), dtype=torch.int32, device="cuda")
    src = torch.full((bsz, l_cap), -5, dtype=torch.int32, device="cuda")
    vxl.gather_bilevel_kv(gl, desc, dk, dv, mask, kmix, vmix, mix_len, src)
    out = torch.full_like(dqd, float("nan"))
    ws3 = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, bsz, t, l_cap))
    vxl.bilevel_decode(desc, dqd, kmix, vmix, mix_len, out, None, ws3)
    torch.cuda.synchronize()
    lens = mix_len.cpu().numpy()
    hsrc = src.cpu().numpy()
    want_out = np.zeros(qd.shape, np.float64)
    for b in range(bsz):                                   # one query at a time keeps the host copy small
        ids = oracle.mixed_source_index(want_mask[b], *lay_args(lay))
        assert lens[b] == len(ids) and np.array_equal(hsrc[b, :len(ids)], ids)
        tid = torch.from_numpy(ids).cuda()
        assert bool((kmix[b, :, :len(ids)] == dk[:, tid]).all()), "gathered K differs"
        assert bool((vmix[b, :, :len(ids)] == dv[:, tid]).all()), "gathered V differs"
        assert bool((kmix[b, :, len(ids):] == 7.0).all())
        want_out[b] = oracle.decode_mixed(qd[b:b + 1], k[None, :, ids], v[None, :, ids], [len(ids)])[0]
    assert_close(vxl.to_host(out), want_out, w.dtype, head_axis=2, what=f"{w.name} decode k={top_k}")
    return want_mask, lens


def test_config2_long_video():
    w = wl.WORKLOADS["config2"]
    lay = wl.make_layout(w)
    k, v, dk, dv, gl = prefill_and_check(w, lay, 0, full_chunks=[0, 128, 255], edge_step=16)
    qd = wl.make_decode_queries(w)
    _, lens = chain_and_check(w, lay, gl, k, v, dk, dv, qd, w.k)
    assert lens[0] == 23808


def test_config4_variable_chunks():
    w = wl.WORKLOADS["config4"]
    lay = wl.make_layout(w)
    c_n = lay.n_chunks
    k, v, dk, dv, gl = prefill_and_check(w, lay, 0, full_chunks=[0, c_n // 2, c_n - 1], edge_step=8)
    qd = wl.make_decode_queries(w)
    planted = set(wl.planted_chunks(w, lay))
    for top_k in (4, 32, c_n):
        mask, lens = chain_and_check(w, lay, gl, k, v, dk, dv, qd, top_k)
        if top_k >= len(planted):
            assert planted <= set(np.nonzero(mask[0])[0])         # query 0 recalls the planted chunks
        if top_k >= c_n:
            assert (lens == lay.n_tokens).all()


@pytest.mark.parametrize("name,layer", [("config2", 0), ("config4", 0), ("config3", 20)])
def test_every_row_at_full_size_against_the_vector_kernel(name, layer):
    """The oracle checks sampled rows at these sizes; the rows it does not reach are checked here on
    the device: EVERY output row of the matrix-core kernel against the fp32 vector-ALU kernel (a
    second implementation with its own tile walk, itself compared with the oracle on the sampled
    rows below), each row bounded on its own as in assert_close."""
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    q, k, v = wl.make_qkv(w, lay, layer=layer)
    gl, desc = make_layout(lay), desc_of(w)
    dq, dk, dv = (vxl.to_device(x, w.dtype) for x in (q, k, v))
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
    out = torch.full_like(dq, float("nan"))
    vxl.chunk_prefill(gl, desc, dq, dk, dv, out, None, ws)
    ref = torch.full_like(dq, float("nan"))
    vxl.debug_force_simple(True)
    try:
        vxl.chunk_prefill(gl, desc, dq, dk, dv, ref, None, ws)
        torch.cuda.synchronize()
    finally:
        vxl.debug_force_simple(False)
    assert bool(torch.isfinite(out).all()) and bool(torch.isfinite(ref).all())
    worst = 0.0
    for h in range(w.n_q_heads):                                   # head by head: fp32 copies of 1/28 of O at a time
        a, b = out[h].float(), ref[h].float()
        row_ref = b.norm(dim=-1)
        floor = 0.05 * float(row_ref.median())
        ratio = (a - b).norm(dim=-1) / torch.clamp(row_ref, min=max(floor, 1e-30))
        worst = max(worst, float(ratio.max()))
        assert float((a - b).abs().max()) <= 2e-2
    assert worst <= 3e-2, f"{name}: worst row of {w.n_q_heads * lay.n_tokens}: ||mfma - vector|| / ||row|| = {worst:.3e}"
    # and the vector kernel itself against the oracle on a sample of rows (all rows of two chunks)
    c_n = lay.n_chunks
    rows = sampled_rows(lay, [1, c_n - 2], max(1, c_n // 8))
    want = oracle.prefill_blk(q, k, v, *lay_args(lay), rows=rows)
    assert_close(vxl.to_host(ref[:, torch.from_numpy(rows).cuda()]), want, w.dtype, what=f"{name}: vector kernel, sampled rows")


@pytest.mark.parametrize("layer", [0, 13, 27])
def test_config3_layers(layer):
    """Three of the 28 independent layers (first, middle, last); the dense-chunk selection is made at layer 0 and reused
    at the other layers (and also checked when made at that layer itself)."""
    w = wl.WORKLOADS["config3"]
    lay = wl.make_layout(w)
    k, v, dk, dv, gl = prefill_and_check(w, lay, layer, full_chunks=[0, 320, 639], edge_step=40)
    qd = wl.make_decode_queries(w, layer)
    mask, lens = chain_and_check(w, lay, gl, k, v, dk, dv, qd, w.k)
    assert lens[0] == 18176
    if layer != 0:
        _, k0, _ = wl.make_qkv(w, lay, layer=0, with_q=False)
        _, mask0 = oracle.select_topk(oracle.chunk_scores(wl.make_decode_queries(w, 0), k0, lay.chunk_bounds), w.k)
        chain_and_check(w, lay, gl, k, v, dk, dv, qd, w.k, mask_from=mask0)


def test_maximum_chunk_count():
    """The largest chunk count the library accepts (the LDS sort runs at its full 4096 slots, the
    gather scan loops 16 times): thousands of chunks of 1..3 tokens, some without kept tokens;
    pre-filling on the same layout (4097 small segments) checked on every row."""
    rng = np.random.default_rng(91)
    c_n = vxl.MAX_CHUNKS
    lens = rng.integers(1, 4, size=c_n)
    kept, s = [], 5
    for ln in lens:
        kept.append(np.array([s], dtype=np.int64) if ln >= 2 else np.zeros(0, np.int64))
        s += int(ln)
    lay = wl.layout_from_lists(5, [int(x) for x in lens], kept)
    w = wl.tiny_workload("bf16", 4, 2, 64, T=2, B=2, k=100, seed=91, value_scale=0.5)
    q, k, v = wl.make_qkv(w, lay)
    gl = make_layout(lay)
    desc = desc_of(w)
    dq, dk, dv = (vxl.to_device(x, w.dtype) for x in (q, k, v))
    out = torch.full_like(dq, float("nan"))
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
    vxl.chunk_prefill(gl, desc, dq, dk, dv, out, None, ws)
    torch.cuda.synchronize()
    rows = np.arange(lay.n_tokens)[::7]
    want = oracle.prefill_blk(q, k, v, *lay_args(lay), rows=rows)
    assert_close(vxl.to_host(out)[:, rows], want, "bf16", what="4096-chunk prefill")
    qd = wl.make_decode_queries(w)
    for top_k in (100, c_n):
        chain_and_check(w, lay, gl, k, v, dk, dv, qd, top_k)
