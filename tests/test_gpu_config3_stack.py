"""Workload config3 as stated: the 28-layer stack with the K and V of ALL layers resident in HBM
(9.4 GB), independent seeded Q/K/V per layer drawn on the device.  Pre-filling runs on every
layer and is compared with the oracle on a few rows per layer (first and last chunk, a middle
one, the prefix: every head); the dense chunks are selected at layer 0, and gather + decode run
on every layer with that selection and are compared in full -- mask, lengths, gathered rows bit
for bit, decode outputs within tolerance.  The oracle sees host copies of the very tensors the
device holds."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_19225_amd import vxl, workloads as wl

from gpu_util import assert_close, desc_of, make_layout

pytestmark = pytest.mark.gpu


def test_config3_all_28_layers_resident():
    w = wl.WORKLOADS["config3"]
    lay = wl.make_layout(w)
    gl = make_layout(lay)
    desc = desc_of(w)
    args = (lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    n_layers, c_n = w.n_layers, lay.n_chunks
    ks, vs, qds = [], [], []
    for layer in range(n_layers):                           # the whole KV cache stays resident
        _, k, v = wl.make_qkv_device(w, lay, layer, with_q=False)
        ks.append(k)
        vs.append(v)
        qds.append(wl.make_decode_queries_device(w, layer))
    resident = sum(k.numel() + v.numel() for k, v in zip(ks, vs)) * 2
    assert resident == 2 * 28 * 4 * 164096 * 128 * 2
    print(f"resident KV: {resident / 1e9:.2f} GB", flush=True)

    # ---- pre-filling, every layer; sampled rows against the oracle ----
    rng = np.random.default_rng(3)
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
    out = None
    for layer in range(n_layers):
        # (Q of one layer at a time: 1.2 GB; only K and V have to stay resident)
        q = wl.make_q_device(w, lay, layer)
        out = torch.full_like(q, float("nan")) if out is None else out.fill_(float("nan"))
        vxl.chunk_prefill(gl, desc, q, ks[layer], vs[layer], out, None, ws)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all()), f"layer {layer}: non-finite pre-filling output"
        picks = [0, int(rng.integers(1, c_n - 1)), c_n - 1]
        rows = [0, lay.n_prefix - 1]
        for c in picks:
            lo, hi = int(lay.chunk_bounds[c]), int(lay.chunk_bounds[c + 1])
            rows += [lo, lo + 1, int(rng.integers(lo, hi)), hi - 1]
        rows = np.array(sorted(set(rows)), dtype=np.int64)
        tid = torch.from_numpy(rows).cuda()
        # the oracle reads q only at `rows`: a host array that is zero elsewhere serves
        hq = np.zeros((w.n_q_heads, lay.n_tokens, w.head_dim), dtype=np.float32)
        hq[:, rows] = vxl.to_host(q[:, tid])
        hk, hv = vxl.to_host(ks[layer]), vxl.to_host(vs[layer])
        want = oracle.prefill_blk(hq, hk, hv, *args, rows=rows)
        assert_close(vxl.to_host(out[:, tid]), want, "bf16", what=f"config3 layer {layer} prefill rows")
        del q, hq
        # ---- the bi-level chain of this layer (selection made at layer 0) ----
        hqd = vxl.to_host(qds[layer])
        if layer == 0:
            bsz, t = hqd.shape[0], hqd.shape[1]
            l_cap = gl.mixed_kv_capacity(w.k)
            idx = torch.zeros((bsz, w.k), dtype=torch.int32, device="cuda")
            mask = torch.zeros((bsz, c_n), dtype=torch.uint8, device="cuda")
            scores = torch.zeros((bsz, c_n), dtype=torch.float32, device="cuda")
            ws1 = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_TOPK, gl, desc, bsz, t))
            vxl.chunk_score_topk(gl, desc, qds[0], ks[0], w.k, idx, mask, scores, workspace=ws1)
            torch.cuda.synchronize()
            want_s = oracle.chunk_scores(hqd, hk, lay.chunk_bounds)
            want_idx, want_mask = oracle.select_topk(want_s, w.k)
            srt = np.sort(want_s, axis=1)[:, ::-1]
            assert (srt[:, w.k - 1] - srt[:, w.k]).min() > 1e-6 * np.abs(want_s).max(), "degenerate seed"
            assert np.abs(scores.cpu().numpy() - want_s).max() <= 2e-5 * np.abs(want_s).max() + 1e-7
            assert np.array_equal(mask.cpu().numpy(), want_mask)
            assert np.array_equal(np.sort(idx.cpu().numpy(), axis=1), np.sort(want_idx, axis=1))
            ids = oracle.mixed_source_index(want_mask[0], *args)
            assert len(ids) == 18176
            tids = torch.from_numpy(ids).cuda()
            kmix = torch.empty((bsz, w.n_kv_heads, l_cap, w.head_dim), dtype=torch.bfloat16, device="cuda")
            vmix = torch.empty_like(kmix)
            mix_len = torch.zeros((bsz,), dtype=torch.int32, device="cuda")
            src = torch.empty((bsz, l_cap), dtype=torch.int32, device="cuda")
            od = torch.empty_like(qds[0])
            ws3 = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, bsz, t, l_cap))
        kmix.fill_(7.0)
        vmix.fill_(7.0)
        src.fill_(-5)
        od.fill_(float("nan"))
        vxl.gather_bilevel_kv(gl, desc, ks[layer], vs[layer], mask, kmix, vmix, mix_len, src)
        vxl.bilevel_decode(desc, qds[layer], kmix, vmix, mix_len, od, None, ws3)
        torch.cuda.synchronize()
        n = len(ids)
        assert int(mix_len[0]) == n and np.array_equal(src[0, :n].cpu().numpy(), ids)
        assert bool((kmix[0, :, :n] == ks[layer][:, tids]).all()) and bool((vmix[0, :, :n] == vs[layer][:, tids]).all())
        assert bool((kmix[0, :, n:] == 7.0).all())
        want_d = oracle.decode_mixed(hqd, hk[None, :, ids], hv[None, :, ids], [n])
        assert_close(vxl.to_host(od), want_d, "bf16", head_axis=2, what=f"config3 layer {layer} decode")
        print(f"layer {layer}: prefill rows, gather and decode match the oracle", flush=True)
