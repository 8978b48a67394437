"""Seeded random sweeps: ragged layouts, head groups, look-back windows, memory layouts, query counts and
selection sizes drawn at random, every call checked against the oracle.  (The fixed cases of the other
files pin the known corner cases; this file walks the space between them.)"""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_19225_amd import vxl, workloads as wl

from gpu_util import (assert_close, check_selection_valid, desc_of, full_sort_selection, gpu_decode,
                      gpu_decode_inplace, gpu_gather, gpu_score_topk, gpu_score_topk_mass, kept_rows, make_layout,
                      storage_round)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_prefill_random_sweep(seed):
    rng = np.random.default_rng(seed)
    for case in range(12):
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        hkv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 2, 3, 4, 7, 8, 9]))
        d = int(rng.choice([64, 128]))
        p = int(rng.choice([0, 1, 17, 64, 130, 300]))
        nc = int(rng.integers(1, 5))
        hi = int(rng.choice([40, 130, 300, 700]))
        lo = int(rng.integers(1, hi + 1))
        window = int(rng.choice([0, 0, 16, 100]))
        tokmaj = bool(rng.random() < 0.4)
        s = int(rng.integers(1 << 30))
        w = wl.tiny_workload(dtype, hkv * group, hkv, d, T=1, B=1, k=1, seed=s,
                             value_scale=float(rng.choice([0.3, 0.6, 1.0])))
        lay = wl.random_layout(np.random.default_rng(s), p, nc, lo, hi)
        q, k, v = wl.make_qkv(w, lay)
        what = (f"seed {seed} case {case}: {dtype} Hkv={hkv} G={group} D={d} P={p} "
                f"chunks={[int(x) for x in np.diff(lay.chunk_bounds)]} window={window} token_major={tokmaj}")
        print(what, flush=True)
        gl = vxl.Layout(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx, window=window)
        desc = vxl.make_desc(w.n_q_heads, w.n_kv_heads, d, dtype, token_major=tokmaj)
        dq, dk, dv = (vxl.to_device(x, dtype) for x in (q, k, v))
        if tokmaj:
            dq, dk, dv = (x.permute(1, 0, 2).contiguous() for x in (dq, dk, dv))
        out = torch.full_like(dq, float("nan"))
        ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
        vxl.chunk_prefill(gl, desc, dq, dk, dv, out, None, ws)
        torch.cuda.synchronize()
        got = vxl.to_host(out.permute(1, 0, 2).contiguous() if tokmaj else out)
        want = oracle.prefill_blk(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx,
                                  window=window)
        assert_close(got, want, dtype, what=what)


@pytest.mark.parametrize("seed", [21, 22])
def test_bilevel_random_sweep(seed):
    rng = np.random.default_rng(seed)
    for case in range(12):
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        hkv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 2, 4, 7, 8]))
        d = int(rng.choice([64, 128]))
        p = int(rng.choice([0, 1, 17, 64, 130]))
        nc = int(rng.integers(1, 12))
        hi = int(rng.choice([40, 130, 300]))
        lo = int(rng.integers(1, hi + 1))
        t_q = int(rng.choice([1, 2, 4, 5, 16, 33, 48, 80]))
        bsz = int(rng.choice([1, 2, 3]))
        k_top = int(rng.integers(0, nc + 2))
        s = int(rng.integers(1 << 30))
        w = wl.tiny_workload(dtype, hkv * group, hkv, d, T=t_q, B=bsz, k=k_top, seed=s,
                             value_scale=float(rng.choice([0.3, 0.6, 1.0])))
        lay = wl.random_layout(np.random.default_rng(s), p, nc, lo, hi)
        q, k, v = wl.make_qkv(w, lay)
        qd = wl.make_decode_queries(w)
        what = (f"seed {seed} case {case}: {dtype} Hkv={hkv} G={group} D={d} P={p} "
                f"chunks={[int(x) for x in np.diff(lay.chunk_bounds)]} T={t_q} B={bsz} k={k_top}")
        print(what, flush=True)
        gl = make_layout(lay)
        idx, mask, sc = gpu_score_topk(w, lay, qd, k, k_top, gl=gl)
        wsc = oracle.chunk_scores(qd, k, lay.chunk_bounds)
        assert np.abs(sc - wsc).max() <= 1e-4 * max(1.0, np.abs(wsc).max()), what
        # the selection: the full sort of the device's own fp32 scores, and valid for the oracle's
        tol = 1e-4 * max(1.0, np.abs(wsc).max())
        own_idx, own_mask = full_sort_selection(sc, k_top)
        assert np.array_equal(idx, own_idx) and np.array_equal(mask, own_mask), what
        check_selection_valid(idx, mask, wsc, oracle.select_topk(wsc, k_top)[1], k_top, tol)
        mask = oracle.select_topk(wsc, k_top)[1]               # what follows takes the oracle's selection on both sides
        midx, mmask, msc = gpu_score_topk_mass(w, lay, qd, k, k_top, gl=gl)
        wms = oracle.chunk_scores_mass(qd, k, lay.n_prefix, lay.chunk_bounds)
        mtol = 1e-4 * np.abs(wms).max()
        assert np.abs(msc - wms).max() <= mtol, what
        own_idx, own_mask = full_sort_selection(msc, k_top)
        assert np.array_equal(midx, own_idx) and np.array_equal(mmask, own_mask), what
        check_selection_valid(midx, mmask, wms, oracle.select_topk(wms, k_top)[1], k_top, mtol)
        l_cap = gl.mixed_kv_capacity(min(k_top, nc))
        kmix, vmix, mix_len, src = gpu_gather(w, lay, k, v, mask, l_cap, gl=gl)
        wk, wv, wlen, wsrc = oracle.gather_bilevel(k, v, mask, lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets,
                                                   lay.sparse_idx, l_cap=l_cap)
        assert np.array_equal(mix_len.cpu().numpy(), wlen), what
        gk, gv = vxl.to_host(kmix), vxl.to_host(vmix)
        for b in range(bsz):
            n = int(wlen[b])
            assert np.array_equal(gk[b, :, :n], wk[b, :, :n]) and np.array_equal(gv[b, :, :n], wv[b, :, :n]), what
            assert np.array_equal(src.cpu().numpy()[b, :n], wsrc[b, :n]), what
        if int(wlen.min()) > 0:
            got = gpu_decode(w, qd, kmix, vmix, mix_len)
            want = oracle.decode_mixed(qd, wk, wv, wlen)
            assert_close(got, want, dtype, head_axis=2, what=what)
            # the same rows read in place: kept rows where they lie, then from a compacted copy
            dk, dv = vxl.to_device(k, dtype), vxl.to_device(v, dtype)
            for sparse in (None, (vxl.to_device(kept_rows(k, lay), dtype), vxl.to_device(kept_rows(v, lay), dtype))):
                got, _, lens = gpu_decode_inplace(w, lay, qd, dk, dv, mask, l_cap, sparse, gl=gl)
                assert np.array_equal(lens, wlen), what
                assert_close(got, want, dtype, head_axis=2, what=what + (" in place" if sparse is None else " in place, compacted"))
            # pooled sparse rows: gather + decode and in place, against the oracle's pooled mixed set
            if lay.sparse_offsets[-1] > 0:
                desc = desc_of(w)
                ksp = torch.empty((hkv, int(lay.sparse_offsets[-1]), d), dtype=dk.dtype, device="cuda")
                vsp = torch.empty_like(ksp)
                vxl.pool_sparse_kv(gl, desc, dk, dv, ksp, vsp)
                torch.cuda.synchronize()
                ok, ov = oracle.pool_sparse_kv(k, v, lay.chunk_bounds, lay.sparse_offsets)
                pk, pv, plen, _ = oracle.gather_bilevel_pooled(k, v, storage_round(w, ok), storage_round(w, ov), mask,
                                                               lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, l_cap=l_cap)
                got, _, lens = gpu_decode_inplace(w, lay, qd, dk, dv, mask, l_cap, (ksp, vsp), gl=gl)
                assert np.array_equal(lens, plen), what
                assert_close(got, oracle.decode_mixed(qd, pk, pv, plen), dtype, head_axis=2, what=what + " in place, pooled")
