"""GPU parity of the pooled sparse KVs (vxl_pool_sparse_kv, vxl_gather_bilevel_kv_pooled) and of
decoding over the mixed set built from them, against the float64 oracle.  Pooled values are
floating point: they are compared to within one unit in the last place of the storage dtype
(the device adds in fp32, the oracle in float64, both round once); everything that is a copy or
an index is compared bit for bit."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_19225_amd import vxl, workloads as wl

from gpu_util import assert_close, desc_of, gpu_decode, make_layout, storage_round

pytestmark = pytest.mark.gpu


def run_pool(w, lay, k, v, gl=None):
    gl = gl or make_layout(lay)
    desc = desc_of(w)
    dk, dv = vxl.to_device(k, w.dtype), vxl.to_device(v, w.dtype)
    s_total = int(lay.sparse_offsets[-1])
    ksp = torch.full((w.n_kv_heads, max(s_total, 1), w.head_dim), 7.0, dtype=dk.dtype, device="cuda")
    vsp = torch.full_like(ksp, 7.0)
    vxl.pool_sparse_kv(gl, desc, dk, dv, ksp, vsp)
    torch.cuda.synchronize()
    return gl, dk, dv, ksp, vsp


def check_pool(w, lay, k, v):
    gl, dk, dv, ksp, vsp = run_pool(w, lay, k, v)
    s_total = int(lay.sparse_offsets[-1])
    wk, wv = oracle.pool_sparse_kv(k, v, lay.chunk_bounds, lay.sparse_offsets)
    # one unit in the last place of the result (its single rounding) plus the fp32 summation error,
    # which scales with the summands, not with the (possibly cancelling) mean
    ulp = 2.0 ** -7 if w.dtype == "bf16" else 2.0 ** -22
    for got, want, src in ((vxl.to_host(ksp)[:, :s_total], wk, k), (vxl.to_host(vsp)[:, :s_total], wv, v)):
        ref = storage_round(w, want).astype(np.float64)
        assert np.isfinite(got).all()
        tol = ulp * np.abs(ref) + 2.0 ** -21 * np.abs(src).max()
        assert (np.abs(got - ref) <= tol).all(), np.abs(got - ref).max()
        if w.dtype == "bf16":
            assert (got == ref).mean() > 0.99                # the two roundings almost always agree
    return gl, dk, dv, ksp, vsp


def test_pool_config0_fp32_and_ragged_groups():
    w = wl.WORKLOADS["config0"]
    lay = wl.make_layout(w)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    check_pool(w, lay, k, v)
    rng = np.random.default_rng(91)
    for dtype, d in (("f32", 128), ("bf16", 64), ("bf16", 128)):
        w = wl.tiny_workload(dtype, 4, 2, d, T=2, B=2, k=2, seed=91)
        # odd chunk lengths and kept counts: groups of unequal size, one row per group, one group
        lay = wl.random_layout(rng, 3, 11, 1, 157, allow_empty_kept=True)
        _, k, v = wl.make_qkv(w, lay, with_q=False)
        check_pool(w, lay, k, v)


@pytest.mark.parametrize("name", ["config0", "config1", "config4"])
def test_pooled_chain(name):
    """select -> pool -> gather (pooled) -> decode, everything on the device; the gathered set is
    checked row by row against its sources, the decode output against the oracle's decode over
    the oracle's own pooled set."""
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    qd = wl.make_decode_queries(w)
    gl, dk, dv, ksp, vsp = check_pool(w, lay, k, v)
    desc = desc_of(w)
    top_k = w.k
    scores = oracle.chunk_scores(qd, k, lay.chunk_bounds)
    _, masks = oracle.select_topk(scores, top_k)
    dm = torch.from_numpy(masks).cuda()
    l_cap = gl.mixed_kv_capacity(top_k)
    bsz = qd.shape[0]
    kmix = torch.full((bsz, w.n_kv_heads, l_cap, w.head_dim), 7.0, dtype=dk.dtype, device="cuda")
    vmix = torch.full_like(kmix, 7.0)
    mix_len = torch.full((bsz,), -1, dtype=torch.int32, device="cuda")
    src = torch.full((bsz, l_cap), -5, dtype=torch.int32, device="cuda")
    vxl.gather_bilevel_kv_pooled(gl, desc, dk, dv, ksp, vsp, dm, kmix, vmix, mix_len, src)
    torch.cuda.synchronize()
    # oracle structure (lengths, source codes) -- pooled values taken from the oracle's own pooling
    ok, ov = oracle.pool_sparse_kv(k, v, lay.chunk_bounds, lay.sparse_offsets)
    ok, ov = storage_round(w, ok), storage_round(w, ov)
    wk, wv, wlen, wsrc = oracle.gather_bilevel_pooled(k, v, ok, ov, masks, lay.n_prefix, lay.chunk_bounds,
                                                      lay.sparse_offsets, l_cap=l_cap)
    assert np.array_equal(mix_len.cpu().numpy(), wlen)
    hsrc = src.cpu().numpy()
    hk, hv = vxl.to_host(kmix), vxl.to_host(vmix)
    dsp_k, dsp_v = vxl.to_host(ksp), vxl.to_host(vsp)
    for b in range(bsz):
        n = int(wlen[b])
        assert np.array_equal(hsrc[b, :n], wsrc[b, :n])
        assert (hsrc[b, n:] == -5).all() and (hk[b, :, n:] == 7.0).all()          # rows beyond untouched
        s = hsrc[b, :n]
        dense = s >= 0
        assert np.array_equal(hk[b][:, :n][:, dense], k[:, s[dense]])             # copies: bit for bit
        assert np.array_equal(hv[b][:, :n][:, dense], v[:, s[dense]])
        assert np.array_equal(hk[b][:, :n][:, ~dense], dsp_k[:, -1 - s[~dense]])
        assert np.array_equal(hv[b][:, :n][:, ~dense], dsp_v[:, -1 - s[~dense]])
    got = gpu_decode(w, qd, kmix, vmix, mix_len)
    want = oracle.decode_mixed(qd, wk, wv, wlen)
    assert_close(got, want, w.dtype, head_axis=2, what=f"{name} decode over pooled mixed KV")


def test_pooled_gather_without_sparse_rows_and_all_dense():
    w = wl.tiny_workload("bf16", 4, 2, 128, T=1, B=1, k=1, seed=92)
    lay = wl.layout_from_lists(4, [40, 24], [np.zeros(0, np.int32)] * 2)           # nothing kept: S_total = 0
    _, k, v = wl.make_qkv(w, lay, with_q=False)
    gl = make_layout(lay)
    desc = desc_of(w)
    dk, dv = vxl.to_device(k, w.dtype), vxl.to_device(v, w.dtype)
    vxl.pool_sparse_kv(gl, desc, dk, dv, None, None)                               # nothing to write
    dm = torch.tensor([[1, 0]], dtype=torch.uint8, device="cuda")
    l_cap = gl.mixed_kv_capacity(1)
    kmix = torch.zeros((1, 2, l_cap, 128), dtype=dk.dtype, device="cuda")
    vmix = torch.zeros_like(kmix)
    mix_len = torch.zeros((1,), dtype=torch.int32, device="cuda")
    vxl.gather_bilevel_kv_pooled(gl, desc, dk, dv, None, None, dm, kmix, vmix, mix_len, None)
    torch.cuda.synchronize()
    assert int(mix_len[0]) == 44
    assert np.array_equal(vxl.to_host(kmix)[0, :, :44], k[:, :44])
