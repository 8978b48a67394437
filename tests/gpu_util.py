"""Helpers of the GPU parity tests: run the four C-ABI calls through the ctypes binding on
seeded inputs and return host arrays; tolerance checks as stated for the path."""
import numpy as np
import torch

from paper_2506_19225_amd import vxl, workloads as wl

# Matching rules: fp32 storage -- max abs error <= 1e-5; bf16 storage with fp32 accumulation --
# max abs error <= 2e-2 and relative Frobenius error <= 1e-2, per query head.  With outputs of
# magnitude 1e-3..1e-2 the absolute bound is vacuous and a head-wide Frobenius ratio averages
# thousands of rows, so one row that lost a key tile would pass both; every output row (the D
# values of one query token and head) is therefore bounded on its own as well:
# ||row error|| <= 3e-2 * ||row||.  A correct row sits at 2e-3..6e-3 (one bf16 rounding of the
# output, 2^-9 relative per element, plus the bf16 rounding of the softmax weights); a row that
# misses a 64-key tile out of the few hundred to few thousand it attends to is off by >= 5e-2.
TOL_F32_ABS = 1e-5
TOL_BF16_ABS = 2e-2
TOL_BF16_REL = 1e-2
TOL_BF16_ROW = 3e-2


def assert_close(got, want, dtype, head_axis=0, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want)
    if dtype == "f32":
        assert err.max() <= TOL_F32_ABS, f"{what}: max abs err {err.max():.3e}"
        return
    assert err.max() <= TOL_BF16_ABS, f"{what}: max abs err {err.max():.3e}"
    g = np.moveaxis(got, head_axis, 0).reshape(got.shape[head_axis], -1)
    w = np.moveaxis(want, head_axis, 0).reshape(want.shape[head_axis], -1)
    rel = np.linalg.norm(g - w, axis=1) / np.maximum(np.linalg.norm(w, axis=1), 1e-30)
    assert rel.max() <= TOL_BF16_REL, f"{what}: rel Frobenius err {rel.max():.3e} (per head {rel})"
    # per output row (last axis); rows whose norm is far below the typical one (cancellation) are
    # measured against a floor of a twentieth of the median row norm
    row_err = np.linalg.norm(got - want, axis=-1)
    row_ref = np.linalg.norm(want, axis=-1)
    floor = 0.05 * float(np.median(row_ref)) if row_ref.size else 0.0
    ratio = row_err / np.maximum(np.maximum(row_ref, floor), 1e-30)
    worst = np.unravel_index(int(np.argmax(ratio)), ratio.shape) if ratio.size else ()
    assert ratio.size == 0 or ratio.max() <= TOL_BF16_ROW, \
        f"{what}: worst row {worst} has ||err||/||row|| = {ratio.max():.3e} (bound {TOL_BF16_ROW})"


def make_layout(lay: wl.Layout, window: int = 0) -> vxl.Layout:
    return vxl.Layout(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx, window=window)


def desc_of(w: wl.Workload, scale: float = 0.0):
    return vxl.make_desc(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype, scale)


def gpu_prefill(w, lay, q, k, v, scale=0.0, want_lse=False, gl=None, dev=None):
    """Returns O (float32 host array [Hq,N,D]) and optionally LSE."""
    gl = gl or make_layout(lay)
    desc = desc_of(w, scale)
    dq, dk, dv = (dev if dev is not None else [vxl.to_device(x, w.dtype) for x in (q, k, v)])
    out = torch.full_like(dq, float("nan"))
    lse = torch.full(dq.shape[:2], float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
    vxl.chunk_prefill(gl, desc, dq, dk, dv, out, lse, ws)
    torch.cuda.synchronize()
    res = vxl.to_host(out)
    return (res, vxl.to_host(lse)) if want_lse else res


def gpu_score_topk(w, lay, qd, k, top_k, gl=None, scale=0.0):
    gl = gl or make_layout(lay)
    desc = desc_of(w, scale)
    dqd, dk = vxl.to_device(qd, w.dtype), vxl.to_device(k, w.dtype)
    bsz, c_n = qd.shape[0], lay.n_chunks
    kk = min(top_k, c_n)
    idx = torch.full((bsz, max(kk, 1)), -7, dtype=torch.int32, device="cuda")
    mask = torch.full((bsz, max(c_n, 1)), 9, dtype=torch.uint8, device="cuda")
    scores = torch.full((bsz, max(c_n, 1)), float("nan"), dtype=torch.float32, device="cuda")
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_TOPK, gl, desc, bsz, qd.shape[1]))
    vxl.chunk_score_topk(gl, desc, dqd, dk, top_k, idx, mask, scores, workspace=ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy()[:, :kk], mask.cpu().numpy()[:, :c_n], scores.cpu().numpy()[:, :c_n]


def gpu_gather(w, lay, k, v, dense_mask, l_cap, gl=None, dev=None):
    """Returns kmix, vmix (float32 host), mix_len, src_idx; untouched rows keep a sentinel."""
    gl = gl or make_layout(lay)
    desc = desc_of(w)
    dk, dv = dev if dev is not None else (vxl.to_device(k, w.dtype), vxl.to_device(v, w.dtype))
    bsz = dense_mask.shape[0]
    dm = torch.from_numpy(np.ascontiguousarray(dense_mask, dtype=np.uint8)).cuda()
    kmix = torch.full((bsz, w.n_kv_heads, l_cap, w.head_dim), 7.0, dtype=dk.dtype, device="cuda")
    vmix = torch.full_like(kmix, 7.0)
    mix_len = torch.full((bsz,), -1, dtype=torch.int32, device="cuda")
    src = torch.full((bsz, l_cap), -5, dtype=torch.int32, device="cuda")
    vxl.gather_bilevel_kv(gl, desc, dk, dv, dm, kmix, vmix, mix_len, src)
    torch.cuda.synchronize()
    return kmix, vmix, mix_len, src


def gpu_decode(w, qd, kmix_dev, vmix_dev, mix_len_dev, scale=0.0, want_lse=False):
    desc = desc_of(w, scale)
    dqd = vxl.to_device(qd, w.dtype)
    out = torch.full_like(dqd, float("nan"))
    lse = torch.full(dqd.shape[:3], float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    bsz, t = qd.shape[0], qd.shape[1]
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, bsz, t, kmix_dev.shape[2]))
    vxl.bilevel_decode(desc, dqd, kmix_dev, vmix_dev, mix_len_dev, out, lse, ws)
    torch.cuda.synchronize()
    res = vxl.to_host(out)
    return (res, vxl.to_host(lse)) if want_lse else res


def gpu_score_topk_mass(w, lay, qd, k, top_k, gl=None, scale=0.0):
    """vxl_chunk_score_topk_mass -> (topk_idx, dense_mask, scores) as host arrays."""
    gl = gl or make_layout(lay)
    desc = desc_of(w, scale)
    dqd, dk = vxl.to_device(qd, w.dtype), vxl.to_device(k, w.dtype)
    bsz, c_n = qd.shape[0], lay.n_chunks
    kk = min(top_k, c_n)
    idx = torch.full((bsz, max(kk, 1)), -7, dtype=torch.int32, device="cuda")
    mask = torch.full((bsz, max(c_n, 1)), 9, dtype=torch.uint8, device="cuda")
    scores = torch.full((bsz, max(c_n, 1)), float("nan"), dtype=torch.float32, device="cuda")
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_MASS, gl, desc, bsz, qd.shape[1]))
    vxl.chunk_score_topk_mass(gl, desc, dqd, dk, top_k, idx, mask, scores, workspace=ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy()[:, :kk], mask.cpu().numpy()[:, :c_n], scores.cpu().numpy()[:, :c_n]


def full_sort_selection(scores, k):
    """(idx [B, min(k, C)] best first, mask [B, C]) that a full sort of `scores` gives: score
    descending, equal scores to the lower chunk id.  Used to check the device's selection against the
    device's OWN fp32 scores -- a property of the selection kernel, in which the oracle has no part."""
    scores = np.asarray(scores)
    bsz, n = scores.shape
    kk = min(k, n)
    idx = np.zeros((bsz, kk), dtype=np.int32)
    mask = np.zeros((bsz, n), dtype=np.uint8)
    for b in range(bsz):
        order = np.lexsort((np.arange(n), -scores[b].astype(np.float64)))     # last key is the primary one
        idx[b] = order[:kk]
        mask[b, order[:kk]] = 1
    return idx, mask


def check_selection_valid(idx, mask, want_scores, want_mask, k, tol):
    """Several selections are correct where oracle scores are closer than the score tolerance: the
    device's must leave out nothing clearly better than what it takes, take exactly min(k, C) chunks,
    agree with its own index list, and equal the oracle's mask wherever the rank-k margin is clear."""
    bsz, n = want_scores.shape
    kk = min(k, n)
    for b in range(bsz):
        assert mask[b].sum() == kk and sorted(idx[b].tolist()) == np.flatnonzero(mask[b]).tolist()
        if 0 < kk < n:
            srt = np.sort(want_scores[b])[::-1]
            assert (want_scores[b, idx[b]] >= srt[kk - 1] - 2 * tol).all()
            assert mask[b][want_scores[b] > srt[kk - 1] + 2 * tol].all()
            if srt[kk - 1] - srt[kk] > 2 * tol:
                assert np.array_equal(mask[b], want_mask[b])
        else:
            assert np.array_equal(mask[b], want_mask[b])


def storage_round(w, x):
    """A float64 result of the oracle as the storage dtype of the workload holds it."""
    return wl.round_to_bf16(x.astype(np.float32)) if w.dtype == "bf16" else x.astype(np.float32)


def kept_rows(k, lay):
    """[Hkv, S_total, D] kept rows in chunk order (host)."""
    return np.ascontiguousarray(k[:, lay.sparse_idx]) if len(lay.sparse_idx) else np.zeros((k.shape[0], 1, k.shape[2]), k.dtype)


def gpu_decode_inplace(w, lay, qd, dk, dv, masks, l_cap, sparse=None, gl=None, desc=None, scale=0.0, want_lse=True):
    """sparse: None (kept rows in place) or (ksp, vsp) device tensors."""
    gl = gl or make_layout(lay)
    desc = desc or desc_of(w, scale)
    dqd = vxl.to_device(qd, w.dtype)
    dm = torch.from_numpy(np.ascontiguousarray(masks, dtype=np.uint8)).cuda()
    bsz, t = qd.shape[0], qd.shape[1]
    out = torch.full_like(dqd, float("nan"))
    lse = torch.full(dqd.shape[:3], float("nan"), dtype=torch.float32, device="cuda")
    lens = torch.full((bsz,), -77, dtype=torch.int32, device="cuda")
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE_INPLACE, gl, desc, bsz, t, l_cap))
    ksp, vsp = sparse if sparse is not None else (None, None)
    vxl.bilevel_decode_inplace(gl, desc, dqd, dk, dv, ksp, vsp, dm, l_cap, out, lse, lens, ws)
    torch.cuda.synchronize()
    first = out.clone()
    # the later tokens of a query reuse the row map that is in the workspace
    out.fill_(float("nan"))
    vxl.bilevel_decode_inplace(gl, desc, dqd, dk, dv, ksp, vsp, dm, l_cap, out, lse, lens, ws, map_ready=True)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.uint8), first.view(torch.uint8)), "map_ready call differs"
    return vxl.to_host(out), vxl.to_host(lse), lens.cpu().numpy()
