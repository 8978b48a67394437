"""Bi-level KV decoding, by definition (test infrastructure).

Paper: Method, "Bi-level KVs Decoding" and its figure caption.  The paper names the
attention-score mechanism as one relevance oracle but prints no formula; the reading taken
here (listed with the other readings in the design notes) is the mean pre-softmax attention
logit of the query tokens onto the dense keys of a chunk:

    score[b, c] = mean over (t, h, j in chunk c) of  scale * Qd[b, t, h, :] . K[g(h), j, :]

which factors into per-chunk mean keys and per-KV-head mean queries.  Selection keeps the
min(k, C) best chunks, ties going to the lower chunk id.  The mixed KV set is the prefix, then
per chunk either all its rows (dense) or its kept rows (sparse), concatenated in temporal order.
Decoding is plain softmax attention of each query token over the mixed set (no mask among the
query tokens: their own KVs are not part of the set).
"""
import numpy as np

from .sets import mixed_source_index


def chunk_scores(qd, k, chunk_bounds, scale=None):
    """score[B, C] float64.  qd [B, T, Hq, D]; k [Hkv, N, D] dense keys."""
    bsz, t, hq, d = qd.shape
    hkv = k.shape[0]
    grp = hq // hkv
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    b = np.asarray(chunk_bounds, dtype=np.int64)
    c_n = len(b) - 1
    k64 = np.asarray(k, dtype=np.float64)
    kbar = np.stack([k64[:, b[c]:b[c + 1], :].mean(axis=1) for c in range(c_n)], axis=1) \
        if c_n else np.zeros((hkv, 0, d))                                  # [Hkv, C, D]
    q64 = np.asarray(qd, dtype=np.float64).reshape(bsz, t, hkv, grp, d)
    qbar = q64.mean(axis=(1, 3))                                            # [B, Hkv, D]
    return scale * np.einsum("bgd,gcd->bc", qbar, kbar) / hkv


def chunk_scores_mass(qd, k, n_prefix, chunk_bounds, scale=None, row_block=64):
    """score[B, C] float64: the second reading of the attention-score relevance oracle -- the
    softmax attention MASS a query token puts on the dense keys of a chunk, averaged over the
    query tokens and query heads:

        p[b,t,h,j] = softmax over ALL tokens j (prefix and every chunk) of scale * Qd[b,t,h].K[g(h),j]
        score[b,c] = mean over (t, h) of  sum_{j in chunk c} p[b,t,h,j]

    The prefix takes part in the softmax but is not scored, so the scores of a query sum to
    1 - (mean mass on the prefix).  qd [B, T, Hq, D]; k [Hkv, N, D]."""
    bsz, t, hq, d = qd.shape
    hkv = k.shape[0]
    grp = hq // hkv
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    b = np.asarray(chunk_bounds, dtype=np.int64)
    assert int(b[0]) == int(n_prefix)
    c_n = len(b) - 1
    k64 = np.asarray(k, dtype=np.float64)
    out = np.zeros((bsz, c_n), dtype=np.float64)
    for bi in range(bsz):
        for h in range(hq):
            kg = k64[h // grp]
            for t0 in range(0, t, row_block):
                q = np.asarray(qd[bi, t0:t0 + row_block, h], dtype=np.float64)      # [rows, D]
                s = scale * (q @ kg.T)                                              # [rows, N]
                s -= s.max(axis=1, keepdims=True)
                p = np.exp(s)
                p /= p.sum(axis=1, keepdims=True)
                for c in range(c_n):
                    out[bi, c] += p[:, b[c]:b[c + 1]].sum()
    return out / (t * hq)


def select_topk(scores, k, decide_dtype=np.float64):
    """(topk_idx [B, k'], dense_mask [B, C] uint8) with k' = min(k, C).

    Full sort of the chunk ids by (score descending, chunk id ascending) on the scores as given
    (float64 by default); the first k' are the dense chunks.  `decide_dtype` is a test option: a
    caller that wants to see what the decision would be on scores rounded to a narrower type (the
    device scores in fp32) passes it explicitly."""
    scores = np.asarray(scores)
    bsz, c_n = scores.shape
    kk = max(0, min(int(k), c_n))
    s = scores.astype(decide_dtype)
    idx = np.zeros((bsz, kk), dtype=np.int32)
    mask = np.zeros((bsz, c_n), dtype=np.uint8)
    for bi in range(bsz):
        order = sorted(range(c_n), key=lambda c: (-float(s[bi, c]), c))     # full sort
        idx[bi] = order[:kk]
        mask[bi, order[:kk]] = 1
    return idx, mask


def gather_bilevel(k, v, dense_mask, n_prefix, chunk_bounds, sparse_offsets, sparse_idx, l_cap=None):
    """Mixed KV of every query.  k, v [Hkv, N, D] (any dtype, copied bit for bit);
    dense_mask [B, C].  Returns (kmix, vmix [B, Hkv, Lcap, D] zero padded, mix_len [B] int32,
    src_idx [B, Lcap] int32 padded with -1)."""
    dense_mask = np.asarray(dense_mask)
    bsz = dense_mask.shape[0]
    srcs = [mixed_source_index(dense_mask[bi], n_prefix, chunk_bounds, sparse_offsets, sparse_idx)
            for bi in range(bsz)]
    lens = np.array([len(s) for s in srcs], dtype=np.int32)
    l_cap = int(lens.max()) if l_cap is None else int(l_cap)
    assert l_cap >= lens.max()
    hkv, _, d = k.shape
    kmix = np.zeros((bsz, hkv, l_cap, d), dtype=k.dtype)
    vmix = np.zeros((bsz, hkv, l_cap, d), dtype=v.dtype)
    src_idx = np.full((bsz, l_cap), -1, dtype=np.int32)
    for bi, s in enumerate(srcs):
        kmix[bi, :, :len(s)] = k[:, s]
        vmix[bi, :, :len(s)] = v[:, s]
        src_idx[bi, :len(s)] = s
    return kmix, vmix, lens, src_idx


def decode_lse(qd, kmix, vmix, mix_len, scale=None):
    """(O [B, T, Hq, D], LSE [B, T, Hq]) float64: softmax attention of every query token over
    the first mix_len[b] rows of its mixed KV."""
    bsz, t, hq, d = qd.shape
    hkv = kmix.shape[1]
    grp = hq // hkv
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    out = np.zeros((bsz, t, hq, d), dtype=np.float64)
    lse = np.zeros((bsz, t, hq), dtype=np.float64)
    for bi in range(bsz):
        ln = int(mix_len[bi])
        for h in range(hq):
            g = h // grp
            kk = np.asarray(kmix[bi, g, :ln], dtype=np.float64)
            vv = np.asarray(vmix[bi, g, :ln], dtype=np.float64)
            s = scale * (np.asarray(qd[bi, :, h, :], dtype=np.float64) @ kk.T)   # [T, ln]
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            l = e.sum(axis=1, keepdims=True)
            out[bi, :, h, :] = (e / l) @ vv
            lse[bi, :, h] = (m + np.log(l))[:, 0]
    return out, lse


def decode_mixed(qd, kmix, vmix, mix_len, scale=None):
    return decode_lse(qd, kmix, vmix, mix_len, scale)[0]


# ---------------------------------------------------------------------------------------------
# Pooled sparse KVs ("Bi-level KVs Decoding": the dense KVs are cut into chunks and a pooling
# operation on each chunk yields its sparse KVs).  The paper gives neither window nor stride; the
# reading taken here: a chunk of len_c rows that is to be represented by s_c sparse rows is cut
# into s_c consecutive groups, group m = rows [floor(m*len_c/s_c), floor((m+1)*len_c/s_c)), and
# sparse row m is the arithmetic mean of the group's rows (K and V alike) -- plain average pooling
# with window len_c/s_c when that divides.  s_c comes from the CSR offsets of the layout.
# ---------------------------------------------------------------------------------------------
def pool_groups(length, count):
    """[(lo, hi)] of the `count` consecutive groups that partition range(length)."""
    return [((m * length) // count, ((m + 1) * length) // count) for m in range(count)]


def pool_sparse_kv(k, v, chunk_bounds, sparse_offsets):
    """(ksp, vsp) float64 [Hkv, S_total, D]: row sparse_offsets[c] + m is the mean of group m of
    chunk c.  (The caller rounds to the storage dtype.)"""
    b = np.asarray(chunk_bounds, dtype=np.int64)
    off = np.asarray(sparse_offsets, dtype=np.int64)
    hkv, _, d = k.shape
    ksp = np.zeros((hkv, int(off[-1]), d), dtype=np.float64)
    vsp = np.zeros_like(ksp)
    for c in range(len(b) - 1):
        cnt = int(off[c + 1] - off[c])
        for m, (lo, hi) in enumerate(pool_groups(int(b[c + 1] - b[c]), cnt)):
            ksp[:, off[c] + m] = np.asarray(k[:, b[c] + lo:b[c] + hi], dtype=np.float64).mean(axis=1)
            vsp[:, off[c] + m] = np.asarray(v[:, b[c] + lo:b[c] + hi], dtype=np.float64).mean(axis=1)
    return ksp, vsp


def gather_bilevel_pooled(k, v, ksp, vsp, dense_mask, n_prefix, chunk_bounds, sparse_offsets, l_cap=None):
    """Mixed KV with pooled sparse rows: the prefix, then per chunk its dense rows (mask 1) or its
    pooled rows (mask 0).  k, v [Hkv, N, D] and ksp, vsp [Hkv, S_total, D] in one dtype, copied bit
    for bit.  Returns (kmix, vmix [B, Hkv, Lcap, D], mix_len [B] int32, src_idx [B, Lcap] int32:
    the token id of a dense row, -1 - (pooled row index) of a pooled row, padding -(2**31))."""
    dense_mask = np.asarray(dense_mask)
    b = np.asarray(chunk_bounds, dtype=np.int64)
    off = np.asarray(sparse_offsets, dtype=np.int64)
    bsz = dense_mask.shape[0]
    srcs = []
    for bi in range(bsz):
        parts = [np.arange(n_prefix, dtype=np.int64)]
        for c in range(len(b) - 1):
            parts.append(np.arange(b[c], b[c + 1], dtype=np.int64) if dense_mask[bi, c]
                         else -1 - np.arange(off[c], off[c + 1], dtype=np.int64))
        srcs.append(np.concatenate(parts))
    lens = np.array([len(s) for s in srcs], dtype=np.int32)
    l_cap = int(lens.max()) if l_cap is None else int(l_cap)
    assert l_cap >= lens.max()
    hkv, _, d = k.shape
    kmix = np.zeros((bsz, hkv, l_cap, d), dtype=k.dtype)
    vmix = np.zeros((bsz, hkv, l_cap, d), dtype=v.dtype)
    src_idx = np.full((bsz, l_cap), -(2 ** 31), dtype=np.int64)
    for bi, s in enumerate(srcs):
        dense = s >= 0
        rows = np.flatnonzero(dense)
        kmix[bi][:, rows] = k[:, s[dense]]
        vmix[bi][:, rows] = v[:, s[dense]]
        rows = np.flatnonzero(~dense)
        kmix[bi][:, rows] = ksp[:, -1 - s[~dense]]
        vmix[bi][:, rows] = vsp[:, -1 - s[~dense]]
        src_idx[bi, :len(s)] = s
    return kmix, vmix, lens, src_idx.astype(np.int64)
