"""Chunk-based pre-filling attention, by definition (test infrastructure).

Paper: Method, "Chunk-based Pre-filling" and its figure caption.  For every query head h
(sharing KV head g = h // (Hq / Hkv)) and every token i,

    O[h, i, :] = sum_{j in A(i)} softmax_j( scale * q_{h,i} . k_{g,j} ) * v_{g,j}

with the allowed set A(i) of `sets.allowed_mask`.  Two forms that must agree:

  prefill_def  one explicit N-column score row block per head, masked with the boolean matrix
               of the set definition;
  prefill_blk  per chunk, the explicit list of visible key ids (prefix, kept ids of earlier
               chunks, own chunk) and an explicit score block with the intra-chunk causal mask.

`window` > 0 adds the dense look-back range of the sliding chunk window (see sets.allowed_mask).

Inputs are float arrays in the caller's storage precision; all arithmetic is float64.
"""
import numpy as np

from .sets import allowed_mask, allowed_keys


def _softmax_rows(s):
    """Row softmax of a float64 matrix that may hold -inf (every row has a finite entry)."""
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    return e / l, (m + np.log(l))[:, 0]


def prefill_def(q, k, v, n_prefix, chunk_bounds, sparse_idx, scale=None, rows=None,
                row_block=512, return_lse=False, return_probs=False, window=0):
    """O[Hq, len(rows), D] (float64) straight from the set definition.

    q [Hq, N, D]; k, v [Hkv, N, D]; rows = query token ids to evaluate (default all).
    return_probs additionally returns the [Hq, len(rows), N] attention probabilities
    (tiny inputs only)."""
    hq, n, d = q.shape
    hkv = k.shape[0]
    assert hq % hkv == 0
    grp = hq // hkv
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    rows = np.arange(n) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.zeros((hq, len(rows), d), dtype=np.float64)
    lse = np.zeros((hq, len(rows)), dtype=np.float64)
    probs = np.zeros((hq, len(rows), n), dtype=np.float64) if return_probs else None
    k64 = np.asarray(k, dtype=np.float64)
    v64 = np.asarray(v, dtype=np.float64)
    for r0 in range(0, len(rows), row_block):
        rr = rows[r0:r0 + row_block]
        mask = allowed_mask(rr, n_prefix, chunk_bounds, sparse_idx, window)
        for h in range(hq):
            g = h // grp
            s = scale * (np.asarray(q[h, rr], dtype=np.float64) @ k64[g].T)
            s[~mask] = -np.inf
            p, l = _softmax_rows(s)
            out[h, r0:r0 + len(rr)] = p @ v64[g]
            lse[h, r0:r0 + len(rr)] = l
            if return_probs:
                probs[h, r0:r0 + len(rr)] = p
    res = (out,)
    if return_lse:
        res += (lse,)
    if return_probs:
        res += (probs,)
    return res[0] if len(res) == 1 else res


def prefill_blk(q, k, v, n_prefix, chunk_bounds, sparse_offsets, sparse_idx, scale=None,
                rows=None, heads=None, return_lse=False, window=0):
    """Same result as prefill_def, organised chunk by chunk (usable at long sequence lengths).

    rows  = query token ids to evaluate (default all), any order; heads = query heads
    (default all).  Returns O[len(heads), len(rows), D] float64 (and LSE[len(heads), len(rows)])
    in the order of `rows`.
    """
    hq, n, d = q.shape
    hkv = k.shape[0]
    grp = hq // hkv
    scale = 1.0 / np.sqrt(d) if scale is None else float(scale)
    b = np.asarray(chunk_bounds, dtype=np.int64)
    rows = np.arange(n) if rows is None else np.asarray(rows, dtype=np.int64)
    heads = list(range(hq)) if heads is None else list(heads)
    out = np.zeros((len(heads), len(rows), d), dtype=np.float64)
    lse = np.zeros((len(heads), len(rows)), dtype=np.float64)
    seg_of = np.searchsorted(b, rows, side="right") - 1                 # -1 = prefix
    for c in np.unique(seg_of):
        sel = np.nonzero(seg_of == c)[0]
        rr = rows[sel]
        lo, hi = (0, n_prefix) if c < 0 else (int(b[c]), int(b[c + 1]))
        hist = allowed_keys(int(c), n_prefix, chunk_bounds, sparse_offsets, sparse_idx, window)
        own = np.arange(lo, hi, dtype=np.int64)
        keys = np.concatenate([hist, own])
        # history keys are all visible; own-chunk key j is visible to query i iff j <= i
        visible = np.concatenate(
            [np.ones((len(rr), len(hist)), dtype=bool), own[None, :] <= rr[:, None]], axis=1)
        for hi_, h in enumerate(heads):
            g = h // grp
            kk = np.asarray(k[g, keys], dtype=np.float64)
            vv = np.asarray(v[g, keys], dtype=np.float64)
            s = scale * (np.asarray(q[h, rr], dtype=np.float64) @ kk.T)
            s[~visible] = -np.inf
            p, l = _softmax_rows(s)
            out[hi_, sel] = p @ vv
            lse[hi_, sel] = l
    return (out, lse) if return_lse else out
