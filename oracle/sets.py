"""Index sets of the method (test infrastructure; see the package docstring).

Token layout: ids 0..P-1 are the system/text prefix; chunk c holds ids b[c]..b[c+1]-1 with
b[0] = P and b[C] = N; S_c is the ascending list of kept (sparse) token ids of chunk c, given
in CSR form (sparse_offsets[C+1], sparse_idx[S_total]).
"""
import numpy as np


def window_start(c, n_prefix, chunk_bounds, window):
    """First token id of the dense look-back range of chunk c: the `window` tokens before the
    chunk, never reaching into the prefix (which is visible anyway)."""
    return max(int(n_prefix), int(chunk_bounds[c]) - int(window))


def allowed_mask(rows, n_prefix, chunk_bounds, sparse_idx, window=0):
    """Boolean [len(rows), N]: entry (r, j) says whether query token rows[r] may attend to key j.

    Pre-filling figure caption + text: the chunk being processed attends to itself, to the
    system prompt and to the kept tokens of preceding chunks; inside a chunk (and inside the
    prefix) attention is causal.  As a set, for query i in chunk c:
        A(i) = [0, P)  u  (S_0 u ... u S_{c-1})  u  [b_c, i]
    and A(i) = [0, i] for a prefix token.

    window > 0 (same paragraph: the chunk to process is placed by a sliding window with a step
    size, so that it also sees the overlapping part of the preceding chunk in full detail):
    chunk c additionally sees every token of [max(P, b_c - window), b_c), i.e.
        A(i) = [0, P)  u  (S_0 u ... u S_{c-1})  u  [max(P, b_c - window), i].
    """
    b = np.asarray(chunk_bounds, dtype=np.int64)
    assert int(b[0]) == int(n_prefix)
    n = int(b[-1])
    chunk_of = np.searchsorted(b, np.arange(n), side="right") - 1      # -1 for prefix tokens
    kept = np.zeros(n, dtype=bool)
    kept[np.asarray(sparse_idx, dtype=np.int64)] = True
    rows = np.asarray(rows, dtype=np.int64)
    ci = chunk_of[rows][:, None]
    cj = chunk_of[None, :]
    j = np.arange(n)[None, :]
    i = rows[:, None]
    same_segment = (cj == ci)
    in_prefix = (j < n_prefix)
    kept_earlier = kept[None, :] & (cj < ci)
    # start of the dense look-back range of every query row (N = none, for prefix rows)
    lo = np.array([window_start(c, n_prefix, b, window) if c >= 0 else n for c in chunk_of[rows]],
                  dtype=np.int64)[:, None]
    looked_back = (j >= lo) & (ci >= 0)
    return (j <= i) & (same_segment | in_prefix | kept_earlier | looked_back)


def allowed_keys(c, n_prefix, chunk_bounds, sparse_offsets, sparse_idx, window=0):
    """Key ids visible to every token of chunk c before its own tokens, ascending: the prefix,
    the kept ids of chunks < c that lie before the look-back range, then the look-back range.
    c = -1 denotes the prefix itself (nothing precedes it)."""
    if c < 0:
        return np.zeros(0, dtype=np.int64)
    lo = window_start(c, n_prefix, chunk_bounds, window)
    hist = np.asarray(sparse_idx, dtype=np.int64)[: int(sparse_offsets[c])]
    hist = hist[hist < lo]
    return np.concatenate([np.arange(n_prefix, dtype=np.int64), hist,
                           np.arange(lo, int(chunk_bounds[c]), dtype=np.int64)])


def allowed_pair_count(n_prefix, chunk_bounds, sparse_offsets, sparse_idx=None, window=0):
    """Number of (query, key) pairs the pre-filling mask allows, in closed form:
    P(P+1)/2 + sum_c [ len_c (P + off_c) + len_c (len_c + 1) / 2 ]  without a window; with one,
    off_c counts only the kept ids before the look-back range and its length is added."""
    b = np.asarray(chunk_bounds, dtype=np.int64)
    off = np.asarray(sparse_offsets, dtype=np.int64)
    p = int(n_prefix)
    total = p * (p + 1) // 2
    for c in range(len(b) - 1):
        ln = int(b[c + 1] - b[c])
        hist = int(off[c])
        back = 0
        if window > 0:
            lo = window_start(c, p, b, window)
            back = int(b[c]) - lo
            hist = int(np.count_nonzero(np.asarray(sparse_idx, dtype=np.int64)[: int(off[c])] < lo))
        total += ln * (p + hist + back) + ln * (ln + 1) // 2
    return total


def mixed_source_index(dense_mask, n_prefix, chunk_bounds, sparse_offsets, sparse_idx):
    """Source token ids of the mixed KV set of one query, in order.

    Bi-level decoding text: dense KVs are loaded for the relevant chunks, sparse KVs for the
    others, and the reloaded pieces are concatenated.  Order: the prefix, then the chunks in
    temporal order, ids ascending inside a chunk.
    """
    b = np.asarray(chunk_bounds, dtype=np.int64)
    off = np.asarray(sparse_offsets, dtype=np.int64)
    sidx = np.asarray(sparse_idx, dtype=np.int64)
    parts = [np.arange(n_prefix, dtype=np.int64)]
    for c in range(len(b) - 1):
        if dense_mask[c]:
            parts.append(np.arange(b[c], b[c + 1], dtype=np.int64))
        else:
            parts.append(sidx[off[c]:off[c + 1]])
    return np.concatenate(parts)
