"""Index sets of the method (test infrastructure; see the package docstring).

Token layout: ids 0..P-1 are the system/text prefix; chunk c holds ids b[c]..b[c+1]-1 with
b[0] = P and b[C] = N; S_c is the ascending list of kept (sparse) token ids of chunk c, given
in CSR form (sparse_offsets[C+1], sparse_idx[S_total]).
"""
import numpy as np


def allowed_mask(rows, n_prefix, chunk_bounds, sparse_idx):
    """Boolean [len(rows), N]: entry (r, j) says whether query token rows[r] may attend to key j.

    Pre-filling figure caption + text: the chunk being processed attends to itself, to the
    system prompt and to the kept tokens of preceding chunks; inside a chunk (and inside the
    prefix) attention is causal.  As a set, for query i in chunk c:
        A(i) = [0, P)  u  (S_0 u ... u S_{c-1})  u  [b_c, i]
    and A(i) = [0, i] for a prefix token.
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
    return (j <= i) & (same_segment | in_prefix | kept_earlier)


def allowed_keys(c, n_prefix, chunk_bounds, sparse_offsets, sparse_idx):
    """Key ids visible to chunk c before its own tokens: prefix, then kept ids of chunks < c.
    c = -1 denotes the prefix itself (nothing precedes it)."""
    if c < 0:
        return np.zeros(0, dtype=np.int64)
    hist = np.asarray(sparse_idx, dtype=np.int64)[: int(sparse_offsets[c])]
    return np.concatenate([np.arange(n_prefix, dtype=np.int64), hist])


def allowed_pair_count(n_prefix, chunk_bounds, sparse_offsets):
    """Number of (query, key) pairs the pre-filling mask allows, in closed form:
    P(P+1)/2 + sum_c [ len_c (P + off_c) + len_c (len_c + 1) / 2 ]."""
    b = np.asarray(chunk_bounds, dtype=np.int64)
    off = np.asarray(sparse_offsets, dtype=np.int64)
    p = int(n_prefix)
    total = p * (p + 1) // 2
    for c in range(len(b) - 1):
        ln = int(b[c + 1] - b[c])
        total += ln * (p + int(off[c])) + ln * (ln + 1) // 2
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
