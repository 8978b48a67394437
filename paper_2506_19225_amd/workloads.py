"""Seeded synthetic video-token workloads (inputs only; none of the method's arithmetic).

The paper evaluates on long videos: a text/system prefix followed by thousands of frames of
visual tokens, split into equal-length chunks (Method, "Chunk-based Pre-filling"), with a
small kept set of tokens per chunk (the timestamp tokens, which are prepended to each frame
group -- "Temporal Information Injection") and a 7B-class GQA decoder (28 query heads, 4 KV
heads, head dim 128 -- "Model Architecture").  The five workloads below have those shapes with
synthetic Gaussian Q/K/V.  This module is the only code shared by the CPU oracle's tests and
the HIP path's tests: it produces bits, and the same bits go to both.

Storage dtypes: "f32" arrays are float32; "bf16" arrays are float32 values that are exactly
representable in bfloat16 (round-to-nearest-even applied here), so `to_bf16_bits` is lossless.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------------------
# storage-dtype helpers
# --------------------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 -> nearest bfloat16 (ties to even), returned as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    b = x.view(np.uint32).copy()
    b += np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))
    b &= np.uint32(0xFFFF0000)
    return b.view(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 holding bf16-representable values -> uint16 bit patterns (lossless)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """uint16 bfloat16 bit patterns -> float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------------------
# layout: prefix + chunks + per-chunk kept (sparse) token lists
# --------------------------------------------------------------------------------------
@dataclass
class Layout:
    """Token layout of one video prompt.

    n_prefix       P, tokens of the system/text prefix (ids 0..P-1)
    chunk_bounds   int32 [C+1], chunk c = tokens chunk_bounds[c] .. chunk_bounds[c+1]-1,
                   chunk_bounds[0] == P, chunk_bounds[C] == N
    sparse_offsets int32 [C+1] CSR offsets into sparse_idx
    sparse_idx     int32 [S_total] absolute token ids kept for chunk c, ascending
    """
    n_prefix: int
    chunk_bounds: np.ndarray
    sparse_offsets: np.ndarray
    sparse_idx: np.ndarray

    @property
    def n_tokens(self) -> int:
        return int(self.chunk_bounds[-1])

    @property
    def n_chunks(self) -> int:
        return len(self.chunk_bounds) - 1

    def chunk_len(self, c: int) -> int:
        return int(self.chunk_bounds[c + 1] - self.chunk_bounds[c])

    def kept(self, c: int) -> np.ndarray:
        return self.sparse_idx[self.sparse_offsets[c]:self.sparse_offsets[c + 1]]


def layout_from_lists(n_prefix: int, chunk_lens: List[int], kept_lists: List[np.ndarray]) -> Layout:
    bounds = np.concatenate([[n_prefix], n_prefix + np.cumsum(chunk_lens)]).astype(np.int32)
    offs = np.concatenate([[0], np.cumsum([len(k) for k in kept_lists])]).astype(np.int32)
    idx = (np.concatenate(kept_lists).astype(np.int32) if len(kept_lists) and offs[-1] > 0
           else np.zeros(0, np.int32))
    return Layout(int(n_prefix), bounds, offs, idx)


def strided_kept(start: int, length: int, count: int) -> np.ndarray:
    """`count` tokens of a chunk at a constant stride, the first one at the chunk start
    (timestamp tokens are prepended to their frame group)."""
    if count <= 0:
        return np.zeros(0, np.int32)
    stride = length // count
    return (start + stride * np.arange(count)).astype(np.int32)


def random_layout(rng: np.random.Generator, n_prefix: int, n_chunks: int,
                  len_lo: int, len_hi: int, allow_empty_kept: bool = True) -> Layout:
    """Small ragged layouts for edge-case tests: odd chunk lengths, random sorted kept sets."""
    lens = [int(rng.integers(len_lo, len_hi + 1)) for _ in range(n_chunks)]
    kept = []
    start = n_prefix
    for ln in lens:
        lo = 0 if allow_empty_kept else 1
        cnt = int(rng.integers(lo, ln + 1))
        kept.append(np.sort(rng.choice(ln, size=cnt, replace=False)).astype(np.int32) + start)
        start += ln
    return layout_from_lists(n_prefix, lens, kept)


# --------------------------------------------------------------------------------------
# the five workloads
# --------------------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    dtype: str                 # "f32" | "bf16"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    n_layers: int
    n_prefix: int
    tokens_per_frame: int
    n_frames: int
    T: int                     # decode/query tokens per query
    B: int                     # independent queries
    k: int                     # dense chunks (top-k); config 4 also sweeps k_sweep
    seed: int
    value_scale: float
    chunk_frames: Optional[int] = None      # fixed chunk = this many frames
    kept_per_chunk: Optional[int] = None    # fixed count, strided unless kept_random
    kept_random: bool = False
    variable_chunks: bool = False           # workload 4
    k_sweep: Tuple[int, ...] = ()
    planted_fraction: float = 0.0
    note: str = ""

    @property
    def n_visual(self) -> int:
        return self.n_frames * self.tokens_per_frame

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


_INV_SQRT128 = 1.0 / float(np.sqrt(128.0))

WORKLOADS: Dict[str, Workload] = {
    "config0": Workload("config0", "f32", 2, 1, 64, 1, 64, 64, 8, T=8, B=1, k=2, seed=0,
                        value_scale=1.0, chunk_frames=2, kept_per_chunk=16,
                        note="tiny fp32 smoke case"),
    "config1": Workload("config1", "bf16", 28, 4, 128, 1, 256, 64, 256, T=32, B=1, k=8, seed=1,
                        value_scale=_INV_SQRT128, chunk_frames=4, kept_per_chunk=32,
                        note="7B-class GQA layer, 16,384 visual tokens"),
    "config2": Workload("config2", "bf16", 28, 4, 128, 1, 256, 64, 2048, T=64, B=1, k=16, seed=2,
                        value_scale=_INV_SQRT128, chunk_frames=8, kept_per_chunk=64,
                        kept_random=True, note="long video, 131,072 visual tokens"),
    "config3": Workload("config3", "bf16", 28, 4, 128, 28, 256, 16, 10240, T=128, B=1, k=32,
                        seed=3, value_scale=_INV_SQRT128, chunk_frames=16, kept_per_chunk=16,
                        note="28-layer stack, 163,840 visual tokens"),
    "config4": Workload("config4", "bf16", 28, 4, 128, 1, 256, 64, 1024, T=32, B=8, k=4, seed=4,
                        value_scale=_INV_SQRT128, variable_chunks=True, k_sweep=(4, 32, -1),
                        planted_fraction=0.05, note="variable chunks, planted relevance"),
}


def make_layout(w: Workload) -> Layout:
    """Chunk bounds and kept lists of a workload (seeded, deterministic)."""
    rng = np.random.default_rng([w.seed, 0x1A70])
    if not w.variable_chunks:
        clen = w.chunk_frames * w.tokens_per_frame
        assert w.n_visual % clen == 0
        n_chunks = w.n_visual // clen
        lens = [clen] * n_chunks
        kept = []
        for c in range(n_chunks):
            start = w.n_prefix + c * clen
            if w.kept_random:
                sel = np.sort(rng.choice(clen, size=w.kept_per_chunk, replace=False))
                kept.append((start + sel).astype(np.int32))
            else:
                kept.append(strided_kept(start, clen, w.kept_per_chunk))
        return layout_from_lists(w.n_prefix, lens, kept)
    # variable chunks: whole frames, 128..1024 tokens, last chunk truncated to end at N
    tpf = w.tokens_per_frame
    lens, total = [], 0
    while total < w.n_visual:
        ln = int(rng.integers(128 // tpf, 1024 // tpf + 1)) * tpf
        ln = min(ln, w.n_visual - total)
        lens.append(ln)
        total += ln
    ratios = rng.choice([4, 8, 32], size=len(lens))
    kept, start = [], w.n_prefix
    for ln, r in zip(lens, ratios):
        kept.append(strided_kept(start, ln, max(1, ln // int(r))))
        start += ln
    return layout_from_lists(w.n_prefix, lens, kept)


def _normal(rng: np.random.Generator, shape, scale: float) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    return x


def _store(w: Workload, x: np.ndarray) -> np.ndarray:
    return round_to_bf16(x) if w.dtype == "bf16" else np.ascontiguousarray(x, np.float32)


def make_decode_queries(w: Workload, layer: int = 0) -> np.ndarray:
    """Qd[B, T, Hq, D] in the storage dtype."""
    rng = np.random.default_rng([w.seed, layer, 0xDEC0])
    return _store(w, _normal(rng, (w.B, w.T, w.n_q_heads, w.head_dim), w.value_scale))


def planted_chunks(w: Workload, layout: Layout) -> np.ndarray:
    """Ids of the chunks whose K carries the planted relevance shift (workload 4)."""
    if w.planted_fraction <= 0.0:
        return np.zeros(0, np.int64)
    rng = np.random.default_rng([w.seed, 0x91A7])
    n = max(1, int(round(w.planted_fraction * layout.n_chunks)))
    return np.sort(rng.choice(layout.n_chunks, size=n, replace=False))


def make_qkv(w: Workload, layout: Layout, layer: int = 0,
             with_q: bool = True) -> Tuple[Optional[np.ndarray], np.ndarray, np.ndarray]:
    """Q[Hq,N,D], K[Hkv,N,D], V[Hkv,N,D] in the storage dtype (Q is None if not with_q).

    Workload 4: the K rows of the planted chunks are shifted by +0.5 * qbar_g before rounding,
    where qbar_g is the mean of query 0's decode tokens over its T tokens and over the query
    heads that share KV head g.
    """
    n = layout.n_tokens
    rk = np.random.default_rng([w.seed, layer, 0x4B])
    rv = np.random.default_rng([w.seed, layer, 0x56])
    k = _normal(rk, (w.n_kv_heads, n, w.head_dim), w.value_scale)
    v = _normal(rv, (w.n_kv_heads, n, w.head_dim), w.value_scale)
    pl = planted_chunks(w, layout)
    if len(pl):
        qd = make_decode_queries(w, layer)[0]                       # [T, Hq, D]
        g = w.n_q_heads // w.n_kv_heads
        qbar = qd.reshape(w.T, w.n_kv_heads, g, w.head_dim).mean(axis=(0, 2), dtype=np.float64)
        for c in pl:
            lo, hi = int(layout.chunk_bounds[c]), int(layout.chunk_bounds[c + 1])
            k[:, lo:hi, :] += (0.5 * qbar[:, None, :]).astype(np.float32)
    q = None
    if with_q:
        rq = np.random.default_rng([w.seed, layer, 0x51])
        q = _store(w, _normal(rq, (w.n_q_heads, n, w.head_dim), w.value_scale))
    return q, _store(w, k), _store(w, v)


def tiny_workload(dtype: str, hq: int, hkv: int, d: int, T: int, B: int, k: int, seed: int,
                  value_scale: float = 1.0) -> Workload:
    """A free-form small workload for edge-case tests (layout supplied separately)."""
    return Workload(f"tiny{seed}", dtype, hq, hkv, d, 1, 0, 1, 0, T=T, B=B, k=k, seed=seed,
                    value_scale=value_scale)


# --------------------------------------------------------------------------------------
# device-side draws for the workloads that are too large to draw on the host
# --------------------------------------------------------------------------------------
def _device_normal(shape, scale: float, dtype: str, seed: int, device):
    """N(0,1) * scale drawn by torch's counter-based generator on `device`, rounded once to the
    storage dtype.  Drawn in slabs along the first axis to bound the fp32 temporary."""
    import torch
    gen = torch.Generator(device=device).manual_seed(int(seed))
    out = torch.empty(shape, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device=device)
    for i in range(shape[0]):
        x = torch.randn(shape[1:], dtype=torch.float32, device=device, generator=gen)
        if scale != 1.0:
            x *= scale
        out[i].copy_(x)                     # bf16: round to nearest even, once
    return out


def _device_seed(w: Workload, layer: int, tag: int) -> int:
    return ((w.seed * 1_000_003 + layer) << 8) + tag


def make_qkv_device(w: Workload, layout: Layout, layer: int = 0, with_q: bool = True, device="cuda"):
    """Q[Hq,N,D], K[Hkv,N,D], V[Hkv,N,D] as DEVICE tensors in the storage dtype, independent seeded
    Gaussians per layer with the value scale of the workload (the 28-layer workload draws 21 G
    elements: minutes on the host, a second on the device).  The values differ from make_qkv's
    (another generator); a test hands the oracle a host copy of exactly these tensors, so both
    sides still compute on the same bits.  Workloads with a planted signal are drawn on the host."""
    assert w.planted_fraction == 0.0, "planted workloads are drawn by make_qkv"
    n = layout.n_tokens
    k = _device_normal((w.n_kv_heads, n, w.head_dim), w.value_scale, w.dtype, _device_seed(w, layer, 0x4B), device)
    v = _device_normal((w.n_kv_heads, n, w.head_dim), w.value_scale, w.dtype, _device_seed(w, layer, 0x56), device)
    q = None
    if with_q:
        q = _device_normal((w.n_q_heads, n, w.head_dim), w.value_scale, w.dtype, _device_seed(w, layer, 0x51), device)
    return q, k, v


def make_q_device(w: Workload, layout: Layout, layer: int = 0, device="cuda"):
    """Q[Hq,N,D] of make_qkv_device alone (the same bits), for callers that keep K and V of many
    layers resident and draw one layer's Q at a time."""
    return _device_normal((w.n_q_heads, layout.n_tokens, w.head_dim), w.value_scale, w.dtype,
                          _device_seed(w, layer, 0x51), device)


def make_decode_queries_device(w: Workload, layer: int = 0, device="cuda"):
    """Qd[B, T, Hq, D] as a device tensor in the storage dtype (see make_qkv_device)."""
    return _device_normal((w.B, w.T, w.n_q_heads, w.head_dim), w.value_scale, w.dtype,
                          _device_seed(w, layer, 0xDE), device)
