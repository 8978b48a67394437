"""ctypes binding of libvxl.so: the same entry points as include/vxl.h, argument marshalling
only.  Every step of the path runs in the HIP kernels of the library; torch is used for device
memory and streams.  Loading fails loudly when the library has not been built -- there is no
fallback path."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np
import torch  # imported before the library so that both use the one HIP runtime torch loaded

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libvxl.so")

VXL_OK, VXL_ERR_INVALID_ARG, VXL_ERR_UNSUPPORTED, VXL_ERR_WORKSPACE, VXL_ERR_HIP, VXL_ERR_ALLOC = range(6)
VXL_F32, VXL_BF16 = 0, 1
OP_PREFILL, OP_SCORE_TOPK, OP_GATHER, OP_DECODE, OP_SCORE_MASS, OP_DECODE_INPLACE = range(6)
MAX_CHUNKS = 4096


class AttnDesc(C.Structure):
    _fields_ = [("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("softmax_scale", C.c_float), ("reserved", C.c_int32),
                ("q_stride_head", C.c_int64), ("q_stride_tok", C.c_int64),
                ("kv_stride_head", C.c_int64), ("kv_stride_tok", C.c_int64)]


class VxlError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().vxl_status_string(status).decode()
        extra = lib().vxl_last_error().decode() if status == VXL_ERR_HIP else ""
        super().__init__(f"{where}: {msg}" + (f" ({extra})" if extra else ""))


_lib = None


def lib() -> C.CDLL:
    """The loaded library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2506_19225_amd.build` "
                           "(or __graft_entry__.build()) first; there is no fallback path")
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    dp = C.POINTER(AttnDesc)
    L.vxl_version.restype = C.c_int
    L.vxl_status_string.restype = C.c_char_p
    L.vxl_status_string.argtypes = [C.c_int]
    L.vxl_last_error.restype = C.c_char_p
    L.vxl_layout_create.restype = C.c_int
    L.vxl_layout_create.argtypes = [i32, i32, i32, vp, vp, vp, vp, C.POINTER(vp)]
    L.vxl_layout_create_windowed.restype = C.c_int
    L.vxl_layout_create_windowed.argtypes = [i32, i32, i32, vp, vp, vp, i32, vp, C.POINTER(vp)]
    L.vxl_layout_destroy.restype = C.c_int
    L.vxl_layout_destroy.argtypes = [vp]
    L.vxl_workspace_bytes.restype = sz
    L.vxl_workspace_bytes.argtypes = [C.c_int, vp, dp, i32, i32, i32]
    L.vxl_mixed_kv_capacity.restype = i32
    L.vxl_mixed_kv_capacity.argtypes = [vp, i32]
    L.vxl_prefill_pair_count.restype = C.c_int64
    L.vxl_prefill_pair_count.argtypes = [vp]
    L.vxl_chunk_prefill.restype = C.c_int
    L.vxl_chunk_prefill.argtypes = [vp, dp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.vxl_chunk_score_topk.restype = C.c_int
    L.vxl_chunk_score_topk.argtypes = [vp, dp, vp, i32, i32, vp, i32, vp, i32, vp, vp, vp, vp, sz, vp]
    L.vxl_chunk_score_topk_mass.restype = C.c_int
    L.vxl_chunk_score_topk_mass.argtypes = [vp, dp, vp, i32, i32, vp, i32, vp, vp, vp, vp, sz, vp]
    L.vxl_gather_bilevel_kv.restype = C.c_int
    L.vxl_gather_bilevel_kv.argtypes = [vp, dp, vp, vp, vp, i32, vp, vp, i32, vp, vp, vp]
    L.vxl_pool_sparse_kv.restype = C.c_int
    L.vxl_pool_sparse_kv.argtypes = [vp, dp, vp, vp, vp, vp, vp]
    L.vxl_gather_bilevel_kv_pooled.restype = C.c_int
    L.vxl_gather_bilevel_kv_pooled.argtypes = [vp, dp, vp, vp, vp, vp, vp, i32, vp, vp, i32, vp, vp, vp]
    L.vxl_kv_store_create.restype = C.c_int
    L.vxl_kv_store_create.argtypes = [vp, dp, C.POINTER(vp)]
    L.vxl_kv_store_destroy.restype = C.c_int
    L.vxl_kv_store_destroy.argtypes = [vp]
    L.vxl_kv_store_host_bytes.restype = sz
    L.vxl_kv_store_host_bytes.argtypes = [vp]
    L.vxl_kv_store_offload.restype = C.c_int
    L.vxl_kv_store_offload.argtypes = [vp, vp, vp, vp, vp, vp]
    L.vxl_kv_store_reload.restype = C.c_int
    L.vxl_kv_store_reload.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, vp]
    L.vxl_bilevel_decode.restype = C.c_int
    L.vxl_bilevel_decode.argtypes = [dp, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    L.vxl_bilevel_decode_inplace.restype = C.c_int
    L.vxl_bilevel_decode_inplace.argtypes = [vp, dp, vp, i32, i32, vp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, sz, vp]
    L.vxl_bilevel_decode_static.restype = C.c_int
    L.vxl_bilevel_decode_static.argtypes = [dp, vp, i32, i32, vp, vp, i32, vp, vp, vp, vp]
    L.vxl_debug_force_simple.argtypes = [C.c_int]
    L.vxl_debug_prefill_variant.argtypes = [C.c_int]
    L.vxl_debug_prefill_events.argtypes = [vp, vp]
    L.vxl_debug_decode_step_waves.argtypes = [C.c_int]
    L.vxl_debug_mfma_stream.argtypes = [vp, C.c_int, C.c_int, vp]
    L.vxl_debug_mfma_stream.restype = C.c_double
    L.vxl_debug_mfma_stream_random.argtypes = [vp, C.c_int, C.c_int, vp]
    L.vxl_debug_mfma_stream_random.restype = C.c_double
    L.vxl_debug_tile_loop_bytes.argtypes = [C.c_int]
    L.vxl_debug_tile_loop_bytes.restype = sz
    L.vxl_debug_tile_loop.argtypes = [C.c_int, vp, vp, C.c_int, C.c_int, vp]
    L.vxl_debug_tile_loop.restype = C.c_double
    L.vxl_debug_read_stream.argtypes = [vp, sz, vp, C.c_int, vp]
    L.vxl_debug_read_stream.restype = C.c_int
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != VXL_OK:
        raise VxlError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def make_desc(n_q_heads: int, n_kv_heads: int, head_dim: int, dtype, softmax_scale: float = 0.0,
              token_major: bool = False) -> AttnDesc:
    """token_major: Q/O are stored [N, Hq, D] and K/V [N, Hkv, D] instead of head-major."""
    if dtype in (torch.bfloat16, "bf16", VXL_BF16):
        code = VXL_BF16
    elif dtype in (torch.float32, "f32", VXL_F32):
        code = VXL_F32
    else:
        raise ValueError(f"unsupported dtype {dtype}")
    if token_major:
        return AttnDesc(n_q_heads, n_kv_heads, head_dim, code, float(softmax_scale), 0,
                        head_dim, n_q_heads * head_dim, head_dim, n_kv_heads * head_dim)
    return AttnDesc(n_q_heads, n_kv_heads, head_dim, code, float(softmax_scale), 0, 0, 0, 0, 0)


def torch_dtype(desc: AttnDesc):
    return torch.bfloat16 if desc.dtype == VXL_BF16 else torch.float32


class Layout:
    """Owns a vxl_layout handle (vxl_layout_create[_windowed] / vxl_layout_destroy)."""

    def __init__(self, n_prefix: int, chunk_bounds, sparse_offsets, sparse_idx, stream=None,
                 n_tokens: Optional[int] = None, window: int = 0):
        self.bounds = np.ascontiguousarray(chunk_bounds, dtype=np.int32)
        self.soff = np.ascontiguousarray(sparse_offsets, dtype=np.int32)
        self.sidx = np.ascontiguousarray(sparse_idx, dtype=np.int32)
        self.n_prefix = int(n_prefix)
        self.n_chunks = len(self.bounds) - 1
        self.n_tokens = int(self.bounds[-1]) if n_tokens is None else int(n_tokens)
        handle = C.c_void_p()
        self.window = int(window)
        if self.window == 0:
            st = lib().vxl_layout_create(
                self.n_tokens, self.n_prefix, self.n_chunks, self.bounds.ctypes.data, self.soff.ctypes.data,
                self.sidx.ctypes.data if self.sidx.size else None, _stream(stream), C.byref(handle))
        else:
            st = lib().vxl_layout_create_windowed(
                self.n_tokens, self.n_prefix, self.n_chunks, self.bounds.ctypes.data, self.soff.ctypes.data,
                self.sidx.ctypes.data if self.sidx.size else None, self.window, _stream(stream),
                C.byref(handle))
        _check(st, "vxl_layout_create")
        self.handle = handle

    def close(self) -> None:
        if getattr(self, "handle", None):
            lib().vxl_layout_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def mixed_kv_capacity(self, k: int) -> int:
        return int(lib().vxl_mixed_kv_capacity(self.handle, int(k)))

    def pair_count(self) -> int:
        return int(lib().vxl_prefill_pair_count(self.handle))


def workspace_bytes(op: int, layout: Optional[Layout], desc: AttnDesc, batch: int = 0,
                    n_q_tokens: int = 0, l_cap: int = 0) -> int:
    return int(lib().vxl_workspace_bytes(op, layout.handle if layout is not None else None,
                                         C.byref(desc), batch, n_q_tokens, l_cap))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def chunk_prefill(layout: Layout, desc: AttnDesc, q, k, v, out, lse=None, workspace=None, stream=None):
    """vxl_chunk_prefill: q/out [Hq,N,D], k/v [Hkv,N,D]; lse float32 [Hq,N] or None."""
    st = lib().vxl_chunk_prefill(layout.handle, C.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                 _ptr(lse), _ptr(workspace), workspace.numel() if workspace is not None else 0,
                                 _stream(stream))
    _check(st, "vxl_chunk_prefill")
    return out


def chunk_score_topk(layout: Layout, desc: AttnDesc, qd, k, top_k: int, topk_idx, dense_mask,
                     scores=None, kbar=None, kbar_ready: bool = False, workspace=None, stream=None):
    """vxl_chunk_score_topk: qd [B,T,Hq,D]; topk_idx int32 [B,min(k,C)]; dense_mask uint8 [B,C]."""
    b, t = int(qd.shape[0]), int(qd.shape[1])
    st = lib().vxl_chunk_score_topk(layout.handle, C.byref(desc), _ptr(qd), b, t, _ptr(k), int(top_k),
                                    _ptr(kbar), int(bool(kbar_ready)), _ptr(topk_idx), _ptr(dense_mask),
                                    _ptr(scores), _ptr(workspace),
                                    workspace.numel() if workspace is not None else 0, _stream(stream))
    _check(st, "vxl_chunk_score_topk")


def chunk_score_topk_mass(layout: Layout, desc: AttnDesc, qd, k, top_k: int, topk_idx, dense_mask,
                          scores=None, workspace=None, stream=None):
    """vxl_chunk_score_topk_mass: arguments as chunk_score_topk, softmax attention-mass score."""
    b, t = int(qd.shape[0]), int(qd.shape[1])
    st = lib().vxl_chunk_score_topk_mass(layout.handle, C.byref(desc), _ptr(qd), b, t, _ptr(k), int(top_k),
                                         _ptr(topk_idx), _ptr(dense_mask), _ptr(scores), _ptr(workspace),
                                         workspace.numel() if workspace is not None else 0, _stream(stream))
    _check(st, "vxl_chunk_score_topk_mass")


def gather_bilevel_kv(layout: Layout, desc: AttnDesc, k, v, dense_mask, kmix, vmix, mix_len,
                      src_idx=None, stream=None):
    """vxl_gather_bilevel_kv: kmix/vmix [B,Hkv,Lcap,D]; mix_len int32 [B]; src_idx int32 [B,Lcap]."""
    b, l_cap = int(kmix.shape[0]), int(kmix.shape[2])
    st = lib().vxl_gather_bilevel_kv(layout.handle, C.byref(desc), _ptr(k), _ptr(v), _ptr(dense_mask), b,
                                     _ptr(kmix), _ptr(vmix), l_cap, _ptr(mix_len), _ptr(src_idx),
                                     _stream(stream))
    _check(st, "vxl_gather_bilevel_kv")


def pool_sparse_kv(layout: Layout, desc: AttnDesc, k, v, ksp, vsp, stream=None):
    """vxl_pool_sparse_kv: k/v [Hkv,N,D] -> ksp/vsp [Hkv,S_total,D]."""
    st = lib().vxl_pool_sparse_kv(layout.handle, C.byref(desc), _ptr(k), _ptr(v), _ptr(ksp), _ptr(vsp),
                                  _stream(stream))
    _check(st, "vxl_pool_sparse_kv")


def gather_bilevel_kv_pooled(layout: Layout, desc: AttnDesc, k, v, ksp, vsp, dense_mask, kmix, vmix, mix_len,
                             src_idx=None, stream=None):
    """vxl_gather_bilevel_kv_pooled: as gather_bilevel_kv, sparse rows taken from ksp/vsp."""
    b, l_cap = int(kmix.shape[0]), int(kmix.shape[2])
    st = lib().vxl_gather_bilevel_kv_pooled(layout.handle, C.byref(desc), _ptr(k), _ptr(v), _ptr(ksp), _ptr(vsp),
                                            _ptr(dense_mask), b, _ptr(kmix), _ptr(vmix), l_cap, _ptr(mix_len),
                                            _ptr(src_idx), _stream(stream))
    _check(st, "vxl_gather_bilevel_kv_pooled")


def bilevel_decode(desc: AttnDesc, qd, kmix, vmix, mix_len, out, lse=None, workspace=None, stream=None):
    """vxl_bilevel_decode: qd/out [B,T,Hq,D]; kmix/vmix [B,Hkv,Lcap,D]; mix_len int32 [B]."""
    b, t = int(qd.shape[0]), int(qd.shape[1])
    l_cap = int(kmix.shape[2])
    st = lib().vxl_bilevel_decode(C.byref(desc), _ptr(qd), b, t, _ptr(kmix), _ptr(vmix), l_cap,
                                  _ptr(mix_len), _ptr(out), _ptr(lse), _ptr(workspace),
                                  workspace.numel() if workspace is not None else 0, _stream(stream))
    _check(st, "vxl_bilevel_decode")
    return out


def bilevel_decode_inplace(layout: Layout, desc: AttnDesc, qd, k, v, ksp, vsp, dense_mask, l_cap: int, out,
                           lse=None, mix_len=None, workspace=None, map_ready: bool = False, stream=None):
    """vxl_bilevel_decode_inplace: gather-free decode; ksp/vsp [Hkv,S_total,D] or None (kept rows in place)."""
    b, t = int(qd.shape[0]), int(qd.shape[1])
    st = lib().vxl_bilevel_decode_inplace(layout.handle, C.byref(desc), _ptr(qd), b, t, _ptr(k), _ptr(v), _ptr(ksp),
                                          _ptr(vsp), _ptr(dense_mask), int(l_cap), int(bool(map_ready)), _ptr(out), _ptr(lse),
                                          _ptr(mix_len), _ptr(workspace),
                                          workspace.numel() if workspace is not None else 0, _stream(stream))
    _check(st, "vxl_bilevel_decode_inplace")
    return out


STATIC_SCRATCH_BYTES = 32 << 20


def bilevel_decode_static(desc: AttnDesc, qd, kmix, vmix, mix_len, out, lse=None, stream=None):
    """vxl_bilevel_decode_static: vxl_bilevel_decode without a workspace (the library's static scratch)."""
    b, t = int(qd.shape[0]), int(qd.shape[1])
    l_cap = int(kmix.shape[2])
    st = lib().vxl_bilevel_decode_static(C.byref(desc), _ptr(qd), b, t, _ptr(kmix), _ptr(vmix), l_cap,
                                         _ptr(mix_len), _ptr(out), _ptr(lse), _stream(stream))
    _check(st, "vxl_bilevel_decode_static")
    return out


class KvStore:
    """Owns a vxl_kv_store handle: pinned host copies of one layer's dense and sparse K/V."""

    def __init__(self, layout: Layout, desc: AttnDesc):
        handle = C.c_void_p()
        _check(lib().vxl_kv_store_create(layout.handle, C.byref(desc), C.byref(handle)), "vxl_kv_store_create")
        self.handle = handle
        self.n_chunks = layout.n_chunks

    def close(self) -> None:
        if getattr(self, "handle", None):
            lib().vxl_kv_store_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def host_bytes(self) -> int:
        return int(lib().vxl_kv_store_host_bytes(self.handle))

    def offload(self, k, v, ksp=None, vsp=None, stream=None) -> None:
        _check(lib().vxl_kv_store_offload(self.handle, _ptr(k), _ptr(v), _ptr(ksp), _ptr(vsp), _stream(stream)),
               "vxl_kv_store_offload")

    def reload(self, dense_mask_host: np.ndarray, kmix, vmix, mix_len=None, stream=None) -> np.ndarray:
        """dense_mask_host: numpy uint8 [B, C]; returns the mixed lengths (numpy int32 [B])."""
        m = np.ascontiguousarray(dense_mask_host, dtype=np.uint8)
        b, l_cap = int(kmix.shape[0]), int(kmix.shape[2])
        assert m.shape == (b, self.n_chunks)
        lens = np.zeros((b,), dtype=np.int32)
        st = lib().vxl_kv_store_reload(self.handle, m.ctypes.data if m.size else None, b, _ptr(kmix), _ptr(vmix),
                                       l_cap, lens.ctypes.data, _ptr(mix_len), _stream(stream))
        _check(st, "vxl_kv_store_reload")
        return lens


def debug_force_simple(on: bool) -> None:
    """Route BF16 calls through the plain vector-ALU kernels (on-device cross-check)."""
    lib().vxl_debug_force_simple(int(bool(on)))


def debug_mfma_stream(out, n_workgroups: int, iters: int, stream=None) -> float:
    """Measurement only: launches a register-resident matrix-instruction stream; returns its FLOP count."""
    return float(lib().vxl_debug_mfma_stream(_ptr(out), int(n_workgroups), int(iters), _stream(stream)))


def debug_mfma_stream_random(out, n_workgroups: int, iters: int, stream=None) -> float:
    """Measurement only: the same stream with pseudo-random bf16 operands that change every instruction."""
    return float(lib().vxl_debug_mfma_stream_random(_ptr(out), int(n_workgroups), int(iters), _stream(stream)))


def debug_tile_loop_bytes(n_workgroups: int) -> int:
    return int(lib().vxl_debug_tile_loop_bytes(int(n_workgroups)))


def debug_tile_loop(mode: int, kv, out, n_workgroups: int, n_tiles: int, stream=None) -> float:
    """Measurement only: the pre-filling tile loop on LDS-resident tiles (mode: see vxl_debug.h); returns its FLOP count."""
    return float(lib().vxl_debug_tile_loop(int(mode), _ptr(kv), _ptr(out), int(n_workgroups), int(n_tiles), _stream(stream)))


def debug_read_stream(src, nbytes: int, out, n_workgroups: int, stream=None) -> None:
    """Measurement only: a bare streaming read of the first nbytes of `src` (out: float32 [n_workgroups*256])."""
    _check(lib().vxl_debug_read_stream(_ptr(src), int(nbytes), _ptr(out), int(n_workgroups), _stream(stream)),
           "vxl_debug_read_stream")


def debug_decode_step_waves(waves: int) -> None:
    """Measurement / cross-check: 0 = the library chooses, 8 = single-buffered 8-wave step kernel,
    4 = double-buffered 4-wave step kernel.  Size the workspace after setting it."""
    lib().vxl_debug_decode_step_waves(int(waves))


def debug_prefill_variant(variant: int) -> None:
    """Cross-check only: 0 = the default instance (8 waves, one workgroup per compute unit);
    1 = the same kernel as two independent 4-wave workgroups per compute unit."""
    lib().vxl_debug_prefill_variant(int(variant))


def debug_prefill_events(start: Optional[torch.cuda.Event], stop: Optional[torch.cuda.Event]) -> None:
    """Measurement hook: record the two events (created with enable_timing=True and already
    recorded once, so that their handles exist) around the main pre-filling kernel of every
    following vxl_chunk_prefill; (None, None) switches it off."""
    lib().vxl_debug_prefill_events(start.cuda_event if start is not None else None,
                                   stop.cuda_event if stop is not None else None)


# ---------------------------------------------------------------------------------------------
# host <-> device marshalling of the storage dtypes (numpy has no bfloat16)
# ---------------------------------------------------------------------------------------------
def to_device(x: np.ndarray, dtype: str, device="cuda") -> torch.Tensor:
    """float32 numpy array holding storage-precision values -> device tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    if dtype == "bf16":
        return t.to(torch.bfloat16).to(device)     # exact: values are bf16-representable
    return t.to(device)


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()
