"""The entry point that allocates nothing (vxl_bilevel_decode_static): same kernels as
vxl_bilevel_decode with the split-KV partial results in the library's static device array.  Its
output must equal the workspace call's bit for bit -- and the oracle within the stated tolerance --
on two calls in a row, the second smaller than the first (the array keeps the first call's
contents), in step mode and batched; a call that needs more than the array holds is rejected."""
import ctypes as C

import numpy as np
import pytest
import torch

import oracle
from paper_2506_19225_amd import vxl, workloads as wl

from gpu_util import assert_close, desc_of

pytestmark = pytest.mark.gpu


def _case(rng, bsz, t_q, hq, hkv, d, l_cap, lens):
    w = wl.tiny_workload("bf16", hq, hkv, d, T=t_q, B=bsz, k=1, seed=int(rng.integers(1 << 30)))
    rnd = lambda *shape: wl.round_to_bf16(rng.standard_normal(shape).astype(np.float32) * np.float32(0.5))
    return w, rnd(bsz, t_q, hq, d), rnd(bsz, hkv, l_cap, d), rnd(bsz, hkv, l_cap, d), np.array(lens, np.int32)


def _both(w, qd, kmix, vmix, mix_len):
    desc = desc_of(w)
    dqd, dk, dv = (vxl.to_device(x, "bf16") for x in (qd, kmix, vmix))
    dlen = torch.from_numpy(mix_len).cuda()
    l_cap = kmix.shape[2]
    nbytes = vxl.workspace_bytes(vxl.OP_DECODE, None, desc, qd.shape[0], qd.shape[1], l_cap)
    assert nbytes <= vxl.STATIC_SCRATCH_BYTES
    ref, ref_lse = torch.full_like(dqd, float("nan")), torch.full(dqd.shape[:3], float("nan"), device="cuda")
    out, out_lse = torch.full_like(dqd, float("nan")), torch.full(dqd.shape[:3], float("nan"), device="cuda")
    vxl.bilevel_decode(desc, dqd, dk, dv, dlen, ref, ref_lse, vxl.alloc_workspace(nbytes))
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    vxl.bilevel_decode_static(desc, dqd, dk, dv, dlen, out, out_lse)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before          # nothing was allocated or freed
    assert torch.equal(out.view(torch.int16), ref.view(torch.int16)), "static-scratch result differs from the workspace call"
    assert torch.equal(out_lse, ref_lse)
    want, wlse = oracle.decode_lse(qd, kmix, vmix, mix_len)
    assert_close(vxl.to_host(out), want, "bf16", head_axis=2, what="static-scratch decode vs oracle")
    assert np.abs(vxl.to_host(out_lse) - wlse).max() < 2e-2


@pytest.mark.parametrize("t_big,t_small", [(1, 1), (40, 8), (8, 1)], ids=["step", "batched", "batched-then-step"])
def test_static_scratch_decode_two_calls_in_a_row(t_big, t_small):
    rng = np.random.default_rng(900 + t_big)
    # a larger call first (more splits, more rows), then a smaller one on the same device array
    _both(*_case(rng, 2, t_big, 14, 2, 128, 5000, [4999, 3100]))
    _both(*_case(rng, 1, t_small, 14, 2, 128, 900, [777]))
    _both(*_case(rng, 1, t_small, 8, 2, 64, 333, [200]))


def test_static_scratch_decode_rejects_what_does_not_fit():
    """64 queries x 64 tokens over a long mixed set need more partial-result bytes than the array
    holds: VXL_ERR_WORKSPACE on the host, nothing launched (no buffer is dereferenced)."""
    desc = vxl.make_desc(28, 4, 128, "bf16")
    need = vxl.workspace_bytes(vxl.OP_DECODE, None, desc, 64, 64, 65536)
    assert need > vxl.STATIC_SCRATCH_BYTES
    fake = C.c_void_p(0x1000)
    st = vxl.lib().vxl_bilevel_decode_static(C.byref(desc), fake, 64, 64, fake, fake, 65536, fake, fake, None, None)
    assert st == vxl.VXL_ERR_WORKSPACE
    assert b"static scratch" in vxl.lib().vxl_last_error()
