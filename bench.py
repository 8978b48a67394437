#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

One step = one pass of all hot-path calls over one batch of synthetic input (workload
"config1": one 7B-class GQA layer, 256 prefix + 16,384 visual tokens in 64 chunks):
    vxl_chunk_prefill -> vxl_chunk_score_topk (per-chunk mean keys recomputed) ->
    vxl_gather_bilevel_kv -> vxl_bilevel_decode (the T query tokens in one call).
Inputs are resident in HBM before the timed region.  `value` = effective pre-filling FLOPs
(4 * D * Hq * allowed pairs) divided by the time of the WHOLE step.  The roofline object is for
the dominant kernel (the matrix-core pre-filling kernel), timed with events recorded around it
on the launch stream.  After the timed region the script also measures, separately, the
bandwidth-bound calls (gather; decode in step mode T=1 and batched) on buffers rotated through
more than the on-package cache, and times the CPU oracle on a bounded sample.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="config1", choices=["config1", "config2", "config4"])
    ap.add_argument("--prefill-variant", type=int, default=0,
                    help="debug: 1 or 2 = the 4-wave register-staged kernel with 1 or 2 row blocks per wave, "
                         "3 = the software-pipelined 4-wave kernel with 64 rows per wave")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the separate gather/decode measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (a dispatch of known size against which "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled)")
    return ap.parse_args()


def cpu_baseline(w, lay, q, k, v):
    """The float64 oracle, as it stands, on a bounded sample of the same workload."""
    import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    # sample: all rows of chunks {0, C/2, C-1}, every query head; grown until ~10 s are spent
    c_n = lay.n_chunks
    order = [0, c_n // 2, c_n - 1] + [int(c) for c in np.random.default_rng(0).permutation(c_n)]
    pairs_done, t_spent, used = 0, 0.0, []
    for c in order:
        if c in used or c < 0 or c >= c_n:
            continue
        lo, hi = int(lay.chunk_bounds[c]), int(lay.chunk_bounds[c + 1])
        rows = np.arange(lo, hi)
        t0 = time.perf_counter()
        oracle.prefill_blk(q, k, v, lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx, rows=rows)
        t_spent += time.perf_counter() - t0
        ln = hi - lo
        pairs_done += ln * (lay.n_prefix + int(lay.sparse_offsets[c])) + ln * (ln + 1) // 2
        used.append(c)
        if t_spent > 12.0:
            break
    flops = 4.0 * w.head_dim * w.n_q_heads * pairs_done
    return {"value": flops / t_spent / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
            "sample": f"oracle.prefill_blk on all rows of {len(used)} of {c_n} chunks (first, middle, last, then a "
                      f"seeded permutation) x all {w.n_q_heads} query heads: {pairs_done} allowed pairs in "
                      f"{t_spent:.1f} s"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_19225_amd import vxl, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py needs a GPU (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    vxl.lib()
    if args.prefill_variant:
        vxl.debug_prefill_variant(args.prefill_variant)

    w = wl.WORKLOADS[args.workload]
    lay = wl.make_layout(w)
    q, k, v = wl.make_qkv(w, lay)
    qd = wl.make_decode_queries(w)
    gl = vxl.Layout(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    desc = vxl.make_desc(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    dq, dk, dv, dqd = (vxl.to_device(x, w.dtype) for x in (q, k, v, qd))
    B, T, C, D, Hq, Hkv = w.B, w.T, lay.n_chunks, w.head_dim, w.n_q_heads, w.n_kv_heads
    top_k = w.k
    l_cap = gl.mixed_kv_capacity(top_k)

    out = torch.empty_like(dq)
    ws_pre = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
    ws_sc = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_TOPK, gl, desc, B, T))
    ws_de = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, B, T, l_cap))
    idx = torch.zeros((B, min(top_k, C)), dtype=torch.int32, device="cuda")
    mask = torch.zeros((B, C), dtype=torch.uint8, device="cuda")
    kmix = torch.zeros((B, Hkv, l_cap, D), dtype=dk.dtype, device="cuda")
    vmix = torch.zeros_like(kmix)
    mix_len = torch.zeros((B,), dtype=torch.int32, device="cuda")
    od = torch.empty_like(dqd)

    def step():
        vxl.chunk_prefill(gl, desc, dq, dk, dv, out, None, ws_pre)
        vxl.chunk_score_topk(gl, desc, dqd, dk, top_k, idx, mask, workspace=ws_sc)
        vxl.gather_bilevel_kv(gl, desc, dk, dv, mask, kmix, vmix, mix_len)
        vxl.bilevel_decode(desc, dqd, kmix, vmix, mix_len, od, None, ws_de)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for a, b in ev:        # materialise the event handles
        a.record()
        b.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        vxl.debug_prefill_events(a, b)
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    vxl.debug_prefill_events(None, None)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernel_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    pairs = gl.pair_count()
    eff_flops = 4.0 * D * Hq * pairs
    value = eff_flops / (ms_per_step * 1e-3) / 1e12
    achieved = eff_flops / (kernel_ms * 1e-3) / 1e12
    mixlen = int(mix_len.cpu()[0])

    kernel_name = {0: "prefill_dma_kernel", 3: "prefill_pipe_kernel"}.get(args.prefill_variant, "prefill_mfma_kernel")
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(args.workload, {}).get(kernel_name)
        except Exception:
            traffic = None

    result = {
        "metric": "chunk-prefill effective TFLOP/s over the whole hot-path step "
                  "(prefill + score/top-k + gather + decode)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "n_tokens": lay.n_tokens, "n_prefix": lay.n_prefix,
                   "n_chunks": C, "q_heads": Hq, "kv_heads": Hkv, "head_dim": D, "decode_tokens": T,
                   "top_k": top_k, "mixed_kv_len": mixlen, "allowed_pairs": pairs,
                   "effective_flops": eff_flops},
        "roofline": {"bound": "mfma", "kernel": kernel_name, "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": traffic, "kernel_ms": kernel_ms},
    }

    if not args.no_extras:
        result["bilevel"] = measure_bilevel(torch, vxl, w, gl, desc, dk, dv, dqd, mask, l_cap, mixlen)
        # the same calls at the shapes on which the bandwidth-bound claim is made: config1's mixed KV
        # (8 MB) is a launch-latency case, these two move 49 MB and 1.08 GB per decode call
        result["bilevel_large"] = {
            "config2": bilevel_case(torch, vxl, wl, "config2", wl.WORKLOADS["config2"].k),
            "config4_k_all": bilevel_case(torch, vxl, wl, "config4", 1 << 30),
        }
        result["widening"] = measure_widening(torch, vxl, w, lay, gl, desc, dk, dv, dqd)
        # one layer of the 28-layer workload: its 28 decode calls per token read 28 distinct mixed
        # KV sets (1.04 GB), which is what the rotating buffers of the measurement stand for
        c3 = bilevel_case(torch, vxl, wl, "config3", wl.WORKLOADS["config3"].k)
        c3["us_per_token_28_layers"] = 28 * c3["decode_step"]["us_per_token"]
        result["bilevel_large"]["config3_per_layer"] = c3
        result["attained_peaks"] = measure_attained_peaks(torch, vxl)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, lay, q, k, v)
    print(json.dumps(result))


def measure_attained_peaks(torch, vxl):
    """What this box attains on the two rooflines with nothing in the way: a register-resident
    stream of the matrix instruction the kernels use, and a plain 1 GiB device-to-device copy."""
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    out = torch.empty((n_cu * 512,), dtype=torch.float32, device="cuda")
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    iters = 100000
    vxl.debug_mfma_stream(out, n_cu, iters)                   # warm-up (clocks)
    torch.cuda.synchronize()
    a.record()
    flops = vxl.debug_mfma_stream(out, n_cu, iters)
    b.record()
    torch.cuda.synchronize()
    mfma = flops / (a.elapsed_time(b) * 1e-3) / 1e12
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    a.record()
    for _ in range(10):
        dst.copy_(src)
    b.record()
    torch.cuda.synchronize()
    copy = 10 * 2.0 * src.numel() * 4 / (a.elapsed_time(b) * 1e-3) / 1e9
    return {"mfma_bf16_stream_TFLOPs": mfma, "mfma_frac_of_published": mfma / PEAK_BF16_TFLOPS,
            "copy_1GiB_GBps_read_plus_write": copy, "copy_frac_of_published": copy / PEAK_HBM_GBS}


def measure_widening(torch, vxl, w, lay, gl, desc, dk, dv, dqd):
    """The calls beyond the four of the step, timed on their own on the step's workload: the
    attention-mass relevance score (streams the dense K once) and the pooling of the dense KVs
    into sparse KVs (streams K and V once)."""
    B, T, C, D, Hkv = w.B, w.T, lay.n_chunks, w.head_dim, w.n_kv_heads
    e = 2
    idx = torch.zeros((B, min(w.k, C)), dtype=torch.int32, device="cuda")
    mask = torch.zeros((B, C), dtype=torch.uint8, device="cuda")
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_MASS, gl, desc, B, T))
    s_total = int(lay.sparse_offsets[-1])
    ksp = torch.empty((Hkv, max(s_total, 1), D), dtype=dk.dtype, device="cuda")
    vsp = torch.empty_like(ksp)

    def timed(fn, iters=50):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / iters

    us_mass = timed(lambda: vxl.chunk_score_topk_mass(gl, desc, dqd, dk, w.k, idx, mask, None, workspace=ws))
    us_pool = timed(lambda: vxl.pool_sparse_kv(gl, desc, dk, dv, ksp, vsp))
    k_bytes = Hkv * lay.n_tokens * D * e
    pool_bytes = 2 * k_bytes + 2 * Hkv * s_total * D * e
    # offline store: the mixed KV of one query rebuilt from pinned host memory (host link, not HBM)
    store = vxl.KvStore(gl, desc)
    store.offload(dk, dv, ksp, vsp)
    torch.cuda.synchronize()
    hmask = np.zeros((B, C), dtype=np.uint8)
    hmask[:, :min(w.k, C)] = 1
    l_cap = gl.mixed_kv_capacity(w.k)
    kmix = torch.empty((B, Hkv, l_cap, D), dtype=dk.dtype, device="cuda")
    vmix = torch.empty_like(kmix)
    mlen = torch.zeros((B,), dtype=torch.int32, device="cuda")
    lens = store.reload(hmask, kmix, vmix, mlen)
    us_reload = timed(lambda: store.reload(hmask, kmix, vmix, mlen), iters=20)
    reload_bytes = 2 * Hkv * int(lens.sum()) * D * e
    return {"timing": "back-to-back launches, inputs cache-resident where they fit",
            "score_mass": {"us": us_mass, "k_bytes": k_bytes, "GBps": k_bytes / us_mass / 1e3},
            "pool_sparse_kv": {"us": us_pool, "bytes": pool_bytes, "GBps": pool_bytes / us_pool / 1e3},
            "store_reload": {"us": us_reload, "bytes_over_host_link": reload_bytes,
                             "GBps": reload_bytes / us_reload / 1e3, "host_store_bytes": store.host_bytes()}}


def bilevel_case(torch, vxl, wl, name, top_k):
    """Gather / decode measurements on the layout and shapes of another workload.  K, V and the
    queries are seeded device-side normals (the values do not matter to these kernels); the dense
    chunks are the first top_k ones."""
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    gl = vxl.Layout(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    desc = vxl.make_desc(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    gen = torch.Generator(device="cuda").manual_seed(w.seed)
    shape_kv = (w.n_kv_heads, lay.n_tokens, w.head_dim)
    dk = (torch.randn(shape_kv, device="cuda", generator=gen) * 0.088).to(torch.bfloat16)
    dv = (torch.randn(shape_kv, device="cuda", generator=gen) * 0.088).to(torch.bfloat16)
    dqd = (torch.randn((w.B, w.T, w.n_q_heads, w.head_dim), device="cuda", generator=gen) * 0.088).to(torch.bfloat16)
    kk = min(top_k, lay.n_chunks)
    mask = torch.zeros((w.B, lay.n_chunks), dtype=torch.uint8, device="cuda")
    mask[:, :kk] = 1
    l_cap = gl.mixed_kv_capacity(kk)
    mixlen = int(lay.n_prefix + sum(int(lay.chunk_bounds[c + 1] - lay.chunk_bounds[c]) if c < kk
                                    else int(lay.sparse_offsets[c + 1] - lay.sparse_offsets[c])
                                    for c in range(lay.n_chunks)))
    res = measure_bilevel(torch, vxl, w, gl, desc, dk, dv, dqd, mask, l_cap, mixlen)
    res.update({"batch": w.B, "decode_tokens": w.T, "mixed_kv_len": mixlen, "dense_chunks": kk})
    return res


def measure_bilevel(torch, vxl, w, gl, desc, dk, dv, dqd, mask, l_cap, mixlen):
    """Gather and decode timed on their own, rotating through distinct mixed-KV buffers whose total
    size exceeds the on-package cache, so the figures are HBM figures."""
    B, T, D, Hkv, Hq = w.B, w.T, w.head_dim, w.n_kv_heads, w.n_q_heads
    e = 2
    kv_bytes = 2 * B * Hkv * mixlen * D * e                 # K and V read once by a decode call
    n_rot = int(max(2, min(128, (1 << 30) // max(1, kv_bytes) + 1)))
    kmixes = [torch.zeros((B, Hkv, l_cap, D), dtype=dk.dtype, device="cuda") for _ in range(n_rot)]
    vmixes = [torch.zeros_like(kmixes[0]) for _ in range(n_rot)]
    mix_len = torch.zeros((B,), dtype=torch.int32, device="cuda")

    def timed(fn, iters):
        """us per call of fn(i), i = 0..iters-1, replayed from one captured HIP graph (the calls
        are a few microseconds long: launched one by one they would measure the host)."""
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(iters):
                fn(i)
        graph.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 3
        a.record()
        for _ in range(reps):
            graph.replay()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / (iters * reps)

    iters = 2 * n_rot
    us_gather = timed(lambda i: vxl.gather_bilevel_kv(gl, desc, dk, dv, mask, kmixes[i % n_rot],
                                                      vmixes[i % n_rot], mix_len), iters)
    gather_bytes = 2 * kv_bytes                             # read + write, K and V
    res = {"mixed_kv_bytes": kv_bytes, "rotating_buffers": n_rot, "timing": "HIP graph replay",
           "gather": {"us": us_gather, "GBps": gather_bytes / us_gather / 1e3,
                      "frac_hbm": gather_bytes / us_gather / 1e3 / PEAK_HBM_GBS}}
    # decode, batched: all T tokens in one call
    od = torch.empty_like(dqd)
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, B, T, l_cap))
    us_b = timed(lambda i: vxl.bilevel_decode(desc, dqd, kmixes[i % n_rot], vmixes[i % n_rot], mix_len, od,
                                              None, ws), iters)
    bytes_b = kv_bytes + 2 * B * T * Hq * D * e
    flops_b = 4.0 * D * Hq * B * T * mixlen
    res["decode_batched"] = {"tokens_per_call": T, "us_per_call": us_b, "us_per_token": us_b / T,
                             "GBps": bytes_b / us_b / 1e3, "frac_hbm": bytes_b / us_b / 1e3 / PEAK_HBM_GBS,
                             "TFLOPs": flops_b / us_b / 1e6}
    # decode, step mode: one token per call (true autoregressive step)
    qd1 = dqd[:, :1].contiguous()
    od1 = torch.empty_like(qd1)
    ws1 = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, B, 1, l_cap))
    us_s = timed(lambda i: vxl.bilevel_decode(desc, qd1, kmixes[i % n_rot], vmixes[i % n_rot], mix_len, od1,
                                              None, ws1), iters)
    bytes_s = kv_bytes + 2 * B * Hq * D * e
    res["decode_step"] = {"us_per_token": us_s, "GBps": bytes_s / us_s / 1e3,
                          "frac_hbm": bytes_s / us_s / 1e3 / PEAK_HBM_GBS}
    return res


if __name__ == "__main__":
    main()
