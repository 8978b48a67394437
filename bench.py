#!/usr/bin/env python3
"""Benchmark of the whole hot path on one MI355X.

Default workload: "config3", the 28-layer stack of 7B-class GQA attention over 10,240 frames
(256 prefix + 163,840 visual tokens in 640 chunks), the largest configuration that one GPU holds.
The K and V of all 28 layers (9.4 GB) and their Q and O stay resident in HBM.  One step = one
pass of the whole hot path over that input:
    28 x vxl_chunk_prefill (one call per layer)
    vxl_chunk_score_topk at layer 0 (per-chunk mean keys recomputed; the selection is reused)
    28 x (vxl_gather_bilevel_kv -> vxl_bilevel_decode, the T query tokens in one call).
`--workload config1|config2|config4` runs the single-layer workloads the same way (one layer).
Inputs are resident in HBM before the timed region.  `value` = effective pre-filling FLOPs
(4 * D * Hq * allowed pairs, all layers) divided by the time of the WHOLE step.  The roofline
object is for the dominant kernel (the matrix-core pre-filling kernel), timed live with events
recorded around every launch of it on the launch stream.  After the timed region the script also
measures, separately, the bandwidth-bound calls (gather; decode in step mode T=1 and batched) on
buffers rotated through more than the on-package cache, the 28-layer decode step over the 28
resident mixed KV sets, short pre-filling runs of the other workloads, and the CPU oracle on a
bounded sample.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import hashlib
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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="config3", choices=["config1", "config2", "config3", "config4"])
    ap.add_argument("--layers", type=int, default=0, help="config3 only: run this many of its 28 layers (0 = all)")
    ap.add_argument("--prefill-variant", type=int, default=0,
                    help="cross-check: 1 = the pre-filling kernel as two 4-wave workgroups per compute unit")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the separate gather/decode measurements")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (a dispatch of known size against which "
                         "the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled)")
    return ap.parse_args()


def kernel_source_hash():
    """Hash of the sources the pre-filling kernel is built from; a stored HBM-traffic figure is
    only reported while it was measured on these very sources."""
    h = hashlib.sha256()
    for f in ("vxl_prefill.hip", "vxl_mfma.h", "vxl_internal.h"):
        h.update(open(os.path.join(ROOT, "paper_2506_19225_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(workload, kernel_name):
    """HBM bytes per launch of the dominant kernel from the rocprofv3 --pmc runs summarised under
    profiles/ (counters cannot be read inside this process), or None when no figure exists for
    this workload or the kernel sources have changed since it was taken."""
    try:
        rec = json.load(open(os.path.join(ROOT, "profiles", "traffic.json")))
        ent = rec.get(workload, {}).get(kernel_name)
        if isinstance(ent, dict) and ent.get("source_hash") == kernel_source_hash():
            return float(ent["bytes_per_launch"])
    except Exception:
        pass
    return None


def cpu_baseline(w, lay, q, k, v):
    """The float64 oracle, as it stands, on a bounded sample of the same workload (one layer)."""
    import oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    # sample: all rows of chunks {0, C/2, C-1}, every query head; grown until ~12 s are spent
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
            "sample": f"oracle.prefill_blk on all rows of {len(used)} of {c_n} chunks of layer 0 (first, middle, "
                      f"last, then a seeded permutation) x all {w.n_q_heads} query heads: {pairs_done} allowed "
                      f"pairs in {t_spent:.1f} s"}


def make_inputs(torch, vxl, wl, w, lay, n_layers):
    """Device-resident Q, K, V and decode queries of every layer.  config3 is drawn on the device
    (21 G elements); the single-layer workloads on the host, as the parity tests draw them."""
    qs, ks, vs, qds = [], [], [], []
    for layer in range(n_layers):
        if w.name == "config3":
            q, k, v = wl.make_qkv_device(w, lay, layer)
            qd = wl.make_decode_queries_device(w, layer)
        else:
            hq, hk, hv = wl.make_qkv(w, lay, layer)
            q, k, v = (vxl.to_device(x, w.dtype) for x in (hq, hk, hv))
            qd = vxl.to_device(wl.make_decode_queries(w, layer), w.dtype)
        qs.append(q); ks.append(k); vs.append(v); qds.append(qd)
    return qs, ks, vs, qds


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
    n_layers = w.n_layers if not args.layers else min(args.layers, w.n_layers)
    gl = vxl.Layout(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    desc = vxl.make_desc(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    dqs, dks, dvs, dqds = make_inputs(torch, vxl, wl, w, lay, n_layers)
    B, T, C, D, Hq, Hkv = w.B, w.T, lay.n_chunks, w.head_dim, w.n_q_heads, w.n_kv_heads
    top_k = w.k
    l_cap = gl.mixed_kv_capacity(top_k)

    outs = [torch.empty_like(q) for q in dqs]
    ws_pre = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
    ws_sc = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_SCORE_TOPK, gl, desc, B, T))
    ws_de = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, B, T, l_cap))
    idx = torch.zeros((B, min(top_k, C)), dtype=torch.int32, device="cuda")
    mask = torch.zeros((B, C), dtype=torch.uint8, device="cuda")
    kmixes = [torch.zeros((B, Hkv, l_cap, D), dtype=dks[0].dtype, device="cuda") for _ in range(n_layers)]
    vmixes = [torch.zeros_like(kmixes[0]) for _ in range(n_layers)]
    mix_lens = [torch.zeros((B,), dtype=torch.int32, device="cuda") for _ in range(n_layers)]
    ods = [torch.empty_like(qd) for qd in dqds]

    def step(events=None):
        for l in range(n_layers):
            if events is not None:
                vxl.debug_prefill_events(*events[l])
            vxl.chunk_prefill(gl, desc, dqs[l], dks[l], dvs[l], outs[l], None, ws_pre)
        # the dense chunks are selected at layer 0 and the selection is reused by every layer
        vxl.chunk_score_topk(gl, desc, dqds[0], dks[0], top_k, idx, mask, workspace=ws_sc)
        for l in range(n_layers):
            vxl.gather_bilevel_kv(gl, desc, dks[l], dvs[l], mask, kmixes[l], vmixes[l], mix_lens[l])
            vxl.bilevel_decode(desc, dqds[l], kmixes[l], vmixes[l], mix_lens[l], ods[l], None, ws_de)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_layers)]
          for _ in range(args.steps)]
    for per_step in ev:        # materialise the event handles
        for a, b in per_step:
            a.record()
            b.record()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for per_step in ev:
        step(per_step)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    vxl.debug_prefill_events(None, None)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    kernel_ms = float(np.mean([a.elapsed_time(b) for per_step in ev for a, b in per_step]))   # per launch = per layer
    pairs = gl.pair_count()
    flops_layer = 4.0 * D * Hq * pairs
    eff_flops = flops_layer * n_layers
    value = eff_flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops_layer / (kernel_ms * 1e-3) / 1e12
    mixlen = int(mix_lens[0].cpu()[0])

    kernel_name = "prefill_dma_kernel"
    result = {
        "metric": "chunk-prefill effective TFLOP/s over the whole hot-path step "
                  "(prefill + score/top-k + gather + decode, all layers)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "layers": n_layers, "n_tokens": lay.n_tokens,
                   "n_prefix": lay.n_prefix, "n_chunks": C, "q_heads": Hq, "kv_heads": Hkv, "head_dim": D,
                   "decode_tokens": T, "top_k": top_k, "mixed_kv_len": mixlen, "allowed_pairs_per_layer": pairs,
                   "effective_flops": eff_flops,
                   "resident_kv_bytes": int(sum(k.numel() + v.numel() for k, v in zip(dks, dvs)) * 2)},
        "roofline": {"bound": "mfma", "kernel": kernel_name, "achieved": achieved,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                     "traffic": stored_traffic(args.workload, kernel_name), "kernel_ms": kernel_ms,
                     "launches_timed": args.steps * n_layers, "flops_per_launch": flops_layer},
    }

    if not args.no_extras:
        result["decode_all_layers"] = measure_layer_stack_decode(torch, vxl, w, desc, dqds, kmixes, vmixes,
                                                                 mix_lens, l_cap, mixlen)
        for tag, compacted in (("decode_all_layers_in_place", False), ("decode_all_layers_in_place_kept_compacted", True)):
            result[tag] = measure_layer_stack_decode_inplace(torch, vxl, w, gl, desc, dqds, dks, dvs, mask, l_cap,
                                                             mixlen, compacted)
        # the same calls per launch shape, on buffers rotated through > 1 GiB
        shapes = {}
        for name, kk in (("config1", None), ("config2", None), ("config3", None), ("config4_k_all", 1 << 30)):
            wn = name.split("_")[0]
            shapes[name] = bilevel_case(torch, vxl, wl, wn, wl.WORKLOADS[wn].k if kk is None else kk)
        result["bilevel"] = shapes
        result["prefill_other_workloads"] = {n: prefill_only(torch, vxl, wl, n) for n in ("config1", "config2", "config4")
                                             if n != args.workload}
        # a diagnostic, not a result: the same launch on all-zero Q, K, V.  The instruction stream is the
        # same; the chip holds its clock on operands that toggle no wires and lowers it on real data.
        result["prefill_clock_diagnostic"] = {"config2_zero_inputs": prefill_only(torch, vxl, wl, "config2", zero=True),
                                              "note": "same kernel and launch as prefill_other_workloads.config2 (or the "
                                                      "headline at --workload config2); inputs all zero"}
        w1 = wl.WORKLOADS["config1"]
        result["widening"] = measure_widening(torch, vxl, wl, w1)
        result["attained_peaks"] = measure_attained_peaks(torch, vxl)
    if not args.no_cpu_baseline:
        hq, hk, hv = (vxl.to_host(x) for x in (dqs[0], dks[0], dvs[0]))
        result["cpu_baseline"] = cpu_baseline(w, lay, hq, hk, hv)
    print(json.dumps(result))


def prefill_only(torch, vxl, wl, name, steps=10, warmup=3, zero=False):
    """vxl_chunk_prefill alone on another workload's layout (device-drawn values of its scale;
    zero = True: all-zero inputs, for the clock diagnostic only)."""
    w = wl.WORKLOADS[name]
    lay = wl.make_layout(w)
    gl = vxl.Layout(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    desc = vxl.make_desc(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    gen = torch.Generator(device="cuda").manual_seed(w.seed)
    draw = lambda h: (torch.randn((h, lay.n_tokens, w.head_dim), device="cuda", generator=gen)
                      * (0.0 if zero else w.value_scale)).to(torch.bfloat16)
    q, k, v = draw(w.n_q_heads), draw(w.n_kv_heads), draw(w.n_kv_heads)
    out = torch.empty_like(q)
    ws = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_PREFILL, gl, desc))
    for _ in range(warmup):
        vxl.chunk_prefill(gl, desc, q, k, v, out, None, ws)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        b.record()
    torch.cuda.synchronize()
    a0, b0 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a0.record()
    for a, b in ev:
        vxl.debug_prefill_events(a, b)
        vxl.chunk_prefill(gl, desc, q, k, v, out, None, ws)
    b0.record()
    torch.cuda.synchronize()
    vxl.debug_prefill_events(None, None)
    kernel_ms = float(np.mean([a.elapsed_time(b) for a, b in ev]))
    flops = 4.0 * w.head_dim * w.n_q_heads * gl.pair_count()
    return {"call_ms": a0.elapsed_time(b0) / steps, "kernel_ms": kernel_ms, "effective_flops": flops,
            "kernel_TFLOPs": flops / kernel_ms / 1e9, "frac_mfma_peak": flops / kernel_ms / 1e9 / PEAK_BF16_TFLOPS,
            "steps": steps, "warmup": warmup}


def measure_layer_stack_decode(torch, vxl, w, desc, dqds, kmixes, vmixes, mix_lens, l_cap, mixlen):
    """One generated token through every layer: n_layers decode calls (T = 1) over the n_layers
    distinct resident mixed KV sets the timed step has built, replayed from one HIP graph."""
    n_layers = len(kmixes)
    B, D, Hkv, Hq = w.B, w.head_dim, w.n_kv_heads, w.n_q_heads
    q1 = [qd[:, :1].contiguous() for qd in dqds]
    o1 = [torch.empty_like(x) for x in q1]
    ws1 = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE, None, desc, B, 1, l_cap))

    def token():
        for l in range(n_layers):
            vxl.bilevel_decode(desc, q1[l], kmixes[l], vmixes[l], mix_lens[l], o1[l], None, ws1)

    for _ in range(3):
        token()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    reps_in_graph = max(1, 64 // n_layers)
    with torch.cuda.graph(graph):
        for _ in range(reps_in_graph):
            token()
    graph.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    a.record()
    for _ in range(reps):
        graph.replay()
    b.record()
    torch.cuda.synchronize()
    us_token = a.elapsed_time(b) * 1e3 / (reps * reps_in_graph)
    bytes_token = n_layers * (2 * B * Hkv * mixlen * D * 2 + 2 * B * Hq * D * 2)
    return {"layers": n_layers, "us_per_token": us_token, "us_per_layer": us_token / n_layers,
            "bytes_per_token": bytes_token, "GBps": bytes_token / us_token / 1e3,
            "frac_hbm": bytes_token / us_token / 1e3 / PEAK_HBM_GBS, "timing": "HIP graph replay",
            "cache_note": "the mixed KV sets of all layers together exceed the on-package cache only when "
                          "layers x bytes per layer > 256 MiB"}


def measure_layer_stack_decode_inplace(torch, vxl, w, gl, desc, dqds, dks, dvs, mask, l_cap, mixlen, compacted):
    """The same token without mixed buffers: every layer's decode reads the dense rows of the
    selected chunks in that layer's resident K / V and the kept rows of the others where they lie
    (compacted = False) or in a compacted copy [Hkv, S_total, D] of them per layer (True), through
    the row map that the layer's first call left in its workspace."""
    n_layers = len(dks)
    sp = [(None, None)] * n_layers
    if compacted and int(gl.soff[-1]) > 0:
        idx = torch.from_numpy(gl.sidx.astype(np.int64)).cuda()
        sp = [(k_[:, idx].contiguous(), v_[:, idx].contiguous()) for k_, v_ in zip(dks, dvs)]
    B, D, Hkv, Hq = w.B, w.head_dim, w.n_kv_heads, w.n_q_heads
    q1 = [qd[:, :1].contiguous() for qd in dqds]
    o1 = [torch.empty_like(x) for x in q1]
    nbytes = vxl.workspace_bytes(vxl.OP_DECODE_INPLACE, gl, desc, B, 1, l_cap)
    wss = [vxl.alloc_workspace(nbytes) for _ in range(n_layers)]
    for l in range(n_layers):                                  # builds the row maps
        vxl.bilevel_decode_inplace(gl, desc, q1[l], dks[l], dvs[l], sp[l][0], sp[l][1], mask, l_cap, o1[l], None, None,
                                   wss[l])

    def token():
        for l in range(n_layers):
            vxl.bilevel_decode_inplace(gl, desc, q1[l], dks[l], dvs[l], sp[l][0], sp[l][1], mask, l_cap, o1[l], None,
                                       None, wss[l], map_ready=True)

    for _ in range(3):
        token()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    reps_in_graph = max(1, 64 // n_layers)
    with torch.cuda.graph(graph):
        for _ in range(reps_in_graph):
            token()
    graph.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 5
    a.record()
    for _ in range(reps):
        graph.replay()
    b.record()
    torch.cuda.synchronize()
    us_token = a.elapsed_time(b) * 1e3 / (reps * reps_in_graph)
    bytes_token = n_layers * (2 * B * Hkv * mixlen * D * 2 + 2 * B * Hq * D * 2 + B * mixlen * 4)
    return {"layers": n_layers, "us_per_token": us_token, "us_per_layer": us_token / n_layers,
            "bytes_per_token": bytes_token, "GBps": bytes_token / us_token / 1e3,
            "frac_hbm": bytes_token / us_token / 1e3 / PEAK_HBM_GBS, "timing": "HIP graph replay",
            "mixed_buffers": "none (row maps of %d bytes per layer)" % (B * l_cap * 4)}


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
    # the same instruction stream with pseudo-random operands that change every instruction (what the
    # attention kernels feed it): the chip lowers its clock under it
    vxl.debug_mfma_stream_random(out, n_cu, iters)
    torch.cuda.synchronize()
    a.record()
    flops_r = vxl.debug_mfma_stream_random(out, n_cu, iters)
    b.record()
    torch.cuda.synchronize()
    mfma_random = flops_r / (a.elapsed_time(b) * 1e-3) / 1e12
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
    res = {"mfma_bf16_stream_TFLOPs": mfma, "mfma_frac_of_published": mfma / PEAK_BF16_TFLOPS,
           "mfma_bf16_stream_random_operands_TFLOPs": mfma_random,
           "mfma_random_operands_frac_of_published": mfma_random / PEAK_BF16_TFLOPS,
           "copy_1GiB_GBps_read_plus_write": copy, "copy_frac_of_published": copy / PEAK_HBM_GBS}
    # the pre-filling kernel's tile loop on its own, one ingredient at a time (vxl_debug.h): what the matrix
    # instructions alone take on this data, and what LDS operands, softmax and ring refills add
    kvbuf = torch.empty(vxl.debug_tile_loop_bytes(n_cu) // 2, dtype=torch.bfloat16, device="cuda").normal_()
    tl = {}
    n_tiles = 4000
    for tag, mode in (("matrix_instructions_only", 0), ("operands_from_registers", 4), ("no_softmax", 3), ("full_tile_code", 1),
                      ("full_tile_code_with_ring_refills", 2), ("alt_16x16x32_matrix_instructions_only", 7),
                      ("alt_16x16x32_full_tile_code", 5), ("alt_16x16x32_full_tile_code_with_ring_refills", 6)):
        vxl.debug_tile_loop(mode, kvbuf, out, n_cu, n_tiles)
        torch.cuda.synchronize()
        a.record()
        fl = vxl.debug_tile_loop(mode, kvbuf, out, n_cu, n_tiles)
        b.record()
        torch.cuda.synchronize()
        ms = a.elapsed_time(b)
        tl[tag] = {"ns_per_tile": ms * 1e6 / n_tiles, "TFLOPs": fl / (ms * 1e-3) / 1e12,
                   "frac_of_published": fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
    res["prefill_tile_loop"] = tl
    del kvbuf
    # a bare streaming read of one decode call's KV bytes (config1 / config3 layer / config2 / 1 GiB), launches
    # replayed from a graph over distinct regions of a 4 GiB buffer: the floor of a split-KV kernel
    del dst
    big = torch.empty(1 << 30, dtype=torch.float32, device="cuda")          # 4 GiB
    big.normal_()
    sink = torch.empty((n_cu * 4 * 256,), dtype=torch.float32, device="cuda")
    for tag, nbytes in (("8MB", 8388608), ("37MB", 37224448), ("49MB", 48758784), ("1GiB", 1 << 30)):
        n_reg = max(1, min(64, (4 << 30) // nbytes))
        views = [big.view(torch.uint8)[i * nbytes:(i + 1) * nbytes] for i in range(n_reg)]
        best = None
        for wgs in (n_cu, 2 * n_cu, 4 * n_cu):
            for v in views[:2]:
                vxl.debug_read_stream(v, nbytes, sink, wgs)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for v in views:
                    vxl.debug_read_stream(v, nbytes, sink, wgs)
            graph.replay()
            torch.cuda.synchronize()
            a.record()
            graph.replay()
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) * 1e3 / n_reg
            if best is None or us < best[0]:
                best = (us, wgs)
        res[f"read_stream_{tag}"] = {"us": best[0], "GBps": nbytes / best[0] / 1e3,
                                     "frac_of_published": nbytes / best[0] / 1e3 / PEAK_HBM_GBS, "workgroups": best[1]}
    return res


def measure_widening(torch, vxl, wl, w):
    """The calls beyond the four of the step, timed on their own on workload config1: the
    attention-mass relevance score (streams the dense K once) and the pooling of the dense KVs
    into sparse KVs (streams K and V once)."""
    lay = wl.make_layout(w)
    gl = vxl.Layout(lay.n_prefix, lay.chunk_bounds, lay.sparse_offsets, lay.sparse_idx)
    desc = vxl.make_desc(w.n_q_heads, w.n_kv_heads, w.head_dim, w.dtype)
    _, hk, hv = wl.make_qkv(w, lay, with_q=False)
    dk, dv = vxl.to_device(hk, w.dtype), vxl.to_device(hv, w.dtype)
    dqd = vxl.to_device(wl.make_decode_queries(w), w.dtype)
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
    # gather-free decode: the same rows read in place through the row map (built once per query,
    # reused by every token: map_ready) -- kept rows where they lie in K / V, and from a compacted
    # copy of the kept rows [Hkv, S_total, D].  K and V themselves are far larger than the cache
    # only for the long workloads; the figures are per call, after one call that builds the map.
    del kmixes, vmixes
    s_total = int(gl.soff[-1])
    idx = torch.from_numpy(gl.sidx.astype(np.int64)).cuda()
    n_in = int(max(1, min(n_rot, 24)))          # distinct copies of K / V (and of the kept rows) to rotate through
    kvs = [(dk, dv)] + [(dk.clone(), dv.clone()) for _ in range(n_in - 1)]
    sps = [(k_[:, idx].contiguous(), v_[:, idx].contiguous()) if s_total else (None, None) for k_, v_ in kvs]
    for tag, use_sp in (("kept_in_place", False), ("kept_compacted", True)):
        for mode, q_, o_, t_ in (("step", qd1, od1, 1), ("batched", dqd, od, T)):
            wsi = vxl.alloc_workspace(vxl.workspace_bytes(vxl.OP_DECODE_INPLACE, gl, desc, B, t_, l_cap))

            def call(i, ready=True):
                k_, v_ = kvs[i % n_in]
                ks_, vs_ = sps[i % n_in] if use_sp else (None, None)
                vxl.bilevel_decode_inplace(gl, desc, q_, k_, v_, ks_, vs_, mask, l_cap, o_, None, None, wsi,
                                           map_ready=ready)
            try:
                call(0, ready=False)            # builds the row map (the same for every copy)
                us = timed(call, iters)
            except vxl.VxlError as err:
                res[f"decode_inplace_{mode}_{tag}"] = {"error": str(err)}
                continue
            nbytes = kv_bytes + 2 * B * t_ * Hq * D * e + 4 * B * mixlen
            res[f"decode_inplace_{mode}_{tag}"] = {"us_per_call": us, "us_per_token": us / t_,
                                                   "GBps": nbytes / us / 1e3,
                                                   "frac_hbm": nbytes / us / 1e3 / PEAK_HBM_GBS}
    res["inplace_copies_rotated"] = n_in
    return res


if __name__ == "__main__":
    main()
