#!/usr/bin/env python3
"""Benchmark of the routed-attention hot path on one MI355X.

A "step" is one decode token of the Llama-3-8B-shaped workload (the second of the five workloads in workloads/configs.py): for each of
the 32 layers, owner layers append the new token's K/V row to their slot (skv_kv_append), then
every layer attends over the slot it is routed to (skv_attn_decode: split-K kernel + merge).
`value` is the algorithmic HBM traffic of the step divided by its wall time.  The causal prefill
workload (the third workload) is measured after it and reported in the "prefill" object of the
same JSON line, because the metric names both.  A third object, "train", times one R-CLA
training pass (Sec. 3.2: sampled route, forward and backward of the attention of every layer) on
the same shape; it is a widening of the path and no part of `value`.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
SETTLE_STEPS = 6          # untimed decode steps after a cache fill, before the warm-up steps (see run_decode)
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


TRAFFIC_FILE = os.path.join("profiles", "hbm_traffic.json")
# sources a kernel is built from: the committed counter summary names their hash, and a summary
# taken from other sources than the ones on disk is not reported
KERNEL_SOURCES = {
    "decode_mfma_kernel": ["decode_mfma.hip"], "append_rows_kernel": ["append.hip"],
    "prefill_pipe_kernel": ["prefill_pipe.hip", "gen_prefill_pipe.py"],
    "dkdv_kernel": ["train_bwd.hip"], "dq_kernel": ["train_bwd.hip"], "delta_kernel": ["train_bwd.hip"],
    "project_append_tile_kernel": ["project_append.hip"], "project_append_kernel": ["project_append.hip"],
    "project_finish_kernel": ["project_append.hip"], "project_small_kernel": ["project_append.hip"],
}


def source_sha(kernel):
    import hashlib
    h = hashlib.sha256()
    for f in KERNEL_SOURCES.get(kernel.split("@")[0], []):
        h.update(open(os.path.join(ROOT, "paper_2604_22782_amd", "csrc", f), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(kernel):
    """HBM bytes per launch of `kernel` (or "kernel@workload" for a launch shape other than the
    headline's) from the committed rocprofv3 counter summary, or None if there is none for the
    kernel's present sources."""
    try:
        t = json.load(open(os.path.join(ROOT, TRAFFIC_FILE)))[kernel]
        if t.get("source_sha16") != source_sha(kernel):
            return None
        return int(t["FETCH_SIZE"]["bytes"] + t["WRITE_SIZE"]["bytes"])
    except Exception:
        return None


def traffic_fields(kernels):
    """`traffic` is not measured by this run (counters need the profiler): it is the committed
    rocprofv3 FETCH_SIZE + WRITE_SIZE summary of the same command, valid only for unchanged sources."""
    parts = [measured_traffic(k) for k in kernels]
    ok = all(p is not None for p in parts)
    return {"traffic": sum(parts) if ok else None,
            "traffic_source": f"{TRAFFIC_FILE} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
                              f"command; " + ("kernel sources unchanged since)" if ok else "none for the present sources)")}


def cpu_baseline_decode(w, seconds_budget=12.0):
    """The float64 oracle, as it stands, on a bounded sample of the decode workload."""
    import torch
    from oracle import skv_oracle as O
    from workloads import gen
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    n_seq = 2
    lens = w.kv_lens[:n_seq]
    n = int(lens.max())
    layer = 1                                   # a routed (non-owner) layer
    src = O.validate_route(w.route)[layer]
    cache = O.Cache([0], n_seq, n, w.n_kv_heads, w.head_dim, np.uint16)
    k = w.kv_rows("k", src, 0, n_seq, 0, n, "cpu")
    v = w.kv_rows("v", src, 0, n_seq, 0, n, "cpu")
    cache.append(0, gen.to_f64(k), gen.to_f64(v), gen.to_bits(k), gen.to_bits(v), np.zeros(n_seq, int), lens)
    q = gen.to_f64(w.q_decode(layer, "cpu")[:n_seq])
    O.decode(cache, 0, q, lens, w.scale)        # warm
    reps, t0 = 0, time.perf_counter()
    while True:
        O.decode(cache, 0, q, lens, w.scale)
        reps += 1
        dt = time.perf_counter() - t0
        if dt > seconds_budget or reps >= 2000:
            break
    row = w.n_kv_heads * w.head_dim * w.elem_bytes
    bytes_per_call = int(lens.sum()) * 2 * row + 2 * n_seq * w.n_q_heads * w.head_dim * w.elem_bytes
    return {"value": round(bytes_per_call * reps / dt / 1e9, 4), "unit": "GB/s", "cores": int(cores),
            "kind": "oracle",
            "sample": f"oracle decode() of 1 routed layer over {n_seq} of {w.batch} sequences x {w.n_q_heads} "
                      f"heads x {n} keys, repeated {reps}x ({dt:.1f} s); bytes counted as for the GPU (16-bit K/V)"}


def _newest_rows(w, which, l, ctx):
    """The K/V row of each sequence's newest position."""
    import torch
    if int(w.kv_lens.min()) == ctx:
        return w.kv_rows(which, l, 0, w.batch, ctx - 1, ctx, "cuda")
    return torch.cat([w.kv_rows(which, l, b, b + 1, int(n) - 1, int(n), "cuda") for b, n in enumerate(w.kv_lens)])


def run_decode(args, torch, skv, H, w, steps, warmup, headline=False):
    """One decode token per step over all layers of workload w: owner layers append the new K/V row,
    every layer attends over its routed slot.  Returns the step rate and the roofline of the call."""
    log(f"[bench] workload {w.name}: B={w.batch} ctx={int(w.kv_lens.max())} layers={w.n_layers} slots={len(w.owner_layers)}")
    cache, _ = H.alloc_cache(w)
    t0 = time.perf_counter()
    # the fill's temporaries grow with the row width: keep them at the size they have for 8 kv heads
    chunk = max(1 << 14, args.fill_chunk_tokens * 1024 // (w.n_kv_heads * w.head_dim))
    if skv.skv_cache_info(cache)[3] * 2 > 128 << 30:      # little memory is left beside the cache
        chunk = min(chunk, 1 << 15)
    H.fill_by_append(cache, w, lens=w.kv_lens - 1, chunk_tokens=chunk)
    log(f"[bench] cache of {skv.skv_cache_info(cache)[3] * 2 / 2**30:.1f} GiB filled through skv_kv_append in {time.perf_counter() - t0:.1f} s")
    ctx = int(w.kv_lens.max())
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    d_start = (d_lens - 1).to(torch.int32)
    ones = torch.ones(w.batch, dtype=torch.int32, device="cuda")
    ws = H.workspace_for(cache, ctx)
    qs = [w.q_decode(l, "cuda") for l in range(w.n_layers)]
    new_k = {l: _newest_rows(w, "k", l, ctx) for l in w.owner_layers}
    new_v = {l: _newest_rows(w, "v", l, ctx) for l in w.owner_layers}
    outs = [torch.empty_like(qs[0]) for _ in range(w.n_layers)]

    def step():
        for l in range(w.n_layers):
            if l in new_k:
                skv.skv_kv_append(cache, l, new_k[l], new_v[l], d_start, ones, 1)
            skv.skv_attn_decode(cache, l, qs[l], outs[l], d_lens, ctx, w.scale, ws)

    # Part of the set-up, like the fill: the first steps over a freshly written cache run up to 80 % slower
    # (5.2, 3.4, 3.1, 3.0, 2.9, 2.9 ... ms on the 8-bit headline workload) while memory clocks and address
    # translation settle; the metric is the steady rate.
    for _ in range(SETTLE_STEPS):
        step()
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    kernel_name = skv.skv_last_kernel_name()
    # Dominant kernel: two HIP events on the launch stream around a region of back-to-back decode calls of
    # all layers (each call = the kernel, plus the clearing and merge launches where the key axis is
    # split), without the appends.  Events around every single call would add their own 3-5 us to a call
    # of 90-160 us (the record is a packet of its own between two launches).
    reps = max(3, min(steps, 10))
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        for l in range(w.n_layers):
            skv.skv_attn_decode(cache, l, qs[l], outs[l], d_lens, ctx, w.scale, ws)
    e1.record()
    torch.cuda.synchronize()
    call_ms = e0.elapsed_time(e1) / (reps * w.n_layers)
    assert skv.skv_cache_device_faults(cache) == 0
    layer_bytes = w.decode_bytes_per_layer()
    # the new rows are read in the activation dtype and written in the slot's element type
    stored = (w.head_dim + 1) if w.kv8 else w.head_dim * w.elem_bytes
    append_bytes = len(w.owner_layers) * 2 * w.batch * w.n_kv_heads * (w.head_dim * w.elem_bytes + stored)
    step_bytes = layer_bytes * w.n_layers + append_bytes
    ms_per_step = dt / steps * 1e3
    value = step_bytes / (dt / steps) / 1e9
    achieved = layer_bytes / (call_ms * 1e-3) / 1e9
    roof = {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4)}
    roof.update(traffic_fields([kernel_name if headline else f"{kernel_name}@{w.name}_b{w.batch}"]))
    roof.update({"launch_us": round(call_ms * 1e3, 2), "algorithmic_bytes_per_launch": layer_bytes})
    res = {"value": round(value, 1), "ms_per_step": round(ms_per_step, 4), "steps": steps, "roofline": roof,
           "config": {"workload": w.name, "batch": w.batch, "max_context": ctx, "layers": w.n_layers,
                      "q_heads": w.n_q_heads, "kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                      "slots": len(w.owner_layers), "sum_kv_len": int(w.kv_lens.sum()), "paged": bool(w.block_size),
                      "dtype": w.dtype, "slots_dtype": "e4m3 + power-of-two scale per (position, kv head)" if w.kv8 else w.dtype,
                      "step": "append(owner)+decode per layer"}}
    cache.free()
    del ws, qs, outs, new_k, new_v
    torch.cuda.empty_cache()
    return res


def run_append(args, torch, skv, H, configs):
    """The cache update of the owner layers (Alg. 2, "Update") alone, against the HBM copy roofline:
    the rows of a whole prompt (the prefill workload: 4 x 8192 rows of 2 KiB, K and V: 128 MiB read and
    128 MiB written per owner layer) and of one decode token (the decode workload: 64 rows).
    Algorithmic bytes = new rows x 2 (K, V) x row bytes, read once and written once."""
    out = {}
    for regime, w, new in (("prompt", configs.llama3_prefill(), None), ("decode_token", configs.llama3_decode(n_layers=8), 1)):
        S = int(w.kv_lens.max())
        new = S if new is None else new
        cache, _ = H.alloc_cache(w)
        owners = w.owner_layers
        # sources and destination slots rotate so that no launch finds its rows in the on-chip caches
        n_src = 4 if regime == "prompt" else len(owners)
        k_new = [w.kv_rows("k", owners[i % len(owners)], 0, w.batch, S - new, S, "cuda") for i in range(n_src)]
        v_new = [w.kv_rows("v", owners[i % len(owners)], 0, w.batch, S - new, S, "cuda") for i in range(n_src)]
        start = torch.full((w.batch,), S - new, dtype=torch.int32, device="cuda")
        lens = torch.full((w.batch,), new, dtype=torch.int32, device="cuda")
        reps = 40 if regime == "prompt" else 400
        for i in range(8):
            skv.skv_kv_append(cache, owners[i % len(owners)], k_new[i % n_src], v_new[i % n_src], start, lens, new)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(reps):
            skv.skv_kv_append(cache, owners[i % len(owners)], k_new[i % n_src], v_new[i % n_src], start, lens, new)
        e1.record()
        torch.cuda.synchronize()
        assert skv.skv_cache_device_faults(cache) == 0
        us = e0.elapsed_time(e1) / reps * 1e3
        nbytes = 2 * (w.batch * new * 2 * w.n_kv_heads * w.head_dim * w.elem_bytes)
        gbs = nbytes / (us * 1e-6) / 1e9
        out[regime] = {"workload": w.name, "rows": w.batch * new, "launch_us": round(us, 2),
                       "roofline": {"bound": "hbm", "kernel": "append_rows_kernel", "achieved": round(gbs, 1),
                                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                                    **traffic_fields([f"append_rows_kernel@{regime}"]),
                                    "algorithmic_bytes_per_launch": nbytes}}
        log(f"[bench] append {regime}: {us:.1f} us, {gbs:.0f} GB/s")
        cache.free()
        del k_new, v_new
        torch.cuda.empty_cache()
    return out


def run_small_launches(args, torch, skv, H, configs):
    """Decode bandwidth against the size of the launch: the decode workload's shape with 1 .. 64
    sequences of 4096 positions per launch (16 MiB .. 1 GiB of K and V), through
    skv_attn_decode_range.  Launches rotate over the 16 slots and over the sequences, so every launch
    reads rows that were last touched at least 1 GiB of traffic ago (nothing is found on chip)."""
    w = configs.llama3_decode()
    cache, _ = H.alloc_cache(w)
    H.fill_by_append(cache, w, chunk_tokens=args.fill_chunk_tokens)
    ctx = int(w.kv_lens.max())
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    q = w.q_decode(0, "cuda")
    out = torch.empty_like(q)
    row = w.n_kv_heads * w.head_dim * w.elem_bytes
    points = []
    for n_seq in (1, 2, 4, 8, 16, 32, 64):
        ws = torch.empty(skv.skv_decode_range_workspace_bytes(cache, n_seq, ctx) // 4 + 1, dtype=torch.float32, device="cuda")
        launches = []
        for i in range(64):            # (layer, first sequence): 64 distinct slices, >= 1 GiB apart in time
            layer = (2 * i) % w.n_layers
            b0 = ((i // 16) * n_seq) % w.batch if n_seq < w.batch else 0
            launches.append((layer, b0))
        def run():
            for layer, b0 in launches:
                skv.skv_attn_decode_range(cache, layer, b0, n_seq, q[b0:], out[b0:], d_lens[b0:], ctx, w.scale, ws)
        run()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 3
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / (reps * len(launches)) * 1e3
        nbytes = n_seq * ctx * 2 * row + 2 * n_seq * w.n_q_heads * w.head_dim * w.elem_bytes
        points.append({"sequences": n_seq, "launch_MiB": round(n_seq * ctx * 2 * row / 2**20, 1), "launch_us": round(us, 2),
                       "GB/s": round(nbytes / (us * 1e-6) / 1e9, 1), "frac": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)})
        log(f"[bench] small launch {points[-1]}")
        del ws
    assert skv.skv_cache_device_faults(cache) == 0
    cache.free()
    torch.cuda.empty_cache()
    return {"shape": "llama3_8b decode: 32 q / 8 kv heads, d 128, 4096 positions per sequence, bf16; "
                     "launch_us includes the merge launch where the key axis is split", "points": points}


def run_cross_layer_reuse(args, torch, skv, H, configs):
    """The closing remark of Sec. 4.3: the layers of a sharing group read the same K, V, so a backend
    could serve the later ones from on-chip memory.  At the sizes of the paper's own benchmark (Tab. 4:
    batch 1, 2K .. 32K positions; Tab. 5: 8K positions, batch 2 .. 16; Qwen3-8B heads; groups of 2, 4, 8)
    a layer's slice of its slot is 8 .. 512 MiB, around the 256 MiB memory-side cache of the device.
    Per point: a stack of n_groups x g layers (enough groups that their slices together exceed 1 GiB,
    so the first reader of a group always finds its slice in HBM only), one decode token through all
    layers in order, HIP events around every call; reported per reader position within the group."""
    import math as _m
    points = []
    row = 8 * 128 * 2
    grid = [(1, T, 4) for T in (2048, 8192, 16384, 32768)] + [(B, 8192, 4) for B in (2, 4, 8, 16)] + \
           [(1, 8192, 2), (1, 8192, 8), (4, 8192, 2), (4, 8192, 8)]
    for batch, ctx, g in grid:
        slice_bytes = batch * ctx * 2 * row
        n_groups = max(2, _m.ceil((1 << 30) / slice_bytes) + 1)
        L = n_groups * g
        w = configs.Workload(f"reuse_b{batch}_t{ctx}_g{g}", "bf16", L, 32, 8, 128, batch, configs.grouped_route(L, g),
                             np.full(batch, ctx), 1.0, 0.5, seed=1100 + g)
        cache, _ = H.alloc_cache(w)
        H.fill_by_append(cache, w, chunk_tokens=args.fill_chunk_tokens)
        d_lens = torch.from_numpy(w.kv_lens).cuda()
        ws = H.workspace_for(cache, ctx)
        q = [w.q_decode(l % 8, "cuda") for l in range(8)]
        out = torch.empty_like(q[0])
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(L)]

        def one_pass(timed):
            for l in range(L):
                if timed:
                    ev[l][0].record()
                skv.skv_attn_decode(cache, l, q[l % 8], out, d_lens, ctx, w.scale, ws)
                if timed:
                    ev[l][1].record()
        one_pass(False)
        per = [[] for _ in range(g)]
        for _ in range(3):
            one_pass(True)
            torch.cuda.synchronize()
            for l in range(L):
                per[l % g].append(ev[l][0].elapsed_time(ev[l][1]) * 1e3)
        assert skv.skv_cache_device_faults(cache) == 0
        nbytes = w.decode_bytes_per_layer()
        first = float(np.mean(per[0]))
        later = float(np.mean([x for r in per[1:] for x in r]))
        group_us = first + (g - 1) * later
        points.append({"batch": batch, "ctx": ctx, "g": g, "slice_MiB": round(slice_bytes / 2**20, 1), "groups": n_groups,
                       "first_reader_us": round(first, 2), "later_readers_us": round(later, 2),
                       "first_reader_GB/s": round(nbytes / first / 1e3, 1), "later_readers_GB/s": round(nbytes / later / 1e3, 1),
                       "group_GB/s": round(g * nbytes / group_us / 1e3, 1)})
        log(f"[bench] reuse {points[-1]}")
        cache.free()
        del ws, q, out
        torch.cuda.empty_cache()
    return {"note": "GB/s = algorithmic bytes of a call / its time between HIP events (kernel + merge launch); above the "
                    "8000 GB/s HBM peak means the slice came from on-chip memory; FETCH_SIZE per reader: "
                    "profiles/decode_mfma_kernel_cross_layer_reuse.txt", "points": points}


def mfma_only_rate(torch, skv):
    """TFLOP/s of back-to-back v_mfma_f32_32x32x16_bf16 and nothing else, one wave per SIMD on all
    256 compute units, with all-zero operands and with Gaussian ones (a different operand pair for
    every instruction, as in attention).  The second figure is what the power limit of the device
    leaves of the first."""
    from paper_2604_22782_amd import calib
    blocks, iters = 256, 6000                      # about 3 ms per launch
    sink = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    gen_ = torch.Generator(device="cpu").manual_seed(1234)
    ops = {"zeros": torch.zeros(8192, dtype=torch.bfloat16, device="cuda"),
           "gaussian": torch.randn(8192, generator=gen_).to(torch.bfloat16).cuda()}
    flops = blocks * 4 * iters * 32 * 32768
    out = {}
    # the third figure: Gaussian operands plus, per MFMA and independent of it, the vector
    # instructions of a softmax and the LDS operand reads of the pre-fill kernel (nothing waits
    # for anything: an estimate of what that instruction mix can reach under the power limit)
    for name, t, mix in (("zeros", ops["zeros"], 0), ("gaussian", ops["gaussian"], 0),
                         ("gaussian_with_softmax_and_lds_reads", ops["gaussian"], 3)):
        best = float("inf")
        for rep in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            calib.skv_calib_mfma_mix_bf16(t, sink, blocks, iters, mix)
            e1.record()
            torch.cuda.synchronize()
            if rep >= 2:
                best = min(best, e0.elapsed_time(e1))
        out[name] = round(flops / (best * 1e-3) / 1e12, 1)
    return out


def run_prefill(args, torch, skv, H, configs):
    w = configs.llama3_prefill()
    S = int(w.kv_lens.max())
    log(f"[bench] workload {w.name}: B={w.batch} S={S} layers={w.n_layers} slots={len(w.owner_layers)}")
    cache, _ = H.alloc_cache(w)
    d_lens = torch.from_numpy(w.kv_lens).cuda()
    zeros = torch.zeros(w.batch, dtype=torch.int32, device="cuda")
    # two query/output buffers are rotated over the layers (a full set would be 16 GiB)
    q = [w.q_prefill(l, 0, w.batch, 0, S, "cuda") for l in range(2)]
    out = [torch.empty_like(q[0]) for _ in range(2)]
    k_new = {l: w.kv_rows("k", l, 0, w.batch, 0, S, "cuda") for l in w.owner_layers[:2]}
    v_new = {l: w.kv_rows("v", l, 0, w.batch, 0, S, "cuda") for l in w.owner_layers[:2]}
    owner_src = w.owner_layers[:2]

    def step():
        for l in range(w.n_layers):
            if w.route[l] == l:   # owner: append its K/V rows of all prompt tokens
                src = owner_src[(l // 4) % 2]
                skv.skv_kv_append(cache, l, k_new[src], v_new[src], zeros, d_lens, S)
            skv.skv_attn_prefill(cache, l, q[l % 2], out[l % 2], d_lens, d_lens, S, S, w.scale)

    steps = max(1, args.steps // 10)
    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    # as for decode: two events around a region of back-to-back calls of all layers, without the appends
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for l in range(w.n_layers):
        skv.skv_attn_prefill(cache, l, q[l % 2], out[l % 2], d_lens, d_lens, S, S, w.scale)
    e1.record()
    torch.cuda.synchronize()
    call_ms = e0.elapsed_time(e1) / w.n_layers
    assert skv.skv_cache_device_faults(cache) == 0
    flops = w.prefill_flops_per_layer()
    tflops_kernel = flops / (call_ms * 1e-3) / 1e12
    tflops_step = flops * w.n_layers / dt / 1e12
    res = {"workload": w.name, "config": {"batch": w.batch, "seq_len": S, "layers": w.n_layers,
                                           "slots": len(w.owner_layers), "dtype": w.dtype},
           "steps": steps, "ms_per_step": round(dt * 1e3, 3), "value": round(tflops_step, 1), "unit": "TFLOP/s",
           "roofline": {"bound": "mfma", "kernel": skv.skv_last_kernel_name(), "achieved": round(tflops_kernel, 1),
                        "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(tflops_kernel / MFMA_BF16_PEAK_TFLOPS, 4),
                        **traffic_fields([skv.skv_last_kernel_name()]),
                        "launch_us": round(call_ms * 1e3, 1), "algorithmic_flops_per_launch": flops}}
    cache.free()
    # the published peak is what "frac" is quoted on; the rates an MFMA-only kernel reaches on this
    # device, measured in the same run, say how much of it any kernel can get
    res["roofline"]["mfma_only_tflops"] = mfma_only_rate(torch, skv)
    return res


def run_project(args, torch, skv, H, configs):
    """The owner layers' K/V projection fused with the cache update (Sec. 4.3), timed in the two
    regimes of the path: the prompt of the prefill workload (compute bound) and one decode token
    of the decode workload (bound by reading the weights).  Hidden size 4096 as in Llama-3-8B."""
    hidden = 4096
    out = {}
    for regime, w, new in (("prefill", configs.llama3_prefill(), None), ("decode", configs.llama3_decode(n_layers=2), 1)):
        S = int(w.kv_lens.max())
        new = S if new is None else new
        cache, _ = H.alloc_cache(w)
        g = torch.Generator(device="cuda").manual_seed(7)
        x = torch.randn(w.batch, new, hidden, generator=g, device="cuda").to(torch.bfloat16)
        F = w.n_kv_heads * w.head_dim
        wk = (torch.randn(F, hidden, generator=g, device="cuda") / hidden ** 0.5).to(torch.bfloat16)
        wv = (torch.randn(F, hidden, generator=g, device="cuda") / hidden ** 0.5).to(torch.bfloat16)
        inv = 10000.0 ** (-torch.arange(w.head_dim // 2, device="cuda", dtype=torch.float64) * 2.0 / w.head_dim)
        ang = torch.arange(S, device="cuda", dtype=torch.float64)[:, None] * inv[None, :]
        cos, sin = torch.cos(ang).float().contiguous(), torch.sin(ang).float().contiguous()
        start = torch.full((w.batch,), S - new, dtype=torch.int32, device="cuda")
        lens = torch.full((w.batch,), new, dtype=torch.int32, device="cuda")
        layer = w.owner_layers[0]
        reps = 40 if regime == "prefill" else 200
        warm = 30 if regime == "prefill" else 50     # ~15 ms of load: the clocks need that long to settle after an idle gap
        ws = torch.empty(max(skv.skv_kv_project_workspace_bytes(cache, new, hidden), 4) // 4, dtype=torch.float32, device="cuda")
        for _ in range(warm):
            skv.skv_kv_project_append(cache, layer, x, wk, wv, cos, sin, start, lens, new, ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            skv.skv_kv_project_append(cache, layer, x, wk, wv, cos, sin, start, lens, new, ws)
        e1.record()
        torch.cuda.synchronize()
        assert skv.skv_cache_device_faults(cache) == 0
        us = e0.elapsed_time(e1) / reps * 1e3
        tokens = w.batch * new
        flops = 2 * tokens * hidden * 2 * F
        nbytes = 2 * (2 * F * hidden + tokens * hidden + 2 * tokens * F)     # weights + x read, K/V rows written
        r = {"tokens": tokens, "hidden": hidden, "launch_us": round(us, 1),
             "tflops": round(flops / (us * 1e-6) / 1e12, 1), "gbs": round(nbytes / (us * 1e-6) / 1e9, 1)}
        if regime == "prefill":
            r["roofline"] = {"bound": "mfma", "kernel": "project_append_tile_kernel", "achieved": r["tflops"],
                             "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                             "frac": round(r["tflops"] / MFMA_BF16_PEAK_TFLOPS, 4),
                             **traffic_fields(["project_append_tile_kernel"]),
                             "algorithmic_flops_per_launch": flops}
        else:
            r["roofline"] = {"bound": "hbm", "kernel": "project_small_kernel + project_finish_kernel", "achieved": r["gbs"],
                             "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(r["gbs"] / HBM_PEAK_GBS, 4),
                             **traffic_fields(["project_small_kernel", "project_finish_kernel"]),
                             "algorithmic_bytes_per_launch": nbytes}
        out[regime] = r
        cache.free()
        torch.cuda.empty_cache()
    return out


def run_e2e(args, torch, skv):
    """The sweep of the paper's inference benchmark (Tab. 4: batch 1, input 2048..32768, 128 new
    tokens; Tab. 5: 8192-token context, batch 2..16, 64 new tokens; group sizes 1 and 4) on a
    synthetic Qwen3-8B-scale decoder: KV-cache MiB, peak device memory, time to first token,
    decode tokens/s.  Context for the paper's tables, not part of `value`."""
    from workloads.e2e_decoder import SyntheticDecoder
    rows = []
    for g in (1, 4):
        torch.cuda.empty_cache()
        m = SyntheticDecoder(group=g, seed=7, qk_norm=True)   # Qwen3's block: q and k heads are RMS-normalised
        w_bytes = sum(t.numel() * t.element_size() for t in m.w.values())
        m.start(1, 2048 + 8)                                  # untimed warm-up: library set-up, GEMM heuristics
        nxt = m.prefill(torch.zeros(1, 2048, dtype=torch.int64, device="cuda")).argmax(-1)
        for _ in range(4):
            nxt = m.decode_step(nxt).argmax(-1)
        torch.cuda.synchronize()
        m.close()
        for table, batch, T, new in ([("tab4", 1, T, 128) for T in (2048, 8192, 16384, 32768)] +
                                     [("tab5", B, 8192, 64) for B in (2, 4, 8, 16)]):
            m.start(batch, T + new)
            gen_ = torch.Generator(device="cuda").manual_seed(T + batch)
            tok = torch.randint(0, m.vocab, (batch, T), generator=gen_, device="cuda")
            torch.cuda.reset_peak_memory_stats()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            nxt = m.prefill(tok).argmax(-1)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            half = (new - 1) // 2
            for _ in range(half):                             # eager: one host call per launch
                nxt = m.decode_step(nxt).argmax(-1)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            m.capture_decode()                                # the same step as one HIP graph
            torch.cuda.synchronize()
            t3 = time.perf_counter()
            for _ in range(new - 1 - half):
                nxt = m.decode_step_graph(nxt).argmax(-1)
            torch.cuda.synchronize()
            t4 = time.perf_counter()
            assert skv.skv_cache_device_faults(m.cache) == 0
            kv = m.kv_cache_bytes(T + new)
            rows.append({"table": table, "batch": batch, "input": T, "new_tokens": new, "g": g,
                         "kv_cache_mib": round(kv / 2 ** 20, 1),
                         "peak_mem_mib": round((torch.cuda.max_memory_allocated() + kv) / 2 ** 20),
                         "weights_mib": round(w_bytes / 2 ** 20),
                         "ttft_ms": round((t1 - t0) * 1e3, 1),
                         "tok_per_s_eager": round(batch * half / (t2 - t1), 1),
                         "tok_per_s": round(batch * (new - 1 - half) / (t4 - t3), 1)})
            log(f"[bench] e2e {rows[-1]}")
            m.close()
        del m
    return rows


def run_train(args, torch, skv, configs):
    """One R-CLA training pass (Sec. 3.2) over the attention of a Llama-3.1-8B-shaped stack at the
    paper's fine-tuning length: sampled route, forward of every layer against its source layer's
    K, V, then the backward in reverse order with the K/V gradients of a source layer collected
    from all its readers.  Activations are synthetic; four layers' worth of buffers are rotated."""
    w = configs.llama3_prefill()
    B, S, Hq, Hkv, D, L = w.batch, int(w.kv_lens.max()), w.n_q_heads, w.n_kv_heads, w.head_dim, w.n_layers
    route = skv.skv_train_sample_route(skv.SKV_TRAIN_RCLA, L, 0, 0.5, 2604, 0)
    log(f"[bench] training pass: B={B} S={S} layers={L} p=0.5 route={route}")
    R = 4
    g = torch.Generator(device="cuda").manual_seed(22782)
    mk = lambda h: torch.randn(B, S, h, D, generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    q, k, v, do = [mk(Hq) for _ in range(R)], [mk(Hkv) for _ in range(R)], [mk(Hkv) for _ in range(R)], [mk(Hq) for _ in range(R)]
    out = [torch.empty_like(q[0]) for _ in range(R)]
    dq = [torch.empty_like(q[0]) for _ in range(R)]
    lse = [torch.empty(B, Hq, S, dtype=torch.float32, device="cuda") for _ in range(R)]
    dk = [torch.zeros(B, S, Hkv, D, dtype=torch.float32, device="cuda") for _ in range(R)]
    dv = [torch.zeros_like(dk[0]) for _ in range(R)]
    lens = torch.full((B,), S, dtype=torch.int32, device="cuda")
    ws = torch.empty(skv.skv_train_bwd_workspace_bytes(B, S, Hq) // 4, dtype=torch.float32, device="cuda")
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(L)]

    def one_pass(timed=False):
        for l in range(L):
            src = route[l] % R
            if timed:
                ev[l][0].record()
            skv.skv_train_attn_fwd(q[l % R], k[src], v[src], out[l % R], lse[l % R], lens, w.scale)
            if timed:
                ev[l][1].record()
        for l in reversed(range(L)):
            src = route[l] % R
            skv.skv_train_attn_bwd(q[l % R], k[src], v[src], out[l % R], lse[l % R], do[l % R], dq[l % R],
                                   dk[src], dv[src], lens, w.scale, ws)
            if timed:
                ev[l][2].record()

    one_pass()
    torch.cuda.synchronize()
    steps = max(1, args.steps // 10)
    t0 = time.perf_counter()
    for _ in range(steps):
        one_pass()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    one_pass(timed=True)
    torch.cuda.synchronize()
    fwd_ms = float(np.mean([ev[l][0].elapsed_time(ev[l][1]) for l in range(L)]))
    # backward calls run back to back in reverse layer order: the gap between the end markers of
    # consecutive calls is one call
    bwd_ms = float(np.mean([ev[l + 1][2].elapsed_time(ev[l][2]) for l in range(L - 1)]))
    assert skv.skv_train_device_faults() == 0
    f_fwd = w.prefill_flops_per_layer()          # two causal products
    f_bwd = f_fwd * 5 // 2                       # five: dV, dP, dQ, dK and the recomputed scores
    return {"workload": "llama3_8b_rcla_train_attention_bf16",
            "config": {"batch": B, "seq_len": S, "layers": L, "p": 0.5, "dtype": "bf16", "route": route},
            "steps": steps, "ms_per_step": round(dt * 1e3, 3),
            "value": round((f_fwd + f_bwd) * L / dt / 1e12, 1), "unit": "TFLOP/s",
            "fwd": {"launch_us": round(fwd_ms * 1e3, 1), "achieved": round(f_fwd / (fwd_ms * 1e-3) / 1e12, 1)},
            "roofline": {"bound": "mfma", "kernel": "delta_kernel + dkdv_kernel + dq_kernel", "achieved": round(f_bwd / (bwd_ms * 1e-3) / 1e12, 1),
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(f_bwd / (bwd_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                         **traffic_fields(["delta_kernel", "dkdv_kernel", "dq_kernel"]),
                         "launch_us": round(bwd_ms * 1e3, 1), "algorithmic_flops_per_launch": f_bwd}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--skip-prefill", action="store_true")
    ap.add_argument("--only", default=None,
                    choices=["prefill", "train", "project", "append", "small-launches", "reuse", "workloads", "e2e"],
                    help="profiling aid: measure only this leg and print its object")
    ap.add_argument("--only-prefill", action="store_true", help="same as --only prefill")
    ap.add_argument("--only-train", action="store_true", help="same as --only train")
    ap.add_argument("--only-project", action="store_true", help="same as --only project")
    ap.add_argument("--e2e", action="store_true",
                    help="only run the end-to-end sweep of the paper's Tab. 4 / Tab. 5 on a synthetic Qwen3-8B-scale decoder")
    ap.add_argument("--skip-train", action="store_true")
    ap.add_argument("--skip-project", action="store_true")
    ap.add_argument("--skip-extras", action="store_true",
                    help="leave out the legs beside the metric: the other decode workloads, append, small launches, reuse")
    ap.add_argument("--skip-cpu-baseline", action="store_true")
    ap.add_argument("--decode-workload", default="llama3_decode", choices=["llama3_decode", "qwen3_paged", "llama2_mha"],
                    help="decode workload of the headline step (default: the one the metric is quoted on)")
    ap.add_argument("--kv8", action="store_true", help="profiling aid: the headline decode workload over 8-bit slots")
    ap.add_argument("--mha-batch", type=int, default=32, help="batch of the llama2_mha workload when it is the headline")
    ap.add_argument("--fill-chunk-tokens", type=int, default=1 << 19,
                    help="tokens generated per append call while the cache is filled (bounds the temporaries)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device copy 5 times (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1")
        sys.exit(2)
    only = args.only or ("prefill" if args.only_prefill else "train" if args.only_train else
                         "project" if args.only_project else "e2e" if args.e2e else None)

    import torch
    import paper_2604_22782_amd as skv
    from workloads import driver as H
    from workloads import configs

    if not torch.cuda.is_available():
        log("bench.py needs a GPU: the hot path has no CPU fallback")
        sys.exit(3)
    skv.lib()
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")    # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    def other_workloads():
        """The remaining decode workloads of the metric: paged + ragged (Qwen3-8B shape) and MHA in
        fp16 (Llama-2-7B shape) at batch 32 and at the largest batch that fits (256 sequences, 256 GiB)."""
        out = {}
        kv8 = {"llama3_8b_kv8": configs.llama3_decode(), "qwen3_8b_paged_kv8": configs.qwen3_paged_decode()}
        for w in kv8.values():          # the same workloads over 8-bit slots: half the bytes per cached position
            w.kv8 = True
            w.name += "_kv8"
        # smallest caches first: the 256 GiB one goes last
        for key, w in (*kv8.items(), ("qwen3_8b_paged", configs.qwen3_paged_decode()),
                       ("llama2_7b_mha_b32", configs.llama2_mha_decode(batch=32)),
                       ("llama2_7b_mha_b256", configs.llama2_mha_decode(batch=256))):
            out[key] = run_decode(args, torch, skv, H, w, steps=max(3, args.steps // 4), warmup=1)
        return out

    legs = {
        "prefill": lambda: run_prefill(args, torch, skv, H, configs),
        "train": lambda: run_train(args, torch, skv, configs),
        "project": lambda: run_project(args, torch, skv, H, configs),
        "append": lambda: run_append(args, torch, skv, H, configs),
        "small-launches": lambda: run_small_launches(args, torch, skv, H, configs),
        "reuse": lambda: run_cross_layer_reuse(args, torch, skv, H, configs),
        "workloads": other_workloads,
        "e2e": lambda: run_e2e(args, torch, skv),
    }
    names = {"project": "project_append", "small-launches": "decode_small_launches", "reuse": "cross_layer_reuse",
             "workloads": "decode_workloads"}
    if only:
        print(json.dumps({names.get(only, only): legs[only]()}), flush=True)
        return

    if args.decode_workload == "qwen3_paged":
        w = configs.qwen3_paged_decode()
    elif args.decode_workload == "llama2_mha":
        w = configs.llama2_mha_decode(batch=args.mha_batch)
    else:
        w = configs.llama3_decode()
    if args.kv8:
        w.kv8 = True
        w.name += "_kv8"
    dec = run_decode(args, torch, skv, H, w, args.steps, args.warmup,
                     headline=args.decode_workload == "llama3_decode" and not args.kv8)
    line = {
        "metric": "routed decode attn HBM GB/s (% of peak) + prefill MFMA util %, 1 MI355X",
        "value": dec["value"], "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dec["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic", "config": dec["config"],
        "pct_of_hbm_peak": round(100 * dec["value"] / HBM_PEAK_GBS, 2),
        "roofline": dec["roofline"],
    }
    # Everything but "prefill" is reported beside the metric, never instead of it.  The HBM-bound legs run
    # first: after the pre-fill and training legs have allocated and freed tens of GiB, the same decode
    # launches are 5-8 % slower (llama3_8b_kv8: 98.6 against 90.8 us per call on one box), so the order of
    # the legs is the order of their sensitivity to the placement of a fresh cache in memory.
    order = [] if args.skip_extras else ["workloads", "append", "small-launches", "reuse"]
    order += [] if args.skip_prefill else ["prefill"]
    order += [] if args.skip_project else ["project"]
    order += [] if args.skip_train else ["train"]
    results = {}
    for key in order:
        try:
            results[key] = legs[key]()
        except Exception as e:  # noqa: BLE001 - the headline line must still be printed
            if key == "prefill":
                raise
            log(f"[bench] {key} leg failed: {e!r}")
            results[key] = {"error": repr(e)}
            torch.cuda.empty_cache()
    for key in ["prefill"] + [k for k in order if k != "prefill"]:     # the line keeps its order of keys
        if key in results:
            line[names.get(key, key)] = results[key]
    if not args.skip_cpu_baseline:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        line["cpu_baseline"] = cpu_baseline_decode(w)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
