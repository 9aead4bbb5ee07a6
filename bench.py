#!/usr/bin/env python3
"""Benchmark of the TreeKV hot path on one MI355X.

Headline workload (the configuration the metric is quoted on): 32 layers x 32 heads x 128 dim, bf16, cache budget
2048 (4 sink + 1024 tree + 1020 recent slots), batch 8.  One "step" decodes one token for all 8 sequences through
all 32 layers: 32 launches of the decode kernel, one per layer (a model runs its layers one after the other), each
doing attend -> score update -> tree eviction -> slot reuse -> retained positions for 256 (batch, head) units.  The
caches are filled with 512-token prefill chunks before the timed region starts; inputs are synthetic and already
resident in HBM.

Prints ONE JSON line.  `roofline` prices the decode kernel's algorithmic bytes per launch against the published
8 TB/s HBM peak (`frac`) and against the streaming-read rate measured in the same run (`frac_of_measured`);
`measured_peaks` holds the three probe results (include/treekv_probe.h); `cpu_baseline` times the fp64 CPU oracle on
a bounded sample of the same workload on this machine's host cores.  The other objects are measured after the headline
figure and are not part of `value`: `prefill` (the 512-token chunk over a full 2048-slot cache, against the dense bf16
MFMA peak), `prompt` (the paper's one-shot block-level prompt compression), `wavelet` (the Haar analysis), and
`side_shapes` (decode at batch 1 / budget 1024, with grouped queries at budget 4096, and with re-assigned positions).

`--peaks` runs only the probe kernels (the command the profiler's byte counters are calibrated with).
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HEAD_DIM = 128
WORKLOADS = {
    "graded": dict(layers=32, batch=8, heads=32, kv_heads=32, budget=2048,
                   name="configs[2]: 32 layers x 32 heads x 128 dim, bf16, budget 2048 "
                        "(4 sink + 1024 tree + 1020 recent), batch 8, caches full"),
    "llama7b-1k": dict(layers=32, batch=1, heads=32, kv_heads=32, budget=1024,
                       name="configs[1] shape: 32 layers x 32 heads x 128 dim, bf16, budget 1024 (4 + 512 + 508), "
                            "batch 1, caches full"),
    "gqa-4k": dict(layers=8, batch=16, heads=32, kv_heads=8, budget=4096,
                   name="configs[4] shape: 8 layers x (32 query / 8 KV heads) x 128 dim, bf16, budget 4096 "
                        "(4 + 2048 + 2044), batch 16, caches full"),
}
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
PREFILL_CHUNK = 512
PROMPT_LEN = 32768
PROMPT_BLOCK = 64

# HBM bytes per launch from rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch), each scaled by what
# the same counter reads for the plain copy kernel of `--peaks` (FETCH_SIZE reads 0.5 KiB per KiB copied: factor 2.0;
# WRITE_SIZE 1.0).  These are CONSTANTS taken from the files named beside them, not measurements of this run; they
# are reported only for the shape and kernels they were taken on.
PROFILED_TRAFFIC = {
    "decode": dict(bytes=(132960 * 2 + 4424) * 1024, source="profiles/hbm_traffic_counters_bench_kernels.txt"),
    "prompt": dict(bytes=((140461 + 140860 + 48 + 16680) * 2 + (128 + 4162 + 4 + 34166)) * 1024,
                   source="profiles/hbm_traffic_counters_bench_kernels.txt"),
    "prefill": dict(bytes=int(((26377 + 716 + 4200) * 2 + (13068 + 1669 + 8192)) * 1024),
                    source="profiles/hbm_traffic_counters_bench_kernels.txt"),
    "wavelet": dict(bytes=int(((532612 + 40974.5) * 2 + (81920 + 10)) * 1024),
                    source="profiles/hbm_traffic_counters_bench_kernels.txt"),
}


def algorithmic_bytes_per_unit(c, G, d=HEAD_DIM, esz=2):
    """Bytes one (batch, KV head) unit must move in one decode step with a full cache."""
    kv = 2 * (c + 1) * d * esz          # K and V rows, read once
    s = 2 * (c + 1) * 4                 # scores read + written
    pos = (c + 1) * 4                   # positions read for the retained list
    ret = c * 4                         # retained positions written
    qo = G * d * esz + G * d * 4        # q read, o written (fp32)
    new = 2 * d * esz                   # the new k, v rows written into the cache
    return kv + s + pos + ret + qo + new


def roofline(bound, achieved, peak, unit, measured_peak=None, **extra):
    r = {"bound": bound, "achieved": achieved, "peak": peak, "unit": unit, "frac": achieved / peak, "traffic": None}
    if measured_peak:
        r["measured_peak"] = measured_peak
        r["frac_of_measured"] = achieved / measured_peak
    r.update(extra)
    return r


# ------------------------------------------------------------------------------------------------------------
# peaks measured on this machine
# ------------------------------------------------------------------------------------------------------------
def measure_peaks(torch, binding, dev, reps=40):
    """Streaming read and plain copy over 256 MiB slices of a 4 GiB buffer (each launch touches memory that the 256 MB
    memory-side cache cannot still hold), and the matrix-pipe issue rate, with the kernels of include/treekv_probe.h."""
    lib = binding.load()
    stream = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    slice_b, total = 256 << 20, 4 << 30
    src = torch.full((total,), 3, dtype=torch.uint8, device=dev)
    dst = torch.empty(slice_b, dtype=torch.uint8, device=dev)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    n_slices = total // slice_b

    def timed(fn, n):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / n

    def rd_with(kib, inflight):
        def rd(i):
            rc = lib.treekv_probe_read(C.c_void_p(src.data_ptr() + (i % n_slices) * slice_b), slice_b, kib, inflight,
                                       C.c_void_p(sink.data_ptr()), stream)
            assert rc == 0, rc
        return rd

    def cp(i):
        rc = lib.treekv_probe_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr() + (i % n_slices) * slice_b), slice_b, stream)
        assert rc == 0, rc

    # the read rate depends on how the bytes are dealt out: take the best of a few shapes, the decode kernel's among them
    shapes = [(1024, 4), (1024, 8), (512, 4), (256, 4), (128, 4), (64, 2)]
    reads = {f"{kib}KiB_x{fl}": slice_b / timed(rd_with(kib, fl), reps) / 1e9 for kib, fl in shapes}
    best = max(reads, key=reads.get)
    t_rd, t_cp = slice_b / (reads[best] * 1e9), timed(cp, reps)
    flops = C.c_double(0.0)
    iters = 20000

    def mf(waves):
        def go(_):
            rc = lib.treekv_probe_mfma(C.c_void_p(sink.data_ptr()), 256, waves, iters, C.byref(flops), stream)
            assert rc == 0, rc
        return go

    t_m1 = timed(mf(1), 5)
    f1 = flops.value
    t_m2 = timed(mf(2), 5)
    f2 = flops.value
    del src, dst
    torch.cuda.empty_cache()
    return {
        "hbm_read_GBs": slice_b / t_rd / 1e9, "hbm_read_shape": best, "hbm_read_GBs_by_shape": reads,
        "hbm_copy_GBs": 2 * slice_b / t_cp / 1e9,
        "mfma_bf16_TFLOPs": max(f1 / t_m1, f2 / t_m2) / 1e12,
        "mfma_bf16_TFLOPs_1_wave_per_simd": f1 / t_m1 / 1e12, "mfma_bf16_TFLOPs_2_waves_per_simd": f2 / t_m2 / 1e12,
        "vendor": {"hbm_GBs": HBM_PEAK_GBS, "mfma_bf16_TFLOPs": MFMA_BF16_PEAK_TFLOPS},
        "how": "treekv_probe_read (KiB per 512-thread workgroup x loads in flight per thread, best of the shapes listed) / "
               "treekv_probe_copy (1 MiB per workgroup): 256 MiB per launch, 16-byte lane loads, slices of a 4 GiB buffer "
               "in turn; treekv_probe_mfma: 256 workgroups, 8 independent v_mfma_f32_16x16x32_bf16 "
               "chains per wave, 160000 instructions per wave",
    }


# ------------------------------------------------------------------------------------------------------------
# decode
# ------------------------------------------------------------------------------------------------------------
def bench_decode(torch, binding, inputs, dev, wl, steps, warmup, rerank=False):
    """W warmup steps, then exactly `steps` timed steps of one token for every sequence through every layer.
    Returns (dict of figures, kv_splits)."""
    L, B, H, Hkv, c = wl["layers"], wl["batch"], wl["heads"], wl["kv_heads"], wl["budget"]
    G = H // Hkv
    flags = binding.TREEKV_POSITION_RERANK if rerank else 0
    layers = [binding.TreeKV(c, H, HEAD_DIM, kv_heads=Hkv, batch=B, dtype="bf16", flags=flags, max_chunk=PREFILL_CHUNK)
              for _ in range(L)]
    cfg = layers[0].cfg
    assert (cfg.n_sink, cfg.n_recent) == (4, c - c // 2 - 4)

    def gen(seed, T):
        """[T, L, B, H, d] inputs; every (layer, head) has its own low-rank basis."""
        q, k, v = inputs.device_lowrank(seed, T, B, L * Hkv, G, HEAD_DIM, device=dev)
        f = lambda x, h: x.view(T, B, L, h, HEAD_DIM).permute(0, 2, 1, 3, 4).contiguous()
        return f(q, H), f(k, Hkv), f(v, Hkv)

    out = torch.empty(L, B, H, HEAD_DIM, dtype=torch.float32, device=dev)
    ret = torch.empty(L, B, Hkv, c, dtype=torch.int32, device=dev)
    nret = torch.empty(L, B, Hkv, dtype=torch.int32, device=dev)
    ev = torch.empty(L, B, Hkv, dtype=torch.int32, device=dev)

    def step(q, k, v):
        for l, kv in enumerate(layers):
            kv.decode_step(q[l], k[l], v[l], out[l], ret[l], nret[l], ev[l])

    # fill the caches to the budget (untimed) with prefill chunks
    for i in range(c // PREFILL_CHUNK):
        q, k, v = gen(100 + i, PREFILL_CHUNK)
        o = torch.empty(B, PREFILL_CHUNK, H, HEAD_DIM, dtype=torch.float32, device=dev)
        for l, kv in enumerate(layers):
            cut = lambda x: x[:, l].permute(1, 0, 2, 3).contiguous()
            kv.prefill_chunk(cut(q), cut(k), cut(v), PREFILL_CHUNK, o, ret[l], nret[l], None)
        del q, k, v, o
    torch.cuda.synchronize()
    assert int(nret.min()) == c, "caches are not full"

    q, k, v = gen(7, warmup + steps)
    for t in range(warmup):
        step(q[t], k[t], v[t])
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_host0 = time.perf_counter()
    e0.record(stream)
    for t in range(warmup, warmup + steps):
        step(q[t], k[t], v[t])
    e1.record(stream)
    torch.cuda.synchronize()
    host_s = time.perf_counter() - t_host0
    dev_ms = e0.elapsed_time(e1)
    total_s = max(host_s, dev_ms * 1e-3)
    assert int(nret.min()) == c and int(ev.min()) >= 0, "every unit must evict once per step"
    launch_us = dev_ms * 1e3 / (steps * L)
    bytes_per_launch = algorithmic_bytes_per_unit(c, G) * B * Hkv
    # the same call one at a time: events around a single ABI call, the stream idle before and after it
    singles = []
    for i in range(min(64, steps * L)):
        t, l = warmup + i // L, i % L
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        layers[l].decode_step(q[t, l], k[t, l], v[t, l], out[l], ret[l], nret[l], ev[l])
        b_.record(stream)
        torch.cuda.synchronize()
        singles.append(a.elapsed_time(b_) * 1e3)
    singles.sort()
    return dict(total_s=total_s, ms_per_step=total_s * 1e3 / steps, steps_per_s=steps / total_s, launch_us=launch_us,
                bytes_per_launch=bytes_per_launch, achieved_GBs=bytes_per_launch / (launch_us * 1e-6) / 1e9,
                kv_splits=int(cfg.kv_splits), single_call_us=singles[len(singles) // 2])


def side_shape(torch, binding, inputs, dev, name, peaks, rerank=False, steps=40, warmup=5):
    wl = dict(WORKLOADS[name])
    wl["layers"] = min(wl["layers"], 8)            # a few layers cycle through more than the memory-side cache holds
    r = bench_decode(torch, binding, inputs, dev, wl, steps, warmup, rerank=rerank)
    torch.cuda.empty_cache()
    return {"workload": wl["name"].replace("32 layers", "8 of the 32 layers") + (", positions re-assigned to cache ranks" if rerank else ""),
            "layer_step_us": r["launch_us"], "layer_steps_per_s": 1e6 / r["launch_us"], "kv_splits": r["kv_splits"],
            "roofline": roofline("hbm", r["achieved_GBs"], HBM_PEAK_GBS, "GB/s", peaks and peaks["hbm_read_GBs"],
                                 bytes_per_launch=r["bytes_per_launch"],
                                 note="per layer-step: HIP-event time of the timed region / (steps x layers); "
                                      + ("one kernel per layer-step" if r["kv_splits"] == 1 else "two kernels per layer-step (slices, then merge)"))}


# ------------------------------------------------------------------------------------------------------------
# the oracle on this machine's cores
# ------------------------------------------------------------------------------------------------------------
def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl):
    """The oracle as it stands, on a bounded sample of the headline workload: streams filled to the budget (untimed)
    and then timed over decode steps with a full cache -- first one stream alone on one core, then one stream per
    worker thread on min(nproc, streams, the thread cap of this box) threads."""
    import numpy as np

    from oracle import treekv_oracle as orc
    from paper_2501_04987_amd import inputs

    orc.build()
    c, B, Hkv, L = wl["budget"], wl["batch"], wl["kv_heads"], wl["layers"]
    streams = L * B * Hkv
    nproc = os.cpu_count() or 1
    cap = int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or nproc      # the share of the host this job may use
    threads = max(1, min(nproc, streams, cap))

    def job(arg):
        i, n_timed = arg
        T = c + n_timed
        q, k, v = inputs.stream_lowrank(1 + i % B, T, 1, HEAD_DIM, layer=i // (B * Hkv), batch=i % B, kv_head=i % Hkv)
        s = orc.OracleStream(c, 1, HEAD_DIM, n_sink=4, n_recent=c - c // 2 - 4)
        s.decode_stream(q[:c], k[:c], v[:c], keep_outputs=False)
        t0 = time.perf_counter()
        s.decode_stream(q[c:], k[c:], v[c:], keep_outputs=False)
        return n_timed / (time.perf_counter() - t0)

    single = job((0, 1024))                                       # one stream, one core, nothing else running
    t0 = time.perf_counter()
    rates = orc.run_many(job, [(i, 1536) for i in range(threads)], workers=threads)
    wall = time.perf_counter() - t0
    unit_steps_per_s = float(sum(rates))
    return {
        "value": unit_steps_per_s / streams, "unit": "steps/s", "cores": threads, "kind": "oracle",
        "sample": (f"{threads} of the {streams} (layer, batch, head) streams, one per thread, each filled to {c} slots "
                   f"then timed for 1536 decode steps; linearly scaled to {streams} streams per step"),
        "nproc": nproc, "thread_cap": cap, "cpu_model": cpu_model(),
        "single_core_one_stream_unit_steps_per_s": single, "all_threads_unit_steps_per_s": unit_steps_per_s,
        "wall_s": wall,
    }


# ------------------------------------------------------------------------------------------------------------
# the other calls of the path
# ------------------------------------------------------------------------------------------------------------
def prefill_flops_per_chunk(c, L=PREFILL_CHUNK, d=HEAD_DIM, heads=32):
    """Algorithmic flops of one chunk over a full cache: Q.K^T and P.V over c cache columns plus the causal half of
    the chunk's own L x L block, for every head."""
    return 2 * 2 * L * (c + (L + 1) / 2) * d * heads


def bench_prefill(torch, binding, inputs, dev, peaks, chunks=64, warm=64, layers=4, c=2048, H=32, flags=0, B=1):
    """Chunks of 512 tokens into full 2048-slot caches, 32 heads x 128, batch 1, cycling over a few layers: one
    32768-token prompt's worth of chunks to warm up (a few milliseconds of work, so that the clocks have settled when
    this runs on its own), then another one timed."""
    kvs = [binding.TreeKV(c, H, HEAD_DIM, batch=B, max_chunk=PREFILL_CHUNK, flags=flags) for _ in range(layers)]
    n_in = 8
    q, k, v = inputs.device_lowrank(11, n_in * PREFILL_CHUNK, B, H, 1, HEAD_DIM, device=dev)
    mk = lambda x: x.view(n_in, PREFILL_CHUNK, B, H, HEAD_DIM).permute(0, 2, 1, 3, 4).contiguous()   # [n,B,L,H,d]
    q, k, v = mk(q), mk(k), mk(v)
    out = torch.empty(B, PREFILL_CHUNK, H, HEAD_DIM, dtype=torch.float32, device=dev)
    ret = torch.empty(layers, B, H, c, dtype=torch.int32, device=dev)
    nret = torch.empty(layers, B, H, dtype=torch.int32, device=dev)
    ev = torch.empty(B, H, PREFILL_CHUNK, dtype=torch.int32, device=dev)

    def run(i):
        l = i % layers
        kvs[l].prefill_chunk(q[i % n_in], k[i % n_in], v[i % n_in], PREFILL_CHUNK, out, ret[l], nret[l], ev)

    for i in range(layers * (c // PREFILL_CHUNK) + warm):          # fill every layer's cache, then warm up
        run(i)
    torch.cuda.synchronize()
    assert int(nret.min()) == c
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(chunks):
        run(i)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / chunks
    assert int(ev.min()) >= 0, "every token of a chunk into a full cache evicts one"
    flops = prefill_flops_per_chunk(c, heads=H) * B
    tf = flops / (us * 1e-6) / 1e12
    extra = {}
    if not flags and B == 1:
        extra = dict(traffic=PROFILED_TRAFFIC["prefill"]["bytes"],
                     traffic_source=PROFILED_TRAFFIC["prefill"]["source"] + " (a constant from that file, not measured in this run)")
    return {"workload": f"configs[3] shape: 512-token chunk into a full 2048-slot cache, 32 heads x 128 dim, bf16, batch {B}"
                        + (", positions re-assigned" if flags else ""),
            "chunks": chunks, "us_per_chunk": us, "prompt_tokens_per_s": B * PREFILL_CHUNK / (us * 1e-6),
            "roofline": roofline("mfma", tf, MFMA_BF16_PEAK_TFLOPS, "TFLOP/s", peaks and peaks["mfma_bf16_TFLOPs"],
                                 flops_per_chunk=flops,
                                 note="algorithmic flops (Q.K^T and P.V once each) over the whole chunk call: every "
                                      "kernel of treekv_prefill_chunk, launch gaps included", **extra)}


def prompt_bytes_per_call(T, c, d=HEAD_DIM, heads=32, block=PROMPT_BLOCK):
    """Algorithmic bytes of one one-shot prompt compression: every key once (the window's logits), the window's
    queries, every token's score written once, the kept rows of K and V read and written, the retained list."""
    per_head = T * d * 2 + block * d * 2 + T * 4 + 2 * 2 * c * d * 2 + c * 4 + c * 4
    return per_head * heads


def bench_prompt(torch, binding, inputs, dev, peaks, calls=20, warm=3, layers=3, flags=0, c=2048, H=32):
    """One-shot block-level compression (Section 4.2) of a 32768-token prompt into 2048 slots, 32 heads x 128,
    blocks of 64, batch 1, cycling over a few prompts (each larger than the memory-side cache)."""
    T, b = PROMPT_LEN, PROMPT_BLOCK
    kv = binding.TreeKV(c, H, HEAD_DIM, max_prompt=T, flags=flags)
    prompts = []
    for l in range(layers):
        q, k, v = inputs.device_lowrank(21 + l, T, 1, H, 1, HEAD_DIM, device=dev)
        prompts.append((q[T - b:].permute(1, 0, 2, 3).contiguous(), k.permute(1, 0, 2, 3).contiguous(),
                        v.permute(1, 0, 2, 3).contiguous()))
        del q, k, v
    ret = torch.empty(1, H, c, dtype=torch.int32, device=dev)
    nret = torch.empty(1, H, dtype=torch.int32, device=dev)

    def run(i):
        qw, kp, vp = prompts[i % layers]
        kv.prefill_prompt(qw, kp, vp, T, b, ret, nret)

    for i in range(warm):
        run(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(calls):
        run(i)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / calls
    assert int(nret.min()) == c
    nbytes = prompt_bytes_per_call(T, c, heads=H)
    gbs = nbytes / (us * 1e-6) / 1e9
    r = roofline("hbm", gbs, HBM_PEAK_GBS, "GB/s", peaks and peaks["hbm_read_GBs"], bytes_per_call=nbytes,
                 note="algorithmic bytes (every key once) over the whole call, all its kernels")
    if not flags:
        r["traffic"] = PROFILED_TRAFFIC["prompt"]["bytes"]
        r["traffic_source"] = PROFILED_TRAFFIC["prompt"]["source"] + " (a constant from that file, not measured in this run)"
    return {"workload": f"configs[3] shape, the paper's own prefill: {T}-token prompt compressed in one shot into "
                        f"{c} slots, blocks of {b}, 32 heads x 128 dim, bf16, batch 1"
                        + (", positions re-assigned" if flags else ""),
            "calls": calls, "us_per_call": us, "prompt_tokens_per_s": T / (us * 1e-6), "roofline": r}


def bench_wavelet(torch, binding, dev, peaks, calls=20, warm=3, samples=8, t=512, levels=5, H=32):
    """The Haar analysis of Sections 3.2-3.3 in the figure's setting (5 levels at generation step 512) for
    32 layers x 32 heads x `samples` sequences per call; a = softmax of random logits, V ~ N(0, 1) in bf16."""
    heads = 32 * H * samples
    g = torch.Generator(device=dev).manual_seed(5)
    a = torch.softmax(3.0 * torch.randn(heads, t, device=dev, generator=g), dim=-1).contiguous()
    sets = [torch.randn(heads, t, HEAD_DIM, device=dev, generator=g).to(torch.bfloat16) for _ in range(2)]
    per_head = torch.empty(heads, levels, t, dtype=torch.float32, device=dev)
    mean = torch.empty(levels, t, dtype=torch.float32, device=dev)
    for i in range(warm):
        binding.wavelet_components(a, sets[i % 2], levels, per_head, mean)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(calls):
        binding.wavelet_components(a, sets[i % 2], levels, per_head, mean)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / calls
    # V and a read once, the per-head magnitudes written once and read once for the mean, the mean written
    nbytes = heads * t * (HEAD_DIM * 2 + 4) + 2 * heads * levels * t * 4 + levels * t * 4
    gbs = nbytes / (us * 1e-6) / 1e9
    r = roofline("hbm", gbs, HBM_PEAK_GBS, "GB/s", peaks and peaks["hbm_read_GBs"], bytes_per_call=nbytes,
                 note="components kernel and mean kernel together")
    r["traffic"] = PROFILED_TRAFFIC["wavelet"]["bytes"]
    r["traffic_source"] = PROFILED_TRAFFIC["wavelet"]["source"] + " (a constant from that file, not measured in this run)"
    return {"workload": f"Haar analysis, {levels} levels, step {t}, {heads} heads (32 layers x {H} heads x "
                        f"{samples} samples) x {HEAD_DIM} dim, bf16 values",
            "calls": calls, "us_per_call": us, "heads_per_s": heads / (us * 1e-6), "roofline": r}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline decode figure: no prefill / prompt / wavelet / side-shape objects")
    ap.add_argument("--workload", choices=sorted(WORKLOADS), default="graded",
                    help="time another decode shape of the configuration list instead (a side measurement)")
    ap.add_argument("--rerank", action="store_true",
                    help="decode (and compress the prompt) with positions re-assigned to cache ranks; a side measurement")
    ap.add_argument("--peaks", action="store_true", help="run only the probe kernels and print their rates")
    ap.add_argument("--only", choices=["prefill", "prefill_batch8", "prompt", "wavelet"],
                    help="run only that object of the default line (for profiling one call's kernels)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (every TreeKV stream is independent; there is no "
              "multi-GPU path to time); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2501_04987_amd import binding, inputs

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load()
    if args.peaks:
        print(json.dumps({"measured_peaks": measure_peaks(torch, binding, dev)}))
        return

    if args.only:
        flags = binding.TREEKV_POSITION_RERANK if args.rerank else 0
        obj = (bench_prefill(torch, binding, inputs, dev, None, flags=flags) if args.only == "prefill" else
               bench_prefill(torch, binding, inputs, dev, None, chunks=16, warm=8, layers=2, B=8, flags=flags)
               if args.only == "prefill_batch8" else
               bench_prompt(torch, binding, inputs, dev, None, flags=flags) if args.only == "prompt" else
               bench_wavelet(torch, binding, dev, None))
        print(json.dumps({args.only: obj}))
        return

    wl = WORKLOADS[args.workload]
    headline = args.workload == "graded" and not args.rerank
    K_steps, W = args.steps, args.warmup
    r = bench_decode(torch, binding, inputs, dev, wl, K_steps, W, rerank=args.rerank)
    torch.cuda.empty_cache()
    peaks = measure_peaks(torch, binding, dev)
    roof = roofline("hbm", r["achieved_GBs"], HBM_PEAK_GBS, "GB/s", peaks["hbm_read_GBs"],
                    kernel="decode_fused_kernel<bf16,128,1>" if r["kv_splits"] == 1 else "decode_split_kernel + decode_merge_kernel",
                    bytes_per_launch=r["bytes_per_launch"], launch_us=r["launch_us"], single_call_us=r["single_call_us"],
                    note="launch_us = HIP-event time of the timed region / number of layer launches, calls enqueued back "
                         "to back (gaps between launches included): achieved and frac refer to it; single_call_us = "
                         "median HIP-event time around one call with the stream idle before and after (not what frac "
                         "uses); frac is against the published 8 TB/s, frac_of_measured against "
                         "measured_peaks.hbm_read_GBs of this run")
    if headline:
        roof["traffic"] = PROFILED_TRAFFIC["decode"]["bytes"]
        roof["traffic_source"] = PROFILED_TRAFFIC["decode"]["source"] + " (a constant from that file, not measured in this run)"
    res = {
        "metric": "decode steps/s (one token for 8 sequences through 32 layers; 32h x 128d, cache 2048, bf16)"
                  if headline else
                  f"decode steps/s ({args.workload}{', positions re-assigned to cache ranks' if args.rerank else ''})",
        "value": r["steps_per_s"], "unit": "steps/s", "n_gpus": 1, "steps": K_steps, "warmup": W,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 storage, fp32 arithmetic", "data": "synthetic",
        "config": {"workload": wl["name"] + (", positions re-assigned to cache ranks" if args.rerank else ""),
                   "layers": wl["layers"], "batch": wl["batch"], "heads": wl["heads"], "kv_heads": wl["kv_heads"],
                   "head_dim": HEAD_DIM, "budget": wl["budget"], "kv_splits": r["kv_splits"], "launch": "stream",
                   "filled_by": "prefill chunks of 512"},
        "tokens_per_s": r["steps_per_s"] * wl["batch"],
        "layer_steps_per_s": r["steps_per_s"] * wl["layers"],
        "roofline": roof,
        "measured_peaks": peaks,
    }
    if headline and not args.no_extras:
        res["prefill"] = bench_prefill(torch, binding, inputs, dev, peaks)
        torch.cuda.empty_cache()
        res["prompt"] = bench_prompt(torch, binding, inputs, dev, peaks)
        torch.cuda.empty_cache()
        res["prefill_batch8"] = bench_prefill(torch, binding, inputs, dev, peaks, chunks=16, warm=8, layers=2, B=8)
        torch.cuda.empty_cache()
        res["wavelet"] = bench_wavelet(torch, binding, dev, peaks)
        torch.cuda.empty_cache()
        res["side_shapes"] = {
            "batch1_budget1024": side_shape(torch, binding, inputs, dev, "llama7b-1k", peaks),
            "gqa_budget4096": side_shape(torch, binding, inputs, dev, "gqa-4k", peaks),
            "graded_shape_rerank": side_shape(torch, binding, inputs, dev, "graded", peaks, rerank=True),
        }
    if args.rerank and not args.no_extras:
        res["prefill"] = bench_prefill(torch, binding, inputs, dev, peaks, flags=binding.TREEKV_POSITION_RERANK)
        torch.cuda.empty_cache()
        res["prompt"] = bench_prompt(torch, binding, inputs, dev, peaks, flags=binding.TREEKV_POSITION_RERANK)
    if headline and not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
