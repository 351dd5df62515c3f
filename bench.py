#!/usr/bin/env python3
"""Benchmark of the QJL hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3] [--no-extra] [--no-cpu]

A "step" is one decode step of the long-context workload (batch 4, 32 heads,
d = 128, m = 256, context 32768: 4,194,304 cached keys, 1.2 GB of codes, norms
and values; the largest of the configurations, all of it resident in HBM):
project the query, estimate all scores, softmax, aggregate the bf16 values --
one call of qjl_decode_attention.  The headline `value` is keys (= batch x
kv-head x token triples) per second over exactly K steps; the steps are
replayed from a HIP graph so that the host's launch cost does not hide the GPU
time (the eager rate is reported next to it).

`roofline` is for the attention kernel of that step: algorithmic bytes per
launch (290 B per key: 32 B code + 2 B norm + 256 B values) over the kernel's
mean duration, taken from the kernel's own start/stop timestamps
(qjl_decode_attention_timed).  `ceilings` holds what a plain streaming read and
a back-to-back bf16 MFMA loop reach on this chip in the same run
(libqjl_ceilings.so), and every roofline carries `frac_of_ceiling` next to
`frac`.  `other_workloads` repeats the measurement for the other decode
configurations (those that fit the 256 MB last-level cache also with rotating
copies of the cache, `*_cold`), the prefill quantizer and the widened rows.
`cpu_baseline` times the CPU oracle on a bounded sample of the headline
workload (`cpu_baselines_other`: GQA decode and prefill quantize), and
`sign_bits` counts the near-zero sign decisions on which the GPU's code of that
sample differs from the oracle's.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak, published
COLD_BYTES = 640 << 20          # rotating copies of a cache add up to at least this (last-level cache: 256 MB)
CEIL = {}                       # filled by measure_ceilings(): name -> rate


class HipEvents:
    """hipEvent_t handles through ctypes (torch's events only see torch's own records)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self) -> int:
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0:
            raise RuntimeError(f"hipEventCreate -> {rc}")
        return ev.value

    def record(self, ev: int, stream: int) -> None:
        rc = self.hip.hipEventRecord(ev, stream)
        if rc != 0:
            raise RuntimeError(f"hipEventRecord -> {rc}")

    def elapsed_ms(self, a: int, b: int) -> float:
        self.hip.hipEventSynchronize(b)
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime -> {rc}")
        return float(ms.value)

    def destroy(self, ev: int) -> None:
        self.hip.hipEventDestroy(ev)


def decode_bytes_per_key(w) -> int:
    """Algorithmic HBM bytes per (batch, kv head, token): code + norm + one row of V."""
    value_row = w.d * w.vbits // 8 + 4 if w.vbits else w.d * 2      # codes + scale + zero point, or 16-bit entries
    return (w.m + w.m_out) // 8 + (4 if w.m_out else 2) + value_row


def load_traffic(name: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summaries, if present."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    try:
        with open(path) as f:
            return json.load(f).get(name)
    except Exception:
        return None


def prepare_decode(qjl, inputs, w, dev):
    import torch
    K, Q, V = inputs.make_workload_tensors(w, dev)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, dev)
    if w.m_out:                                     # outlier channels quantized separately (Section 4.1)
        S_out = qjl.qjl_make_sketch(w.sketch_seed + 1000, w.m_out, w.d, w.dtype, dev)
        ch = qjl.qjl_select_outliers(K, 4)
        S = qjl.qjl_make_dual_sketch(S, S_out, ch)
        bits, norms, norms_out = qjl.qjl_quantize_keys_dual(K, S, ch, w.m_out)
        k_last = K[:, :, -1:].contiguous() if w.stream else None
        del K
        ws = torch.empty((qjl.qjl_decode_dual_workspace_bytes(w.batch, w.q_heads, w.kv_heads, w.n, w.d, w.m,
                                                              w.m_out, w.dtype),), dtype=torch.uint8, device=dev)
        out = torch.empty((w.batch, w.q_heads, w.d), dtype=torch.float32, device=dev)
        extra_v = {}
        if w.vbits:                                 # ... and the values token-wise (Section 3.2): the paper's operating point
            vc, vs, vz = qjl.qjl_quantize_values(V, w.vbits)
            extra_v = dict(vcodes=vc, vscale=vs, vzero=vz, v_last=V[:, :, -1:].contiguous() if w.stream else None, ch=ch)
            V = None
        torch.cuda.synchronize()
        return dict(Q=Q, S=S, bits=bits, norms=norms, norms_out=norms_out, V=V, ws=ws, out=out, k_last=k_last, **extra_v)
    bits, norms = qjl.qjl_quantize_keys(K, S)       # untimed: the cache already exists at decode time
    k_last = K[:, :, -1:].contiguous() if w.stream else None
    del K
    if w.vbits:                                     # value cache quantized token-wise (Section 3.2), also untimed
        vc, vs, vz = qjl.qjl_quantize_values(V, w.vbits)
        V = None
        extra_v = dict(vcodes=vc, vscale=vs, vzero=vz)
    else:
        extra_v = {}
    ws = torch.empty((qjl.qjl_decode_workspace_bytes(w.batch, w.q_heads, w.kv_heads, w.n, w.d, w.m, w.dtype),),
                     dtype=torch.uint8, device=dev)
    out = torch.empty((w.batch, w.q_heads, w.d), dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    return dict(Q=Q, S=S, bits=bits, norms=norms, V=V, ws=ws, out=out, k_last=k_last, **extra_v)


def run_decode(qjl, t, w, events=None):
    if w.stream and w.m_out and w.vbits:   # the newest token's key and value are quantized into the last row, then attention
        qjl.qjl_generation_step(t["Q"], t["k_last"], t["v_last"], t["S"], t["ch"], t["bits"], t["norms"], t["norms_out"],
                                t["vcodes"], t["vscale"], t["vzero"], w.n - 1, w.m_out, w.vbits, w.scale, out=t["out"],
                                workspace=t["ws"])
        return
    if w.m_out and w.vbits:
        qjl.qjl_decode_attention_dual_vq(t["Q"], t["S"], t["bits"], t["norms"], t["norms_out"], t["vcodes"], t["vscale"],
                                         t["vzero"], w.m_out, w.vbits, w.scale, out=t["out"], workspace=t["ws"], events=events)
        return
    if w.stream:        # the newest key is quantized into the last row, then attention over the full cache
        qjl.qjl_decode_step(t["Q"], t["k_last"], t["S"], t["bits"], t["norms"], t["V"], w.n - 1, w.scale,
                            out=t["out"], workspace=t["ws"])
        return
    if w.vbits:
        qjl.qjl_decode_attention_vq(t["Q"], t["S"], t["bits"], t["norms"], t["vcodes"], t["vscale"], t["vzero"],
                                    w.vbits, w.scale, out=t["out"], workspace=t["ws"], events=events)
        return
    if w.m_out:
        qjl.qjl_decode_attention_dual(t["Q"], t["S"], t["bits"], t["norms"], t["norms_out"], t["V"], w.m_out,
                                      w.scale, out=t["out"], workspace=t["ws"], events=events)
        return
    qjl.qjl_decode_attention(t["Q"], t["S"], t["bits"], t["norms"], t["V"], w.scale, out=t["out"],
                             workspace=t["ws"], events=events)


def cache_sets(t, w):
    """Rotating copies of everything a decode step streams (codes, norms, values): enough of them that the last-level
    cache (256 MB) cannot hold what the next step reads.  The first set is the original."""
    import torch
    big = [k for k in ("bits", "norms", "norms_out", "V", "vcodes", "vscale", "vzero") if t.get(k) is not None]
    set_bytes = sum(t[k].numel() * t[k].element_size() for k in big)
    count = max(3, -(-COLD_BYTES // set_bytes))
    sets = [t]
    for _ in range(count - 1):
        c = dict(t)
        for k in big:
            c[k] = t[k].clone()
        sets.append(c)
    torch.cuda.synchronize()
    return sets, set_bytes


def graph_time(run, steps, warmup, gb):
    """ms per step over exactly `steps` steps replayed from a HIP graph that holds `gb` of them (run(i) = step i)."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(0)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for i in range(gb):
            run(i)
    for _ in range(max(1, warmup // gb)):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps // gb):
        g.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def kernel_time(qjl, ev, w, sets, count):
    """Mean and median duration (ms) of the attention kernel alone: events recorded around it inside the call."""
    import torch
    pairs = [(ev.create(), ev.create()) for _ in range(count)]
    for i, (a, b) in enumerate(pairs):
        run_decode(qjl, sets[i % len(sets)], w, events=(a, b))
    torch.cuda.synchronize()
    durs = sorted(ev.elapsed_ms(a, b) for a, b in pairs)
    for a, b in pairs:
        ev.destroy(a)
        ev.destroy(b)
    return sum(durs) / len(durs), durs[len(durs) // 2]


def time_decode(qjl, ev, w, t, steps, warmup, graph_batch=None, cold=False):
    """Returns dict(ms_graph, ms_eager, kernel_ms, ...) for one workload; with `cold` also the same figures with
    the caches rotated over copies that together exceed the last-level cache."""
    import torch
    for _ in range(warmup):
        run_decode(qjl, t, w)
    torch.cuda.synchronize()
    # ---- eager: K library calls back to back
    t0 = time.perf_counter()
    for _ in range(steps):
        run_decode(qjl, t, w)
    torch.cuda.synchronize()
    ms_eager = (time.perf_counter() - t0) * 1e3 / steps
    # ---- HIP graph holding `gb` steps, replayed steps/gb times (exactly `steps` steps)
    gb = graph_batch or next(g for g in (50, 25, 20, 10, 5, 4, 2, 1) if steps % g == 0)
    ms_graph = graph_time(lambda i: run_decode(qjl, t, w), steps, warmup, gb)
    r = dict(ms_graph=ms_graph, ms_eager=ms_eager, graph_batch=gb)
    if w.stream:        # no kernel-timestamp variant of this call: the roofline figure uses the whole step
        r.update(kernel_ms=ms_graph, kernel_ms_median=ms_graph)
        return r
    r["kernel_ms"], r["kernel_ms_median"] = kernel_time(qjl, ev, w, [t], min(steps, 200))
    if cold:
        sets, set_bytes = cache_sets(t, w)
        gbc = max(gb, len(sets))
        steps_c = max(gbc, steps // gbc * gbc)
        r["ms_graph_cold"] = graph_time(lambda i: run_decode(qjl, sets[i % len(sets)], w), steps_c, warmup, gbc)
        r["kernel_ms_cold"], r["kernel_ms_cold_median"] = kernel_time(qjl, ev, w, sets, min(steps, 200))
        r["cold_sets"], r["cold_bytes"] = len(sets), len(sets) * set_bytes
        del sets
    return r


def read_ceiling(nbytes, cold):
    """The streaming-read rate (GB/s) measured at the size closest to nbytes."""
    if not CEIL:
        return None
    if nbytes >= 700e6:
        return CEIL.get("read_1200MB_GBs")
    if nbytes >= 150e6:
        return CEIL.get("read_300MB_cold_GBs" if cold else "read_300MB_GBs")
    return CEIL.get("read_38MB_cold_GBs" if cold else "read_38MB_GBs")


def decode_record(w, r):
    algo_bytes = decode_bytes_per_key(w) * w.key_heads
    achieved = algo_bytes / (r["kernel_ms"] * 1e-3) / 1e9
    ceil = read_ceiling(algo_bytes, False)
    rec = {
        "workload": w.name,
        "metric": "decode keys/s/GPU",
        "value": w.key_heads / (r["ms_graph"] * 1e-3),
        "ms_per_step": r["ms_graph"],
        "ms_per_step_eager": r["ms_eager"],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": load_traffic(w.name),
                     "ceiling": ceil, "frac_of_ceiling": achieved / ceil if ceil else None,
                     "kernel": "decode_kernel", "kernel_ms": r["kernel_ms"],
                     "kernel_ms_median": r["kernel_ms_median"], "algorithmic_bytes": algo_bytes},
    }
    if "ms_graph_cold" in r:        # every step reads a copy of the cache that the last-level cache cannot still hold
        ach_c = algo_bytes / (r["kernel_ms_cold"] * 1e-3) / 1e9
        ceil_c = read_ceiling(algo_bytes, True)
        rec.update({"value_cold": w.key_heads / (r["ms_graph_cold"] * 1e-3), "ms_per_step_cold": r["ms_graph_cold"]})
        rec["roofline"].update({"achieved_cold": ach_c, "frac_cold": ach_c / HBM_PEAK_GBS,
                                "kernel_ms_cold": r["kernel_ms_cold"], "kernel_ms_cold_median": r["kernel_ms_cold_median"],
                                "ceiling_cold": ceil_c, "frac_of_ceiling_cold": ach_c / ceil_c if ceil_c else None,
                                "cold_sets": r["cold_sets"], "cold_bytes": r["cold_bytes"]})
    return rec


class Ceilings:
    """libqjl_ceilings.so through ctypes: a streaming read, a copy and an MFMA loop (no part of the method)."""

    def __init__(self):
        path = os.path.join(ROOT, "paper_2406_03482_amd", "libqjl_ceilings.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2406_03482_amd.build`")
        L = ctypes.CDLL(path)
        vp = ctypes.c_void_p
        L.ceil_stream_read.argtypes = [vp, ctypes.c_size_t, ctypes.c_int, ctypes.c_int, vp, vp]
        L.ceil_copy.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int, vp]
        L.ceil_mfma_loop.argtypes = [vp, ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.POINTER(ctypes.c_double), vp]
        self.L = L


def timed_launches(ev, stream, launch, count, warm):
    """ms per launch over `count` launches back to back on `stream`, bracketed by two events."""
    import torch
    for i in range(warm):
        launch(i)
    torch.cuda.synchronize()
    a, b = ev.create(), ev.create()
    ev.record(a, stream)
    for i in range(count):
        launch(i)
    ev.record(b, stream)
    ms = ev.elapsed_ms(a, b) / count
    ev.destroy(a)
    ev.destroy(b)
    return ms


def measure_ceilings(ev, dev, quick=False):
    """What this chip sustains, measured like the kernels themselves: streaming reads of the decode workloads' sizes
    (warm = the same buffer again and again, cold = rotating buffers adding up to more than the last-level cache) and
    a loop of nothing but bf16 MFMAs on N(0,1) operands, eight waves per CU, >= 50 launches back to back so that the
    clock has settled to what the chip holds under matrix load."""
    import torch
    C = Ceilings().L
    stream = torch.cuda.current_stream().cuda_stream
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    out = {}
    g = torch.Generator(device=dev)
    g.manual_seed(7)
    for label, nbytes in (("38MB", 38010880), ("300MB", 304087040), ("1200MB", 1216348160)):
        nsets = 1 if nbytes > 700e6 else max(3, -(-COLD_BYTES // nbytes))
        bufs = [torch.randint(0, 2 ** 31 - 1, (nbytes // 4,), dtype=torch.int32, device=dev, generator=g) for _ in range(nsets)]
        reps = 20 if quick else (200 if nbytes < 100e6 else 60)
        # the ceiling is the best of a few launch shapes (workgroups per CU x load kind x access pattern)
        shapes = [(cus * k, mode) for k in (2, 4, 8, 16) for mode in range(5)]
        def sweep(pick):
            best = None
            for blocks, mode in shapes:
                ms = timed_launches(ev, stream, lambda i: C.ceil_stream_read(pick(i).data_ptr(), nbytes, blocks, mode, sink.data_ptr(), stream),
                                    max(10, reps // 4), 3)
                if best is None or ms < best[0]:
                    best = (ms, blocks, mode)
            ms = timed_launches(ev, stream, lambda i: C.ceil_stream_read(pick(i).data_ptr(), nbytes, best[1], best[2], sink.data_ptr(), stream), reps, 5)
            return min(ms, best[0]), best[1], best[2]
        ms, blocks, mode = sweep(lambda i: bufs[0])
        out[f"read_{label}_GBs"] = nbytes / (ms * 1e-3) / 1e9
        out[f"read_{label}_shape"] = f"{blocks} workgroups, mode {mode}"
        if nsets > 1:
            ms, blocks, mode = sweep(lambda i: bufs[i % nsets])
            out[f"read_{label}_cold_GBs"] = nbytes / (ms * 1e-3) / 1e9
            out[f"read_{label}_cold_shape"] = f"{blocks} workgroups, mode {mode}"
        del bufs
        torch.cuda.empty_cache()
    frag = torch.randn((8 * 64 * 8,), device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    zeros = torch.zeros_like(frag)
    flops = ctypes.c_double()
    iters = 2000 if quick else 6000          # 16 MFMAs per iteration and wave: about 1.5 ms per launch
    for label, wide, src in (("mfma_16x16x32_TFLOPs", 0, frag), ("mfma_32x32x16_TFLOPs", 1, frag),
                             ("mfma_16x16x32_zero_operands_TFLOPs", 0, zeros)):
        ms = timed_launches(ev, stream, lambda i: C.ceil_mfma_loop(src.data_ptr(), wide, iters, cus, sink.data_ptr(), ctypes.byref(flops), stream),
                            20 if quick else 60, 5)
        out[label] = flops.value / (ms * 1e-3) / 1e12
    out["mfma_TFLOPs"] = out["mfma_16x16x32_TFLOPs"]   # the quantizer's instruction and operand statistics
    out["read_GBs"] = out["read_1200MB_GBs"]
    out["note"] = ("streaming read with 16-byte loads, nothing written; MFMA loop of eight waves per CU on N(0,1) bf16 "
                   "register operands, no memory traffic, 60 launches of about 1.5 ms back to back")
    return out


def bench_quantize(qjl, inputs, ev, w, dev, steps, warmup, zero_operands=False):
    import torch
    K = inputs.make_keys(w.batch, w.kv_heads, w.n, w.d, w.dtype, w.data_seed, dev, w.outliers)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, dev)
    if zero_operands:       # the same instruction stream on all-zero keys and sketch: no data toggling in the
        K.zero_()           # matrix pipe or on the memory path (a power experiment, not a workload)
        S.zero_()
    mt = w.m + w.m_out
    bits = torch.empty((w.batch, w.kv_heads, w.n, mt // 8), dtype=torch.uint8, device=dev)
    norms = torch.empty((w.batch, w.kv_heads, w.n), dtype=torch.float16, device=dev)
    if w.m_out:      # timed: the quantizer itself; channel selection and the stacked sketch are one-off prompt-phase steps
        S_out = qjl.qjl_make_sketch(w.sketch_seed + 1000, w.m_out, w.d, w.dtype, dev)
        ch = qjl.qjl_select_outliers(K, 4)
        S = qjl.qjl_make_dual_sketch(S, S_out, ch)
        norms_out = torch.empty_like(norms)
        call = lambda: qjl.qjl_quantize_keys_dual(K, S, ch, w.m_out, bits, norms, norms_out)
    else:
        call = lambda: qjl.qjl_quantize_keys(K, S, bits, norms)
    stream = torch.cuda.current_stream().cuda_stream
    # one kernel per call, back to back: events bracket the kernels.  The warm-up is long enough (tens of
    # milliseconds) for the clocks to settle to what the chip holds under this load: the first hundred launches
    # after an idle stretch run about 10 % slower than the steady state that follows.
    ms = timed_launches(ev, stream, lambda i: call(), steps, warmup)
    rows = w.batch * w.kv_heads * w.n
    flops = 2.0 * w.d * mt * rows
    achieved = flops / (ms * 1e-3) / 1e12
    algo_bytes = rows * (w.d * 2 + mt // 8 + (4 if w.m_out else 2))
    return {
        "workload": w.name + ("_zero_operands" if zero_operands else ""),
        "metric": "prefill quantize tokens/s",
        "value": w.batch * w.n / (ms * 1e-3),
        "rows_per_s": rows / (ms * 1e-3),
        "ms_per_step": ms,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": load_traffic(w.name),
                     "ceiling": CEIL.get("mfma_TFLOPs"),
                     "frac_of_ceiling": achieved / CEIL["mfma_TFLOPs"] if CEIL.get("mfma_TFLOPs") else None,
                     "launches_back_to_back": steps,
                     "kernel": "quantize_slds_kernel" if mt <= 512 else "quantize_mfma_kernel", "kernel_ms": ms, "flops": flops,
                     "algorithmic_bytes": algo_bytes, "hbm_GBs": algo_bytes / (ms * 1e-3) / 1e9},
    }


def bench_scores(qjl, inputs, ev, w, dev, steps, warmup):
    """The estimator on its own (Eq. (4) for every cached key): S q, then one fp32 score per key and query head
    written to HBM.  34 bytes read per key and kv head, 4 written per key and query head."""
    import torch
    K = inputs.make_keys(w.batch, w.kv_heads, w.n, w.d, w.dtype, w.data_seed, dev, w.outliers)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, dev)
    bits, norms = qjl.qjl_quantize_keys(K, S)
    del K
    Q = inputs.make_normal((w.batch, w.q_heads, w.d), w.dtype, w.data_seed + 7919, dev)
    sq = torch.empty((w.batch, w.q_heads, w.m), dtype=torch.float32, device=dev)
    out = torch.empty((w.batch, w.q_heads, w.n), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream

    def step():
        qjl.qjl_project_query(Q, S, sq)
        qjl.qjl_scores(sq, bits, norms, w.scale, out=out)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    a, b = ev.create(), ev.create()
    ev.record(a, stream)
    for _ in range(steps):
        step()
    ev.record(b, stream)
    ms = ev.elapsed_ms(a, b) / steps
    ev.destroy(a)
    ev.destroy(b)
    algo_bytes = w.batch * w.n * (w.kv_heads * (w.m // 8 + 2) + w.q_heads * 4)
    achieved = algo_bytes / (ms * 1e-3) / 1e9
    return {
        "workload": w.name + "_scores_only",
        "metric": "estimated scores keys/s/GPU",
        "value": w.key_heads / (ms * 1e-3),
        "ms_per_step": ms,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "project128_kernel + scores_kernel",
                     "kernel_ms": ms, "algorithmic_bytes": algo_bytes},
    }


def bench_value_quantize(qjl, inputs, ev, w, dev, steps, warmup):
    """Token-wise 4-bit quantization of a value cache of the prefill workload's shape (HBM-bound)."""
    import torch
    V = inputs.make_normal((w.batch, w.kv_heads, w.n, w.d), w.dtype, w.data_seed + 104729, dev)
    vc = torch.empty((w.batch, w.kv_heads, w.n, w.d // 2), dtype=torch.uint8, device=dev)
    vs = torch.empty((w.batch, w.kv_heads, w.n), dtype=torch.float16, device=dev)
    vz = torch.empty_like(vs)
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(warmup):
        qjl.qjl_quantize_values(V, 4, vc, vs, vz)
    torch.cuda.synchronize()
    a, b = ev.create(), ev.create()
    ev.record(a, stream)
    for _ in range(steps):
        qjl.qjl_quantize_values(V, 4, vc, vs, vz)
    ev.record(b, stream)
    ms = ev.elapsed_ms(a, b) / steps
    ev.destroy(a)
    ev.destroy(b)
    rows = w.batch * w.kv_heads * w.n
    algo_bytes = rows * (w.d * 2 + w.d // 2 + 4)
    achieved = algo_bytes / (ms * 1e-3) / 1e9
    return {
        "workload": w.name + "_values_v4",
        "metric": "prefill value quantize tokens/s",
        "value": w.batch * w.n / (ms * 1e-3),
        "rows_per_s": rows / (ms * 1e-3),
        "ms_per_step": ms,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel": "value_quant_kernel",
                     "kernel_ms": ms, "algorithmic_bytes": algo_bytes},
    }


def bench_sketches(qjl, ev, dev):
    """One-off set-up kernels: the Gaussian sketch and its orthogonalised variant (Section 4.1), 256 x 128 bf16."""
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    out = {"workload": "sketch_256x128_bf16", "metric": "set-up kernel time", "unit": "us"}
    for name, fn in (("make_sketch_us", qjl.qjl_make_sketch), ("make_sketch_orthogonal_us", qjl.qjl_make_sketch_orthogonal)):
        for _ in range(3):
            fn(1, 256, 128, torch.bfloat16, dev)
        torch.cuda.synchronize()
        a, b = ev.create(), ev.create()
        ev.record(a, stream)
        for _ in range(20):
            fn(1, 256, 128, torch.bfloat16, dev)
        ev.record(b, stream)
        out[name] = ev.elapsed_ms(a, b) / 20 * 1e3
        ev.destroy(a)
        ev.destroy(b)
    return out


def bench_outlier_setup(qjl, inputs, ev, w, dev):
    """Prompt-phase set-up of the two-part code (Section 4.1) on the prefill keys: the per-channel magnitude pass
    with the selection of the outlier channels (reads every key once: 256 B per key and head against HBM), and
    the stacked per-head sketch."""
    import torch
    stream = torch.cuda.current_stream().cuda_stream
    K = inputs.make_keys(w.batch, w.kv_heads, w.n, w.d, w.dtype, w.data_seed, dev, w.outliers)
    S_in = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, dev)
    S_out = qjl.qjl_make_sketch(w.sketch_seed + 1000, w.m_out, w.d, w.dtype, dev)
    ch = torch.empty((w.batch, w.kv_heads, 4), dtype=torch.int32, device=dev)
    ws = torch.empty((1 << 24,), dtype=torch.uint8, device=dev)
    S_dual = qjl.qjl_make_dual_sketch(S_in, S_out, qjl.qjl_select_outliers(K, 4, channels=ch, workspace=ws))
    ms_sel = timed_launches(ev, stream, lambda i: qjl.qjl_select_outliers(K, 4, channels=ch, workspace=ws), 20, 3)
    ms_dual = timed_launches(ev, stream, lambda i: qjl.qjl_make_dual_sketch(S_in, S_out, ch, S_dual), 20, 3)
    nbytes = K.numel() * K.element_size()
    return {"workload": w.name + "_outlier_setup", "metric": "set-up kernel time", "unit": "us",
            "select_outliers_us": ms_sel * 1e3, "select_outliers_GBs": nbytes / (ms_sel * 1e-3) / 1e9,
            "select_outliers_frac_of_hbm_peak": nbytes / (ms_sel * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "make_dual_sketch_us": ms_dual * 1e3}


def _oracle_threads():
    from threadpoolctl import threadpool_info
    return max([p.get("num_threads", 1) for p in threadpool_info()] + [1])


def cpu_decode_baseline(qjl, inputs, w, dev, budget_s=10.0, units=None):
    """The oracle, as it stands, on the host cores: the same decode step (project -> scores -> softmax -> values) on a
    bounded sample of the workload -- the first batch entry (and, if `units` is given, its first `units` kv heads with
    their query heads), at the full context length.  The sample's keys are also quantized on the GPU and the two codes
    compared: the second return value counts the sign decisions that differ (Definition 3.1 with sign(0) = +1; entries
    with |(S k)_i| < 1e-5 ||s_i|| ||k|| are the near-zero band in which fp32 rounding may decide differently)."""
    import dataclasses
    import numpy as np
    import torch
    from threadpoolctl import threadpool_limits
    from oracle import qjl_oracle as orc
    G = w.q_heads // w.kv_heads
    kvh = min(units or w.kv_heads, w.kv_heads)
    ws = dataclasses.replace(w, batch=1, kv_heads=kvh, q_heads=kvh * G)
    K, Q, V = inputs.make_workload_tensors(ws, "cpu")
    S = orc.gaussian_sketch(w.sketch_seed, w.m, w.d, "bf16")
    K64, Q64, V64 = inputs.to_f64(K), inputs.to_f64(Q), inputs.to_f64(V)
    cores = min(16, os.cpu_count() or 1)
    with threadpool_limits(limits=cores):
        bits, nu16, P = orc.quantize_keys(K64, S)             # untimed, as on the GPU
        S_dev = torch.from_numpy(S).to(dev).to(w.dtype)       # exact: the oracle's sketch is already rounded to bf16
        gbits, _ = qjl.qjl_quantize_keys(K.to(dev), S_dev)
        diff = orc.unpack_signs(gbits.cpu().numpy(), w.m) != orc.unpack_signs(bits, w.m)
        band = np.abs(P) < 1e-5 * np.linalg.norm(S, axis=1) * np.linalg.norm(K64, axis=-1, keepdims=True)
        signs = {"sample": f"{ws.key_heads} keys x {w.m} projections of {w.name} (batch entry 0, {kvh} kv heads), GPU code against the oracle's",
                 "entries": int(diff.size), "near_zero_entries": int(band.sum()),
                 "near_zero_flips": int((diff & band).sum()), "mismatches_outside_band": int((diff & ~band).sum())}
        del P, diff, band, gbits
        orc.decode_attention(Q64, S, bits, nu16, V64, w.scale)   # warm-up
        reps, t0 = 0, time.perf_counter()
        while True:
            orc.decode_attention(Q64, S, bits, nu16, V64, w.scale)
            reps += 1
            el = time.perf_counter() - t0
            if el >= budget_s or reps >= 500:
                break
        used = _oracle_threads()
    base = {"value": ws.key_heads * reps / el, "unit": "keys/s", "cores": int(min(cores, used)), "kind": "oracle",
            "workload": w.name,
            "sample": f"{reps} decode steps over batch entry 0 of {w.batch}, {kvh} of {w.kv_heads} kv heads with their "
                      f"{kvh * G} query heads, full context {w.n} ({ws.key_heads} of {w.key_heads} keys per step), "
                      f"numpy float64, {el:.1f} s of CPU work"}
    return base, signs


def cpu_quantize_baseline(inputs, w, stride=16, budget_s=10.0):
    """The oracle's key quantizer (project, sign, pack, norm) on 1/stride of the prefill workload's tokens."""
    import dataclasses
    from threadpoolctl import threadpool_limits
    from oracle import qjl_oracle as orc
    ws = dataclasses.replace(w, n=w.n // stride)
    K = inputs.make_keys(ws.batch, ws.kv_heads, ws.n, ws.d, ws.dtype, ws.data_seed, "cpu", ws.outliers)
    S = orc.gaussian_sketch(w.sketch_seed, w.m, w.d, "bf16")
    K64 = inputs.to_f64(K)
    cores = min(16, os.cpu_count() or 1)
    with threadpool_limits(limits=cores):
        reps, t0 = 0, time.perf_counter()
        while True:
            orc.quantize_keys(K64, S)
            reps += 1
            el = time.perf_counter() - t0
            if el >= budget_s or reps >= 100:
                break
        used = _oracle_threads()
    return {"value": ws.batch * ws.n * reps / el, "unit": "tokens/s", "cores": int(min(cores, used)), "kind": "oracle",
            "workload": w.name,
            "sample": f"{reps} passes over {ws.n} of {w.n} tokens per head (1/{stride} of the workload, all {w.kv_heads} heads, "
                      f"{ws.batch * ws.kv_heads * ws.n} keys per pass), numpy float64, {el:.1f} s of CPU work"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="c3", help="headline workload: c3 (default: the largest configuration that one "
                    "GPU holds), c2, c5a, c5b (decode), c4 (prefill quantize), or c2d / c3d / c4d (the same with the outlier channels "
                    "quantized separately), c2v / c3v / c5bv (decode on a 4-bit value cache; c3v2, c3v8: 2 and 8 bits), c2s (append + decode), for profiling single kernels; "
                    "'copy' runs a plain 1 GiB device copy to calibrate the HBM byte counters; 'ceilings' only the calibration kernels")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baselines")
    ap.add_argument("--no-ceilings", action="store_true", help="skip the streaming-read and MFMA-loop calibration")
    ap.add_argument("--zero-operands", action="store_true", help="c4 / c4d only: time the quantizer on all-zero keys and sketch "
                    "(same instructions, no data toggling: shows how far the kernel is limited by power rather than by issue)")
    ap.add_argument("--cold", action="store_true", help="with --no-extra: also time the headline workload on rotating copies of its cache")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the hot path has no cross-GPU step); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2406_03482_amd as qjl
    from paper_2406_03482_amd import inputs
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    qjl.lib()                                   # fail loudly if the HIP library is missing
    dev = "cuda:0"
    ev = HipEvents()

    if args.workload == "copy":
        # calibration aid for the HBM counters: a plain device copy of known size
        # (1 GiB read + 1 GiB written per launch), nothing of the method
        C = Ceilings().L
        src = torch.ones((1 << 29,), dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        stream = torch.cuda.current_stream().cuda_stream
        for _ in range(max(1, args.steps)):
            C.ceil_copy(src.data_ptr(), dst.data_ptr(), src.numel() * 2, 256 * 8, stream)
        torch.cuda.synchronize()
        print(json.dumps({"workload": "copy", "kernel": "copy_kernel", "bytes_read_per_launch": src.numel() * 2,
                          "bytes_written_per_launch": src.numel() * 2, "launches": max(1, args.steps)}))
        return 0
    if not args.no_ceilings or args.workload == "ceilings":
        CEIL.update(measure_ceilings(ev, dev, quick=args.no_extra and args.workload != "ceilings"))
        torch.cuda.empty_cache()
    if args.workload == "ceilings":
        print(json.dumps({"workload": "ceilings", "ceilings": CEIL}))
        return 0
    names = {k.split("_")[0]: k for k in inputs.WORKLOADS}
    if args.workload not in names or args.workload == "c1":
        print(f"bench.py: unknown workload {args.workload!r}", file=sys.stderr)
        return 2
    w = inputs.WORKLOADS[names[args.workload]]
    if args.workload.startswith("c4"):
        head = bench_quantize(qjl, inputs, ev, w, dev, args.steps, args.warmup, zero_operands=args.zero_operands)
        head["ms_per_step_eager"] = head["ms_per_step"]
        r = {"graph_batch": 0}
    else:
        t = prepare_decode(qjl, inputs, w, dev)
        # the full run times the headline on rotating copies of its caches as well: even 1.2 GB replayed from one
        # buffer set is not quite what a step on caches last touched a model step ago sees (1-2 % apart)
        r = time_decode(qjl, ev, w, t, args.steps, args.warmup, cold=args.cold or not args.no_extra)
        head = decode_record(w, r)
        del t
    torch.cuda.empty_cache()

    line = {
        "metric": head["metric"],
        "value": head["value"],
        "unit": "tokens/s" if args.workload.startswith("c4") else "keys/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "ms_per_step_eager": head["ms_per_step_eager"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": head.get("workload", w.name), "batch": w.batch, "q_heads": w.q_heads, "kv_heads": w.kv_heads,
                   "context": w.n, "d": w.d, "m": w.m, "m_out": w.m_out, "vbits": w.vbits, "launch": f"hip graph of {r['graph_batch']} steps" if r["graph_batch"] else "eager, one kernel per step"},
        "roofline": head["roofline"],
        "ceilings": dict(CEIL) if CEIL else None,
    }
    for k in ("value_cold", "ms_per_step_cold"):
        if k in head:
            line[k] = head[k]

    if not args.no_extra:
        extra = []
        # (workload, steps, warm-up, also on rotating copies of the cache)
        for name, steps, warm, cold in [("c2_llama2_7b_decode_4k", 2000, 200, True), ("c5a_llama3_8b_gqa_b1_128k", 200, 20, True),
                                        ("c5b_llama3_8b_gqa_b16_8k", 200, 20, True), ("c3_long_context_b4_32k", 100, 20, False),
                                        ("c2d_llama2_7b_decode_4k_dual", 400, 40, False),
                                        ("c3d_long_context_b4_32k_dual", 100, 20, False), ("c2v_llama2_7b_decode_4k_v4", 400, 40, False),
                                        ("c3v_long_context_b4_32k_v4", 100, 20, False), ("c5bv_llama3_8b_gqa_b16_8k_v4", 200, 20, False),
                                        ("c2s_llama2_7b_decode_step_4k", 400, 40, False),
                                        ("c3o_long_context_b4_32k_dual_v4", 100, 20, False),
                                        ("c5bo_llama3_8b_gqa_b16_8k_dual_v4", 200, 20, False),
                                        ("c2o_llama2_7b_generation_step_4k_dual_v4", 400, 40, False)]:
            wx = inputs.WORKLOADS[name]
            if wx.name == w.name:
                continue
            tx = prepare_decode(qjl, inputs, wx, dev)
            extra.append(decode_record(wx, time_decode(qjl, ev, wx, tx, steps, warm, cold=cold)))
            del tx
            torch.cuda.empty_cache()
        if not args.workload.startswith("c4"):
            extra.append(bench_quantize(qjl, inputs, ev, inputs.WORKLOADS["c4_prefill_quantize_64k"], dev, 200, 100))
        extra.append(bench_quantize(qjl, inputs, ev, inputs.WORKLOADS["c4d_prefill_quantize_64k_dual"], dev, 200, 100))
        extra.append(bench_value_quantize(qjl, inputs, ev, inputs.WORKLOADS["c4_prefill_quantize_64k"], dev, 50, 5))
        extra.append(bench_scores(qjl, inputs, ev, inputs.WORKLOADS["c3_long_context_b4_32k"], dev, 100, 10))
        line["setup_kernels"] = bench_sketches(qjl, ev, dev)
        line["setup_kernels_outliers"] = bench_outlier_setup(qjl, inputs, ev, inputs.WORKLOADS["c4d_prefill_quantize_64k_dual"], dev)
        line["other_workloads"] = extra

    line["cpu_baseline"] = None
    if not args.no_cpu:
        plain = lambda x: not x.m_out and not x.vbits and not x.stream
        if args.workload.startswith("c4") and not w.m_out:
            line["cpu_baseline"] = cpu_quantize_baseline(inputs, w)
        elif plain(w):
            line["cpu_baseline"], line["sign_bits"] = cpu_decode_baseline(qjl, inputs, w, dev)
        if not args.no_extra:
            others = []
            w5, w4 = inputs.WORKLOADS["c5a_llama3_8b_gqa_b1_128k"], inputs.WORKLOADS["c4_prefill_quantize_64k"]
            if w.name != w5.name:
                others.append(cpu_decode_baseline(qjl, inputs, w5, dev, budget_s=8.0, units=2)[0])
            if w.name != w4.name:
                others.append(cpu_quantize_baseline(inputs, w4, budget_s=8.0))
            line["cpu_baselines_other"] = others
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
