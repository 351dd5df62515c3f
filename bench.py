#!/usr/bin/env python3
"""Benchmark of the QJL hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-extra] [--no-cpu]

A "step" is one decode step of the Llama-2-7B-shaped workload (batch 1, 32
heads, d = 128, m = 256, context 4096; keys already quantized and everything
resident in HBM): project the query, estimate all scores, softmax, aggregate
the bf16 values -- one call of qjl_decode_attention.  The headline `value` is
keys (= batch x kv-head x token triples) per second over exactly K steps; the
steps are replayed from a HIP graph so that the host's launch cost does not
hide the GPU time (the eager rate is reported next to it).

The `roofline` object is for the attention kernel of that step: algorithmic
bytes per launch (290 B per key: 32 B code + 2 B norm + 256 B values) over the
kernel's mean duration measured with HIP events recorded around the kernel
itself (qjl_decode_attention_timed).  `other_workloads` repeats the
measurement for the long-context, GQA and prefill-quantize configurations.
`cpu_baseline` times the CPU oracle on the same workload.
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
        del K
        ws = torch.empty((qjl.qjl_decode_dual_workspace_bytes(w.batch, w.q_heads, w.kv_heads, w.n, w.d, w.m,
                                                              w.m_out, w.dtype),), dtype=torch.uint8, device=dev)
        out = torch.empty((w.batch, w.q_heads, w.d), dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        return dict(Q=Q, S=S, bits=bits, norms=norms, norms_out=norms_out, V=V, ws=ws, out=out)
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


def time_decode(qjl, ev, w, t, steps, warmup, graph_batch=None):
    """Returns dict(ms_graph, ms_eager, kernel_ms) for one workload."""
    import torch
    stream = torch.cuda.current_stream().cuda_stream
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
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_decode(qjl, t, w)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(gb):
            run_decode(qjl, t, w)
    for _ in range(max(1, warmup // gb)):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps // gb):
        g.replay()
    torch.cuda.synchronize()
    ms_graph = (time.perf_counter() - t0) * 1e3 / steps
    if w.stream:        # no kernel-timestamp variant of this call: the roofline figure uses the whole step
        return dict(ms_graph=ms_graph, ms_eager=ms_eager, kernel_ms=ms_graph, kernel_ms_median=ms_graph, graph_batch=gb)
    # ---- the attention kernel alone: events recorded around it inside the library call
    nk = min(steps, 200)
    pairs = [(ev.create(), ev.create()) for _ in range(nk)]
    for a, b in pairs:
        run_decode(qjl, t, w, events=(a, b))
    torch.cuda.synchronize()
    durs = sorted(ev.elapsed_ms(a, b) for a, b in pairs)
    for a, b in pairs:
        ev.destroy(a)
        ev.destroy(b)
    kernel_ms = sum(durs) / len(durs)
    return dict(ms_graph=ms_graph, ms_eager=ms_eager, kernel_ms=kernel_ms, kernel_ms_median=durs[len(durs) // 2],
                graph_batch=gb)


def decode_record(w, r):
    algo_bytes = decode_bytes_per_key(w) * w.key_heads
    achieved = algo_bytes / (r["kernel_ms"] * 1e-3) / 1e9
    return {
        "workload": w.name,
        "metric": "decode keys/s/GPU",
        "value": w.key_heads / (r["ms_graph"] * 1e-3),
        "ms_per_step": r["ms_graph"],
        "ms_per_step_eager": r["ms_eager"],
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": load_traffic(w.name),
                     "kernel": "decode_kernel", "kernel_ms": r["kernel_ms"],
                     "kernel_ms_median": r["kernel_ms_median"], "algorithmic_bytes": algo_bytes},
    }


def bench_quantize(qjl, inputs, ev, w, dev, steps, warmup):
    import torch
    K = inputs.make_keys(w.batch, w.kv_heads, w.n, w.d, w.dtype, w.data_seed, dev, w.outliers)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, dev)
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
    for _ in range(warmup):
        call()
    torch.cuda.synchronize()
    a, b = ev.create(), ev.create()
    ev.record(a, stream)
    for _ in range(steps):
        call()
    ev.record(b, stream)
    ms = ev.elapsed_ms(a, b) / steps          # one kernel per call, back to back: events bracket the kernels
    ev.destroy(a)
    ev.destroy(b)
    rows = w.batch * w.kv_heads * w.n
    flops = 2.0 * w.d * mt * rows
    achieved = flops / (ms * 1e-3) / 1e12
    algo_bytes = rows * (w.d * 2 + mt // 8 + (4 if w.m_out else 2))
    return {
        "workload": w.name,
        "metric": "prefill quantize tokens/s",
        "value": w.batch * w.n / (ms * 1e-3),
        "rows_per_s": rows / (ms * 1e-3),
        "ms_per_step": ms,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": load_traffic(w.name),
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


def cpu_baseline(inputs, w, budget_s=12.0):
    """The oracle, as it stands, on the host cores: the same decode step
    (project -> scores -> softmax -> values) on the same workload."""
    import numpy as np
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import qjl_oracle as orc
    K, Q, V = inputs.make_workload_tensors(w, "cpu")
    S = orc.gaussian_sketch(w.sketch_seed, w.m, w.d, "bf16")
    K64, Q64, V64 = inputs.to_f64(K), inputs.to_f64(Q), inputs.to_f64(V)
    bits, nu16, _ = orc.quantize_keys(K64, S)             # untimed, as on the GPU
    cores = min(16, os.cpu_count() or 1)
    with threadpool_limits(limits=cores):
        orc.decode_attention(Q64, S, bits, nu16, V64, w.scale)   # warm-up
        reps, t0 = 0, time.perf_counter()
        while True:
            orc.decode_attention(Q64, S, bits, nu16, V64, w.scale)
            reps += 1
            el = time.perf_counter() - t0
            if el >= budget_s or reps >= 500:
                break
        used = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    return {"value": w.key_heads * reps / el, "unit": "keys/s", "cores": int(min(cores, used)), "kind": "oracle",
            "sample": f"{reps} full decode steps of {w.name} (all {w.key_heads} keys each), numpy float64, "
                      f"{el:.1f} s of CPU work"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="c2", help="headline workload: c2 (default, the configuration the "
                    "metric is quoted on), c3, c5a, c5b (decode), c4 (prefill quantize), or c2d / c3d / c4d (the same with the outlier channels "
                    "quantized separately), c2v / c3v / c5bv (decode on a 4-bit value cache; c3v2, c3v8: 2 and 8 bits), c2s (append + decode), for profiling single kernels; "
                    "'copy' runs a plain 1 GiB device copy to calibrate the HBM byte counters")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
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
        src = torch.ones((1 << 29,), dtype=torch.bfloat16, device=dev)
        dst = torch.empty_like(src)
        for _ in range(max(1, args.steps)):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"workload": "copy", "bytes_read_per_launch": src.numel() * 2,
                          "bytes_written_per_launch": src.numel() * 2, "launches": max(1, args.steps)}))
        return 0
    names = {k.split("_")[0]: k for k in inputs.WORKLOADS}
    if args.workload not in names or args.workload == "c1":
        print(f"bench.py: unknown workload {args.workload!r}", file=sys.stderr)
        return 2
    w = inputs.WORKLOADS[names[args.workload]]
    if args.workload.startswith("c4"):
        head = bench_quantize(qjl, inputs, ev, w, dev, args.steps, args.warmup)
        head["ms_per_step_eager"] = head["ms_per_step"]
        r = {"graph_batch": 0}
    else:
        t = prepare_decode(qjl, inputs, w, dev)
        r = time_decode(qjl, ev, w, t, args.steps, args.warmup)
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
        "config": {"workload": w.name, "batch": w.batch, "q_heads": w.q_heads, "kv_heads": w.kv_heads,
                   "context": w.n, "d": w.d, "m": w.m, "m_out": w.m_out, "vbits": w.vbits, "launch": f"hip graph of {r['graph_batch']} steps" if r["graph_batch"] else "eager, one kernel per step"},
        "roofline": head["roofline"],
    }

    if not args.no_extra:
        extra = []
        for name, steps, warm in [("c3_long_context_b4_32k", 100, 20), ("c5a_llama3_8b_gqa_b1_128k", 200, 20),
                                  ("c5b_llama3_8b_gqa_b16_8k", 200, 20), ("c2d_llama2_7b_decode_4k_dual", 400, 40),
                                  ("c3d_long_context_b4_32k_dual", 100, 20), ("c2v_llama2_7b_decode_4k_v4", 400, 40),
                                  ("c3v_long_context_b4_32k_v4", 100, 20), ("c5bv_llama3_8b_gqa_b16_8k_v4", 200, 20),
                                  ("c2s_llama2_7b_decode_step_4k", 400, 40)]:
            wx = inputs.WORKLOADS[name]
            tx = prepare_decode(qjl, inputs, wx, dev)
            extra.append(decode_record(wx, time_decode(qjl, ev, wx, tx, steps, warm)))
            del tx
            torch.cuda.empty_cache()
        extra.append(bench_quantize(qjl, inputs, ev, inputs.WORKLOADS["c4_prefill_quantize_64k"], dev, 50, 5))
        extra.append(bench_quantize(qjl, inputs, ev, inputs.WORKLOADS["c4d_prefill_quantize_64k_dual"], dev, 50, 5))
        extra.append(bench_value_quantize(qjl, inputs, ev, inputs.WORKLOADS["c4_prefill_quantize_64k"], dev, 50, 5))
        extra.append(bench_scores(qjl, inputs, ev, inputs.WORKLOADS["c3_long_context_b4_32k"], dev, 100, 10))
        line["setup_kernels"] = bench_sketches(qjl, ev, dev)
        line["other_workloads"] = extra

    if not args.no_cpu and not args.workload.startswith("c4") and not w.m_out and not w.vbits and not w.stream:
        line["cpu_baseline"] = cpu_baseline(inputs, w)
    else:
        line["cpu_baseline"] = None
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
