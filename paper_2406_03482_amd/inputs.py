"""Seeded synthetic inputs shaped like the paper's workloads.

Serves the tests, the smoke check and the benchmark, and is the only module
that both the GPU-side callers and the oracle-side callers use.  It contains
no part of the method: only shapes and random tensors.

Recipe: keys, queries and values are i.i.d. N(0,1) drawn in fp32 and rounded
to the storage dtype; in every KV head four channel indices (fixed for all
tokens and batches, drawn without replacement from the seed) carry keys scaled
by 15, mimicking the few large fixed channels the paper observes in deep
layers (Section 4.1, Figure 2).  Stand-in for real model activations, which
need weights and datasets that are not available here.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict

import torch


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    q_heads: int
    kv_heads: int
    n: int
    d: int
    m: int
    dtype: torch.dtype
    scale: float
    data_seed: int
    sketch_seed: int
    outliers: int = 4
    m_out: int = 0          # > 0: outlier channels get a second sketch of m_out rows (m is the inlier sketch)
    vbits: int = 0          # > 0: the value cache is quantized token-wise to vbits bits per entry
    stream: bool = False    # a generation step: the last key is quantized and appended, then attention runs

    @property
    def key_heads(self) -> int:
        """(batch, kv head, token) triples: the unit of the decode metric."""
        return self.batch * self.kv_heads * self.n


_RS = 1.0 / math.sqrt(128.0)

WORKLOADS: Dict[str, Workload] = {w.name: w for w in [
    # single head, everything N(0,1), fp32, the paper's softmax without 1/sqrt(d)
    Workload("c1_single_head", 1, 1, 1, 1024, 128, 256, torch.float32, 1.0, 1001, 1, outliers=0),
    # Llama-2-7B-shaped decode step
    Workload("c2_llama2_7b_decode_4k", 1, 32, 32, 4096, 128, 256, torch.bfloat16, _RS, 1002, 2),
    # long-context decode
    Workload("c3_long_context_b4_32k", 4, 32, 32, 32768, 128, 256, torch.bfloat16, _RS, 1003, 3),
    # prefill quantize
    Workload("c4_prefill_quantize_64k", 1, 32, 32, 65536, 128, 512, torch.bfloat16, _RS, 1004, 4),
    # Llama-3-8B-shaped grouped-query decode, two shapes
    Workload("c5a_llama3_8b_gqa_b1_128k", 1, 32, 8, 131072, 128, 256, torch.bfloat16, _RS, 1005, 5),
    Workload("c5b_llama3_8b_gqa_b16_8k", 16, 32, 8, 8192, 128, 256, torch.bfloat16, _RS, 1006, 5),
    # the same shapes with the outlier channels quantized separately: 256 + 128 bits = 3 bits per coordinate
    Workload("c2d_llama2_7b_decode_4k_dual", 1, 32, 32, 4096, 128, 256, torch.bfloat16, _RS, 1002, 2, m_out=128),
    Workload("c3d_long_context_b4_32k_dual", 4, 32, 32, 32768, 128, 256, torch.bfloat16, _RS, 1003, 3, m_out=128),
    Workload("c4d_prefill_quantize_64k_dual", 1, 32, 32, 65536, 128, 256, torch.bfloat16, _RS, 1004, 4, m_out=128),
    # the decode shapes with a 4-bit value cache as well (Section 3.2)
    Workload("c2v_llama2_7b_decode_4k_v4", 1, 32, 32, 4096, 128, 256, torch.bfloat16, _RS, 1002, 2, vbits=4),
    Workload("c3v_long_context_b4_32k_v4", 4, 32, 32, 32768, 128, 256, torch.bfloat16, _RS, 1003, 3, vbits=4),
    Workload("c5bv_llama3_8b_gqa_b16_8k_v4", 16, 32, 8, 8192, 128, 256, torch.bfloat16, _RS, 1006, 5, vbits=4),
    # the long-context shape with 2-bit and 8-bit value codes
    Workload("c3v2_long_context_b4_32k_v2", 4, 32, 32, 32768, 128, 256, torch.bfloat16, _RS, 1003, 3, vbits=2),
    Workload("c3v8_long_context_b4_32k_v8", 4, 32, 32, 32768, 128, 256, torch.bfloat16, _RS, 1003, 3, vbits=8),
    # the paper's operating point: 256 + 128 code bits per key (3 bits per coordinate) and 4-bit values, on the
    # long-context and grouped-query shapes; and a whole generation step (append key and value, then attend)
    Workload("c3o_long_context_b4_32k_dual_v4", 4, 32, 32, 32768, 128, 256, torch.bfloat16, _RS, 1003, 3, m_out=128, vbits=4),
    Workload("c5bo_llama3_8b_gqa_b16_8k_dual_v4", 16, 32, 8, 8192, 128, 256, torch.bfloat16, _RS, 1006, 5, m_out=128, vbits=4),
    Workload("c2o_llama2_7b_generation_step_4k_dual_v4", 1, 32, 32, 4096, 128, 256, torch.bfloat16, _RS, 1002, 2, m_out=128,
             vbits=4, stream=True),
    # a whole generation step on the headline shape: append the newest key (Algorithm 1's loop), then attend
    Workload("c2s_llama2_7b_decode_step_4k", 1, 32, 32, 4096, 128, 256, torch.bfloat16, _RS, 1002, 2, stream=True),
]}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def outlier_channels(kv_heads: int, d: int, count: int, seed: int) -> torch.Tensor:
    """[kv_heads, count] channel indices, distinct inside a head (CPU, int64)."""
    g = _gen("cpu", seed ^ 0x5EED)
    return torch.stack([torch.randperm(d, generator=g)[:count] for _ in range(kv_heads)])


def make_keys(batch: int, kv_heads: int, n: int, d: int, dtype: torch.dtype, seed: int,
              device="cpu", outliers: int = 4, outlier_scale: float = 15.0) -> torch.Tensor:
    g = _gen(device, seed)
    K = torch.empty((batch, kv_heads, n, d), dtype=dtype, device=device)
    ch = outlier_channels(kv_heads, d, outliers, seed).to(device) if outliers > 0 else None
    for b in range(batch):                      # one batch entry at a time bounds the fp32 transient
        x = torch.randn((kv_heads, n, d), generator=g, device=device, dtype=torch.float32)
        if ch is not None:
            mult = torch.ones((kv_heads, 1, d), device=device)
            mult.scatter_(2, ch[:, None, :], outlier_scale)
            x *= mult
        K[b] = x.to(dtype)
    return K


def make_normal(shape, dtype: torch.dtype, seed: int, device="cpu") -> torch.Tensor:
    g = _gen(device, seed)
    lead = shape[0]
    out = torch.empty(shape, dtype=dtype, device=device)
    for b in range(lead):
        out[b] = torch.randn(shape[1:], generator=g, device=device, dtype=torch.float32).to(dtype)
    return out


def make_workload_tensors(w: Workload, device="cpu", need_values: bool = True):
    """(K, Q, V) for a workload; V is None when need_values is False."""
    K = make_keys(w.batch, w.kv_heads, w.n, w.d, w.dtype, w.data_seed, device, w.outliers)
    Q = make_normal((w.batch, w.q_heads, w.d), w.dtype, w.data_seed + 7919, device)
    V = make_normal((w.batch, w.kv_heads, w.n, w.d), w.dtype, w.data_seed + 104729, device) \
        if need_values else None
    return K, Q, V


def to_f64(t: torch.Tensor):
    """Exact float64 numpy view of a stored tensor (for the oracle side)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
