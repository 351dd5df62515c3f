"""GPU-vs-oracle parity, through the C ABI (python binding = marshalling only).

Tolerances (stated by the build's goal):
  * packed sign bits: bit-exact, except entries with |(S k)_i| < 1e-5 ||s_i|| ||k||,
    which are counted and reported;
  * norms and scores: 1e-3 relative (scores: relative to max(|ref|, 1e-2 rms of
    the head's scores), since an unbiased estimate of a small inner product can
    be arbitrarily close to zero);
  * attention outputs: 2e-3 max absolute error.
Each stage is fed the oracle's own outputs of the stage before it, so that no
oracle input comes from the GPU.
"""
import math
import os

import numpy as np
import pytest
import torch

import paper_2406_03482_amd as qjl
from paper_2406_03482_amd import inputs
from oracle import qjl_oracle as orc

pytestmark = pytest.mark.gpu

DEV = "cuda"
DT = {"bf16": torch.bfloat16, "f16": torch.float16, "f32": torch.float32}


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    assert os.path.exists(qjl.lib_path()), "libqjl.so must be built before the GPU tests run"
    qjl.lib()


# ------------------------------------------------------------------ comparison helpers
def bits_report(bits_gpu: np.ndarray, K64: np.ndarray, S64: np.ndarray):
    """(mismatches outside the near-zero band, flips inside it, entries inside it)."""
    ref_bits, _, P = orc.quantize_keys(K64, S64)
    m = S64.shape[0]
    diff = orc.unpack_signs(bits_gpu, m) != orc.unpack_signs(ref_bits, m)
    band = np.abs(P) < 1e-5 * np.linalg.norm(S64, axis=1) * np.linalg.norm(K64, axis=-1, keepdims=True)
    return int((diff & ~band).sum()), int((diff & band).sum()), int(band.sum())


def assert_norms(norms_gpu: np.ndarray, K64: np.ndarray):
    ref = np.linalg.norm(K64, axis=-1)
    got = norms_gpu.astype(np.float64)
    assert np.all(np.abs(got - ref) <= 1e-3 * ref + 1e-30)
    # and never further than one binary16 step from the oracle's stored value
    ref16 = orc.key_norms(K64)
    step = np.abs(np.nextafter(ref16, np.float16(np.inf)).astype(np.float64) - ref16.astype(np.float64))
    assert np.all(np.abs(got - ref16.astype(np.float64)) <= step)
    return float(np.mean(norms_gpu == ref16))


def assert_scores(got: np.ndarray, ref: np.ndarray):
    rms = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    tol = 1e-3 * np.maximum(np.abs(ref), 1e-2 * rms)
    err = np.abs(got.astype(np.float64) - ref)
    assert np.all(err <= tol), f"score error {float((err / tol).max()):.3g} x tolerance"
    return float((err / tol).max())


def assert_attention(got: np.ndarray, ref: np.ndarray):
    err = float(np.max(np.abs(got.astype(np.float64) - ref)))
    assert err <= 2e-3, f"attention max abs error {err:.3g}"
    return err


def oracle_cache(K, S):
    """Oracle-quantized cache of K, uploaded: (bits, norms) device tensors + numpy twins."""
    bits, nu16, _ = orc.quantize_keys(inputs.to_f64(K), inputs.to_f64(S))
    return (torch.from_numpy(bits).to(DEV), torch.from_numpy(nu16).to(DEV)), (bits, nu16)


# ------------------------------------------------------------------ a0: the sketch
@pytest.mark.parametrize("dt", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("m,d,seed", [(256, 128, 1), (512, 128, 4), (40, 24, 99)])
def test_make_sketch_matches_oracle_generator(dt, m, d, seed):
    say(f"[sketch] dt={dt} m={m} d={d} seed={seed}")
    S = qjl.qjl_make_sketch(seed, m, d, DT[dt], DEV)
    got = inputs.to_f64(S)
    ref = orc.gaussian_sketch(seed, m, d, dt)
    exact = float(np.mean(got == ref))
    ulp = {"f32": 2.0 ** -23, "bf16": 2.0 ** -7, "f16": 2.0 ** -10}[dt]
    assert np.all(np.abs(got - ref) <= ulp * np.maximum(np.abs(ref), 2.0 ** -14))
    assert exact > 0.999                      # libm differences may move a rounding, rarely
    S2 = qjl.qjl_make_sketch(seed, m, d, DT[dt], DEV)
    assert torch.equal(S, S2)
    say(f"  exact fraction {exact:.6f}")


# ------------------------------------------------------------------ a1-a3: quantize keys
QUANT_CASES = [
    # dt, B, Hkv, n, d, m, outliers
    ("bf16", 1, 2, 1000, 128, 256, 4),       # MFMA, ragged last tile
    ("bf16", 2, 3, 257, 128, 512, 4),        # MFMA m=512 (128 projections per wave)
    ("bf16", 1, 1, 95, 128, 128, 4),         # MFMA m=128 (32 projections per wave, 16-bit stores)
    ("bf16", 1, 1, 70, 128, 384, 0),         # three blocks of 128 projections
    ("bf16", 1, 1, 33, 128, 1024, 0),        # two blocks of 512 projections
    ("bf16", 2, 2, 1500, 128, 1024, 4),      # the same over many tiles: sketch rows in registers, keys through LDS
    ("f16", 1, 3, 700, 128, 768, 4),         # two blocks of 384 projections (three computing waves per workgroup)
    ("bf16", 1, 2, 300, 128, 640, 4),        # 640 = 5 x 128: 32 projections per wave
    ("f16", 1, 2, 513, 128, 256, 4),         # fp16 MFMA
    ("f16", 1, 1, 64, 128, 512, 0),
    ("bf16", 1, 1, 1, 128, 256, 0),          # a single key
    ("bf16", 1, 1, 31, 128, 256, 4),         # fewer keys than one tile
    ("f32", 1, 1, 1024, 128, 256, 0),        # config 1 keys: fp32 FMA path
    ("f32", 2, 2, 37, 128, 512, 4),
    ("bf16", 1, 2, 50, 64, 96, 0),           # generic path: other d, m % 32 == 0
    ("f16", 1, 1, 19, 40, 32, 0),
    ("f32", 1, 1, 9, 8, 32, 0),
]


@pytest.mark.parametrize("dt,B,Hkv,n,d,m,outl", QUANT_CASES)
def test_quantize_keys_parity(dt, B, Hkv, n, d, m, outl):
    say(f"[quantize] dt={dt} B={B} Hkv={Hkv} n={n} d={d} m={m}")
    K = inputs.make_keys(B, Hkv, n, d, DT[dt], 7 + n, DEV, outliers=outl)
    S = qjl.qjl_make_sketch(3, m, d, DT[dt], DEV)
    bits, norms = qjl.qjl_quantize_keys(K, S)
    torch.cuda.synchronize()
    K64, S64 = inputs.to_f64(K), inputs.to_f64(S)
    bad, flips, inband = bits_report(bits.cpu().numpy(), K64, S64)
    say(f"  bits: {bad} mismatches outside the band, {flips} flips among {inband} near-zero entries "
        f"of {B * Hkv * n * m}")
    assert bad == 0
    same = assert_norms(norms.cpu().numpy(), K64)
    say(f"  norms: {same:.4f} identical to the oracle's binary16 value")
    bits2, norms2 = qjl.qjl_quantize_keys(K, S)
    assert torch.equal(bits, bits2) and torch.equal(norms, norms2)      # deterministic


def test_quantize_zero_and_tiny_keys():
    """||k|| = 0 -> norm 0 and all bits 1 (sign(0) := +1); -k flips every bit."""
    say("[quantize] zero keys and negation")
    K = inputs.make_keys(1, 1, 64, 128, torch.bfloat16, 5, DEV)
    K[0, 0, 3] = 0
    K[0, 0, 40] = 0
    S = qjl.qjl_make_sketch(3, 256, 128, torch.bfloat16, DEV)
    bits, norms = qjl.qjl_quantize_keys(K, S)
    assert bits[0, 0, 3].eq(255).all() and bits[0, 0, 40].eq(255).all()
    assert norms[0, 0, 3] == 0 and norms[0, 0, 40] == 0
    nb, nn = qjl.qjl_quantize_keys(-K, S)
    keep = torch.ones(64, dtype=torch.bool, device=DEV)
    keep[3] = keep[40] = False
    assert torch.equal(nb[0, 0, keep], ~bits[0, 0, keep]) and torch.equal(nn, norms)
    K32 = K.float()
    S32 = S.float()
    b32, n32 = qjl.qjl_quantize_keys(K32, S32)                          # same values via the fp32 path
    bad, flips, _ = bits_report(b32.cpu().numpy(), inputs.to_f64(K32), inputs.to_f64(S32))
    assert bad == 0
    assert b32[0, 0, 3].eq(255).all() and n32[0, 0, 3] == 0


# ------------------------------------------------------------------ b1: project the query
@pytest.mark.parametrize("dt,B,Hq,d,m", [("bf16", 1, 32, 128, 256), ("f32", 1, 1, 128, 256),
                                         ("f16", 3, 5, 128, 512), ("bf16", 2, 3, 128, 40),
                                         ("f32", 2, 2, 24, 40), ("bf16", 1, 4, 64, 96)])
def test_project_query_parity(dt, B, Hq, d, m):
    say(f"[project] dt={dt} B={B} Hq={Hq} d={d} m={m}")
    Q = inputs.make_normal((B, Hq, d), DT[dt], 21, DEV)
    S = qjl.qjl_make_sketch(8, m, d, DT[dt], DEV)
    SQ = qjl.qjl_project_query(Q, S).cpu().numpy()
    ref = orc.project_query(inputs.to_f64(Q), inputs.to_f64(S))
    scale = np.linalg.norm(inputs.to_f64(Q), axis=-1, keepdims=True) * np.linalg.norm(inputs.to_f64(S), axis=1)
    assert np.all(np.abs(SQ - ref) <= 1e-5 * scale)


# ------------------------------------------------------------------ b2: scores
@pytest.mark.parametrize("B,Hq,Hkv,n,m,scale", [
    (1, 1, 1, 1024, 256, 1.0), (1, 4, 4, 3000, 256, 0.0884), (2, 8, 2, 777, 256, 0.0884),
    (1, 6, 3, 300, 512, 1.0), (1, 3, 3, 65, 128, 0.5), (1, 8, 1, 2500, 128, 1.0),
    (1, 2, 1, 1, 256, 1.0)])
def test_scores_parity(B, Hq, Hkv, n, m, scale):
    say(f"[scores] B={B} Hq={Hq} Hkv={Hkv} n={n} m={m} scale={scale}")
    d = 128
    K = inputs.make_keys(B, Hkv, n, d, torch.bfloat16, 31 + n, DEV)
    Q = inputs.make_normal((B, Hq, d), torch.bfloat16, 32, DEV)
    S = qjl.qjl_make_sketch(9, m, d, torch.bfloat16, DEV)
    (bits_d, nu_d), (bits, nu16) = oracle_cache(K, S)
    SQ64 = orc.project_query(inputs.to_f64(Q), inputs.to_f64(S))
    SQ_d = torch.from_numpy(SQ64.astype(np.float32)).to(DEV)
    got = qjl.qjl_scores(SQ_d, bits_d, nu_d, scale).cpu().numpy()
    ref = orc.estimate_scores(SQ64.astype(np.float32).astype(np.float64), bits, nu16, scale)
    worst = assert_scores(got, ref)
    say(f"  worst error / tolerance = {worst:.3g}")


# ------------------------------------------------------------------ c1-c3: decode attention
DECODE_CASES = [
    # dt, B, Hq, Hkv, n, m, scale
    ("f32", 1, 1, 1, 1024, 256, 1.0),            # config 1
    ("f32", 2, 8, 2, 777, 256, 0.0884),          # fp32, GQA x4
    ("f32", 1, 2, 1, 300, 512, 0.0884),          # fp32, m = 512, GQA x2
    ("f32", 1, 4, 1, 1100, 128, 1.0),            # fp32, m = 128, GQA x4
    ("bf16", 1, 4, 4, 4096, 256, 0.0884),        # config-2 heads
    ("bf16", 2, 8, 2, 1500, 256, 0.0884),        # GQA x4, ragged
    ("bf16", 1, 8, 4, 333, 256, 1.0),            # GQA x2, paper-literal scale
    ("bf16", 1, 3, 1, 700, 256, 0.0884),         # GQA x3 -> one head at a time
    ("f16", 1, 4, 1, 260, 512, 0.0884),          # m=512, fp16
    ("bf16", 1, 4, 1, 129, 128, 0.0884),         # m=128
    ("bf16", 1, 2, 2, 1, 256, 1.0),              # n = 1: out = v_1
    ("bf16", 1, 1, 1, 63, 256, 0.0884),
    ("bf16", 1, 1, 1, 65, 256, 0.0884),
    ("bf16", 1, 2, 1, 20000, 256, 0.0884),       # many chunks
]


@pytest.mark.parametrize("dt,B,Hq,Hkv,n,m,scale", DECODE_CASES)
def test_decode_attention_parity(dt, B, Hq, Hkv, n, m, scale):
    say(f"[decode] dt={dt} B={B} Hq={Hq} Hkv={Hkv} n={n} m={m} scale={scale}")
    d = 128
    K = inputs.make_keys(B, Hkv, n, d, DT[dt], 41 + n, DEV, outliers=0 if dt == "f32" else 4)
    Q = inputs.make_normal((B, Hq, d), DT[dt], 42, DEV)
    V = inputs.make_normal((B, Hkv, n, d), DT[dt], 43, DEV)
    S = qjl.qjl_make_sketch(10, m, d, DT[dt], DEV)
    (bits_d, nu_d), (bits, nu16) = oracle_cache(K, S)
    ref = orc.decode_attention(inputs.to_f64(Q), inputs.to_f64(S), bits, nu16, inputs.to_f64(V), scale)
    out = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale)
    err = assert_attention(out.cpu().numpy(), ref)
    say(f"  max abs error {err:.3g}")
    # a second call on the same workspace-free path gives the same bits
    out2 = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale)
    assert torch.equal(out, out2)


@pytest.mark.parametrize("splits", [1, 2, 7, 64])
def test_decode_split_count_does_not_matter(splits):
    say(f"[decode] forced chunk count {splits}")
    B, Hq, Hkv, n, d, m = 1, 8, 2, 5000, 128, 256
    K = inputs.make_keys(B, Hkv, n, d, torch.bfloat16, 51, DEV)
    Q = inputs.make_normal((B, Hq, d), torch.bfloat16, 52, DEV)
    V = inputs.make_normal((B, Hkv, n, d), torch.bfloat16, 53, DEV)
    S = qjl.qjl_make_sketch(11, m, d, torch.bfloat16, DEV)
    (bits_d, nu_d), (bits, nu16) = oracle_cache(K, S)
    ref = orc.decode_attention(inputs.to_f64(Q), inputs.to_f64(S), bits, nu16, inputs.to_f64(V), 0.0884)
    need, _, got_splits, _ = qjl.qjl_decode_plan(B, Hq, Hkv, n, d, m, 0, splits)
    assert got_splits == (splits if splits < 64 else 10)   # 8 waves x 64 keys per chunk at least: 5000 keys -> 10
    ws = torch.full((need,), 0xAB, dtype=torch.uint8, device=DEV)   # dirty workspace: contents must not matter
    for _ in range(3):                                # counters must be usable call after call
        out = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, 0.0884, workspace=ws, splits=splits)
        assert_attention(out.cpu().numpy(), ref)


def test_decode_degenerate_queries():
    """q = 0 -> uniform weights -> out = mean of V (an oracle pin, checked on the GPU too)."""
    say("[decode] q = 0")
    B, Hq, Hkv, n, d, m = 1, 4, 4, 999, 128, 256
    K = inputs.make_keys(B, Hkv, n, d, torch.bfloat16, 61, DEV)
    V = inputs.make_normal((B, Hkv, n, d), torch.bfloat16, 63, DEV)
    S = qjl.qjl_make_sketch(12, m, d, torch.bfloat16, DEV)
    (bits_d, nu_d), _ = oracle_cache(K, S)
    Q = torch.zeros((B, Hq, d), dtype=torch.bfloat16, device=DEV)
    out = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, 1.0).cpu().numpy()
    assert_attention(out, inputs.to_f64(V).mean(axis=2))


def test_pipeline_end_to_end_config1():
    """Config 1 run as a chain on the GPU (quantize -> project -> scores, and
    quantize -> decode) against the same chain in the oracle."""
    w = inputs.WORKLOADS["c1_single_head"]
    say(f"[chain] {w.name}")
    K, Q, V = inputs.make_workload_tensors(w, DEV)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, DEV)
    K64, Q64, V64, S64 = map(inputs.to_f64, (K, Q, V, S))
    bits_d, nu_d = qjl.qjl_quantize_keys(K, S)
    bad, flips, inband = bits_report(bits_d.cpu().numpy(), K64, S64)
    say(f"  bits: {bad} outside band, {flips} flips of {inband} near-zero entries")
    assert bad == 0
    if flips:
        pytest.skip(f"{flips} near-zero sign decisions differ; the chained comparison needs equal codes")
    bits, nu16, _ = orc.quantize_keys(K64, S64)
    SQ = qjl.qjl_project_query(Q, S)
    sc = qjl.qjl_scores(SQ, bits_d, nu_d, w.scale).cpu().numpy()
    ref_sc = orc.estimate_scores(orc.project_query(Q64, S64), bits, nu16, w.scale)
    # the GPU's norms may sit one binary16 step from the oracle's: allow for it
    step = 2.0 ** -10
    rms = np.sqrt(np.mean(ref_sc ** 2))
    assert np.all(np.abs(sc - ref_sc) <= (1e-3 + step) * np.maximum(np.abs(ref_sc), 1e-2 * rms))
    out = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, w.scale).cpu().numpy()
    ref = orc.decode_attention(Q64, S64, bits_d.cpu().numpy(), nu_d.cpu().numpy(), V64, w.scale)
    assert_attention(out, ref)


# ------------------------------------------------------------------ full-size configurations, sampled
def _sample_units(B, Hkv, count, seed):
    rng = np.random.default_rng(seed)
    flat = rng.choice(B * Hkv, size=min(count, B * Hkv), replace=False)
    return [(int(u // Hkv), int(u % Hkv)) for u in sorted(flat)]


@pytest.mark.parametrize("name,units", [("c2_llama2_7b_decode_4k", 32), ("c3_long_context_b4_32k", 32),
                                        ("c5a_llama3_8b_gqa_b1_128k", 8), ("c5b_llama3_8b_gqa_b16_8k", 32)])
def test_full_size_decode_sampled(name, units):
    """The benchmark's launch configuration at full size.  c2 and c5a: every
    (batch, kv head) unit goes through the oracle; c3 and c5b: 32 of the 128
    units, drawn from the seed.  The keys of those units are quantized by the
    oracle, the GPU consumes exactly those codes for them, and the attention
    outputs of all their query heads are compared; the other units get the
    properties that hold at any size."""
    w = inputs.WORKLOADS[name]
    say(f"[full decode] {name}")
    K, Q, V = inputs.make_workload_tensors(w, DEV)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, DEV)
    S64, Q64 = inputs.to_f64(S), inputs.to_f64(Q)
    bits_d, nu_d = qjl.qjl_quantize_keys(K, S)
    G = w.q_heads // w.kv_heads
    picked = _sample_units(w.batch, w.kv_heads, units, w.data_seed)
    refs = {}
    tot_bad = tot_flip = 0
    for (b, g) in picked:
        K64 = inputs.to_f64(K[b, g])[None, None]
        bad, flips, _ = bits_report(bits_d[b, g].cpu().numpy()[None, None], K64, S64)
        tot_bad += bad
        tot_flip += flips
        assert_norms(nu_d[b, g].cpu().numpy()[None, None], K64)
        bits, nu16, _ = orc.quantize_keys(K64, S64)
        bits_d[b, g] = torch.from_numpy(bits[0, 0]).to(DEV)            # both sides use the oracle's code
        nu_d[b, g] = torch.from_numpy(nu16[0, 0]).to(DEV)
        refs[(b, g)] = orc.decode_attention(Q64[b:b + 1, g * G:(g + 1) * G], S64, bits, nu16,
                                            inputs.to_f64(V[b, g])[None, None], w.scale)[0]
    say(f"  quantize on {len(picked)} of {w.batch * w.kv_heads} units: {tot_bad} outside band, {tot_flip} near-zero flips")
    assert tot_bad == 0
    del K
    out = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, w.scale).cpu().numpy()
    worst = 0.0
    for (b, g), ref in refs.items():
        worst = max(worst, assert_attention(out[b, g * G:(g + 1) * G], ref))
    assert np.all(np.isfinite(out))
    # property that holds for every head at any size: outputs are convex
    # combinations of the values, so they lie inside V's per-channel range
    vmax = V.float().amax(dim=2).cpu().numpy().repeat(G, axis=1)
    vmin = V.float().amin(dim=2).cpu().numpy().repeat(G, axis=1)
    assert np.all(out <= vmax + 1e-3) and np.all(out >= vmin - 1e-3)
    say(f"  worst attention error over {len(refs) * G} heads: {worst:.3g}")


def test_full_size_decode_step_sampled():
    """The streaming workload as bench.py runs it: the newest key goes into the last row of a full cache and is
    attended to in the same launch.  Sampled (batch, kv head) units against the oracle's stream."""
    w = inputs.WORKLOADS["c2s_llama2_7b_decode_step_4k"]
    say(f"[full decode step] {w.name}")
    K, Q, V = inputs.make_workload_tensors(w, DEV)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, DEV)
    S64, Q64 = inputs.to_f64(S), inputs.to_f64(Q)
    pos = w.n - 1
    bits_d, nu_d = qjl.qjl_quantize_keys(K, S)
    bits_d[:, :, pos] = 0                                               # the row the step has to write
    nu_d[:, :, pos] = 0
    G = w.q_heads // w.kv_heads
    picked = _sample_units(w.batch, w.kv_heads, 6, w.data_seed)
    refs = {}
    for (b, g) in picked:
        K64 = inputs.to_f64(K[b, g])[None, None]
        ob, on, _ = orc.quantize_keys(K64[:, :, :pos], S64)             # the oracle's cache before the step
        cb = np.zeros((1, 1, w.n, w.m // 8), dtype=np.uint8); cn = np.zeros((1, 1, w.n), dtype=np.float16)
        cb[:, :, :pos] = ob; cn[:, :, :pos] = on
        bits_d[b, g, :pos] = torch.from_numpy(ob[0, 0]).to(DEV)         # both sides start from the oracle's codes
        nu_d[b, g, :pos] = torch.from_numpy(on[0, 0]).to(DEV)
        refs[(b, g)] = orc.decode_step(Q64[b:b + 1, g * G:(g + 1) * G], S64, cb, cn,
                                       inputs.to_f64(V[b, g])[None, None], K64[:, :, pos:pos + 1], pos, w.scale)[0]
    out = qjl.qjl_decode_step(Q, K[:, :, pos:pos + 1].contiguous(), S, bits_d, nu_d, V, pos, w.scale).cpu().numpy()
    worst = 0.0
    for (b, g), ref in refs.items():
        worst = max(worst, assert_attention(out[b, g * G:(g + 1) * G], ref))
        K64 = inputs.to_f64(K[b, g, pos:pos + 1])[None, None]
        bad, _, _ = bits_report(bits_d[b, g, pos:pos + 1].cpu().numpy()[None, None], K64, S64)
        assert bad == 0
        assert_norms(nu_d[b, g, pos:pos + 1].cpu().numpy()[None, None], K64)
    # every head's new row was written, and is what the bulk quantizer gives
    ref_b, ref_n = qjl.qjl_quantize_keys(K[:, :, pos:pos + 1].contiguous(), S)
    assert torch.equal(nu_d[:, :, pos:pos + 1], ref_n)
    assert float((bits_d[:, :, pos:pos + 1] != ref_b).float().mean()) < 1e-3      # near-zero projections may differ
    say(f"  worst attention error over {len(refs) * G} heads: {worst:.3g}")


def test_full_size_prefill_quantize_sampled():
    """Config 4 at full size (2,097,152 keys, m = 512): every 16th row (131,072 rows, each of the 64 rows of a
    tile position is hit in turn) plus the ends and a head boundary against the oracle, and whole-tensor
    properties (norm range, bit balance)."""
    w = inputs.WORKLOADS["c4_prefill_quantize_64k"]
    say(f"[full quantize] {w.name}")
    K = inputs.make_keys(w.batch, w.kv_heads, w.n, w.d, w.dtype, w.data_seed, DEV, w.outliers)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, DEV)
    bits_d, nu_d = qjl.qjl_quantize_keys(K, S)
    torch.cuda.synchronize()
    S64 = inputs.to_f64(S)
    total = w.kv_heads * w.n
    i16 = np.arange(total // 16)
    strided = 16 * i16 + (i16 // 4) % 16                                # one row in 16, every position of a 64-row tile
    rows = np.unique(np.concatenate([strided, np.arange(0, 64), np.arange(total - 64, total),
                                     np.arange(w.n - 40, w.n + 40)]))   # ends and a head boundary
    bad = flips = inband = 0
    for part in np.array_split(rows, 8):                                # bounded float64 transients on the host
        idx = torch.from_numpy(part).to(DEV)
        Kr = inputs.to_f64(K.view(-1, w.d)[idx])[None, None]
        b1, f1, i1 = bits_report(bits_d.view(-1, w.m // 8)[idx].cpu().numpy()[None, None], Kr, S64)
        bad += b1; flips += f1; inband += i1
        assert_norms(nu_d.view(-1)[idx].cpu().numpy()[None, None], Kr)
    say(f"  {rows.size} rows (1/16 stride): {bad} outside band, {flips} flips of {inband} near-zero entries")
    assert bad == 0
    # whole tensor: norms equal the fp32 norm computed by torch within fp16 rounding; bits are balanced
    ref_n = K.float().norm(dim=-1)
    assert torch.all((nu_d.float() - ref_n).abs() <= 1e-3 * ref_n)
    ones = 0
    for h in range(w.kv_heads):
        ones += int(torch.sum(_popcount8(bits_d[0, h])))
    frac = ones / (w.kv_heads * w.n * w.m)
    say(f"  fraction of +1 signs: {frac:.5f}")
    assert abs(frac - 0.5) < 5e-3


_POP = None


def _popcount8(t: torch.Tensor) -> torch.Tensor:
    global _POP
    if _POP is None:
        _POP = torch.tensor([bin(i).count("1") for i in range(256)], dtype=torch.int64, device=DEV)
    return _POP[t.long()]


# ------------------------------------------------------------------ streams and graphs
def test_decode_on_side_stream_and_in_a_graph():
    """The calls enqueue on the caller's stream only, so a decode step can be
    captured in a HIP graph: every replay (with other eager work and
    synchronisations in between, and new queries written into the captured
    buffers) must equal the eager result for the same inputs."""
    say("[graph] decode step captured and replayed")
    B, Hq, Hkv, n, d, m, scale = 1, 8, 2, 3000, 128, 256, 0.0884
    K = inputs.make_keys(B, Hkv, n, d, torch.bfloat16, 71, DEV)
    V = inputs.make_normal((B, Hkv, n, d), torch.bfloat16, 73, DEV)
    S = qjl.qjl_make_sketch(13, m, d, torch.bfloat16, DEV)
    (bits_d, nu_d), (bits, nu16) = oracle_cache(K, S)
    Qs = [inputs.make_normal((B, Hq, d), torch.bfloat16, 80 + i, DEV) for i in range(4)]
    Q = Qs[0].clone()
    ws = torch.empty((qjl.qjl_decode_workspace_bytes(B, Hq, Hkv, n, d, m),), dtype=torch.uint8, device=DEV)
    out = torch.empty((B, Hq, d), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # eager on a non-default stream
        qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale, out=out, workspace=ws)
    side.synchronize()
    ref0 = orc.decode_attention(inputs.to_f64(Q), inputs.to_f64(S), bits, nu16, inputs.to_f64(V), scale)
    assert_attention(out.cpu().numpy(), ref0)
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale, out=out, workspace=ws)
    for i, q in enumerate(Qs):
        Q.copy_(q)                                     # eager work between replays
        out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = out.clone()
        eager = qjl.qjl_decode_attention(q, S, bits_d, nu_d, V, scale)
        assert torch.equal(got, eager), f"replay {i} differs from the eager result"
        ref = orc.decode_attention(inputs.to_f64(q), inputs.to_f64(S), bits, nu16, inputs.to_f64(V), scale)
        assert_attention(got.cpu().numpy(), ref)


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (16, 4), (8, 8)])
def test_uneven_chunk_pairs_agree_whoever_takes_them(Hq, Hkv):
    """Long chunks are cut into uneven pairs and the workgroups of a launch agree at run time, through a word in
    the workspace, on who takes which (the slower XCDs take the small ones).  The chunks and their records are
    the same either way, so the result must not depend on the outcome: eager calls, calls on a workspace full
    of ones or of noise, and replays from a graph (whose workgroups land on other XCDs) all have to give the
    same bits, and the oracle's numbers."""
    say(f"[uneven chunks] Hq={Hq} Hkv={Hkv}")
    B, n, d, m, scale, splits = 1, 20000, 128, 256, 0.0884, 4
    total, gt, nsplit, chunk = qjl.qjl_decode_plan(B, Hq, Hkv, n, d, m, splits=splits)
    assert nsplit == 4 and chunk >= 2048               # what the uneven cut needs: long chunks, an even count
    K = inputs.make_keys(B, Hkv, n, d, torch.bfloat16, 171, DEV)
    V = inputs.make_normal((B, Hkv, n, d), torch.bfloat16, 173, DEV)
    S = qjl.qjl_make_sketch(17, m, d, torch.bfloat16, DEV)
    (bits_d, nu_d), (bits, nu16) = oracle_cache(K, S)
    Q = inputs.make_normal((B, Hq, d), torch.bfloat16, 180, DEV)
    ref = orc.decode_attention(inputs.to_f64(Q), inputs.to_f64(S), bits, nu16, inputs.to_f64(V), scale)
    ws = torch.empty((total,), dtype=torch.uint8, device=DEV)
    out = torch.empty((B, Hq, d), dtype=torch.float32, device=DEV)
    first = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale, workspace=ws, splits=splits).clone()
    assert_attention(first.cpu().numpy(), ref)
    for fill in ("ones", "noise", "as left"):
        if fill == "ones":
            ws.fill_(255)
        elif fill == "noise":
            ws.copy_(torch.randint(0, 256, (total,), dtype=torch.uint8, device=DEV))
        for _ in range(3):
            out.zero_()
            qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale, out=out, workspace=ws, splits=splits)
            assert torch.equal(out, first), fill
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale, out=out, workspace=ws, splits=splits)
        qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale, out=out, workspace=ws, splits=splits)
    for i in range(4):
        out.zero_()
        if i == 2:
            ws.fill_(0)                                # eager work on the workspace between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, first), f"replay {i}"
    # the same keys cut evenly (an odd number of chunks): other sums, the same attention
    odd = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale, splits=3)
    assert_attention(odd.cpu().numpy(), ref)


def test_many_small_units():
    """Many (batch, head) units with a short context: one workgroup per unit, no chunking."""
    say("[decode] B=24 Hq=16 Hkv=16 n=200")
    B, Hq, Hkv, n, d, m, scale = 24, 16, 16, 200, 128, 256, 0.0884
    K = inputs.make_keys(B, Hkv, n, d, torch.bfloat16, 91, DEV)
    Q = inputs.make_normal((B, Hq, d), torch.bfloat16, 92, DEV)
    V = inputs.make_normal((B, Hkv, n, d), torch.bfloat16, 93, DEV)
    S = qjl.qjl_make_sketch(15, m, d, torch.bfloat16, DEV)
    (bits_d, nu_d), (bits, nu16) = oracle_cache(K, S)
    ref = orc.decode_attention(inputs.to_f64(Q), inputs.to_f64(S), bits, nu16, inputs.to_f64(V), scale)
    out = qjl.qjl_decode_attention(Q, S, bits_d, nu_d, V, scale)
    assert_attention(out.cpu().numpy(), ref)
    sc = qjl.qjl_scores(qjl.qjl_project_query(Q, S), bits_d, nu_d, scale).cpu().numpy()
    SQ32 = orc.project_query(inputs.to_f64(Q), inputs.to_f64(S)).astype(np.float32).astype(np.float64)
    # the GPU's own S q differs from the oracle's by fp32 rounding only: compare the scores loosely here,
    # the strict comparison (same S q on both sides) is test_scores_parity
    ref_sc = orc.estimate_scores(SQ32, bits, nu16, scale)
    rms = np.sqrt(np.mean(ref_sc ** 2, axis=-1, keepdims=True))
    assert np.all(np.abs(sc - ref_sc) <= 2e-3 * np.maximum(np.abs(ref_sc), 1e-2 * rms))


# ------------------------------------------------------------------ orthogonalised sketch (Section 4.1)
@pytest.mark.parametrize("dt", ["f32", "bf16", "f16"])
@pytest.mark.parametrize("m,d,seed", [(256, 128, 2), (512, 128, 4), (128, 128, 9), (100, 128, 5), (40, 24, 99), (300, 128, 6)])
def test_orthogonal_sketch_matches_oracle(dt, m, d, seed):
    """Both sides orthogonalise the same Gaussian draws in float64 (Gram-Schmidt twice here, Householder QR in the
    oracle); after rounding to the storage type the matrices must agree to the last bit almost everywhere, and
    nowhere by more than one unit in the last place."""
    say(f"[orth sketch] dt={dt} m={m} d={d} seed={seed}")
    S = qjl.qjl_make_sketch_orthogonal(seed, m, d, DT[dt], DEV)
    got = inputs.to_f64(S)
    ref = orc.orthogonal_sketch(seed, m, d, dt)
    same = float(np.mean(got == ref))
    ulp = {"f32": 2.0 ** -23, "bf16": 2.0 ** -7, "f16": 2.0 ** -10}[dt]
    worst = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-30)))
    say(f"  identical entries: {same:.6f}, worst relative difference {worst:.3g}")
    assert same >= 0.999 and worst <= 1.01 * ulp
    # structure, independent of the oracle: float32 storage keeps the rows of a block orthogonal to rounding
    if dt == "f32":
        for r0 in range(0, m, d):
            Sb = got[r0:r0 + d]
            gram = Sb @ Sb.T
            off = gram - np.diag(np.diag(gram))
            assert np.max(np.abs(off)) <= 1e-4
    assert torch.equal(S, qjl.qjl_make_sketch_orthogonal(seed, m, d, DT[dt], DEV))


def test_orthogonal_sketch_is_a_drop_in_and_lowers_the_error():
    """The whole path runs unchanged on the orthogonalised sketch, and on the same data its attention output is
    closer to exact attention (Section 4.1 reports that it almost always helps)."""
    B, H, n, d, m, scale = 1, 8, 4096, 128, 256, 0.0884
    K = inputs.make_keys(B, H, n, d, torch.bfloat16, 91, DEV, outliers=0)
    Q = inputs.make_normal((B, H, d), torch.bfloat16, 92, DEV)
    V = inputs.make_normal((B, H, n, d), torch.bfloat16, 93, DEV)
    K64, Q64, V64 = inputs.to_f64(K), inputs.to_f64(Q), inputs.to_f64(V)
    exact = orc.attention_from_scores(scale * np.einsum("bhd,bhnd->bhn", Q64, K64), V64)
    errs = {}
    for name, make in (("iid", qjl.qjl_make_sketch), ("orthogonal", qjl.qjl_make_sketch_orthogonal)):
        tot = 0.0
        for seed in range(6):
            S = make(100 + seed, m, d, torch.bfloat16, DEV)
            bits, norms = qjl.qjl_quantize_keys(K, S)
            out = qjl.qjl_decode_attention(Q, S, bits, norms, V, scale).cpu().numpy().astype(np.float64)
            if seed == 0:      # parity of the path on this sketch
                rb, rn, _ = orc.quantize_keys(K64, inputs.to_f64(S))
                ref = orc.decode_attention(Q64, inputs.to_f64(S), rb, rn, V64, scale)
                assert np.max(np.abs(out - ref)) <= 2e-3
            tot += float(np.mean((out - exact) ** 2))
        errs[name] = (tot / 6) ** 0.5
    say(f"[orth drop-in] rms error to exact attention: iid {errs['iid']:.4f}, orthogonalised {errs['orthogonal']:.4f}")
    assert errs["orthogonal"] < errs["iid"]


# ------------------------------------------------------------------ streaming (Algorithm 1 as a loop)
@pytest.mark.parametrize("dt,B,Hkv,t,m,pos", [("bf16", 2, 3, 1, 256, 5), ("bf16", 1, 32, 1, 256, 4095), ("f16", 1, 2, 7, 512, 0),
                                              ("f32", 1, 1, 3, 128, 10), ("bf16", 1, 2, 4, 192, 1), ("bf16", 1, 8, 64, 384, 36)])
def test_append_keys_parity(dt, B, Hkv, t, m, pos):
    say(f"[append] dt={dt} B={B} Hkv={Hkv} t={t} m={m} pos={pos}")
    d, cap = 128, pos + t + 3
    K_new = inputs.make_keys(B, Hkv, t, d, DT[dt], 200 + t, DEV, outliers=4)
    S = qjl.qjl_make_sketch(5, m, d, DT[dt], DEV)
    bits = torch.full((B, Hkv, cap, m // 8), 0xA5, dtype=torch.uint8, device=DEV)
    norms = torch.full((B, Hkv, cap), 77.0, dtype=torch.float16, device=DEV)
    qjl.qjl_append_keys(K_new, S, bits, norms, pos)
    torch.cuda.synchronize()
    K64, S64 = inputs.to_f64(K_new), inputs.to_f64(S)
    bad, flips, inband = bits_report(bits[:, :, pos:pos + t].cpu().numpy(), K64, S64)
    say(f"  bits: {bad} mismatches outside the band, {flips} flips among {inband} near-zero entries")
    assert bad == 0
    assert_norms(norms[:, :, pos:pos + t].cpu().numpy(), K64)
    untouched = torch.ones(cap, dtype=torch.bool); untouched[pos:pos + t] = False
    assert torch.all(bits[:, :, untouched.to(DEV)] == 0xA5) and torch.all(norms[:, :, untouched.to(DEV)] == 77.0)
    # the bulk quantizer and the append kernel agree on every bit of these keys outside the near-zero band
    b2, n2 = qjl.qjl_quantize_keys(K_new, S)
    bad2, _, _ = bits_report(b2.cpu().numpy(), K64, S64)
    assert bad2 == 0


@pytest.mark.parametrize("dt,B,Hq,Hkv,cap,m,n0", [
    ("bf16", 1, 8, 4, 300, 256, 292),        # two query heads per kv head
    ("f16", 1, 4, 1, 132, 512, 125),         # four query heads per kv head, steps across a 128-key boundary
    ("bf16", 2, 2, 2, 68, 128, 61),          # fewer projections than threads, steps across a 64-key boundary
    ("bf16", 1, 3, 1, 5, 256, 0),            # from an empty cache
    ("f32", 1, 2, 1, 40, 256, 36),           # fp32: the key is appended by a kernel of its own
])
def test_decode_steps_stream_into_a_cache(dt, B, Hq, Hkv, cap, m, n0):
    """Generation steps from a prefilled cache: after every step the cache rows and the attention output
    match the oracle's stream, which in turn equals quantizing everything at once."""
    d, scale = 128, 0.0884
    say(f"[stream] dt={dt} B={B} Hq={Hq} Hkv={Hkv} cap={cap} m={m} from {n0}")
    K = inputs.make_keys(B, Hkv, cap, d, DT[dt], 301, DEV, outliers=4)
    V = inputs.make_normal((B, Hkv, cap, d), DT[dt], 302, DEV)
    Qs = inputs.make_normal((cap, B * Hq, d), DT[dt], 303, DEV).view(cap, B, Hq, d)
    S = qjl.qjl_make_sketch(6, m, d, DT[dt], DEV)
    K64, V64, S64 = inputs.to_f64(K), inputs.to_f64(V), inputs.to_f64(S)
    ob = np.zeros((B, Hkv, cap, m // 8), dtype=np.uint8); on = np.zeros((B, Hkv, cap), dtype=np.float16)
    if n0 > 0:
        rb, rn, _ = orc.quantize_keys(K64[:, :, :n0], S64)                   # the oracle's prefill
        ob[:, :, :n0] = rb; on[:, :, :n0] = rn
    bits = torch.from_numpy(ob.copy()).to(DEV); norms = torch.from_numpy(on.copy()).to(DEV)
    ws = torch.empty((qjl.qjl_decode_workspace_bytes(B, Hq, Hkv, cap, d, m, DT[dt]),), dtype=torch.uint8, device=DEV)
    worst = 0.0
    for pos in range(n0, cap):
        out = qjl.qjl_decode_step(Qs[pos].contiguous(), K[:, :, pos:pos + 1].contiguous(), S, bits, norms, V, pos, scale, workspace=ws)
        ref = orc.decode_step(inputs.to_f64(Qs[pos]), S64, ob, on, V64, K64[:, :, pos:pos + 1], pos, scale)
        bad, _, _ = bits_report(bits[:, :, pos:pos + 1].cpu().numpy(), K64[:, :, pos:pos + 1], S64)
        assert bad == 0
        assert_norms(norms[:, :, pos:pos + 1].cpu().numpy(), K64[:, :, pos:pos + 1])
        bits[:, :, pos] = torch.from_numpy(ob[:, :, pos]).to(DEV)          # keep both sides on the oracle's code
        norms[:, :, pos] = torch.from_numpy(on[:, :, pos]).to(DEV)
        worst = max(worst, assert_attention(out.cpu().numpy(), ref))
    say(f"[stream] worst attention error over {cap - n0} steps: {worst:.3g}")
    assert torch.all(bits[:, :, :n0].cpu() == torch.from_numpy(ob[:, :, :n0]))   # earlier rows never rewritten
