"""GPU-vs-oracle parity of the quantized value cache (Section 3.2), through the C ABI.

The bar for the codes is the oracle's definition in exact arithmetic (`value_codes_exact`): identical outside
the band of quotients within 2^-20 relative of a half-integer, where float32 may round to the neighbour; entries
in the band are counted and reported.  The library also promises the float32 subtract / divide / round of its
header, so as an extra check its codes must equal `quantize_values` (the same three operations) bit for bit, and
so must the stored binary16 scale and zero point.  Attention outputs on a quantized value cache: 2e-3 absolute,
like every other attention output.
"""
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


@pytest.mark.parametrize("vbits", [4, 2, 8])
@pytest.mark.parametrize("dt,B,Hkv,n", [("bf16", 2, 3, 333), ("f16", 1, 2, 1000), ("f32", 1, 1, 257),
                                        ("bf16", 1, 1, 1), ("bf16", 1, 32, 4096)])
def test_quantize_values_is_bit_exact(dt, B, Hkv, n, vbits):
    say(f"[values] dt={dt} B={B} Hkv={Hkv} n={n} vbits={vbits}")
    V = inputs.make_normal((B, Hkv, n, 128), DT[dt], 900 + n, DEV)
    V[0, 0, 0] = 0.75                                          # a constant row: scale 0
    if n > 2:
        V[0, 0, 1] *= 37.0                                     # a wide row
        V[0, 0, 2, 5:] = V[0, 0, 2, 4]                         # two distinct values only
    codes, sc, z = qjl.qjl_quantize_values(V, vbits)
    torch.cuda.synchronize()
    rc, rs, rz = orc.quantize_values(inputs.to_f64(V), vbits)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), rs.view(np.uint16))
    assert np.array_equal(z.cpu().numpy().view(np.uint16), rz.view(np.uint16))
    diff = int((codes.cpu().numpy() != rc).sum())
    say(f"  code bytes differing: {diff} of {rc.size}")
    assert diff == 0
    c2, s2, z2 = qjl.qjl_quantize_values(V, vbits)
    assert torch.equal(codes, c2) and torch.equal(sc, s2) and torch.equal(z, z2)


@pytest.mark.parametrize("vbits", [4, 2, 8])
@pytest.mark.parametrize("dt,B,Hkv,n", [("bf16", 2, 3, 700), ("f16", 1, 2, 1000), ("f32", 1, 2, 513)])
def test_quantize_values_against_the_definition_in_exact_arithmetic(dt, B, Hkv, n, vbits):
    say(f"[values, exact form] dt={dt} B={B} Hkv={Hkv} n={n} vbits={vbits}")
    V = inputs.make_normal((B, Hkv, n, 128), DT[dt], 950 + n, DEV)
    V[0, 0, :40] = torch.round(V[0, 0, :40] * 4) / 4           # few distinct values per row: exact ties
    codes, sc, z = qjl.qjl_quantize_values(V, vbits)
    torch.cuda.synchronize()
    V64 = inputs.to_f64(V)
    sc_x, z_x, near_c = orc.value_constants_exact(V64, vbits)
    sc_g, z_g = sc.cpu().numpy(), z.cpu().numpy()
    assert np.array_equal(z_g.view(np.uint16), z_x.view(np.uint16))
    same_scale = sc_g.view(np.uint16) == sc_x.view(np.uint16)
    assert np.all(same_scale | near_c)
    # the codes against the constants the GPU stored (each stage is checked on what the stage before it left)
    want, near = orc.value_codes_exact(V64, sc_g, z_g, vbits)
    got = orc.unpack_value_codes(codes.cpu().numpy(), vbits)
    diff = got != want
    say(f"  scales off the exact rounding: {int((~same_scale).sum())} of {same_scale.size} rows (all near a binary16 midpoint); "
        f"codes differing inside the tie band: {int((diff & near).sum())} of {int(near.sum())} near-tie entries of {want.size}; outside: {int((diff & ~near).sum())}")
    assert not (diff & ~near).any()


VQ_CASES = [
    # dtype, B, Hq, Hkv, n, m, scale
    ("bf16", 1, 4, 4, 4096, 256, 0.0884),
    ("bf16", 2, 8, 2, 1500, 256, 0.0884),        # GQA x4, ragged
    ("bf16", 1, 8, 4, 333, 256, 1.0),            # GQA x2
    ("bf16", 1, 3, 1, 700, 256, 0.0884),         # GQA x3 -> one head at a time
    ("f16", 1, 4, 1, 260, 512, 0.0884),
    ("bf16", 1, 4, 1, 129, 128, 0.0884),
    ("bf16", 1, 2, 2, 1, 256, 1.0),              # n = 1: out = the stored v_1
    ("bf16", 1, 1, 1, 65, 256, 0.0884),
    ("bf16", 1, 2, 1, 20000, 256, 0.0884),       # many chunks
]


@pytest.mark.parametrize("vbits", [4, 2, 8])
@pytest.mark.parametrize("dt,B,Hq,Hkv,n,m,scale", VQ_CASES)
def test_decode_attention_vq_parity(dt, B, Hq, Hkv, n, m, scale, vbits):
    say(f"[decode vq] dt={dt} B={B} Hq={Hq} Hkv={Hkv} n={n} m={m} scale={scale} vbits={vbits}")
    d = 128
    K = inputs.make_keys(B, Hkv, n, d, DT[dt], 700 + n, DEV, outliers=4)
    Q = inputs.make_normal((B, Hq, d), DT[dt], 71, DEV)
    V = inputs.make_normal((B, Hkv, n, d), DT[dt], 72, DEV)
    S = qjl.qjl_make_sketch(10, m, d, DT[dt], DEV)
    S64 = inputs.to_f64(S)
    bits, nu16, _ = orc.quantize_keys(inputs.to_f64(K), S64)            # the oracle's caches
    vc, vs, vz = orc.quantize_values(inputs.to_f64(V), vbits)
    ref = orc.decode_attention_vq(inputs.to_f64(Q), S64, bits, nu16, vc, vs, vz, vbits, scale)
    up = lambda a: torch.from_numpy(a).to(DEV)
    args = (Q, S, up(bits), up(nu16), up(vc), up(vs), up(vz), vbits, scale)
    out = qjl.qjl_decode_attention_vq(*args)
    err = float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref)))
    say(f"  max abs error {err:.3g}")
    assert err <= 2e-3
    assert torch.equal(out, qjl.qjl_decode_attention_vq(*args))
    if n == 1:
        assert np.allclose(out.cpu().numpy()[0, 0], orc.dequantize_values(vc, vs, vz, vbits)[0, 0, 0], atol=2e-3)


@pytest.mark.parametrize("vbits,max_shift", [(4, 0.1), (2, 0.4), (8, 0.01)])
def test_vq_pipeline_on_the_gpu_and_distance_to_unquantized_values(vbits, max_shift):
    B, Hq, Hkv, n, d, m, scale = 1, 8, 8, 2048, 128, 256, 0.0884
    K = inputs.make_keys(B, Hkv, n, d, torch.bfloat16, 81, DEV, outliers=4)
    Q = inputs.make_normal((B, Hq, d), torch.bfloat16, 82, DEV)
    V = inputs.make_normal((B, Hkv, n, d), torch.bfloat16, 83, DEV)
    S = qjl.qjl_make_sketch(11, m, d, torch.bfloat16, DEV)
    bits, norms = qjl.qjl_quantize_keys(K, S)
    vc, vs, vz = qjl.qjl_quantize_values(V, vbits)
    out = qjl.qjl_decode_attention_vq(Q, S, bits, norms, vc, vs, vz, vbits, scale).cpu().numpy().astype(np.float64)
    full = qjl.qjl_decode_attention(Q, S, bits, norms, V, scale).cpu().numpy().astype(np.float64)
    ref = orc.decode_attention_vq(inputs.to_f64(Q), inputs.to_f64(S), bits.cpu().numpy(), norms.cpu().numpy(),
                                  *[t.cpu().numpy() for t in (vc, vs, vz)], vbits, scale)
    assert float(np.max(np.abs(out - ref))) <= 2e-3
    # the output moves by a fraction of a quantization step (N(0,1) rows: step ~ 5 / (2^b - 1))
    shift = float(np.sqrt(np.mean((out - full) ** 2)))
    say(f"[vq chain] {vbits}-bit values: rms distance to attention on bf16 values: {shift:.4f}")
    assert shift < max_shift


@pytest.mark.parametrize("name,units", [("c2_llama2_7b_decode_4k", 8), ("c3_long_context_b4_32k", 3)])
def test_full_size_vq_sampled(name, units):
    """The benchmark's configuration at full size: every code byte, scale and zero point of sampled units
    against the oracle; attention of those units on the oracle's caches."""
    w = inputs.WORKLOADS[name]
    say(f"[full vq] {name}")
    K, Q, V = inputs.make_workload_tensors(w, DEV)
    S = qjl.qjl_make_sketch(w.sketch_seed, w.m, w.d, w.dtype, DEV)
    S64, Q64 = inputs.to_f64(S), inputs.to_f64(Q)
    bits_d, nu_d = qjl.qjl_quantize_keys(K, S)
    vc_d, vs_d, vz_d = qjl.qjl_quantize_values(V, 4)
    rng = np.random.default_rng(w.data_seed + 5)
    picked = sorted(rng.choice(w.batch * w.kv_heads, size=units, replace=False).tolist())
    refs = {}
    for u in picked:
        b, g = divmod(u, w.kv_heads)
        K64 = inputs.to_f64(K[b, g])[None, None]
        V64 = inputs.to_f64(V[b, g])[None, None]
        rc, rs, rz = orc.quantize_values(V64, 4)
        assert np.array_equal(vc_d[b, g].cpu().numpy(), rc[0, 0])
        assert np.array_equal(vs_d[b, g].cpu().numpy().view(np.uint16), rs[0, 0].view(np.uint16))
        assert np.array_equal(vz_d[b, g].cpu().numpy().view(np.uint16), rz[0, 0].view(np.uint16))
        rb, rn, _ = orc.quantize_keys(K64, S64)
        bits_d[b, g] = torch.from_numpy(rb[0, 0]).to(DEV)
        nu_d[b, g] = torch.from_numpy(rn[0, 0]).to(DEV)
        refs[(b, g)] = orc.decode_attention_vq(Q64[b:b + 1, g:g + 1], S64, rb, rn, rc, rs, rz, 4, w.scale)[0]
        say(f"  unit b={b} kv={g}: oracle done")
    del K, V
    out = qjl.qjl_decode_attention_vq(Q, S, bits_d, nu_d, vc_d, vs_d, vz_d, 4, w.scale).cpu().numpy()
    worst = max(float(np.max(np.abs(out[b, g:g + 1].astype(np.float64) - ref))) for (b, g), ref in refs.items())
    say(f"  worst attention error over {len(refs)} heads: {worst:.3g}")
    assert worst <= 2e-3 and np.all(np.isfinite(out))


@pytest.mark.parametrize("vbits", [4, 2, 8])
def test_quantize_values_on_rows_full_of_ties(vbits):
    """Rows whose entries sit exactly on, or one bf16 step away from, the midpoints between codes: the kernel's
    division-free shortcut must hand every such entry to the exact path."""
    V = torch.zeros((1, 4, 4096, 128), dtype=torch.bfloat16, device=DEV)
    g = torch.Generator(device=DEV); g.manual_seed(5)
    V[0, 0] = (torch.arange(128, device=DEV).float() % 31 * 0.25).to(torch.bfloat16)          # scale 0.5: every second entry is a tie
    V[0, 1] = (torch.randint(0, 61, (4096, 128), device=DEV, generator=g).float() * 0.125).to(torch.bfloat16)
    V[0, 2] = (torch.randn((4096, 128), device=DEV, generator=g) * 3).to(torch.bfloat16)
    V[0, 3] = (torch.randint(-40, 41, (4096, 128), device=DEV, generator=g).float() * 0.0625).to(torch.bfloat16)
    if vbits == 8:                                   # steps of 1/4 over a range of 255/2: entries on every midpoint
        V[0, 0] = (torch.arange(128, device=DEV).float() * 0.25).to(torch.bfloat16)
        V[0, 0, :, 127] = 127.5
        V[0, 1] = (torch.randint(0, 511, (4096, 128), device=DEV, generator=g).float() * 0.25).to(torch.bfloat16)
        V[0, 1, :, 0] = 0.0
        V[0, 1, :, 1] = 127.5
    if vbits == 2:                                   # steps of 1/2 over a range of 3: every second entry is a tie
        V[0, 0] = (torch.arange(128, device=DEV).float() % 7 * 0.5).to(torch.bfloat16)
        V[0, 1] = (torch.randint(0, 13, (4096, 128), device=DEV, generator=g).float() * 0.25).to(torch.bfloat16)
    codes, sc, z = qjl.qjl_quantize_values(V, vbits)
    rc, rs, rz = orc.quantize_values(inputs.to_f64(V), vbits)
    assert np.array_equal(sc.cpu().numpy().view(np.uint16), rs.view(np.uint16))
    assert np.array_equal(z.cpu().numpy().view(np.uint16), rz.view(np.uint16))
    assert int((codes.cpu().numpy() != rc).sum()) == 0
