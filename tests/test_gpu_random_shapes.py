"""GPU-vs-oracle parity on shapes drawn from a seed instead of picked by hand: every decode entry point and both
key quantizers, over head counts, group sizes, code sizes, storage types and context lengths around the tile
edges (multiples of 64 and their neighbours, one key, a few thousand keys).  Bars as everywhere: attention 2e-3
absolute, code bits exact outside the near-zero band, norms 1e-3 relative.  The oracle builds every cache the GPU
reads.  The draws are fixed by the seeds below, so a failure names a case that can be run again."""
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
LENGTHS = [1, 2, 5, 63, 64, 65, 127, 129, 255, 256, 257, 511, 513, 1000, 1023, 1025, 2047, 2500, 4097]
SCALE = 0.0884


def say(*a):
    print(*a, flush=True)


@pytest.fixture(scope="module", autouse=True)
def _need_gpu_and_lib():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    assert os.path.exists(qjl.lib_path()), "libqjl.so must be built before the GPU tests run"
    qjl.lib()


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _err(out, ref):
    return float(np.max(np.abs(out.cpu().numpy().astype(np.float64) - ref)))


def _draw_decode_cases(seed, count):
    rng = np.random.default_rng(seed)
    cases = []
    for it in range(count):
        mode = ["plain", "vq", "step", "dual", "dual_vq", "generation"][it % 6]
        dt = "f32" if (mode in ("plain", "dual") and it % 5 == 0) else ["bf16", "f16"][int(rng.integers(0, 2))]
        Hkv = int(rng.choice([1, 2, 3, 8]))
        G = int(rng.choice([1, 2, 3, 4, 8]))
        B = int(rng.integers(1, 3))
        n = int(rng.choice(LENGTHS))
        if mode in ("dual", "dual_vq", "generation"):
            m, m_out = [(128, 128), (256, 128)][int(rng.integers(0, 2))]
        else:
            m, m_out = int(rng.choice([128, 256, 512])), 0
        vbits = int(rng.choice([2, 4, 8])) if mode in ("vq", "dual_vq", "generation") else 0
        cases.append((it, mode, dt, B, Hkv * G, Hkv, n, m, m_out, vbits))
    return cases


DECODE_CASES = _draw_decode_cases(20240603, 48)


@pytest.mark.parametrize("it,mode,dt,B,Hq,Hkv,n,m,m_out,vbits", DECODE_CASES)
def test_decode_paths_on_drawn_shapes(it, mode, dt, B, Hq, Hkv, n, m, m_out, vbits):
    say(f"[drawn decode {it}] {mode} dt={dt} B={B} Hq={Hq} Hkv={Hkv} n={n} m={m}+{m_out} vbits={vbits}")
    d = 128
    K = inputs.make_keys(B, Hkv, n, d, DT[dt], 3000 + it, DEV, outliers=4)
    V = inputs.make_normal((B, Hkv, n, d), DT[dt], 3100 + it, DEV)
    Q = inputs.make_normal((B, Hq, d), DT[dt], 3200 + it, DEV)
    K64, V64, Q64 = inputs.to_f64(K), inputs.to_f64(V), inputs.to_f64(Q)
    if m_out == 0:
        S = qjl.qjl_make_sketch(it, m, d, DT[dt], DEV)
        S64 = inputs.to_f64(S)
        if mode == "plain":
            rb, rn, _ = orc.quantize_keys(K64, S64)
            ref = orc.decode_attention(Q64, S64, rb, rn, V64, SCALE)
            out = qjl.qjl_decode_attention(Q, S, _dev(rb), _dev(rn), V, SCALE)
        elif mode == "vq":
            rb, rn, _ = orc.quantize_keys(K64, S64)
            vc, vs, vz = orc.quantize_values(V64, vbits)
            ref = orc.decode_attention_vq(Q64, S64, rb, rn, vc, vs, vz, vbits, SCALE)
            out = qjl.qjl_decode_attention_vq(Q, S, _dev(rb), _dev(rn), _dev(vc), _dev(vs), _dev(vz), vbits, SCALE)
        else:                                           # append the last key, then attend
            pos = n - 1
            cb = np.full((B, Hkv, n, m // 8), 0x5A, dtype=np.uint8)
            cn = np.full((B, Hkv, n), 3.0, dtype=np.float16)
            if pos > 0:
                rb, rn, _ = orc.quantize_keys(K64[:, :, :pos], S64)
                cb[:, :, :pos] = rb
                cn[:, :, :pos] = rn
            bits, norms = _dev(cb), _dev(cn)
            ref = orc.decode_step(Q64, S64, cb, cn, V64, K64[:, :, pos:pos + 1], pos, SCALE)
            out = qjl.qjl_decode_step(Q, K[:, :, pos:pos + 1].contiguous(), S, bits, norms, V, pos, SCALE)
    else:
        S_in = qjl.qjl_make_sketch(2 * it, m, d, DT[dt], DEV)
        S_out = qjl.qjl_make_sketch(2 * it + 1, m_out, d, DT[dt], DEV)
        S_in64, S_out64 = inputs.to_f64(S_in), inputs.to_f64(S_out)
        ch = orc.select_outlier_channels(K64, 4)
        ch_d = _dev(ch.astype(np.int32))
        S_dual = qjl.qjl_make_dual_sketch(S_in, S_out, ch_d)
        if mode == "dual":
            rb, ri, ro, _, _ = orc.quantize_keys_dual(K64, S_in64, S_out64, ch)
            ref = orc.decode_attention_dual(Q64, S_in64, S_out64, ch, rb, ri, ro, V64, SCALE)
            out = qjl.qjl_decode_attention_dual(Q, S_dual, _dev(rb), _dev(ri), _dev(ro), V, m_out, SCALE)
        elif mode == "dual_vq":
            rb, ri, ro, _, _ = orc.quantize_keys_dual(K64, S_in64, S_out64, ch)
            vc, vs, vz = orc.quantize_values(V64, vbits)
            ref = orc.decode_attention_dual_vq(Q64, S_in64, S_out64, ch, rb, ri, ro, vc, vs, vz, vbits, SCALE)
            out = qjl.qjl_decode_attention_dual_vq(Q, S_dual, _dev(rb), _dev(ri), _dev(ro), _dev(vc), _dev(vs),
                                                   _dev(vz), m_out, vbits, SCALE)
        else:                                           # append the last token (key and value), then attend
            pos = n - 1
            rb, ri, ro, _, _ = orc.quantize_keys_dual(K64, S_in64, S_out64, ch)
            vc, vs, vz = orc.quantize_values(V64, vbits)
            caches = [np.ascontiguousarray(x.copy()) for x in (rb, ri, ro, vc, vs, vz)]
            for x in caches:                            # row pos holds stale contents until the step writes it
                x[:, :, pos:] = np.asarray(77).astype(x.dtype)
            dc = [_dev(x) for x in caches]
            ref = orc.generation_step(Q64, S_in64, S_out64, ch, *caches, K64[:, :, pos:pos + 1],
                                      V64[:, :, pos:pos + 1], pos, vbits, SCALE)
            out = qjl.qjl_generation_step(Q, K[:, :, pos:pos + 1].contiguous(), V[:, :, pos:pos + 1].contiguous(),
                                          S_dual, ch_d, *dc, pos, m_out, vbits, SCALE)
            torch.cuda.synchronize()
            assert np.array_equal(dc[3].cpu().numpy(), vc) and np.array_equal(dc[4].cpu().numpy(), vs) and \
                np.array_equal(dc[5].cpu().numpy(), vz)
    err = _err(out, ref)
    say(f"  max abs error {err:.3g}")
    assert err <= 2e-3


def _draw_quantize_cases(seed, count):
    rng = np.random.default_rng(seed)
    cases = []
    for it in range(count):
        dt = ["bf16", "f16"][it % 2] if it % 7 else "f32"
        B, H = int(rng.integers(1, 4)), int(rng.integers(1, 5))
        n = int(rng.choice(LENGTHS + [700, 1500, 2049]))
        dual = it % 3 == 0
        if dual:
            m, m_out = [(128, 128), (256, 128), (512, 128), (256, 256)][int(rng.integers(0, 4))]
        else:
            m, m_out = int(rng.choice([128, 256, 384, 512, 1024])), 0
        cases.append((it, dt, B, H, n, m, m_out))
    return cases


QUANT_CASES = _draw_quantize_cases(603, 42)


@pytest.mark.parametrize("it,dt,B,H,n,m,m_out", QUANT_CASES)
def test_quantizers_on_drawn_shapes(it, dt, B, H, n, m, m_out):
    say(f"[drawn quantize {it}] dt={dt} B={B} H={H} n={n} m={m}+{m_out}")
    d = 128
    K = inputs.make_keys(B, H, n, d, DT[dt], 4000 + it, DEV, outliers=4)
    K64 = inputs.to_f64(K)
    kn = np.linalg.norm(K64, axis=-1)
    if m_out == 0:
        S = qjl.qjl_make_sketch(it, m, d, DT[dt], DEV)
        S64 = inputs.to_f64(S)
        bits, norms = qjl.qjl_quantize_keys(K, S)
        rb, _, P = orc.quantize_keys(K64, S64)
        diff = orc.unpack_signs(bits.cpu().numpy(), m) != orc.unpack_signs(rb, m)
        band = np.abs(P) < 1e-5 * np.linalg.norm(S64, axis=1) * kn[..., None]
        assert int((diff & ~band).sum()) == 0
        assert np.all(np.abs(norms.cpu().numpy().astype(np.float64) - kn) <= 1e-3 * kn)
        say(f"  {int((diff & band).sum())} near-zero sign flips")
    else:
        S_in = qjl.qjl_make_sketch(2 * it, m, d, DT[dt], DEV)
        S_out = qjl.qjl_make_sketch(2 * it + 1, m_out, d, DT[dt], DEV)
        S_in64, S_out64 = inputs.to_f64(S_in), inputs.to_f64(S_out)
        ch = orc.select_outlier_channels(K64, 4)
        ch_d = _dev(ch.astype(np.int32))
        S_dual = qjl.qjl_make_dual_sketch(S_in, S_out, ch_d)
        bits, nin, nout = qjl.qjl_quantize_keys_dual(K, S_dual, ch_d, m_out)
        rb, _, _, P_in, P_out = orc.quantize_keys_dual(K64, S_in64, S_out64, ch)
        K_in, K_out = orc.split_channels(K64, ch)
        got, ref = bits.cpu().numpy(), rb
        flips = 0
        for lo, mm, P, S64, Kp, is_out in ((0, m, P_in, S_in64, K_in, False), (m // 8, m_out, P_out, S_out64, K_out, True)):
            diff = orc.unpack_signs(got[..., lo:lo + mm // 8], mm) != orc.unpack_signs(ref[..., lo:lo + mm // 8], mm)
            for b in range(B):
                for h in range(H):
                    mask = np.zeros(d)
                    mask[ch[b, h]] = 1.0
                    Sm = S64 * (mask if is_out else 1 - mask)
                    band = np.abs(P[b, h]) < 1e-5 * np.linalg.norm(Sm, axis=1) * np.linalg.norm(Kp[b, h], axis=-1)[:, None]
                    assert not (diff[b, h] & ~band).any(), (b, h)
                    flips += int((diff[b, h] & band).sum())
        for g16, Kp in ((nin, K_in), (nout, K_out)):
            refn = np.linalg.norm(Kp, axis=-1)
            assert np.all(np.abs(g16.cpu().numpy().astype(np.float64) - refn) <= 1e-3 * refn + 1e-6)
        say(f"  {flips} near-zero sign flips")
