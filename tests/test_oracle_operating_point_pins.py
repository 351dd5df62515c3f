"""Pins for the oracle's composition of two-part key codes (Section 4.1), few-bit values (Section 3.2) and the
token stream (Algorithm 1): `decode_attention_dual_vq`, `append_token`, `generation_step`.  CPU only.

The parts are pinned on their own elsewhere; what is pinned here is the composition: which rows are written,
which rows are attended to, that the new token's own (quantized) key and value take part in its step, and that
the result is the written-out formula  softmax_j( scale * (Prod_in + Prod_out) ) . (zero_j + scale_j code_j)."""
import math

import numpy as np
import pytest
import torch

from oracle import qjl_oracle as orc


def _setup(seed=0, B=2, Hq=4, Hkv=2, cap=10, d=16, m=32, m_out=16, count=2):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((B, Hkv, cap, d))
    ch = np.stack([np.stack([rng.permutation(d)[:count] for _ in range(Hkv)]) for _ in range(B)])
    for b in range(B):
        for h in range(Hkv):
            K[b, h][:, ch[b, h]] *= 12.0
    V = rng.standard_normal((B, Hkv, cap, d)).astype(np.float32).astype(np.float64)
    Q = rng.standard_normal((cap, B, Hq, d))
    S_in = rng.standard_normal((m, d))
    S_out = rng.standard_normal((m_out, d))
    return K, V, Q, S_in, S_out, ch


def _empty_caches(B, Hkv, cap, d, m, m_out, vbits):
    return (np.full((B, Hkv, cap, (m + m_out) // 8), 0xA5, dtype=np.uint8), np.full((B, Hkv, cap), 7.0, dtype=np.float16),
            np.full((B, Hkv, cap), 9.0, dtype=np.float16), np.full((B, Hkv, cap, d * vbits // 8), 0x5A, dtype=np.uint8),
            np.full((B, Hkv, cap), 3.0, dtype=np.float16), np.full((B, Hkv, cap), -2.0, dtype=np.float16))


@pytest.mark.parametrize("vbits", [2, 4, 8])
def test_streaming_at_the_operating_point_equals_quantizing_everything_at_once(vbits):
    K, V, Q, S_in, S_out, ch = _setup()
    B, Hkv, cap, d = K.shape
    m, m_out = S_in.shape[0], S_out.shape[0]
    caches = _empty_caches(B, Hkv, cap, d, m, m_out, vbits)          # stale contents must not matter
    all_bits, all_in, all_out, _, _ = orc.quantize_keys_dual(K, S_in, S_out, ch)
    all_c, all_s, all_z = orc.quantize_values(V, vbits)
    for pos in range(cap):
        out = orc.generation_step(Q[pos], S_in, S_out, ch, *caches, K[:, :, pos:pos + 1], V[:, :, pos:pos + 1], pos, vbits, 0.3)
        e = pos + 1
        for got, want in zip(caches, (all_bits, all_in, all_out, all_c, all_s, all_z)):
            assert np.array_equal(got[:, :, :e], want[:, :, :e])
        if e < cap:                                                  # rows not yet written are untouched
            assert np.all(caches[0][:, :, e:] == 0xA5) and np.all(caches[3][:, :, e:] == 0x5A)
            assert np.all(caches[1][:, :, e:] == np.float16(7.0)) and np.all(caches[5][:, :, e:] == np.float16(-2.0))
        want = orc.decode_attention_dual_vq(Q[pos], S_in, S_out, ch, all_bits[:, :, :e], all_in[:, :, :e], all_out[:, :, :e],
                                            all_c[:, :, :e], all_s[:, :, :e], all_z[:, :, :e], vbits, 0.3)
        assert np.array_equal(out, want)


def test_the_step_is_the_written_out_formula():
    """Brute force in Python loops and math.*: per query head h (kv head g = h // G), per cached token j,
    score_j = scale sqrt(pi/2) ( nu_in_j/m <S_in q_in, s_in_j> + nu_out_j/m_out <S_out q_out, s_out_j> ),
    p = softmax(score), out = sum_j p_j (zero_j + scale_j code_j)."""
    K, V, Q, S_in, S_out, ch = _setup(3, B=1, Hq=4, Hkv=2, cap=5, d=8, m=16, m_out=8, count=2)
    vbits, scale = 4, 0.7
    B, Hkv, cap, d = K.shape
    m, m_out = 16, 8
    caches = _empty_caches(B, Hkv, cap, d, m, m_out, vbits)
    for pos in range(cap):
        out = orc.generation_step(Q[pos], S_in, S_out, ch, *caches, K[:, :, pos:pos + 1], V[:, :, pos:pos + 1], pos, vbits, scale)
    pos = cap - 1
    bits, nu_in, nu_out, vc, vs, vz = caches
    for h in range(4):
        g = h // 2
        q = Q[pos][0, h]
        outl = set(int(t) for t in ch[0, g])
        q_in = [0.0 if t in outl else q[t] for t in range(d)]
        q_out = [q[t] if t in outl else 0.0 for t in range(d)]
        sq_in = [sum(S_in[i, t] * q_in[t] for t in range(d)) for i in range(m)]
        sq_out = [sum(S_out[i, t] * q_out[t] for t in range(d)) for i in range(m_out)]
        scores = []
        for j in range(cap):
            row = bits[0, g, j]
            sgn = [1.0 if (int(row[i // 8]) >> (i % 8)) & 1 else -1.0 for i in range(m + m_out)]
            a = sum(sq_in[i] * sgn[i] for i in range(m))
            b = sum(sq_out[i] * sgn[m + i] for i in range(m_out))
            scores.append(scale * math.sqrt(math.pi / 2) * (float(nu_in[0, g, j]) / m * a + float(nu_out[0, g, j]) / m_out * b))
        mx = max(scores)
        w = [math.exp(x - mx) for x in scores]
        tot = sum(w)
        for t in range(d):
            acc = 0.0
            for j in range(cap):
                code = (int(vc[0, g, j, t // 2]) >> (4 * (t % 2))) & 15
                acc += w[j] / tot * (float(vz[0, g, j]) + float(vs[0, g, j]) * code)
            assert abs(acc - out[0, h, t]) < 1e-12


def test_reduces_to_its_parts():
    K, V, Q, S_in, S_out, ch = _setup(5)
    B, Hkv, cap, d = K.shape
    bits, nu_in, nu_out, _, _ = orc.quantize_keys_dual(K, S_in, S_out, ch)
    # values that an 8-bit code represents exactly: the step equals the two-part decode on those values
    rng = np.random.default_rng(1)
    codes = rng.integers(0, 256, size=(B, Hkv, cap, d))
    codes[..., 0] = 0
    codes[..., 1] = 255                                  # every row spans the whole range: min = zero, (max - min)/255 = scale
    Vx = -1.5 + codes * (2.0 ** -6)
    vc, vs, vz = orc.quantize_values(Vx, 8)
    assert np.array_equal(orc.dequantize_values(vc, vs, vz, 8), Vx)
    a = orc.decode_attention_dual_vq(Q[0], S_in, S_out, ch, bits, nu_in, nu_out, vc, vs, vz, 8, 0.2)
    assert np.array_equal(a, orc.decode_attention_dual(Q[0], S_in, S_out, ch, bits, nu_in, nu_out, Vx, 0.2))
    # no outlier channels: the inlier quantizer is the whole method and the step equals the one-sketch decode on quantized values
    none = np.zeros((B, Hkv, 0), dtype=np.int64)
    b0, i0, o0, _, _ = orc.quantize_keys_dual(K, S_in, S_out, none)
    assert not o0.any()
    vc4, vs4, vz4 = orc.quantize_values(V, 4)
    got = orc.decode_attention_dual_vq(Q[1], S_in, S_out, none, b0, i0, o0, vc4, vs4, vz4, 4, 0.2)
    m = S_in.shape[0]
    assert np.allclose(got, orc.decode_attention_vq(Q[1], S_in, b0[..., : m // 8], i0, vc4, vs4, vz4, 4, 0.2), rtol=0, atol=1e-14)
    # torch float64 softmax on the oracle's own scores
    sc = orc.estimate_scores_dual(Q[2], S_in, S_out, ch, bits, nu_in, nu_out, 0.2)
    G = Q.shape[2] // Hkv
    Vd = np.repeat(orc.dequantize_values(vc4, vs4, vz4, 4), G, axis=1)
    want = torch.einsum("bhn,bhnd->bhd", torch.softmax(torch.from_numpy(sc), dim=-1), torch.from_numpy(Vd)).numpy()
    assert np.allclose(orc.decode_attention_dual_vq(Q[2], S_in, S_out, ch, bits, nu_in, nu_out, vc4, vs4, vz4, 4, 0.2), want, rtol=0, atol=1e-13)


def test_degenerate_steps():
    K, V, Q, S_in, S_out, ch = _setup(7)
    B, Hkv, cap, d = K.shape
    caches = _empty_caches(B, Hkv, cap, d, S_in.shape[0], S_out.shape[0], 4)
    # the first step sees one token: the output is that token's value as stored (not the unquantized one)
    o0 = orc.generation_step(Q[0], S_in, S_out, ch, *caches, K[:, :, :1], V[:, :, :1], 0, 4)
    stored = orc.dequantize_values(caches[3][:, :, :1], caches[4][:, :, :1], caches[5][:, :, :1], 4)[:, :, 0]
    assert np.allclose(o0, np.repeat(stored, 2, axis=1), rtol=0, atol=1e-15)
    assert not np.allclose(o0, np.repeat(V[:, :, 0], 2, axis=1), rtol=0, atol=1e-3)
    # q = 0: every score is 0, the output is the mean of the stored values
    for pos in range(1, 4):
        o = orc.generation_step(np.zeros_like(Q[0]), S_in, S_out, ch, *caches, K[:, :, pos:pos + 1], V[:, :, pos:pos + 1], pos, 4)
    stored = orc.dequantize_values(caches[3][:, :, :4], caches[4][:, :, :4], caches[5][:, :, :4], 4)
    assert np.allclose(o, np.repeat(stored.mean(axis=2), 2, axis=1), rtol=0, atol=1e-14)
    with pytest.raises(ValueError):
        orc.append_token(*caches, K[:, :, :1], V[:, :, :1], S_in, S_out, ch, cap, 4)
    with pytest.raises(ValueError):
        orc.append_token(*caches, K[:, :, :2], V[:, :, :2], S_in, S_out, ch, 0, 4)


def test_planted_mistakes_are_caught(monkeypatch):
    run = lambda: (test_streaming_at_the_operating_point_equals_quantizing_everything_at_once(4),
                   test_the_step_is_the_written_out_formula(), test_degenerate_steps())
    run()
    orig_append = orc.append_token

    def value_not_quantized_into_its_row(bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, K_new, V_new, S_in, S_out, channels, pos, vbits=4):
        keep = vcodes[:, :, pos].copy()
        orig_append(bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, K_new, V_new, S_in, S_out, channels, pos, vbits)
        vcodes[:, :, pos] = keep

    def row_off_by_one(bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, K_new, V_new, S_in, S_out, channels, pos, vbits=4):
        orig_append(bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, K_new, V_new, S_in, S_out, channels, min(pos + 1, bits.shape[2] - 1), vbits)

    def norms_swapped(bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, K_new, V_new, S_in, S_out, channels, pos, vbits=4):
        orig_append(bits, nu_out16, nu_in16, vcodes, vscale16, vzero16, K_new, V_new, S_in, S_out, channels, pos, vbits)

    for bad in (value_not_quantized_into_its_row, row_off_by_one, norms_swapped):
        monkeypatch.setattr(orc, "append_token", bad)
        with pytest.raises(AssertionError):
            run()
    monkeypatch.setattr(orc, "append_token", orig_append)
    orig_dec = orc.decode_attention_dual_vq

    def new_token_left_out(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, vbits=4, scale=1.0):
        e = max(1, bits.shape[2] - 1)
        return orig_dec(Q, S_in, S_out, channels, bits[:, :, :e], nu_in16[:, :, :e], nu_out16[:, :, :e], vcodes[:, :, :e],
                        vscale16[:, :, :e], vzero16[:, :, :e], vbits, scale)

    def outlier_estimate_dropped(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, vbits=4, scale=1.0):
        return orig_dec(Q, S_in, S_out, channels, bits, nu_in16, np.zeros_like(nu_out16), vcodes, vscale16, vzero16, vbits, scale)

    def zero_point_dropped(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, vbits=4, scale=1.0):
        return orig_dec(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, vcodes, vscale16, np.zeros_like(vzero16), vbits, scale)

    for bad in (new_token_left_out, outlier_estimate_dropped, zero_point_dropped):
        monkeypatch.setattr(orc, "decode_attention_dual_vq", bad)
        with pytest.raises(AssertionError):
            test_the_step_is_the_written_out_formula()
    monkeypatch.setattr(orc, "decode_attention_dual_vq", orig_dec)
    run()
