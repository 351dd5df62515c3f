"""Pins for the oracle's value-cache quantizer (Section 3.2): a hand-worked row,
the round-trip error bound, structural properties, and planted mistakes.  CPU only."""
import json
import os

import numpy as np
import pytest

from oracle import qjl_oracle as orc


def _golden():
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "golden", "value_quant_worked_example.json")) as f:
        return json.load(f)


def _f32(x):
    return np.asarray(x, dtype=np.float32).astype(np.float64)


def test_worked_rows():
    g = _golden()
    V = _f32(g["row"])[None, None, None]
    codes, sc, z = orc.quantize_values(V, 4)
    assert codes.dtype == np.uint8 and sc.dtype == np.float16 and z.dtype == np.float16
    assert float(sc[0, 0, 0]) == g["scale"] and float(z[0, 0, 0]) == g["zero"]
    assert codes[0, 0, 0].tolist() == g["packed_bytes"]
    assert np.allclose(orc.dequantize_values(codes, sc, z, 4)[0, 0, 0], g["dequantized"], atol=0, rtol=0)
    V2 = _f32(g["row2_2bit"])[None, None, None]
    c2, s2, z2 = orc.quantize_values(V2, 2)
    assert c2[0, 0, 0].tolist() == g["row2_packed"] and float(s2[0, 0, 0]) == 1.0 and float(z2[0, 0, 0]) == -1.0
    assert orc.dequantize_values(c2, s2, z2, 2)[0, 0, 0].tolist() == g["row2_dequantized"]


def _unpack_loops(codes_row, vbits, d):
    out = []
    for t in range(d):
        bit = t * vbits
        out.append((int(codes_row[bit // 8]) >> (bit % 8)) & ((1 << vbits) - 1))
    return out


@pytest.mark.parametrize("vbits", [2, 4, 8])
def test_roundtrip_bound_and_structure(vbits):
    rng = np.random.default_rng(3 + vbits)
    V = _f32(rng.standard_normal((2, 3, 17, 32)) * rng.uniform(0.1, 30.0, size=(2, 3, 17, 1)))
    codes, sc, z = orc.quantize_values(V, vbits)
    assert codes.shape == (2, 3, 17, 32 * vbits // 8)
    back = orc.dequantize_values(codes, sc, z, vbits)
    s64, z64 = sc.astype(np.float64)[..., None], z.astype(np.float64)[..., None]
    lo, hi = V.min(-1, keepdims=True), V.max(-1, keepdims=True)
    levels = (1 << vbits) - 1
    # stored constants are the binary16 neighbours of the exact ones
    assert np.all(np.abs(z64 - lo) <= 2.0 ** -10 * np.abs(lo) + 1e-7)
    assert np.all(np.abs(s64 - (hi - lo) / levels) <= 2.0 ** -10 * (hi - lo) / levels + 1e-7)
    # error: half a step, plus what the rounding of zero and scale can add at the top of the range
    bound = 0.5 * s64 + np.abs(z64 - lo) + levels * np.abs(s64 - (hi - lo) / levels) + 1e-6
    assert np.all(np.abs(back - V) <= bound)
    for idx in [(0, 0, 0), (1, 2, 16)]:
        q = _unpack_loops(codes[idx], vbits, 32)
        assert min(q) == 0 and max(q) == levels            # the extremes of a row hit the ends of the range
        order = np.argsort(V[idx], kind="stable")
        assert all(q[a] <= q[b] for a, b in zip(order[:-1], order[1:]))   # monotone
        assert np.allclose(back[idx], float(z[idx]) + np.asarray(q) * float(sc[idx]), rtol=0, atol=0)


def test_constant_and_degenerate_rows():
    V = np.zeros((1, 1, 3, 8))
    V[0, 0, 1] = 2.5
    V[0, 0, 2, 3] = 1e-9                                     # range underflows binary16 -> scale 0
    V = _f32(V)
    codes, sc, z = orc.quantize_values(V, 4)
    assert not codes.any() and not sc.any()
    assert z[0, 0].tolist() == [0.0, 2.5, 0.0]
    assert np.array_equal(orc.dequantize_values(codes, sc, z, 4)[0, 0, 1], np.full(8, 2.5))


def test_power_of_two_affine_equivariance_and_sign_flip():
    rng = np.random.default_rng(9)
    V = _f32(rng.standard_normal((1, 2, 9, 16)))
    c1, s1, z1 = orc.quantize_values(V, 4)
    c2, s2, z2 = orc.quantize_values(4.0 * V, 4)             # exact scaling: same codes, constants x4
    assert np.array_equal(c1, c2) and np.array_equal(s2.astype(np.float64), 4 * s1.astype(np.float64))
    assert np.array_equal(z2.astype(np.float64), 4 * z1.astype(np.float64))
    b1 = orc.dequantize_values(c1, s1, z1, 4)
    b3 = orc.dequantize_values(*orc.quantize_values(-V, 4), 4)
    assert np.max(np.abs(b1 - V)) <= 0.51 * float(s1.max()) + 2e-3 and np.max(np.abs(b3 + V)) <= 0.51 * float(s1.max()) + 2e-3


def test_attention_on_stored_values_matches_the_algebra():
    """sum_j p_j (zero_j + scale_j c_j) = sum_j (p_j scale_j) c_j + sum_j p_j zero_j, and it stays close to
    attention on the unquantized values."""
    rng = np.random.default_rng(10)
    B, Hq, Hkv, n, d, m = 1, 4, 2, 50, 16, 64
    K = _f32(rng.standard_normal((B, Hkv, n, d)))
    V = _f32(rng.standard_normal((B, Hkv, n, d)))
    Q = _f32(rng.standard_normal((B, Hq, d)))
    S = _f32(rng.standard_normal((m, d)))
    bits, nu, _ = orc.quantize_keys(K, S)
    codes, sc, z = orc.quantize_values(V, 4)
    out = orc.decode_attention_vq(Q, S, bits, nu, codes, sc, z, 4, scale=0.25)
    p = orc.softmax(orc.estimate_scores(orc.project_query(Q, S), bits, nu, 0.25))
    for h in range(Hq):
        g = h // 2
        q = np.array([_unpack_loops(codes[0, g, j], 4, d) for j in range(n)], dtype=np.float64)
        want = (p[0, h] * sc[0, g].astype(np.float64)) @ q + p[0, h] @ z[0, g].astype(np.float64)
        assert np.allclose(out[0, h], want, rtol=1e-12, atol=1e-12)
    full = orc.decode_attention(Q, S, bits, nu, V, scale=0.25)
    assert np.max(np.abs(out - full)) <= 0.5 * float(sc.max()) + 1e-3


# ---- planted mistakes
_orig_q = orc.quantize_values
_orig_d = orc.dequantize_values


def _swap_nibbles(V, vbits=4):
    c, s, z = _orig_q(V, vbits)
    if vbits == 4:
        c = ((c << 4) | (c >> 4)).astype(np.uint8)
    return c, s, z


def _truncate(V, vbits=4):
    c, s, z = _orig_q(V, vbits)
    V32 = np.asarray(V, dtype=np.float32)
    sc = s.astype(np.float32)[..., None]
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.floor((V32 - z.astype(np.float32)[..., None]) / sc)
    q = np.where(sc > 0, np.clip(q, 0, (1 << vbits) - 1), 0).astype(np.uint8)
    per = 8 // vbits
    g = q.reshape(q.shape[:-1] + (q.shape[-1] // per, per)).astype(np.uint16)
    p = np.zeros(g.shape[:-1], dtype=np.uint16)
    for t in range(per):
        p |= g[..., t] << (vbits * t)
    return p.astype(np.uint8), s, z


def _scale_over_levels_plus_one(V, vbits=4):
    V32 = np.asarray(V, dtype=np.float32)
    c, s, z = _orig_q(V, vbits)
    return c, ((V32.max(-1) - V32.min(-1)) / np.float32(1 << vbits)).astype(np.float16), z


def _dequant_without_zero(codes, scale16, zero16, vbits=4):
    return _orig_d(codes, scale16, np.zeros_like(zero16), vbits)


PINS = [test_worked_rows, lambda: test_roundtrip_bound_and_structure(4), lambda: test_roundtrip_bound_and_structure(2),
        test_constant_and_degenerate_rows, test_power_of_two_affine_equivariance_and_sign_flip,
        test_attention_on_stored_values_matches_the_algebra]
MUTATIONS = [("quantize_values", _swap_nibbles, "element order inside a byte reversed"),
             ("quantize_values", _truncate, "truncation instead of round-to-nearest-even"),
             ("quantize_values", _scale_over_levels_plus_one, "scale = range / 2^b"),
             ("dequantize_values", _dequant_without_zero, "zero point dropped when reading back")]


@pytest.mark.parametrize("name,replacement,what", MUTATIONS, ids=[m[2] for m in MUTATIONS])
def test_planted_mistake_in_value_functions_is_caught(monkeypatch, name, replacement, what):
    monkeypatch.setattr(orc, name, replacement)
    failed = 0
    for pin in PINS:
        try:
            pin()
        except (AssertionError, ValueError, IndexError):
            failed += 1
    assert failed >= 1, f"no pin noticed: {what}"


# ------------------------------------------------------------------ the definition in exact arithmetic
@pytest.mark.parametrize("vbits", [2, 4, 8])
def test_exact_codes_against_rational_arithmetic(vbits):
    """`value_codes_exact` against Python's Fraction: (v - zero) / scale as an exact rational, rounded half to even,
    clipped.  Rows with many exact ties (few-bit inputs) are included on purpose."""
    from fractions import Fraction
    rng = np.random.default_rng(40 + vbits)
    rows = [rng.standard_normal(16).astype(np.float32), np.round(rng.standard_normal(16) * 4) / 8,
            np.arange(16, dtype=np.float64) * 0.25 - 1.0, np.full(16, 0.75),
            np.array([0.0, (1 << vbits) - 1, 0.5, 1.5, 2.5, 0.25, 0.75, 1.0, 2.0, 0.5, 1.5, 2.5, 0.0, 1.25, 2.75, 0.5])]   # scale 1: exact ties
    V = np.stack(rows).astype(np.float32).astype(np.float64)[None, None]
    sc16, z16, _ = orc.value_constants_exact(V, vbits)
    codes, near = orc.value_codes_exact(V, sc16, z16, vbits)
    levels = (1 << vbits) - 1
    ties = 0
    for r in range(V.shape[2]):
        s, z = Fraction(float(sc16[0, 0, r])), Fraction(float(z16[0, 0, r]))
        for t in range(16):
            if s == 0:
                want = 0
            else:
                q = (Fraction(float(V[0, 0, r, t])) - z) / s
                fl = q.numerator // q.denominator
                rem = q - fl
                want = fl + 1 if rem > Fraction(1, 2) else fl if rem < Fraction(1, 2) else fl + (fl % 2)
                ties += rem == Fraction(1, 2)
                want = min(max(want, 0), levels)
            assert int(codes[0, 0, r, t]) == want, (r, t)
    assert ties > 0                                            # the half-even rule was exercised
    assert near[0, 0, 4, 2:5].all()                            # and those entries are flagged as near a tie


@pytest.mark.parametrize("vbits", [2, 4, 8])
def test_float32_form_agrees_with_the_definition_outside_the_tie_band(vbits):
    """`quantize_values` (three float32 operations) may differ from the exact definition only where the definition
    itself flags a near-tie; constants likewise only on rows flagged as near a binary16 midpoint."""
    rng = np.random.default_rng(50 + vbits)
    V = (rng.standard_normal((2, 2, 400, 128)) * rng.uniform(0.05, 40.0, size=(2, 2, 400, 1))).astype(np.float32)
    V[0, 0, :50] = np.round(V[0, 0, :50] * 8) / 8              # bf16-like inputs: exact ties occur
    V = V.astype(np.float64)
    packed, sc, z = orc.quantize_values(V, vbits)
    sc_x, z_x, near_c = orc.value_constants_exact(V, vbits)
    assert np.array_equal(z.view(np.uint16), z_x.view(np.uint16))
    assert np.array_equal(sc.view(np.uint16)[~near_c], sc_x.view(np.uint16)[~near_c])
    codes_x, near = orc.value_codes_exact(V, sc, z, vbits)      # against the constants that were stored
    got = orc.unpack_value_codes(packed, vbits)
    diff = got != codes_x
    assert not (diff & ~near).any()
    assert int(np.abs(got.astype(int) - codes_x.astype(int)).max()) <= 1
    assert near.mean() < 0.02                                  # the band is thin


def test_unpack_value_codes_is_the_inverse_of_the_packing():
    rng = np.random.default_rng(9)
    for vbits in (2, 4, 8):
        V = rng.standard_normal((1, 2, 5, 32)).astype(np.float32).astype(np.float64)
        packed, sc, z = orc.quantize_values(V, vbits)
        per = orc.unpack_value_codes(packed, vbits)
        for idx in [(0, 0, 0), (0, 1, 4)]:
            assert per[idx].tolist() == _unpack_loops(packed[idx], vbits, 32)
        assert np.array_equal(orc.dequantize_values(packed, sc, z, vbits),
                              z.astype(np.float64)[..., None] + per * sc.astype(np.float64)[..., None])
