"""Pins for the oracle's streaming functions (Algorithm 1 as a loop over the token stream).  CPU only."""
import numpy as np
import pytest

from oracle import qjl_oracle as orc


def _setup(seed=0, B=2, Hq=4, Hkv=2, cap=12, d=16, m=32):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((B, Hkv, cap, d))
    V = rng.standard_normal((B, Hkv, cap, d))
    Q = rng.standard_normal((cap, B, Hq, d))
    S = rng.standard_normal((m, d))
    return K, V, Q, S


def test_streaming_equals_quantizing_everything_at_once():
    K, V, Q, S = _setup()
    B, Hkv, cap, d = K.shape
    m = S.shape[0]
    bits = np.full((B, Hkv, cap, m // 8), 0xA5, dtype=np.uint8)      # stale contents must not matter
    nu = np.full((B, Hkv, cap), 77.0, dtype=np.float16)
    all_bits, all_nu, _ = orc.quantize_keys(K, S)
    for pos in range(cap):
        out = orc.decode_step(Q[pos], S, bits, nu, V, K[:, :, pos:pos + 1], pos, scale=0.3)
        assert np.array_equal(bits[:, :, :pos + 1], all_bits[:, :, :pos + 1])
        assert np.array_equal(nu[:, :, :pos + 1], all_nu[:, :, :pos + 1])
        if pos + 1 < cap:                                            # rows not yet written are untouched
            assert np.all(bits[:, :, pos + 1:] == 0xA5) and np.all(nu[:, :, pos + 1:] == np.float16(77.0))
        want = orc.decode_attention(Q[pos], S, all_bits[:, :, :pos + 1], all_nu[:, :, :pos + 1], V[:, :, :pos + 1], 0.3)
        assert np.array_equal(out, want)
    # the first step sees one key: the output is that key's value
    bits0 = np.zeros_like(bits); nu0 = np.zeros_like(nu)
    o0 = orc.decode_step(Q[0], S, bits0, nu0, V, K[:, :, :1], 0)
    assert np.allclose(o0, np.repeat(V[:, :, 0], 2, axis=1))


def test_append_several_tokens_and_bounds():
    K, V, Q, S = _setup(1)
    B, Hkv, cap, d = K.shape
    bits = np.zeros((B, Hkv, cap, 4), dtype=np.uint8); nu = np.zeros((B, Hkv, cap), dtype=np.float16)
    orc.append_keys(bits, nu, K[:, :, 3:8], S, 3)
    ref_b, ref_n, _ = orc.quantize_keys(K[:, :, 3:8], S)
    assert np.array_equal(bits[:, :, 3:8], ref_b) and np.array_equal(nu[:, :, 3:8], ref_n)
    assert not bits[:, :, :3].any() and not bits[:, :, 8:].any()
    with pytest.raises(ValueError):
        orc.append_keys(bits, nu, K[:, :, :5], S, cap - 4)
    with pytest.raises(ValueError):
        orc.append_keys(bits, nu, K[:, :, :1], S, -1)


def test_planted_mistakes_are_caught(monkeypatch):
    orig = orc.append_keys

    def off_by_one(bits, nu16, K_new, S, pos):
        return orig(bits, nu16, K_new, S, min(pos + 1, bits.shape[2] - K_new.shape[2]))

    monkeypatch.setattr(orc, "append_keys", off_by_one)
    with pytest.raises(AssertionError):
        test_streaming_equals_quantizing_everything_at_once()
    monkeypatch.setattr(orc, "append_keys", orig)
    orig_dec = orc.decode_attention

    def too_many_keys(Q, S, bits, nu16, V, scale=1.0):               # attends over one key too few
        return orig_dec(Q, S, bits[:, :, :max(1, bits.shape[2] - 1)], nu16[:, :, :max(1, bits.shape[2] - 1)],
                        V[:, :, :max(1, bits.shape[2] - 1)], scale)

    monkeypatch.setattr(orc, "decode_attention", too_many_keys)
    with pytest.raises(AssertionError):
        K, V, Q, S = _setup()
        bits = np.zeros((2, 2, 12, 4), dtype=np.uint8); nu = np.zeros((2, 2, 12), dtype=np.float16)
        out = orc.decode_step(Q[0], S, bits, nu, V, K[:, :, :1], 0)
        o1 = orc.decode_step(Q[1], S, bits, nu, V, K[:, :, 1:2], 1)
        ab, an, _ = orc.quantize_keys(K, S)
        assert np.array_equal(o1, orig_dec(Q[1], S, ab[:, :, :2], an[:, :, :2], V[:, :, :2]))
