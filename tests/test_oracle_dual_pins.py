"""Pins for the oracle's outlier/inlier functions (Section 4.1 "Outliers"):
a hand-worked example, reductions to the single-sketch functions, brute force,
and the statistics that two independent unbiased estimators must obey.  CPU only.
"""
import json
import math
import os

import numpy as np
import pytest

from oracle import qjl_oracle as orc

C = orc.SQRT_HALF_PI


def _golden():
    here = os.path.dirname(os.path.abspath(__file__))
    with open(os.path.join(here, "golden", "dual_worked_example.json")) as f:
        return json.load(f)


def _as4(x):
    return np.asarray(x, dtype=np.float64)[None, None]


def test_worked_example_selection():
    g = _golden()
    K = _as4(g["K"])
    assert np.allclose(np.mean(np.abs(K[0, 0]), axis=0), g["mean_abs_per_channel"])
    assert orc.select_outlier_channels(K, 1)[0, 0].tolist() == g["top1_channels"]
    assert orc.select_outlier_channels(K, 2)[0, 0].tolist() == g["top2_channels"]
    assert orc.select_outlier_channels(K, 0).shape == (1, 1, 0)


def test_worked_example_codes_norms_scores_attention():
    g = _golden()
    K, S_in, S_out = _as4(g["K"]), np.asarray(g["S_in"], float), np.asarray(g["S_out"], float)
    ch = np.asarray(g["top1_channels"], dtype=np.int64)[None, None]
    bits, nu_in, nu_out, P_in, P_out = orc.quantize_keys_dual(K, S_in, S_out, ch)
    assert P_in[0, 0].tolist() == g["P_in"]
    assert P_out[0, 0].tolist() == g["P_out"]
    assert bits.dtype == np.uint8 and bits[0, 0].tolist() == g["code_bytes"]
    assert nu_in.dtype == np.float16 and nu_in[0, 0].tolist() == g["norms_in"]
    assert nu_out.dtype == np.float16 and nu_out[0, 0].tolist() == g["norms_out"]
    Q = np.asarray(g["q"], float)[None, None]
    Q_in, Q_out = orc.split_channels(Q, ch)
    assert orc.project_query(Q_in, S_in)[0, 0].tolist() == g["Sq_in"]
    assert orc.project_query(Q_out, S_out)[0, 0].tolist() == g["Sq_out"]
    s = orc.estimate_scores_dual(Q, S_in, S_out, ch, bits, nu_in, nu_out)
    want = [C / 8.0 * (g["norms_in"][j] * g["inner_in"][j] + g["norms_out"][j] * g["inner_out"][j]) for j in range(2)]
    assert np.allclose(s[0, 0], want, rtol=1e-14)
    assert np.allclose(s[0, 0] / C, g["score_over_sqrt_half_pi"], rtol=1e-14)
    # attention: two keys, identity values -> the softmax weights themselves
    a = g["attention_scale"]
    out = orc.decode_attention_dual(Q, S_in, S_out, ch, bits, nu_in, nu_out, _as4(g["V"]), scale=a)
    s0, s1 = (a * C * x for x in g["score_over_sqrt_half_pi"])
    p0 = 1.0 / (1.0 + math.exp(s1 - s0))
    assert np.allclose(out[0, 0], [p0, 1.0 - p0], rtol=1e-13)


def test_selection_matches_sort_and_tie_rule():
    rng = np.random.default_rng(5)
    K = rng.standard_normal((2, 3, 40, 12))
    K[0, 1, :, 4] *= 9.0
    K[1, 2, :, [0, 11]] *= 7.0
    got = orc.select_outlier_channels(K, 4)
    for b in range(2):
        for h in range(3):
            mean_abs = np.abs(K[b, h]).mean(axis=0)
            assert got[b, h].tolist() == np.argsort(-mean_abs, kind="stable")[:4].tolist()
    assert got[0, 1, 0] == 4 and set(got[1, 2, :2].tolist()) == {0, 11}
    # exact ties: equal columns -> lower index first
    T = np.ones((1, 1, 6, 5))
    T[..., 3] = 2.0
    assert orc.select_outlier_channels(T, 3)[0, 0].tolist() == [3, 0, 1]
    # sign must not matter, only magnitude
    assert orc.select_outlier_channels(-K, 4).tolist() == got.tolist()


def test_split_is_a_partition_and_follows_gqa():
    rng = np.random.default_rng(6)
    ch = np.array([[[1, 5], [0, 2]]])                      # B=1, Hkv=2
    X = rng.standard_normal((1, 4, 3, 8))                  # 4 heads -> heads 0,1 use kv 0; 2,3 use kv 1
    X_in, X_out = orc.split_channels(X, ch)
    assert np.array_equal(X_in + X_out, X)
    for h, idx in [(0, [1, 5]), (1, [1, 5]), (2, [0, 2]), (3, [0, 2])]:
        rest = [t for t in range(8) if t not in idx]
        assert np.array_equal(X_out[0, h][..., idx], X[0, h][..., idx])
        assert not X_out[0, h][..., rest].any()
        assert not X_in[0, h][..., idx].any()
        assert np.array_equal(X_in[0, h][..., rest], X[0, h][..., rest])
    with pytest.raises(ValueError):
        orc.split_channels(X, np.array([[[1, 1], [0, 2]]]))


def test_no_outliers_reduces_to_the_single_sketch():
    rng = np.random.default_rng(7)
    K = rng.standard_normal((1, 2, 9, 16))
    Q = rng.standard_normal((1, 4, 16))
    V = rng.standard_normal((1, 2, 9, 16))
    S_in = rng.standard_normal((32, 16))
    S_out = rng.standard_normal((8, 16))
    none = np.zeros((1, 2, 0), dtype=np.int64)
    bits, nu_in, nu_out, _, P_out = orc.quantize_keys_dual(K, S_in, S_out, none)
    b1, nu1, _ = orc.quantize_keys(K, S_in)
    assert np.array_equal(bits[..., :4], b1) and np.array_equal(nu_in, nu1)
    assert not P_out.any() and np.all(bits[..., 4:] == 0xFF) and not nu_out.any()   # sign(0) = +1, zero norm
    s = orc.estimate_scores_dual(Q, S_in, S_out, none, bits, nu_in, nu_out, scale=0.3)
    assert np.array_equal(s, orc.estimate_scores(orc.project_query(Q, S_in), b1, nu1, scale=0.3))
    o = orc.decode_attention_dual(Q, S_in, S_out, none, bits, nu_in, nu_out, V, scale=0.3)
    assert np.array_equal(o, orc.decode_attention(Q, S_in, b1, nu1, V, scale=0.3))


def test_all_channels_outliers_reduces_to_the_outlier_sketch():
    rng = np.random.default_rng(8)
    K = rng.standard_normal((1, 1, 7, 8))
    Q = rng.standard_normal((1, 1, 8))
    S_in = rng.standard_normal((16, 8))
    S_out = rng.standard_normal((24, 8))
    every = np.arange(8)[None, None]
    bits, nu_in, nu_out, _, _ = orc.quantize_keys_dual(K, S_in, S_out, every)
    b2, nu2, _ = orc.quantize_keys(K, S_out)
    assert np.array_equal(bits[..., 2:], b2) and np.array_equal(nu_out, nu2) and not nu_in.any()
    s = orc.estimate_scores_dual(Q, S_in, S_out, every, bits, nu_in, nu_out)
    assert np.array_equal(s, orc.estimate_scores(orc.project_query(Q, S_out), b2, nu2))


def test_bruteforce_tiny_python_loops():
    """Everything recomputed with Python integers and loops, no numpy arithmetic."""
    rng = np.random.default_rng(9)
    d, m_in, m_out, n = 6, 16, 8, 5
    K = rng.integers(-9, 10, size=(n, d)).tolist()
    for row in K:
        row[2] *= 11
    S_in = rng.integers(-4, 5, size=(m_in, d)).tolist()
    S_out = rng.integers(-4, 5, size=(m_out, d)).tolist()
    q = rng.integers(-5, 6, size=d).tolist()
    # selection: largest sum of |k| (same ranking as the mean), ties to the lower index
    tot = [sum(abs(K[j][t]) for j in range(n)) for t in range(d)]
    order = sorted(range(d), key=lambda t: (-tot[t], t))[:2]
    Kn = np.asarray(K, float)[None, None]
    ch = orc.select_outlier_channels(Kn, 2)
    assert ch[0, 0].tolist() == order and order[0] == 2
    bits, nu_in, nu_out, _, _ = orc.quantize_keys_dual(Kn, np.asarray(S_in, float), np.asarray(S_out, float), ch)
    s = orc.estimate_scores_dual(np.asarray(q, float)[None, None], np.asarray(S_in, float), np.asarray(S_out, float),
                                 ch, bits, nu_in, nu_out)
    inl = [t for t in range(d) if t not in order]
    for j in range(n):
        total = 0.0
        col = 0
        for S, m, idx in ((S_in, m_in, inl), (S_out, m_out, order)):
            inner = 0
            for i in range(m):
                p = sum(S[i][t] * K[j][t] for t in idx)
                bit = 1 if p >= 0 else 0
                assert (int(bits[0, 0, j, col + i // 8]) >> (i % 8)) & 1 == bit
                inner += (1 if bit else -1) * sum(S[i][t] * q[t] for t in idx)
            nrm = float(np.float16(math.sqrt(sum(K[j][t] ** 2 for t in idx))))
            total += C / m * nrm * inner
            col += m // 8
        assert abs(s[0, 0, j] - total) <= 1e-12 * max(1.0, abs(total))


def test_matches_sum_of_two_definitions():
    """estimate_scores_dual = Prod_QJL(q_in,k_in;S_in) + Prod_QJL(q_out,k_out;S_out) (up to the binary16 norms)."""
    rng = np.random.default_rng(10)
    d = 16
    K = rng.standard_normal((1, 1, 6, d)); K[..., [3, 9]] *= 12
    q = rng.standard_normal(d)
    S_in, S_out = rng.standard_normal((64, d)), rng.standard_normal((32, d))
    ch = orc.select_outlier_channels(K, 2)
    bits, nu_in, nu_out, _, _ = orc.quantize_keys_dual(K, S_in, S_out, ch)
    s = orc.estimate_scores_dual(q[None, None], S_in, S_out, ch, bits, nu_in, nu_out)[0, 0]
    mask = np.zeros(d); mask[ch[0, 0]] = 1.0
    for j in range(6):
        k = K[0, 0, j]
        want = orc.prod_qjl(q * (1 - mask), k * (1 - mask), S_in) + orc.prod_qjl(q * mask, k * mask, S_out)
        assert abs(s[j] - want) <= 1.5e-3 * (abs(want) + 1.0)


def _dual_samples(q, k, mask, m_in, m_out, T, rng):
    d = len(q)
    vals = np.empty(T)
    for t in range(T):
        S_in = rng.standard_normal((m_in, d))
        S_out = rng.standard_normal((m_out, d))
        vals[t] = orc.prod_qjl(q * (1 - mask), k * (1 - mask), S_in) + orc.prod_qjl(q * mask, k * mask, S_out)
    return vals


def test_unbiased_with_the_sum_of_the_two_variances():
    """Lemma 3.2 for each copy => the sum is unbiased for <q,k>; the copies are independent, so the
    variance is the sum of the two exact variances ((pi/2)|q|^2|k|^2 - <q,k>^2)/m of each part."""
    rng = np.random.default_rng(11)
    d, m_in, m_out, T = 32, 64, 32, 6000
    k = rng.standard_normal(d); k[[5, 20]] *= 15
    q = rng.standard_normal(d)
    mask = np.zeros(d); mask[[5, 20]] = 1.0
    vals = _dual_samples(q, k, mask, m_in, m_out, T, rng)

    def var(qq, kk, m):
        return ((math.pi / 2) * (qq @ qq) * (kk @ kk) - (qq @ kk) ** 2) / m

    v = var(q * (1 - mask), k * (1 - mask), m_in) + var(q * mask, k * mask, m_out)
    assert abs(vals.mean() - q @ k) <= 4.0 * math.sqrt(v / T)
    assert abs(vals.var(ddof=1) / v - 1.0) <= 0.08


def test_split_beats_one_sketch_of_the_same_size_on_outlier_keys():
    """Section 4.1: isolating the outlier channels lowers the distortion (at equal total bits)."""
    rng = np.random.default_rng(12)
    d, T = 32, 3000
    k = rng.standard_normal(d); k[[1, 7, 19, 30]] *= 15
    q = rng.standard_normal(d)
    mask = np.zeros(d); mask[[1, 7, 19, 30]] = 1.0
    dual = _dual_samples(q, k, mask, 64, 32, T, rng)
    single = np.array([orc.prod_qjl(q, k, rng.standard_normal((96, d))) for _ in range(T)])
    assert dual.var() < 0.8 * single.var()
    # closed forms say the same
    one = ((math.pi / 2) * (q @ q) * (k @ k) - (q @ k) ** 2) / 96
    qi, ki, qo, ko = q * (1 - mask), k * (1 - mask), q * mask, k * mask
    two = ((math.pi / 2) * (qi @ qi) * (ki @ ki) - (qi @ ki) ** 2) / 64 + ((math.pi / 2) * (qo @ qo) * (ko @ ko) - (qo @ ko) ** 2) / 32
    assert two < one


def test_scaling_invariance():
    rng = np.random.default_rng(13)
    K = rng.standard_normal((1, 1, 5, 8)); K[..., 6] *= 20
    Q = rng.standard_normal((1, 1, 8))
    S_in, S_out = rng.standard_normal((16, 8)), rng.standard_normal((8, 8))
    ch = orc.select_outlier_channels(K, 1)
    assert ch[0, 0].tolist() == [6]
    b1, i1, o1, _, _ = orc.quantize_keys_dual(K, S_in, S_out, ch)
    b2, i2, o2, _, _ = orc.quantize_keys_dual(4.0 * K, S_in, S_out, orc.select_outlier_channels(4.0 * K, 1))
    assert np.array_equal(b1, b2)
    assert np.allclose(i2.astype(float), 4 * i1.astype(float), rtol=1e-3) and np.allclose(o2.astype(float), 4 * o1.astype(float), rtol=1e-3)


# ---- the pins must bite: planted mistakes in the dual functions
def _sel_by_max(K, count):
    K = np.asarray(K, dtype=np.float64)
    mx = np.max(np.abs(K), axis=2)
    return np.argsort(-mx, axis=-1, kind="stable")[..., :count].astype(np.int64)


def _sel_ties_high(K, count):
    K = np.asarray(K, dtype=np.float64)
    mean_abs = np.mean(np.abs(K), axis=2)
    B, H, d = mean_abs.shape
    out = np.empty((B, H, count), dtype=np.int64)
    for b in range(B):
        for h in range(H):
            out[b, h] = sorted(range(d), key=lambda t: (-mean_abs[b, h, t], -t))[:count]
    return out


_orig_split = orc.split_channels
_orig_quant_dual = orc.quantize_keys_dual
_orig_est = orc.estimate_scores


def _split_without_zeroing(X, channels):
    X_in, X_out = _orig_split(X, channels)
    return np.asarray(X, dtype=np.float64), X_out            # inlier copy still sees the outliers


def _split_kv_head_zero_only(X, channels):
    ch0 = np.repeat(np.asarray(channels)[:, :1], np.asarray(channels).shape[1], axis=1)
    return _orig_split(X, ch0)                               # every head uses the channels of kv head 0


def _quant_dual_swapped_order(K, S_in, S_out, channels):
    bits, nu_in, nu_out, P_in, P_out = _orig_quant_dual(K, S_in, S_out, channels)
    m_in = np.asarray(S_in).shape[0]
    return np.concatenate([bits[..., m_in // 8:], bits[..., : m_in // 8]], axis=-1), nu_in, nu_out, P_in, P_out


def _quant_dual_swapped_norms(K, S_in, S_out, channels):
    bits, nu_in, nu_out, P_in, P_out = _orig_quant_dual(K, S_in, S_out, channels)
    return bits, nu_out, nu_in, P_in, P_out


DUAL_PINS = [
    test_worked_example_selection, test_worked_example_codes_norms_scores_attention,
    test_selection_matches_sort_and_tie_rule, test_split_is_a_partition_and_follows_gqa,
    test_no_outliers_reduces_to_the_single_sketch, test_all_channels_outliers_reduces_to_the_outlier_sketch,
    test_bruteforce_tiny_python_loops, test_matches_sum_of_two_definitions,
]
DUAL_MUTATIONS = [
    ("select_outlier_channels", _sel_by_max, "channels ranked by max |k| instead of mean |k|"),
    ("select_outlier_channels", _sel_ties_high, "ties to the higher index"),
    ("split_channels", _split_without_zeroing, "inlier copy not cleared of outlier coordinates"),
    ("split_channels", _split_kv_head_zero_only, "every head uses kv head 0's channels"),
    ("quantize_keys_dual", _quant_dual_swapped_order, "outlier code stored before the inlier code"),
    ("quantize_keys_dual", _quant_dual_swapped_norms, "the two norms swapped"),
]


@pytest.mark.parametrize("name,replacement,what", DUAL_MUTATIONS, ids=[m[2] for m in DUAL_MUTATIONS])
def test_planted_mistake_in_dual_functions_is_caught(monkeypatch, name, replacement, what):
    monkeypatch.setattr(orc, name, replacement)
    failed = 0
    for pin in DUAL_PINS:
        try:
            pin()
        except (AssertionError, ValueError, IndexError):
            failed += 1
    assert failed >= 1, f"no pin noticed: {what}"
