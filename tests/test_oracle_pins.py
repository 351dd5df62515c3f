"""Pins for the CPU oracle: each test ties an oracle function to something the
paper or plain mathematics fixes (hand-worked values, closed forms, textbook
routines, invariants, Monte Carlo against Lemma 3.2 / Lemma 3.5), never to the
oracle's own formula retyped.  CPU only.
"""
import json
import math
import os

import numpy as np
import pytest
import torch
from scipy import stats

from oracle import qjl_oracle as orc

RT_HALF_PI = math.sqrt(math.pi / 2.0)


def _load_example(golden_dir):
    with open(os.path.join(golden_dir, "def31_worked_example.json")) as f:
        return json.load(f)


# ---------------------------------------------------------------- worked example
def test_worked_example_bits_norms_scores(golden_dir):
    """Definition 3.1 worked by hand on d=4, m=8 integers (see the fixture)."""
    ex = _load_example(golden_dir)
    S = np.array(ex["S"], dtype=np.float64)
    K = np.array(ex["keys"], dtype=np.float64)[None, None]          # [1,1,2,4]
    Q = np.array(ex["query"], dtype=np.float64)[None, None]         # [1,1,4]
    bits, nu, P = orc.quantize_keys(K, S)
    assert P[0, 0].tolist() == ex["Sk"]
    assert bits.shape == (1, 1, 2, 1) and bits.dtype == np.uint8
    assert bits[0, 0, :, 0].tolist() == ex["packed_bytes"]          # 0x5B, 0x67
    assert nu.dtype == np.float16 and nu[0, 0].tolist() == ex["norms"]
    assert orc.unpack_signs(bits, 8)[0, 0].tolist() == ex["signs"]
    SQ = orc.project_query(Q, S)
    assert SQ[0, 0].tolist() == ex["Sq"]
    sc = orc.estimate_scores(SQ, bits, nu, scale=1.0)
    want = [c * RT_HALF_PI for c in ex["prod_qjl_over_sqrt_half_pi"]]
    np.testing.assert_allclose(sc[0, 0], want, rtol=1e-15)
    for j in range(2):
        assert orc.prod_qjl(Q[0, 0], K[0, 0, j], S) == pytest.approx(want[j], rel=1e-15)


def test_worked_example_attention(golden_dir):
    ex = _load_example(golden_dir)
    S = np.array(ex["S"], dtype=np.float64)
    K = np.array(ex["keys"], dtype=np.float64)[None, None]
    Q = np.array(ex["query"], dtype=np.float64)[None, None]
    V = np.array(ex["values"], dtype=np.float64)[None, None]
    bits, nu, _ = orc.quantize_keys(K, S)
    out = orc.decode_attention(Q, S, bits, nu, V, scale=ex["softmax_scale"])
    p2 = 1.0 / (1.0 + math.exp(1.6875 * RT_HALF_PI))
    want = (1.0 - p2) * V[0, 0, 0] + p2 * V[0, 0, 1]
    np.testing.assert_allclose(out[0, 0], want, rtol=1e-14)


# ---------------------------------------------------------------- brute force, tiny sizes
def test_bruteforce_tiny_python_loops():
    """d <= 8, m <= 16, small integers: every step redone with Python ints and
    loops (exact), including the bit placement."""
    rng = np.random.default_rng(7)
    for d, m, n in [(3, 8, 5), (8, 16, 9), (5, 16, 4)]:
        S = rng.integers(-3, 4, size=(m, d))
        K = rng.integers(-4, 5, size=(n, d))
        K[0] = 0                                                    # the zero key
        q = rng.integers(-3, 4, size=d)
        bits, nu, _ = orc.quantize_keys(K[None, None].astype(float), S.astype(float))
        SQ = orc.project_query(q[None, None].astype(float), S.astype(float))
        sc = orc.estimate_scores(SQ, bits, nu)
        for j in range(n):
            code = 0
            inner = 0
            for i in range(m):
                p = sum(int(S[i, t]) * int(K[j, t]) for t in range(d))
                sq = sum(int(S[i, t]) * int(q[t]) for t in range(d))
                if p >= 0:
                    code |= 1 << i
                    inner += sq
                else:
                    inner -= sq
            got = sum(int(bits[0, 0, j, b]) << (8 * b) for b in range(m // 8))
            assert got == code
            nrm = float(np.float16(math.sqrt(sum(int(x) ** 2 for x in K[j]))))
            assert float(nu[0, 0, j]) == nrm
            assert sc[0, 0, j] == pytest.approx(RT_HALF_PI / m * nrm * inner, rel=1e-14, abs=1e-300)
        assert np.all(bits[0, 0, 0] == 0xFF) and nu[0, 0, 0] == 0 and sc[0, 0, 0] == 0


def test_pack_is_little_endian_bit_order():
    rng = np.random.default_rng(3)
    b = rng.random((4, 7, 64)) < 0.5
    got = orc.pack_sign_bits(b)
    np.testing.assert_array_equal(got, np.packbits(b, axis=-1, bitorder="little"))
    one = np.zeros(32, dtype=bool)
    one[11] = True                                                  # byte 1, bit 3
    assert orc.pack_sign_bits(one).tolist() == [0, 8, 0, 0]
    sig = orc.unpack_signs(got, 64)
    np.testing.assert_array_equal(sig > 0, b)
    assert set(np.unique(sig)) == {-1.0, 1.0}


# ---------------------------------------------------------------- special cases -> library routines
def test_identity_sketch_reduces_to_sign_of_key():
    rng = np.random.default_rng(11)
    d = 16
    K = rng.standard_normal((1, 2, 9, d))
    Q = rng.standard_normal((1, 2, d))
    S = np.eye(d)
    bits, nu, _ = orc.quantize_keys(K, S)
    np.testing.assert_array_equal(bits, np.packbits(K >= 0, axis=-1, bitorder="little"))
    sc = orc.estimate_scores(orc.project_query(Q, S), bits, nu)
    nu64 = np.linalg.norm(K, axis=-1).astype(np.float16).astype(np.float64)
    want = RT_HALF_PI / d * nu64 * np.einsum("bht,bhjt->bhj", Q, np.sign(K))
    np.testing.assert_allclose(sc, want, rtol=1e-13)


def test_self_product_is_l1_norm_of_projection():
    """q = k: Prod_QJL(k,k) = sqrt(pi/2)/m * ||k|| * ||S k||_1 (first line of
    the proof of Lemma 3.2 with q = k) -- never touches the bit code."""
    rng = np.random.default_rng(5)
    S = rng.standard_normal((64, 24))
    for _ in range(5):
        k = rng.standard_normal(24) * 3
        want = RT_HALF_PI / 64 * np.linalg.norm(k) * np.abs(S @ k).sum()
        assert orc.prod_qjl(k, k, S) == pytest.approx(want, rel=1e-13)


def test_proof_decomposition_matches_estimator():
    """Proof of Lemma 3.2: Prod = sqrt(pi/2)/m * sum_i [ <q,k>/||k|| |s_i.k| +
    ||k|| s_i.q_perp sign(s_i.k) ] with q_perp = q - <q,k>/||k||^2 k."""
    rng = np.random.default_rng(6)
    m, d = 48, 20
    S = rng.standard_normal((m, d))
    for _ in range(5):
        q, k = rng.standard_normal(d), rng.standard_normal(d) * 2
        nk = np.linalg.norm(k)
        qp = q - (q @ k) / nk ** 2 * k
        total = 0.0
        for i in range(m):
            sk = S[i] @ k
            total += (q @ k) / nk * abs(sk) + nk * (S[i] @ qp) * (1.0 if sk >= 0 else -1.0)
        assert orc.prod_qjl(q, k, S) == pytest.approx(RT_HALF_PI / m * total, rel=1e-12)


def test_packed_path_equals_definition_path():
    """estimate_scores (packed bits + fp16 norm) against prod_qjl (definition,
    float64 norm): equal up to the binary16 rounding of the norm."""
    rng = np.random.default_rng(8)
    m, d, n = 64, 32, 50
    S = rng.standard_normal((m, d))
    K = rng.standard_normal((1, 1, n, d))
    Q = rng.standard_normal((1, 1, d))
    bits, nu, _ = orc.quantize_keys(K, S)
    sc = orc.estimate_scores(orc.project_query(Q, S), bits, nu)[0, 0]
    for j in range(n):
        ref = orc.prod_qjl(Q[0, 0], K[0, 0, j], S)
        ratio = float(nu[0, 0, j]) / np.linalg.norm(K[0, 0, j])
        assert sc[j] == pytest.approx(ref * ratio, rel=1e-12)
        assert abs(ratio - 1) <= 2.0 ** -11


def test_norms_match_numpy_and_fp16_rne():
    rng = np.random.default_rng(9)
    K = rng.standard_normal((2, 3, 17, 128)) * rng.uniform(0.01, 40, size=(2, 3, 17, 1))
    nu = orc.key_norms(K)
    assert nu.dtype == np.float16
    ref = np.linalg.norm(K, axis=-1)
    np.testing.assert_array_equal(nu, ref.astype(np.float16))
    assert np.max(np.abs(nu.astype(np.float64) / ref - 1)) <= 2.0 ** -11
    # RNE tie: 2049 lies halfway between the binary16 neighbours 2048 and 2050
    assert float(orc.key_norms(np.array([[2049.0, 0.0]]))[0]) == 2048.0
    assert float(orc.key_norms(np.array([[2051.0, 0.0]]))[0]) == 2052.0


def test_project_query_is_matrix_vector_product():
    rng = np.random.default_rng(10)
    S = rng.standard_normal((40, 12))
    Q = rng.standard_normal((2, 5, 12))
    got = orc.project_query(Q, S)
    for b in range(2):
        for h in range(5):
            np.testing.assert_allclose(got[b, h], S @ Q[b, h], rtol=1e-12, atol=1e-13)
    # not transposed: a basis vector picks a column of S
    e3 = np.zeros((1, 1, 12))
    e3[0, 0, 3] = 1
    np.testing.assert_array_equal(orc.project_query(e3, S)[0, 0], S[:, 3])


def test_softmax_and_value_aggregation_match_torch_float64():
    rng = np.random.default_rng(12)
    B, Hq, Hkv, n, d = 2, 8, 2, 33, 16
    sc = rng.standard_normal((B, Hq, n)) * 30
    V = rng.standard_normal((B, Hkv, n, d))
    p = orc.softmax(sc)
    pt = torch.softmax(torch.from_numpy(sc), dim=-1)
    np.testing.assert_allclose(p, pt.numpy(), rtol=1e-13, atol=1e-300)
    np.testing.assert_allclose(p.sum(-1), 1.0, rtol=1e-14)
    Vrep = torch.from_numpy(V).repeat_interleave(Hq // Hkv, dim=1)   # contiguous groups
    want = torch.einsum("bhj,bhjt->bht", pt, Vrep).numpy()
    np.testing.assert_allclose(orc.attention_from_scores(sc, V), want, rtol=1e-12, atol=1e-14)


def test_gqa_head_mapping_is_contiguous_groups():
    """Query head h must read KV head h // G: make KV heads distinguishable."""
    rng = np.random.default_rng(13)
    B, Hq, Hkv, n, d, m = 1, 6, 2, 10, 8, 16
    S = rng.standard_normal((m, d))
    K = rng.standard_normal((B, Hkv, n, d))
    V = rng.standard_normal((B, Hkv, n, d))
    Q = rng.standard_normal((B, Hq, d))
    bits, nu, _ = orc.quantize_keys(K, S)
    out = orc.decode_attention(Q, S, bits, nu, V, scale=0.3)
    for h in range(Hq):
        g = h // 3
        single = orc.decode_attention(Q[:, h:h + 1], S, bits[:, g:g + 1], nu[:, g:g + 1],
                                      V[:, g:g + 1], scale=0.3)
        np.testing.assert_allclose(out[0, h], single[0, 0], rtol=1e-13)


# ---------------------------------------------------------------- invariants
def test_invariants_scaling_negation_linearity_permutation():
    rng = np.random.default_rng(14)
    m, d, n = 64, 32, 40
    S = rng.standard_normal((m, d))
    K = rng.standard_normal((1, 1, n, d))
    Q = rng.standard_normal((1, 2, d))
    # norms chosen exactly representable in binary16 so that scaling by 4 is exact
    bits, nu, _ = orc.quantize_keys(K, S)
    SQ = orc.project_query(Q[:, :1], S)
    sc = orc.estimate_scores(SQ, bits, nu)
    b4, nu4, _ = orc.quantize_keys(4.0 * K, S)
    np.testing.assert_array_equal(b4, bits)                         # k -> a k keeps the code
    np.testing.assert_array_equal(nu4.astype(np.float64), 4.0 * nu.astype(np.float64))
    np.testing.assert_allclose(orc.estimate_scores(SQ, b4, nu4), 4.0 * sc, rtol=1e-14)
    bn, nun, _ = orc.quantize_keys(-K, S)                           # k -> -k flips every bit
    np.testing.assert_array_equal(bn, ~bits)
    np.testing.assert_allclose(orc.estimate_scores(SQ, bn, nun), -sc, rtol=1e-14)
    # linear in q
    SQ2 = orc.project_query(Q[:, 1:], S)
    SQc = orc.project_query(2.0 * Q[:, :1] - 3.0 * Q[:, 1:], S)
    np.testing.assert_allclose(orc.estimate_scores(SQc, bits, nu),
                               2.0 * sc - 3.0 * orc.estimate_scores(SQ2, bits, nu),
                               rtol=1e-11, atol=1e-11)
    # permuting the rows of S permutes code bits and leaves the scores alone
    perm = rng.permutation(m)
    bp, nup, _ = orc.quantize_keys(K, S[perm])
    np.testing.assert_array_equal(orc.unpack_signs(bp, m), orc.unpack_signs(bits, m)[..., perm])
    np.testing.assert_allclose(orc.estimate_scores(orc.project_query(Q[:, :1], S[perm]), bp, nup),
                               sc, rtol=1e-12)
    # scale multiplies the logits
    np.testing.assert_allclose(orc.estimate_scores(SQ, bits, nu, scale=0.25), 0.25 * sc, rtol=1e-15)


def test_attention_degenerate_cases():
    rng = np.random.default_rng(15)
    m, d, n = 32, 16, 21
    S = rng.standard_normal((m, d))
    K = rng.standard_normal((1, 1, n, d))
    V = rng.standard_normal((1, 1, n, d))
    bits, nu, _ = orc.quantize_keys(K, S)
    out0 = orc.decode_attention(np.zeros((1, 1, d)), S, bits, nu, V)   # q = 0 -> uniform
    np.testing.assert_allclose(out0[0, 0], V[0, 0].mean(0), rtol=1e-13)
    out1 = orc.decode_attention(rng.standard_normal((1, 1, d)), S, bits[:, :, :1], nu[:, :, :1],
                                V[:, :, :1])
    np.testing.assert_allclose(out1[0, 0], V[0, 0, 0], rtol=1e-15)     # n = 1 -> v_1
    out = orc.decode_attention(rng.standard_normal((1, 1, d)), S, bits, nu, V, scale=0.2)
    assert np.all(out[0, 0] <= V[0, 0].max(0) + 1e-12) and np.all(out[0, 0] >= V[0, 0].min(0) - 1e-12)


# ---------------------------------------------------------------- Lemma 3.2 / Lemma 3.5 (Monte Carlo)
def _pairs(d, rng):
    q = rng.standard_normal(d)
    k = rng.standard_normal(d)
    k_out = k.copy()
    k_out[[1, 5, 7, 11]] *= 15.0                                       # outlier channels
    q_perp = q - (q @ k) / (k @ k) * k
    return [(q, k), (q, k_out), (k * 0.7, k), (q_perp, k), (-2.0 * k + 0.1 * q, k)]


@pytest.mark.parametrize("source", ["numpy_rng", "oracle_sketch"])
def test_unbiased_and_variance_closed_form(source):
    """Lemma 3.2: E_S[Prod_QJL] = <q,k>.  The proof of Lemma 3.5 gives
    E z_i^2 = (pi/2)||q||^2||k||^2 for the m i.i.d. terms, hence
    Var[Prod_QJL] = ((pi/2)||q||^2||k||^2 - <q,k>^2)/m exactly."""
    d, m, T = 16, 32, 20000
    rng = np.random.default_rng(2024)
    if source == "numpy_rng":
        Ss = rng.standard_normal((T, m, d))
    else:
        Ss = np.stack([orc.gaussian_sketch(1000 + t, m, d, "f32") for t in range(T)])
    for q, k in _pairs(d, rng):
        SK = Ss @ k                                                    # [T,m]
        SQ = Ss @ q
        est = RT_HALF_PI / m * np.linalg.norm(k) * np.sum(SQ * np.where(SK >= 0, 1.0, -1.0), axis=1)
        # spot-check that this vectorised form is the oracle's prod_qjl
        for t in (0, 17, T - 1):
            assert est[t] == pytest.approx(orc.prod_qjl(q, k, Ss[t]), rel=1e-12, abs=1e-12)
        var = ((math.pi / 2) * (q @ q) * (k @ k) - (q @ k) ** 2) / m
        assert abs(est.mean() - q @ k) <= 4.5 * math.sqrt(var / T)
        assert est.var(ddof=1) == pytest.approx(var, rel=0.05)


def test_tail_bound_lemma_3_5():
    """Lemma 3.5 bounds Pr[|Prod - <q,k>| > eps ||q|| ||k||] with Bernstein's
    inequality from the moments E|z_i|^l it states.  Those moments give
    variance proxy v = m (pi/2) N^2 and scale c = (2/3) N  (N = ||q|| ||k||),
    hence the bound 2 exp(-m eps^2 / (pi + 4 eps / 3)).  The display printed
    in the paper, 2 exp(-(3/4) m eps^2 / (1 + eps)) (its minus sign is also
    lost in print), has 4/3 where the derivation has pi, and is too small:
    for q orthogonal to k the estimator is close to N(0, (pi/2) N^2 / m), so
    at m = 64, eps = 0.5 the exceedance is about 1.4e-3 against a printed
    bound of 6.7e-4.  The test holds the oracle to the derivable bound and
    checks that Gaussian-tail prediction, which is what pins the estimator's
    spread here (together with the exact variance above)."""
    d, m, T = 16, 64, 20000
    rng = np.random.default_rng(77)
    Ss = rng.standard_normal((T, m, d))
    for q, k in _pairs(d, rng):
        est = RT_HALF_PI / m * np.linalg.norm(k) * np.sum(
            (Ss @ q) * np.where(Ss @ k >= 0, 1.0, -1.0), axis=1)
        N = np.linalg.norm(q) * np.linalg.norm(k)
        err = np.abs(est - q @ k) / N
        sd = math.sqrt(((math.pi / 2) - (q @ k / N) ** 2) / m)
        for eps in (0.1, 0.2, 0.3, 0.4, 0.5):
            bound = 2.0 * math.exp(-m * eps * eps / (math.pi + 4.0 * eps / 3.0))
            freq = float(np.mean(err > eps))
            assert freq <= bound
            clt = 2.0 * stats.norm.sf(eps / sd)                        # normal approximation
            assert abs(freq - clt) <= 0.35 * clt + 5.0 * math.sqrt(clt / T) + 2e-4


def test_theorem_3_6_score_distortion():
    """Theorem 3.6: ||q||,||k_j|| <= r and m >= 2 r^2 eps^-2 log n  =>  every
    softmax score is within (1 +- 3 eps) of the exact one (w.h.p.)."""
    rng = np.random.default_rng(5150)
    d, n, r, eps = 16, 64, 1.0, 0.5
    m = int(math.ceil(2 * r * r / eps ** 2 * math.log(n)))            # 34
    m += (-m) % 8
    worst = 0.0
    for trial in range(20):
        K = rng.standard_normal((n, d))
        K /= np.linalg.norm(K, axis=1, keepdims=True)
        q = rng.standard_normal(d)
        q /= np.linalg.norm(q)
        S = rng.standard_normal((m, d))
        bits, nu, _ = orc.quantize_keys(K[None, None], S)
        est = orc.softmax(orc.estimate_scores(orc.project_query(q[None, None], S), bits, nu))[0, 0]
        exact = orc.softmax(K @ q)
        worst = max(worst, float(np.max(np.abs(est - exact) / exact)))
    assert worst <= 3 * eps


# ---------------------------------------------------------------- the sketch generator
def test_splitmix64_published_vector():
    """First five outputs of SplitMix64 seeded with 1234567 (the widely
    published check values of the reference generator)."""
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    assert [int(x) for x in orc.splitmix64_at(1234567, np.arange(5))] == want


def test_sketch_is_standard_normal_and_seeded():
    S = orc.gaussian_sketch(42, 512, 128, "f32")
    assert S.shape == (512, 128)
    x = S.ravel()
    n = x.size
    assert abs(x.mean()) < 4 / math.sqrt(n)
    assert abs(x.var() - 1) < 4 * math.sqrt(2 / n)
    assert stats.kstest(x, "norm").pvalue > 1e-3
    assert abs(stats.kurtosis(x)) < 0.1 and abs(stats.skew(x)) < 0.05
    np.testing.assert_array_equal(S, orc.gaussian_sketch(42, 512, 128, "f32"))
    S2 = orc.gaussian_sketch(43, 512, 128, "f32")
    assert abs(np.corrcoef(x, S2.ravel())[0, 1]) < 4 / math.sqrt(n)
    # rows are uncorrelated: S S^T / d is close to the identity
    gram = S @ S.T / 128
    off = gram - np.diag(np.diag(gram))
    assert np.abs(off).max() < 6 / math.sqrt(128)
    # entry e depends only on (seed, e): a smaller sketch is a prefix
    np.testing.assert_array_equal(orc.gaussian_sketch(42, 4, 128, "f32"), S[:4])


def test_round_to_storage_types():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -9, -3.14159, 65504.0, 1e-3])
    bf = orc.round_to_storage(x, "bf16")
    want = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64)
    np.testing.assert_array_equal(bf, want.numpy())
    assert bf[1] == 1.0 and bf[2] == 1.0 + 2.0 ** -7                   # ties to even
    h = orc.round_to_storage(x, "f16")
    np.testing.assert_array_equal(h, x.astype(np.float32).astype(np.float16).astype(np.float64))
    np.testing.assert_array_equal(orc.round_to_storage(x, "f32"), x.astype(np.float32).astype(np.float64))


def test_memory_claim_arithmetic():
    """Abstract / Section 4: 3 bits per number against 16 is 'around 81%'
    less and 'more than fivefold'; the key code here costs (m + 16)/d bits."""
    assert 1 - 3 / 16 == pytest.approx(0.8125) and 16 / 3 > 5
    assert (256 + 16) / 128 == 2.125
