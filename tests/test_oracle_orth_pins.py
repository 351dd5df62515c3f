"""Pins for the oracle's orthogonalised sketch (Section 4.1): an independent Gram-Schmidt in plain loops,
structural identities, and the statistics the construction promises.  CPU only."""
import math

import numpy as np
import pytest

from oracle import qjl_oracle as orc


def _gram_schmidt_loops(G):
    """Modified Gram-Schmidt on the rows of G, one block, plain Python loops on float64."""
    r, d = G.shape
    Q = []
    for i in range(r):
        v = [float(x) for x in G[i]]
        for q in Q:
            c = sum(a * b for a, b in zip(q, v))
            v = [a - c * b for a, b in zip(v, q)]
        nrm = math.sqrt(sum(a * a for a in v))
        Q.append([a / nrm for a in v])
    out = np.array(Q)
    return out * np.linalg.norm(G, axis=1)[:, None]


@pytest.mark.parametrize("m,d", [(8, 8), (5, 8), (20, 8), (16, 16), (40, 12)])
def test_matches_gram_schmidt_written_out(m, d):
    S = orc.orthogonal_sketch(7, m, d, "f64")
    G = orc.gaussian_sketch(7, m, d, "f32")
    for r0 in range(0, m, d):
        want = _gram_schmidt_loops(G[r0:r0 + d])
        assert np.allclose(S[r0:r0 + d], want, rtol=0, atol=1e-11)


def test_structure():
    m, d = 3 * 32 + 7, 32
    S = orc.orthogonal_sketch(11, m, d, "f64")
    G = orc.gaussian_sketch(11, m, d, "f32")
    assert np.allclose(np.linalg.norm(S, axis=1), np.linalg.norm(G, axis=1), rtol=1e-13)      # lengths kept
    for r0 in range(0, m, d):
        Sb, Gb = S[r0:r0 + d], G[r0:r0 + d]
        gram = Sb @ Sb.T
        off = gram - np.diag(np.diag(gram))
        assert np.max(np.abs(off)) <= 1e-10                                                   # orthogonal inside a block
        assert np.allclose(Sb[0], Gb[0], rtol=1e-13)                                          # first row untouched
        for i in (1, len(Sb) // 2, len(Sb) - 1):                                              # row i stays in span(g_0..g_i), on g_i's side
            coef, res, _, _ = np.linalg.lstsq(Gb[: i + 1].T, Sb[i], rcond=None)
            assert np.allclose(Gb[: i + 1].T @ coef, Sb[i], atol=1e-9) and coef[-1] > 0
    # rows of different blocks are not orthogonalised against each other
    assert abs(S[0] @ S[d]) > 1e-3
    # determinism and dependence on the seed; storage rounding is the generator's
    assert np.array_equal(S, orc.orthogonal_sketch(11, m, d, "f64"))
    assert not np.allclose(S, orc.orthogonal_sketch(12, m, d, "f64"))
    assert np.array_equal(orc.orthogonal_sketch(11, m, d, "bf16"), orc.round_to_storage(S, "bf16"))


def test_rows_keep_gaussian_marginals_and_the_estimator_its_mean_with_less_variance():
    d, m, T = 16, 16, 3000
    rng = np.random.default_rng(3)
    k = rng.standard_normal(d)
    q = 0.6 * k / np.linalg.norm(k) * np.linalg.norm(k) + 0.8 * rng.standard_normal(d)
    ortho = np.empty(T); iid = np.empty(T)
    ent = []
    for t in range(T):
        So = orc.orthogonal_sketch(1000 + t, m, d, "f64")
        ortho[t] = orc.prod_qjl(q, k, So)
        iid[t] = orc.prod_qjl(q, k, orc.gaussian_sketch(1000 + t, m, d, "f32"))
        ent.append(So[3, 5])
    v_iid = ((math.pi / 2) * (q @ q) * (k @ k) - (q @ k) ** 2) / m
    assert abs(iid.mean() - q @ k) <= 4 * math.sqrt(v_iid / T)
    assert abs(ortho.mean() - q @ k) <= 4 * math.sqrt(v_iid / T)              # still unbiased (Lemma 3.2 needs only the marginals)
    assert abs(iid.var() / v_iid - 1) < 0.1
    assert ortho.var() < 0.9 * iid.var()                                      # and less noisy
    ent = np.array(ent)
    assert abs(ent.mean()) < 4 / math.sqrt(T) and abs(ent.var() - 1) < 0.1    # an entry of a later row is still N(0,1)


# ---- planted mistakes
_orig = orc.orthogonal_sketch


def _no_sign_fix(seed, m, d, dtype="f32"):
    G = orc.gaussian_sketch(seed, m, d, "f32")
    S = np.empty_like(G)
    for r0 in range(0, m, d):
        Gb = G[r0:r0 + d]
        Qt, _ = np.linalg.qr(Gb.T)
        S[r0:r0 + d] = np.linalg.norm(Gb, axis=1)[:, None] * Qt.T
    return S if dtype == "f64" else orc.round_to_storage(S, dtype)


def _unit_rows(seed, m, d, dtype="f32"):
    S = _orig(seed, m, d, "f64")
    S = S / np.linalg.norm(S, axis=1, keepdims=True) * math.sqrt(d)
    return S if dtype == "f64" else orc.round_to_storage(S, dtype)


def _columns_instead_of_rows(seed, m, d, dtype="f32"):
    G = orc.gaussian_sketch(seed, m, d, "f32")
    S = np.empty_like(G)
    for r0 in range(0, m, d):
        Gb = G[r0:r0 + d]
        Q, R = np.linalg.qr(Gb)
        S[r0:r0 + d] = (Q * np.sign(np.diag(R))[None, :]) * np.linalg.norm(Gb, axis=1)[:, None] if Q.shape == Gb.shape else Gb
    return S if dtype == "f64" else orc.round_to_storage(S, dtype)


def _whole_matrix_at_once(seed, m, d, dtype="f32"):
    return _orig(seed, min(m, d), d, dtype) if m <= d else np.concatenate(
        [_orig(seed, d, d, dtype), orc.gaussian_sketch(seed, m, d, "f32")[d:] if dtype == "f64" else
         orc.round_to_storage(orc.gaussian_sketch(seed, m, d, "f32")[d:], dtype)])


PINS = [lambda: test_matches_gram_schmidt_written_out(20, 8), lambda: test_matches_gram_schmidt_written_out(16, 16), test_structure]
MUTATIONS = [("orthogonal_sketch", _no_sign_fix, "signs left as the QR routine returns them"),
             ("orthogonal_sketch", _unit_rows, "rows rescaled to a common length"),
             ("orthogonal_sketch", _columns_instead_of_rows, "columns orthogonalised instead of rows"),
             ("orthogonal_sketch", _whole_matrix_at_once, "only the first block orthogonalised")]


@pytest.mark.parametrize("name,replacement,what", MUTATIONS, ids=[m[2] for m in MUTATIONS])
def test_planted_mistake_in_orthogonal_sketch_is_caught(monkeypatch, name, replacement, what):
    monkeypatch.setattr(orc, name, replacement)
    failed = 0
    for pin in PINS:
        try:
            pin()
        except (AssertionError, ValueError, IndexError):
            failed += 1
    assert failed >= 1, f"no pin noticed: {what}"
