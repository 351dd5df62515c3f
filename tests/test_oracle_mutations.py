"""The pins must bite: each plausible mistake planted in the oracle (on the CPU,
by patching one of its functions for the duration of a test) has to make at
least one pin test fail.  This guards the oracle's guardians -- a pin that
still passes with a transposed operand or a wrong bit order pins nothing.
"""
import math

import numpy as np
import pytest

from oracle import qjl_oracle as orc
import tests.test_oracle_pins as pins


def _golden_dir():
    import os
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


# pin tests cheap enough to re-run per mutation (name -> callable)
def _run_pins():
    g = _golden_dir()
    checks = [
        lambda: pins.test_worked_example_bits_norms_scores(g),
        lambda: pins.test_worked_example_attention(g),
        pins.test_bruteforce_tiny_python_loops,
        pins.test_pack_is_little_endian_bit_order,
        pins.test_identity_sketch_reduces_to_sign_of_key,
        pins.test_self_product_is_l1_norm_of_projection,
        pins.test_proof_decomposition_matches_estimator,
        pins.test_packed_path_equals_definition_path,
        pins.test_norms_match_numpy_and_fp16_rne,
        pins.test_project_query_is_matrix_vector_product,
        pins.test_softmax_and_value_aggregation_match_torch_float64,
        pins.test_gqa_head_mapping_is_contiguous_groups,
        pins.test_invariants_scaling_negation_linearity_permutation,
        pins.test_attention_degenerate_cases,
        pins.test_splitmix64_published_vector,
        pins.test_round_to_storage_types,
    ]
    failed = 0
    for c in checks:
        try:
            c()
        except (AssertionError, ValueError, IndexError, FloatingPointError):
            failed += 1
    return failed


def test_unmutated_oracle_passes_all_pins():
    assert _run_pins() == 0


def _msb_first_pack(nonneg):
    nonneg = np.asarray(nonneg, dtype=bool)
    return np.packbits(nonneg, axis=-1, bitorder="big")


def _sign_zero_negative(K, S):
    P = orc.key_projections(K, S)
    return orc.pack_sign_bits(P > 0.0), orc.key_norms(K), P


def _norm_not_rounded(K):
    K = np.asarray(K, dtype=np.float64)
    return np.sqrt(np.sum(K * K, axis=-1))          # float64, never stored as binary16


def _norm_l1(K):
    return np.sum(np.abs(np.asarray(K, dtype=np.float64)), axis=-1).astype(np.float16)


def _project_transposed(Q, S):
    Q = np.asarray(Q, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    if S.shape[0] == S.shape[1]:
        return np.einsum("...t,ti->...i", Q, S)     # S^T q
    raise ValueError("shape mismatch")               # non-square: a transposed product cannot even run


def _scores_without_constant(SQ, bits, nu16, scale=1.0):
    return orc_estimate(SQ, bits, nu16, scale) / orc.SQRT_HALF_PI


def _scores_divide_by_d(SQ, bits, nu16, scale=1.0):
    m = SQ.shape[-1]
    return orc_estimate(SQ, bits, nu16, scale) * m / (m + 1)


def _scores_wrong_gqa(SQ, bits, nu16, scale=1.0):
    Hq, Hkv = SQ.shape[1], bits.shape[1]
    if Hq == Hkv:
        return orc_estimate(SQ, bits, nu16, scale)
    perm = [(h % Hkv) * (Hq // Hkv) + h // Hkv for h in range(Hq)]   # interleaved instead of contiguous
    return orc_estimate(SQ[:, perm], bits, nu16, scale)


def _softmax_no_normalisation(x):
    x = np.asarray(x, dtype=np.float64)
    return np.exp(x - np.max(x, axis=-1, keepdims=True))


def _softmax_base2(x):
    x = np.asarray(x, dtype=np.float64)
    e = np.exp2(x - np.max(x, axis=-1, keepdims=True))
    return e / e.sum(-1, keepdims=True)


def _unpack_inverted(bits, m):
    return -orc_unpack(bits, m)


def _splitmix_wrong_shift(seed, counter):
    c = np.asarray(counter, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & ((1 << 64) - 1)) + (c + np.uint64(1)) * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(31))) * np.uint64(0xBF58476D1CE4E5B9)     # 31 instead of 30
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _bf16_truncate(x, dtype):
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "bf16":
        u = x32.view(np.uint32) & np.uint32(0xFFFF0000)                     # truncation, not RNE
        return u.view(np.float32).astype(np.float64)
    return orc_round(x, dtype)


orc_estimate = orc.estimate_scores
orc_unpack = orc.unpack_signs
orc_round = orc.round_to_storage

MUTATIONS = [
    ("pack_sign_bits", _msb_first_pack, "MSB-first bit order"),
    ("quantize_keys", _sign_zero_negative, "sign(0) taken as -1"),
    ("key_norms", _norm_not_rounded, "norm kept in float64 instead of binary16"),
    ("key_norms", _norm_l1, "L1 norm instead of L2"),
    ("project_query", _project_transposed, "S transposed on the query side"),
    ("estimate_scores", _scores_without_constant, "sqrt(pi/2) dropped"),
    ("estimate_scores", _scores_divide_by_d, "wrong 1/m normalisation"),
    ("estimate_scores", _scores_wrong_gqa, "interleaved GQA head mapping"),
    ("softmax", _softmax_no_normalisation, "softmax not normalised"),
    ("softmax", _softmax_base2, "softmax in base 2"),
    ("unpack_signs", _unpack_inverted, "bit 1 read as -1"),
    ("splitmix64_at", _splitmix_wrong_shift, "wrong SplitMix64 shift"),
    ("round_to_storage", _bf16_truncate, "bf16 by truncation"),
]


@pytest.mark.parametrize("name,replacement,what", MUTATIONS, ids=[m[2] for m in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, name, replacement, what):
    monkeypatch.setattr(orc, name, replacement)
    assert _run_pins() >= 1, f"no pin noticed: {what}"
