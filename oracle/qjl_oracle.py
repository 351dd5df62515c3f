"""CPU oracle for the QJL key-cache hot path.  TEST INFRASTRUCTURE ONLY.

This module is a plain, slow, float64 restatement of what the QJL paper
(arXiv 2406.03482) defines.  It exists so that the GPU library can be checked
against something that is obviously the paper's mathematics.  Nothing in the
product path may import it: only the tests, the smoke check and the
`cpu_baseline` leg of the benchmark do.  It shares no code, table, constant
generator or helper with the HIP library.

Every function names the passage it follows:

  * Definition 3.1, Eq. (3)      H_S(k) = sign(S k)
  * Definition 3.1, Eq. (4)      Prod_QJL(q,k) = sqrt(pi/2)/m * ||k||_2 * <S q, H_S(k)>
  * Algorithm 1, steps 1-4       draw S; per key store sign(S k) and nu = ||k||_2
  * Algorithm 1, EstimateScores  estimator for every cached key, then softmax
  * Section 2, Eq. (1), (2)      o_n = sum_i Score(i) v_i ,  Score = softmax(.)

Readings of points the paper leaves open (all restated where they are used):

  * sign(0) := +1, i.e. bit 1 iff the projection is >= 0 (the codomain of
    H_S is {-1,+1}, so zero needs a side).
  * Packing: projection i of a key lives in byte i//8, bit i%8 (LSB first);
    bit 1 <-> +1.
  * Algorithm 1 prints nu_i inside a formula indexed by j; it is nu_j, the
    norm of the key whose code is being used (as in Eq. (4)).
  * The norm is stored in IEEE binary16 (round-to-nearest-even), and the
    score estimator uses that stored value.
  * Eq. (2) has no 1/sqrt(d); a `scale` factor multiplies the estimator
    before the softmax, and scale = 1 is the paper's literal definition.
  * Grouped-query attention: query head h reads the cache of key/value head
    h // (Hq // Hkv).
  * The sketch S is data: Algorithm 1 step 1 only asks for i.i.d. N(0,1)
    entries.  `gaussian_sketch` fixes one reproducible way to draw them
    (SplitMix64 counter -> Box-Muller in float64 -> rounding to the storage
    type).  Its exact values are pinned by a published SplitMix64 test
    vector, by determinism and by distribution tests only: beyond that the
    *values* of S are "parity unpinned" (any i.i.d. N(0,1) matrix is a valid
    S).  Every other function here is pinned by tests/test_oracle_pins.py.
  * Outlier channels (Section 4.1, "Outliers"; end of Section 1): the paper
    says that the channels are identified in the prompt phase and that two
    independent copies of the quantizer are applied to outliers and inliers,
    the outlier copy with more bits per coordinate; it gives no selection
    rule, no sizes and no layout.  Read here as: per (batch, kv head) the
    `count` channels with the largest mean |k| over the prompt's tokens
    (Figure 2 ranks channels by exactly that), ties to the lower index; the
    inlier copy sees the key with those coordinates set to zero, the outlier
    copy sees only those coordinates (left in place), each with its own
    i.i.d. sketch ([m_in,d] and [m_out,d]) and its own binary16 norm; the
    query is split the same way and the two Eq. (4) estimates are added; a
    cache row is the inlier code followed by the outlier code.  These
    functions are pinned by tests/test_oracle_dual_pins.py.
  * Value cache (Section 3.2): the paper says only "normalizing each token's
    entries and then rounding each entry to a few-bit integer".  Read here as
    the standard asymmetric token-wise scheme: per (batch, kv head, token)
    zero point = the row's minimum, scale = (max - min)/(2^b - 1), both stored
    in binary16; code = round-to-nearest-even of (v - min)/scale clipped to
    [0, 2^b - 1], taken against the *stored* zero point and scale; b = 2, 4 or 8;
    element t of a row occupies bits [b*t, b*t + b) of the row's bytes, LSB
    first; a value is read back as min + code * scale.  The code is an integer
    decided by floating point.  Its definition is `value_codes_exact`: the
    quotient in exact arithmetic (float64 on exactly represented operands),
    rounded half to even; entries whose quotient is within 2^-20 relative of
    a half-integer form the band in which a float32 evaluation may
    legitimately differ.  `quantize_values` is one such evaluation, with the
    three float32 operations written out, kept because an implementation that
    performs the same three operations must then match it bit for bit; it is
    itself held to `value_codes_exact` outside the band.  Everything after
    the code is float64.  Pinned by tests/test_oracle_value_pins.py (exact
    rational arithmetic on small rows, round-trip bound, worked example,
    invariances); the choice of scheme itself is this build's reading.
  * Orthogonalised sketch (Section 4.1, "Orthogonalized JL transform"): the
    paper draws S i.i.d. Gaussian and orthogonalises its rows by QR; with
    m > d not all rows can be orthogonal, and the paper does not say what a
    row's length becomes.  Read here as: rows are taken in blocks of d; inside
    a block row i is replaced by the i-th Gram-Schmidt direction of the
    block's rows (the Q factor of the QR decomposition of the block's
    transpose, signs fixed so that R has a positive diagonal), scaled back to
    the length the Gaussian row had.  Row lengths and directions of a Gaussian
    matrix are independent, so every row is still N(0, I) on its own and
    Lemma 3.2 holds unchanged; only rows of the same block are now orthogonal.
    Pinned by tests/test_oracle_orth_pins.py.
  * Streaming (Algorithm 1's loop over the token stream): a key is quantized
    when it arrives and appended to the cache; the estimator then runs over
    the keys stored so far.  `decode_step` is one iteration in a cache of
    fixed capacity: row `pos` receives the new key's code and norm, attention
    covers rows 0..pos.  Rows are quantized independently, so streaming must
    give exactly what quantizing all keys at once gives
    (tests/test_oracle_stream_pins.py).

  * The paper's operating point (Section 4.1: "in all experiments" the keys get
    the outlier/inlier codes; Section 3.2: the values are quantized token-wise;
    Algorithm 1: both caches grow as the stream arrives): `generation_step` is
    one iteration with all three at once -- the new token's key gets its
    two-part code, its value row its few-bit code, both go to row `pos`, and
    attention over rows 0..pos uses the sum of the two Eq. (4) estimates and
    the values as stored.  It is a composition of the functions above and
    nothing else; pinned by tests/test_oracle_operating_point_pins.py.

Array conventions (all dense, C order):
    K, V  [B, Hkv, n, d]     Q   [B, Hq, d]      S      [m, d]
    bits  [B, Hkv, n, m/8]   nu  [B, Hkv, n]     SQ     [B, Hq, m]
    scores[B, Hq, n]         out [B, Hq, d]
Inputs that were stored in bf16/fp16/fp32 are passed in already converted,
exactly, to float64.
"""
from __future__ import annotations

import math

import numpy as np

SQRT_HALF_PI = math.sqrt(math.pi / 2.0)

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_MIX1 = 0xBF58476D1CE4E5B9
_MIX2 = 0x94D049BB133111EB


# --------------------------------------------------------------------------
# Algorithm 1, step 1: the sketch
# --------------------------------------------------------------------------
def splitmix64_at(seed: int, counter: np.ndarray) -> np.ndarray:
    """The `counter`-th output (0-based) of the SplitMix64 stream started at
    `seed` (Steele, Lea, Flood 2014): state = seed + (counter+1)*golden, then
    the two xor-shift-multiply rounds and a final xor-shift."""
    c = np.asarray(counter, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & _MASK64) + (c + np.uint64(1)) * np.uint64(_GOLDEN)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_MIX1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_MIX2)
        z = z ^ (z >> np.uint64(31))
    return z


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the storage type and return them as float64.
    f32: one RNE rounding.  f16 / bf16: RNE to float32 first, then RNE to the
    16-bit type (the same two steps a float32 pipeline performs)."""
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32)
    if dtype == "f32":
        return x32.astype(np.float64)
    if dtype == "f16":
        return x32.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        u = x32.view(np.uint32).astype(np.uint64)
        lsb = (u >> np.uint64(16)) & np.uint64(1)
        u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
        return u.astype(np.uint32).view(np.float32).astype(np.float64)
    raise ValueError(f"unknown storage dtype {dtype!r}")


def gaussian_sketch(seed: int, m: int, d: int, dtype: str = "f32") -> np.ndarray:
    """Algorithm 1 step 1 / Definition 3.1: S in R^{m x d}, i.i.d. N(0,1).

    Entry e = i*d + j uses SplitMix64 outputs 2e and 2e+1 of the stream
    `seed`:  U1 = ((a >> 11) + 1) / 2^53 in (0,1],  U2 = (b >> 11) / 2^53 in
    [0,1),  z = sqrt(-2 ln U1) * cos(2 pi U2)  (Box-Muller, float64), then
    `round_to_storage`.
    """
    e = np.arange(m * d, dtype=np.uint64)
    a = splitmix64_at(seed, np.uint64(2) * e)
    b = splitmix64_at(seed, np.uint64(2) * e + np.uint64(1))
    u1 = ((a >> np.uint64(11)).astype(np.float64) + 1.0) * 2.0 ** -53
    u2 = (b >> np.uint64(11)).astype(np.float64) * 2.0 ** -53
    z = np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * np.pi * u2)
    return round_to_storage(z, dtype).reshape(m, d)


# --------------------------------------------------------------------------
# Definition 3.1 Eq. (3) and Algorithm 1 steps 3-4: quantize keys
# --------------------------------------------------------------------------
def key_projections(K: np.ndarray, S: np.ndarray) -> np.ndarray:
    """P[..., j, i] = <s_i, k_j> = (S k_j)_i in float64 (Eq. (3) before sign)."""
    K = np.asarray(K, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    return np.einsum("...jt,it->...ji", K, S)


def pack_sign_bits(nonneg: np.ndarray) -> np.ndarray:
    """Pack a boolean array [..., m] (True <-> +1) into uint8 [..., m/8]:
    projection i -> byte i//8, bit i%8."""
    nonneg = np.asarray(nonneg, dtype=bool)
    m = nonneg.shape[-1]
    if m % 8:
        raise ValueError("m must be a multiple of 8")
    grouped = nonneg.reshape(nonneg.shape[:-1] + (m // 8, 8)).astype(np.uint16)
    out = np.zeros(grouped.shape[:-1], dtype=np.uint16)
    for t in range(8):
        out |= grouped[..., t] << t
    return out.astype(np.uint8)


def unpack_signs(bits: np.ndarray, m: int) -> np.ndarray:
    """Inverse of `pack_sign_bits`, returned as float64 values in {-1,+1}."""
    bits = np.asarray(bits, dtype=np.uint8)
    if bits.shape[-1] * 8 != m:
        raise ValueError("bits last dim must be m/8")
    sig = np.empty(bits.shape[:-1] + (m,), dtype=np.float64)
    for t in range(8):
        sig[..., t::8] = ((bits >> t) & 1).astype(np.float64) * 2.0 - 1.0
    return sig


def key_norms(K: np.ndarray) -> np.ndarray:
    """nu_j = ||k_j||_2 (Algorithm 1 step 3) in float64, stored as binary16."""
    K = np.asarray(K, dtype=np.float64)
    return np.sqrt(np.sum(K * K, axis=-1)).astype(np.float16)


def quantize_keys(K: np.ndarray, S: np.ndarray):
    """Algorithm 1 steps 3-4 for every key: returns (bits, nu16, P).

    bits  uint8  [..., n, m/8]   packed H_S(k_j) = sign(S k_j), sign(0) = +1
    nu16  float16[..., n]        stored key norms
    P     float64[..., n, m]     the projections themselves (so a caller can
                                 see how close to zero a sign decision was)
    """
    P = key_projections(K, S)
    return pack_sign_bits(P >= 0.0), key_norms(K), P


# --------------------------------------------------------------------------
# Definition 3.1 Eq. (4) and Algorithm 1 EstimateScores
# --------------------------------------------------------------------------
def project_query(Q: np.ndarray, S: np.ndarray) -> np.ndarray:
    """SQ[b,h,:] = S q  -- the query side of Eq. (4), not quantized."""
    Q = np.asarray(Q, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    return np.einsum("...t,it->...i", Q, S)


def estimate_scores(SQ: np.ndarray, bits: np.ndarray, nu16: np.ndarray,
                    scale: float = 1.0) -> np.ndarray:
    """scale * Prod_QJL(q_h, k_j) for every query head h and cached key j:

        scale * sqrt(pi/2)/m * nu_j * <S q_h, H_S(k_j)>      (Eq. (4))

    SQ [B,Hq,m], bits [B,Hkv,n,m/8], nu16 [B,Hkv,n] -> [B,Hq,n].
    """
    SQ = np.asarray(SQ, dtype=np.float64)
    B, Hq, m = SQ.shape
    Hkv = bits.shape[1]
    if Hq % Hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    G = Hq // Hkv
    sig = unpack_signs(bits, m)                          # [B,Hkv,n,m]
    nu = np.asarray(nu16, dtype=np.float16).astype(np.float64)
    out = np.empty((B, Hq, bits.shape[2]), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            g = h // G
            inner = sig[b, g] @ SQ[b, h]                 # <S q, H_S(k_j)> for all j
            out[b, h] = scale * (SQRT_HALF_PI / m) * nu[b, g] * inner
    return out


def softmax(x: np.ndarray) -> np.ndarray:
    """softmax over the last axis (Eq. (2)), computed with the maximum
    subtracted, which does not change its value."""
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - np.max(x, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_from_scores(scores: np.ndarray, V: np.ndarray) -> np.ndarray:
    """o = sum_j softmax(scores)_j v_j (Eq. (1)); scores [B,Hq,n], V
    [B,Hkv,n,d] -> [B,Hq,d]."""
    V = np.asarray(V, dtype=np.float64)
    B, Hq, _ = scores.shape
    Hkv = V.shape[1]
    G = Hq // Hkv
    p = softmax(scores)
    out = np.empty((B, Hq, V.shape[-1]), dtype=np.float64)
    for b in range(B):
        for h in range(Hq):
            out[b, h] = p[b, h] @ V[b, h // G]
    return out


def decode_attention(Q: np.ndarray, S: np.ndarray, bits: np.ndarray,
                     nu16: np.ndarray, V: np.ndarray,
                     scale: float = 1.0) -> np.ndarray:
    """One decode step on a quantized key cache: project the query, estimate
    all scores (Algorithm 1, EstimateScores), softmax, aggregate values
    (Eq. (1))."""
    SQ = project_query(Q, S)
    return attention_from_scores(estimate_scores(SQ, bits, nu16, scale), V)


def prod_qjl(q: np.ndarray, k: np.ndarray, S: np.ndarray) -> float:
    """Eq. (4) for one pair of vectors, written straight from the definition
    (no packing, float64 norm): used by the statistical tests of Lemma 3.2
    and Lemma 3.5."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    m = S.shape[0]
    h = np.where(S @ k >= 0.0, 1.0, -1.0)
    return SQRT_HALF_PI / m * math.sqrt(float(k @ k)) * float((S @ q) @ h)


# --------------------------------------------------------------------------
# Section 4.1 "Outliers": two independent quantizers for outlier and inlier
# channels.  Everything below is the single-sketch definitions above applied
# to two sub-vectors; only the channel choice and the split are new.
# --------------------------------------------------------------------------
def select_outlier_channels(K: np.ndarray, count: int) -> np.ndarray:
    """For every (batch, kv head): the `count` channels whose mean |k| over the
    n tokens of K [B,Hkv,n,d] is largest, in decreasing order of that mean,
    ties to the lower channel index.  Returns int64 [B,Hkv,count]."""
    K = np.asarray(K, dtype=np.float64)
    B, H, n, d = K.shape
    if not 0 <= count <= d:
        raise ValueError("count must be in [0, d]")
    mean_abs = np.mean(np.abs(K), axis=2)                  # [B,H,d]
    out = np.empty((B, H, count), dtype=np.int64)
    for b in range(B):
        for h in range(H):
            order = sorted(range(d), key=lambda t: (-mean_abs[b, h, t], t))
            out[b, h] = order[:count]
    return out


def split_channels(X: np.ndarray, channels: np.ndarray):
    """X [B,H,...,d] -> (X_in, X_out) with X_in + X_out = X: X_out keeps only the
    coordinates listed in channels[b, h // (H // Hkv)], X_in has them zeroed.
    (H may be the number of query heads: a query head uses the channels of its
    kv head.)"""
    X = np.asarray(X, dtype=np.float64)
    channels = np.asarray(channels, dtype=np.int64)
    B, H = X.shape[:2]
    Hkv = channels.shape[1]
    if H % Hkv:
        raise ValueError("head count must be a multiple of the kv head count")
    G = H // Hkv
    X_out = np.zeros_like(X)
    for b in range(B):
        for h in range(H):
            idx = channels[b, h // G]
            if len(set(idx.tolist())) != len(idx):
                raise ValueError("outlier channels must be distinct")
            X_out[b, h][..., idx] = X[b, h][..., idx]
    return X - X_out, X_out


def quantize_keys_dual(K: np.ndarray, S_in: np.ndarray, S_out: np.ndarray,
                       channels: np.ndarray):
    """Two independent copies of Algorithm 1 steps 3-4, one on the inlier part
    of every key and one on its outlier part.  Returns

        bits    uint8  [B,Hkv,n,(m_in+m_out)/8]   inlier code, then outlier code
        nu_in   float16[B,Hkv,n]   ||k_in||_2     nu_out float16 ||k_out||_2
        P_in, P_out                               the projections (float64)
    """
    K_in, K_out = split_channels(K, channels)
    b_in, nu_in, P_in = quantize_keys(K_in, S_in)
    b_out, nu_out, P_out = quantize_keys(K_out, S_out)
    return np.concatenate([b_in, b_out], axis=-1), nu_in, nu_out, P_in, P_out


def estimate_scores_dual(Q: np.ndarray, S_in: np.ndarray, S_out: np.ndarray,
                         channels: np.ndarray, bits: np.ndarray, nu_in16: np.ndarray,
                         nu_out16: np.ndarray, scale: float = 1.0) -> np.ndarray:
    """scale * (Prod_QJL on the inlier parts + Prod_QJL on the outlier parts)
    for every query head and cached key: Q [B,Hq,d] -> [B,Hq,n]."""
    m_in = np.asarray(S_in).shape[0]
    Q_in, Q_out = split_channels(Q, channels)
    bits = np.asarray(bits, dtype=np.uint8)
    s_in = estimate_scores(project_query(Q_in, S_in), bits[..., : m_in // 8], nu_in16, scale)
    s_out = estimate_scores(project_query(Q_out, S_out), bits[..., m_in // 8:], nu_out16, scale)
    return s_in + s_out


def decode_attention_dual(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, V,
                          scale: float = 1.0) -> np.ndarray:
    """One decode step on a cache quantized by `quantize_keys_dual`."""
    return attention_from_scores(
        estimate_scores_dual(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, scale), V)


# --------------------------------------------------------------------------
# Section 3.2: token-wise quantization of the value cache
# --------------------------------------------------------------------------
def quantize_values(V: np.ndarray, vbits: int = 4):
    """V [B,Hkv,n,d] (already exact in float32) -> (codes uint8 [B,Hkv,n,d*vbits/8],
    scale float16 [B,Hkv,n], zero float16 [B,Hkv,n]).

    Per row, in float32 (the precision in which the code is decided):
        lo, hi   = min, max of the row
        scale16  = binary16( (hi - lo) / (2^b - 1) )        zero16 = binary16(lo)
        code_t   = clip( rint( (v_t - zero16) / scale16 ), 0, 2^b - 1 )   (0 if scale16 == 0)
    """
    if vbits not in (2, 4, 8):
        raise ValueError("vbits must be 2, 4 or 8")
    V32 = np.asarray(V, dtype=np.float32)
    if not np.array_equal(V32.astype(np.float64), np.asarray(V, dtype=np.float64)):
        raise ValueError("values must be exactly representable in float32")
    levels = np.float32((1 << vbits) - 1)
    lo = V32.min(axis=-1)
    hi = V32.max(axis=-1)
    scale16 = ((hi - lo) / levels).astype(np.float16)
    zero16 = lo.astype(np.float16)
    sc = scale16.astype(np.float32)[..., None]
    z = zero16.astype(np.float32)[..., None]
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint((V32 - z) / sc)                       # float32 subtract, divide, round-half-even
    q = np.where(sc > 0, np.clip(q, np.float32(0), levels), np.float32(0)).astype(np.uint8)
    per = 8 // vbits                                      # elements per byte
    d = q.shape[-1]
    if d % per:
        raise ValueError("d * vbits must be a multiple of 8")
    grouped = q.reshape(q.shape[:-1] + (d // per, per)).astype(np.uint16)
    packed = np.zeros(grouped.shape[:-1], dtype=np.uint16)
    for t in range(per):
        packed |= grouped[..., t] << (vbits * t)
    return packed.astype(np.uint8), scale16, zero16


def value_codes_exact(V: np.ndarray, scale16: np.ndarray, zero16: np.ndarray, vbits: int = 4):
    """Section 3.2's rounding step with no float32 in it: against stored constants scale16 / zero16 [B,Hkv,n], the
    code of entry t is  clip( round_half_even( (v_t - zero) / scale ), 0, 2^b - 1 )  with the quotient formed in
    float64 from exactly represented operands (its error, 2^-52 relative, is far below anything float32 can
    resolve).  Returns (codes_per_entry uint8 [B,Hkv,n,d], near_tie bool [B,Hkv,n,d]): near_tie marks the entries
    whose quotient lies within 2^-20 * max(1, quotient) of a half-integer -- there, and only there, an evaluation
    of the same three operations in float32 (subtract 2^-24, divide 2^-24 relative) may round to the neighbouring
    code.  This is the definition that `quantize_values` (which fixes float32) is held to outside that band."""
    if vbits not in (2, 4, 8):
        raise ValueError("vbits must be 2, 4 or 8")
    V = np.asarray(V, dtype=np.float64)
    sc = np.asarray(scale16, dtype=np.float16).astype(np.float64)[..., None]
    z = np.asarray(zero16, dtype=np.float16).astype(np.float64)[..., None]
    levels = float((1 << vbits) - 1)
    with np.errstate(divide="ignore", invalid="ignore"):
        q = (V - z) / sc
    q = np.where(sc > 0, q, 0.0)
    codes = np.clip(np.rint(q), 0.0, levels).astype(np.uint8)
    frac = np.abs(q - np.floor(q) - 0.5)
    inside = (q > -0.5 - 1e-3) & (q < levels + 0.5 + 1e-3)          # ties beyond the clip change nothing
    near_tie = (frac <= 2.0 ** -20 * np.maximum(1.0, np.abs(q))) & inside & (sc > 0)
    return codes, near_tie


def value_constants_exact(V: np.ndarray, vbits: int = 4):
    """The stored constants of a row from float64 arithmetic: zero16 = binary16(min), scale16 =
    binary16((max - min) / (2^b - 1)), and `near_tie` [B,Hkv,n]: rows whose exact scale lies within 2^-21 relative of
    the midpoint of two neighbouring binary16 numbers, where forming it in float32 first (two roundings of 2^-24)
    may land on the neighbour."""
    V = np.asarray(V, dtype=np.float64)
    levels = float((1 << vbits) - 1)
    lo, hi = V.min(axis=-1), V.max(axis=-1)
    exact = (hi - lo) / levels
    scale16 = exact.astype(np.float16)
    zero16 = lo.astype(np.float16)
    s = scale16.astype(np.float64)
    up = np.nextafter(scale16, np.float16(np.inf)).astype(np.float64)
    dn = np.nextafter(scale16, np.float16(-np.inf)).astype(np.float64)
    with np.errstate(invalid="ignore"):
        d_mid = np.minimum(np.abs(exact - 0.5 * (s + up)), np.abs(exact - 0.5 * (s + dn)))
    near_tie = d_mid <= 2.0 ** -21 * np.abs(exact)
    return scale16, zero16, near_tie


def unpack_value_codes(codes: np.ndarray, vbits: int = 4) -> np.ndarray:
    """Packed code bytes [..., d*vbits/8] -> one code per entry, uint8 [..., d] (element t in bits
    [vbits*t, vbits*t + vbits) of the row, LSB first)."""
    codes = np.asarray(codes, dtype=np.uint8)
    per = 8 // vbits
    mask = (1 << vbits) - 1
    out = np.empty(codes.shape[:-1] + (codes.shape[-1] * per,), dtype=np.uint8)
    for t in range(per):
        out[..., t::per] = (codes >> (vbits * t)) & mask
    return out


def dequantize_values(codes: np.ndarray, scale16: np.ndarray, zero16: np.ndarray, vbits: int = 4) -> np.ndarray:
    """Values as the cache represents them: zero + code * scale, float64 [B,Hkv,n,d]."""
    codes = np.asarray(codes, dtype=np.uint8)
    per = 8 // vbits
    mask = (1 << vbits) - 1
    q = np.empty(codes.shape[:-1] + (codes.shape[-1] * per,), dtype=np.float64)
    for t in range(per):
        q[..., t::per] = ((codes >> (vbits * t)) & mask).astype(np.float64)
    sc = np.asarray(scale16, dtype=np.float16).astype(np.float64)[..., None]
    z = np.asarray(zero16, dtype=np.float16).astype(np.float64)[..., None]
    return z + q * sc


def decode_attention_vq(Q, S, bits, nu16, vcodes, vscale16, vzero16, vbits: int = 4,
                        scale: float = 1.0) -> np.ndarray:
    """One decode step with both caches quantized: Algorithm 1's scores from the
    key code, softmax, and Eq. (1) on the values as stored (Section 3.2)."""
    SQ = project_query(Q, S)
    return attention_from_scores(estimate_scores(SQ, bits, nu16, scale),
                                 dequantize_values(vcodes, vscale16, vzero16, vbits))


# --------------------------------------------------------------------------
# Section 4.1: orthogonalised rows
# --------------------------------------------------------------------------
def orthogonal_sketch(seed: int, m: int, d: int, dtype: str = "f32") -> np.ndarray:
    """The Gaussian sketch of `gaussian_sketch(seed, m, d, "f32")` with the rows of
    every block of d rows orthogonalised (QR) and rescaled to their original
    lengths; float64 arithmetic, then rounded to the storage type ("f64": not
    rounded at all)."""
    G = gaussian_sketch(seed, m, d, "f32")
    S = np.empty_like(G)
    for r0 in range(0, m, d):
        Gb = G[r0:r0 + d]                                   # [r, d], r <= d
        Qt, R = np.linalg.qr(Gb.T)                          # Gb^T = Qt R ; columns of Qt: orthonormalised rows of Gb, in order
        Qt = Qt * np.sign(np.diag(R))[None, :]              # Gram-Schmidt's choice of sign: R_ii > 0
        S[r0:r0 + d] = np.linalg.norm(Gb, axis=1)[:, None] * Qt.T
    return S if dtype == "f64" else round_to_storage(S, dtype)


# --------------------------------------------------------------------------
# Algorithm 1 as a stream: append one key, then estimate over the keys so far
# --------------------------------------------------------------------------
def append_keys(bits: np.ndarray, nu16: np.ndarray, K_new: np.ndarray, S: np.ndarray, pos: int):
    """Algorithm 1 steps 3-4 for the tokens K_new [B,Hkv,t,d] arriving at positions pos..pos+t-1 of caches
    bits [B,Hkv,cap,m/8], nu16 [B,Hkv,cap] (modified in place and returned)."""
    t = K_new.shape[2]
    if pos < 0 or pos + t > bits.shape[2]:
        raise ValueError("append outside the cache")
    b_new, nu_new, _ = quantize_keys(K_new, S)
    bits[:, :, pos:pos + t] = b_new
    nu16[:, :, pos:pos + t] = nu_new
    return bits, nu16


def decode_step(Q, S, bits, nu16, V, K_new, pos: int, scale: float = 1.0) -> np.ndarray:
    """One generation step: the new token's key K_new [B,Hkv,1,d] is quantized into row `pos` of the caches, then
    attention runs over rows 0..pos (V must already hold the new token's value in row pos)."""
    append_keys(bits, nu16, K_new, S, pos)
    return decode_attention(Q, S, bits[:, :, :pos + 1], nu16[:, :, :pos + 1], np.asarray(V)[:, :, :pos + 1], scale)


# --------------------------------------------------------------------------
# The paper's operating point: two-part key codes (Section 4.1), few-bit
# values (Section 3.2) and a cache that grows with the stream (Algorithm 1)
# --------------------------------------------------------------------------
def decode_attention_dual_vq(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, vcodes, vscale16, vzero16,
                             vbits: int = 4, scale: float = 1.0) -> np.ndarray:
    """One decode step on a cache with two-part key codes and quantized values: the sum of the two Eq. (4)
    estimates (Section 4.1), softmax, and Eq. (1) on the values as stored (Section 3.2)."""
    scores = estimate_scores_dual(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, scale)
    return attention_from_scores(scores, dequantize_values(vcodes, vscale16, vzero16, vbits))


def append_token(bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, K_new, V_new, S_in, S_out, channels,
                 pos: int, vbits: int = 4):
    """Algorithm 1's loop body without the estimate: the token arriving at position `pos` (K_new, V_new
    [B,Hkv,1,d]) is quantized -- the key by the two quantizers of Section 4.1, the value row token-wise as in
    Section 3.2 -- and written to row `pos` of the six cache arrays (modified in place)."""
    if K_new.shape[2] != 1 or V_new.shape[2] != 1:
        raise ValueError("one token per step")
    if pos < 0 or pos >= bits.shape[2]:
        raise ValueError("append outside the cache")
    b_new, in_new, out_new, _, _ = quantize_keys_dual(K_new, S_in, S_out, channels)
    c_new, s_new, z_new = quantize_values(V_new, vbits)
    bits[:, :, pos] = b_new[:, :, 0]
    nu_in16[:, :, pos] = in_new[:, :, 0]
    nu_out16[:, :, pos] = out_new[:, :, 0]
    vcodes[:, :, pos] = c_new[:, :, 0]
    vscale16[:, :, pos] = s_new[:, :, 0]
    vzero16[:, :, pos] = z_new[:, :, 0]


def generation_step(Q, S_in, S_out, channels, bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, K_new, V_new,
                    pos: int, vbits: int = 4, scale: float = 1.0) -> np.ndarray:
    """One generation step at the paper's operating point: append the new token (key and value) at row `pos`,
    then attend over rows 0..pos of the caches of capacity bits.shape[2]."""
    append_token(bits, nu_in16, nu_out16, vcodes, vscale16, vzero16, K_new, V_new, S_in, S_out, channels, pos, vbits)
    e = pos + 1
    return decode_attention_dual_vq(Q, S_in, S_out, channels, bits[:, :, :e], nu_in16[:, :, :e], nu_out16[:, :, :e],
                                    vcodes[:, :, :e], vscale16[:, :, :e], vzero16[:, :, :e], vbits, scale)
