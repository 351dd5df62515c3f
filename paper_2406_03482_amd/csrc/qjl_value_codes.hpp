// The arithmetic of the token-wise value quantizer (Section 3.2), shared by the
// bulk quantizer and by the generation step that quantizes one new row: given
// eight entries of a row and the row's minimum and maximum, the stored scale and
// zero point (binary16) and the eight codes.
#pragma once

#include "qjl_common.hpp"

namespace qjl {

// scale = (max - min) / (2^b - 1), zero = min, both rounded to binary16; code =
// (x - zero) / scale rounded to nearest (ties to even), clipped to [0, 2^b - 1],
// taken in IEEE float32 against the stored constants.
template <int BITS>
__device__ __forceinline__ void value_codes8(const float (&x)[8], float lo, float hi, uint16_t& s16, uint16_t& z16,
                                             uint32_t (&q8)[8]) {
  constexpr float kLevels = (float)((1 << BITS) - 1);
  s16 = float_to_f16_bits((hi - lo) / kLevels);
  z16 = float_to_f16_bits(lo);
  const float sc = f16_bits_to_float(s16), z = f16_bits_to_float(z16);
#pragma unroll
  for (int e = 0; e < 8; ++e) q8[e] = 0u;
  if (sc > 0.f) {
    // rint((x - z) / sc) without a division per entry: q0 = rint((x - z) * (1/sc)) is accepted when the
    // remainder (x - z) - q0 * sc (one fused multiply-add: exact up to 2^-25 of a step) is clear of half
    // a step by a margin.  Then the true quotient lies within 0.5 - margin of q0, and so does its float32
    // rounding, which is off by at most |quotient| * 2^-24: below 2^-19 for the quotients up to 16.5
    // that can still round to a code below the clip (b <= 4), below 2^-15 up to 256.5 (b = 8).  Entries
    // near a tie take the division itself, so every code is the one the definition gives.
    const float inv = 1.0f / sc;
    const float clear = (0.5f - (BITS == 8 ? 0x1.0p-14f : 0x1.0p-18f)) * sc;
#pragma unroll
    for (int e = 0; e < 8; ++e) {                  // a branch per entry: exact ties are common enough with
      const float t = x[e] - z;                    // 8- to 11-bit inputs that one branch for all eight
      float q = rintf(t * inv);                    // would send most waves through eight divisions
      if (!(fabsf(fmaf(-q, sc, t)) < clear)) q = rintf(t / sc);
      q8[e] = (uint32_t)__builtin_amdgcn_fmed3f(q, 0.f, kLevels);
    }
  }
}

// The same for N entries of a row held by one lane, with the stored constants already formed (sc, z: the
// binary16 scale and zero point as floats).  The estimate of the quotient uses v_rcp_f32: any estimate will do,
// the exact remainder decides whether it is accepted.  (One branch per lane instead of one per entry, the
// flagged lanes redoing their N entries with the division, was slower: 141 against 133 us for 2 M rows --
// with 8-bit mantissas enough entries sit near a tie that most waves then divide sixteen times.)
template <int BITS, int N>
__device__ __forceinline__ void value_codes_n(const float (&x)[N], float sc, float z, uint32_t (&q)[N]) {
  constexpr float kLevels = (float)((1 << BITS) - 1);
#pragma unroll
  for (int e = 0; e < N; ++e) q[e] = 0u;
  if (sc > 0.f) {
    const float inv = __builtin_amdgcn_rcpf(sc);
    const float clear = (0.5f - (BITS == 8 ? 0x1.0p-14f : 0x1.0p-18f)) * sc;
#pragma unroll
    for (int e = 0; e < N; ++e) {
      const float t = x[e] - z;
      float qf = rintf(t * inv);
      if (!(fabsf(fmaf(-qf, sc, t)) < clear)) qf = rintf(t / sc);
      q[e] = (uint32_t)__builtin_amdgcn_fmed3f(qf, 0.f, kLevels);
    }
  }
}

}  // namespace qjl
