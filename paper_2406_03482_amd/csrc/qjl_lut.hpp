// Byte-indexed partial-sum tables for <S q, sign bits> (Definition 3.1 Eq. (4)).
//
// For byte position p of a key's code and byte value b,
//     T[p][b] = sum_{t<8} (bit t of b ? +1 : -1) * (S q)[8p + t],
// so the inner product with one key is the sum of m/8 table entries selected
// by the key's code bytes.  Tables for GT query heads that share a KV head are
// interleaved (GT consecutive floats per entry) so one LDS read serves all.
// The tables are built in two stages from 4-bit tables so that each entry
// costs one add.
#pragma once

#include "qjl_common.hpp"

namespace qjl {

// GT floats as one value.  Clang vector types (not HIP's float2/float4 structs):
// arithmetic on the whole vector keeps an LDS access one ds_read_b64/b128; with
// per-component use the backend would split it into GT 32-bit reads.
template <int GT> struct vecf { typedef float type __attribute__((ext_vector_type(GT))); };
template <> struct vecf<1> { using type = float; };

template <int GT> __device__ __forceinline__ float vget(const typename vecf<GT>::type& v, int g) {
  if constexpr (GT == 1) return v; else return v[g];
}
template <int GT> __device__ __forceinline__ void vset(typename vecf<GT>::type& v, int g, float x) {
  if constexpr (GT == 1) v = x; else v[g] = x;
}

// LDS floats needed: sq GT*m, 4-bit tables 4*m*GT, byte tables 32*m*GT.
template <int GT> __host__ __device__ constexpr size_t lut_lds_floats(int m) {
  return (size_t)GT * m * (1 + 4 + 32);
}

// sq: [GT][m] in LDS (already filled, visible to all threads).
// nib: [(m/4)][16][GT], lut: [(m/8)][256][GT].  Ends with a barrier.
template <int GT>
__device__ __forceinline__ void build_lut(const float* sq, float* nib, float* lut, int m, int tid,
                                          int nthreads) {
  const int n_nib = (m >> 2) << 4;
  for (int e = tid; e < n_nib; e += nthreads) {
    const int q = e >> 4, x = e & 15;
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      const float* s = sq + g * m + 4 * q;
      float v0 = (x & 1) ? s[0] : -s[0];
      float v1 = (x & 2) ? s[1] : -s[1];
      float v2 = (x & 4) ? s[2] : -s[2];
      float v3 = (x & 8) ? s[3] : -s[3];
      nib[e * GT + g] = (v0 + v1) + (v2 + v3);
    }
  }
  __syncthreads();
  using V = typename vecf<GT>::type;
  const V* nibv = reinterpret_cast<const V*>(nib);
  V* lutv = reinterpret_cast<V*>(lut);
  const int n_byte = (m >> 3) << 8;
  if constexpr (GT == 1) {
    // four consecutive byte values share the high nibble: one 16-byte read of the
    // low table, one broadcast read of the high table, one 16-byte write
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4* nib4 = reinterpret_cast<const f4*>(nib);
    f4* lut4 = reinterpret_cast<f4*>(lut);
    for (int e4 = tid; e4 < (n_byte >> 2); e4 += nthreads) {
      const int p = e4 >> 6, b0 = (e4 & 63) << 2;
      lut4[e4] = nib4[(2 * p) * 4 + ((b0 & 15) >> 2)] + nib[(2 * p + 1) * 16 + (b0 >> 4)];
    }
  } else {
    for (int e = tid; e < n_byte; e += nthreads) {
      const int p = e >> 8, b = e & 255;
      lutv[e] = nibv[(2 * p) * 16 + (b & 15)] + nibv[(2 * p + 1) * 16 + (b >> 4)];
    }
  }
  __syncthreads();
}

// <S q_g, signs of one key> for g < GT, from the key's MW code words.
// Words [W0, W1) of the code only (W0 = 0, W1 = MW: the whole code).
template <int GT, int MW, int W0 = 0, int W1 = MW>
__device__ __forceinline__ typename vecf<GT>::type key_inner(const uint32_t (&w)[MW], const float* lut) {
  using V = typename vecf<GT>::type;
  const V* lutv = reinterpret_cast<const V*>(lut);
  V a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;         // four chains: adds do not wait on each other
#pragma unroll
  for (int wi = W0; wi < W1; ++wi) {
    a0 += lutv[(wi * 4 + 0) * 256 + (w[wi] & 255u)];
    a1 += lutv[(wi * 4 + 1) * 256 + ((w[wi] >> 8) & 255u)];
    a2 += lutv[(wi * 4 + 2) * 256 + ((w[wi] >> 16) & 255u)];
    a3 += lutv[(wi * 4 + 3) * 256 + (w[wi] >> 24)];
  }
  return (a0 + a1) + (a2 + a3);
}

// Load the MW code words of one key (row `row` of bits[*, MW*4 bytes]).
template <int MW>
__device__ __forceinline__ void load_code(const uint8_t* __restrict__ bits, size_t row,
                                          uint32_t (&w)[MW]) {
  const uint4* p = reinterpret_cast<const uint4*>(bits + row * (size_t)(MW * 4));
#pragma unroll
  for (int i = 0; i < MW / 4; ++i) {
    uint4 r = p[i];
    w[4 * i + 0] = r.x; w[4 * i + 1] = r.y; w[4 * i + 2] = r.z; w[4 * i + 3] = r.w;
  }
}

}  // namespace qjl
