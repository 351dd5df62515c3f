// Value cache quantization (Section 3.2): every token's row of V is normalised
// and rounded to a few-bit integer.  Scheme: zero point = the row's minimum,
// scale = (max - min) / (2^b - 1), both stored as binary16; the code of an
// entry is (v - zero) / scale rounded to the nearest integer (ties to even) and
// clipped to [0, 2^b - 1], taken against the stored zero point and scale, so
// that zero + code * scale is the nearest representable value.  b = 2, 4 or 8;
// the first entry's code sits in the lowest bits of a byte.
//
// The code is an integer decided by floating point: subtract, divide and round
// are IEEE float32 operations in exactly this order (the kernel takes a shortcut
// only where it provably gives the same integer).
#include "qjl_common.hpp"
#include "qjl_value_codes.hpp"

namespace qjl {
namespace {

// d == 128: eight lanes share a row (16 entries each, two 16-byte loads); minimum and maximum by three DPP
// steps; the row's constants (one division, four conversions) are formed once per 16 entries; a lane packs its
// sixteen b-bit codes into 2 b bytes, so a row's 16 b code bytes leave as one contiguous piece.
template <typename T, int BITS>
__global__ void __launch_bounds__(256)
value_quant_kernel(const void* __restrict__ V, uint8_t* __restrict__ codes,
                   uint16_t* __restrict__ vscale, uint16_t* __restrict__ vzero, long rows) {
  constexpr float kLevels = (float)((1 << BITS) - 1);
  const int c = threadIdx.x & 7, r = threadIdx.x >> 3;
  for (long row0 = (long)blockIdx.x * 32; row0 < rows; row0 += (long)gridDim.x * 32) {
    const long row = min(row0 + r, rows - 1);          // rows past the end are computed on the last row and not stored
    float x[16];
    {
      float lo8[8], hi8[8];
      load8<T>(V, (size_t)row * 128 + c * 16, lo8);
      load8<T>(V, (size_t)row * 128 + c * 16 + 8, hi8);
#pragma unroll
      for (int e = 0; e < 8; ++e) { x[e] = lo8[e]; x[8 + e] = hi8[e]; }
    }
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) { lo = fminf(lo, x[e]); hi = fmaxf(hi, x[e]); }
    lo = fminf(lo, QJL_DPP_F(lo, 0xB1)); hi = fmaxf(hi, QJL_DPP_F(hi, 0xB1));      // quad_perm [1,0,3,2]
    lo = fminf(lo, QJL_DPP_F(lo, 0x4E)); hi = fmaxf(hi, QJL_DPP_F(hi, 0x4E));      // quad_perm [2,3,0,1]
    lo = fminf(lo, QJL_DPP_F(lo, 0x141)); hi = fmaxf(hi, QJL_DPP_F(hi, 0x141));    // row_half_mirror: the other quad of the eight
    const uint16_t s16 = float_to_f16_bits((hi - lo) / kLevels);
    const uint16_t z16 = float_to_f16_bits(lo);
    uint32_t q[16];
    value_codes_n<BITS, 16>(x, f16_bits_to_float(s16), f16_bits_to_float(z16), q);
    if (row0 + r < rows) {
      uint8_t* dst = codes + (size_t)row * (16 * BITS) + c * (2 * BITS);
      if constexpr (BITS == 8) {
        uint4 w;
        w.x = q[0] | (q[1] << 8) | (q[2] << 16) | (q[3] << 24);
        w.y = q[4] | (q[5] << 8) | (q[6] << 16) | (q[7] << 24);
        w.z = q[8] | (q[9] << 8) | (q[10] << 16) | (q[11] << 24);
        w.w = q[12] | (q[13] << 8) | (q[14] << 16) | (q[15] << 24);
        *reinterpret_cast<uint4*>(dst) = w;
      } else if constexpr (BITS == 4) {
        uint2 w = make_uint2(0u, 0u);
#pragma unroll
        for (int e = 0; e < 8; ++e) { w.x |= q[e] << (4 * e); w.y |= q[8 + e] << (4 * e); }
        *reinterpret_cast<uint2*>(dst) = w;
      } else {
        uint32_t w = 0;
#pragma unroll
        for (int e = 0; e < 16; ++e) w |= q[e] << (2 * e);
        *reinterpret_cast<uint32_t*>(dst) = w;
      }
      if (c == 0) { vscale[row] = s16; vzero[row] = z16; }
    }
  }
}

template <typename T>
void launch_bits(int vbits, unsigned blocks, hipStream_t st, const void* V, uint8_t* codes, uint16_t* vscale,
                 uint16_t* vzero, long rows) {
  if (vbits == 2) hipLaunchKernelGGL((value_quant_kernel<T, 2>), dim3(blocks), dim3(256), 0, st, V, codes, vscale, vzero, rows);
  else if (vbits == 4) hipLaunchKernelGGL((value_quant_kernel<T, 4>), dim3(blocks), dim3(256), 0, st, V, codes, vscale, vzero, rows);
  else hipLaunchKernelGGL((value_quant_kernel<T, 8>), dim3(blocks), dim3(256), 0, st, V, codes, vscale, vzero, rows);
}

}  // namespace

int launch_quantize_values(const qjl_shape& sh, int vbits, const void* V, uint8_t* codes,
                           uint16_t* vscale, uint16_t* vzero, hipStream_t st) {
  if ((vbits != 2 && vbits != 4 && vbits != 8) || sh.d != 128) return QJL_ERR_UNSUPPORTED;
  const long rows = (long)sh.batch * sh.kv_heads * sh.n;
  long blocks = (rows + 31) / 32;
  const long cap = 32L * device_cu_count();        // grid-stride beyond this
  if (blocks > cap) blocks = cap;
  switch (sh.dtype) {
    case QJL_F32: launch_bits<f32_t>(vbits, (unsigned)blocks, st, V, codes, vscale, vzero, rows); break;
    case QJL_F16: launch_bits<f16_t>(vbits, (unsigned)blocks, st, V, codes, vscale, vzero, rows); break;
    default: launch_bits<bf16_t>(vbits, (unsigned)blocks, st, V, codes, vscale, vzero, rows); break;
  }
  return launch_status();
}

}  // namespace qjl
