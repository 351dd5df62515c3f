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

// d == 128: sixteen lanes share a row (8 entries each); minimum and maximum by
// 16-lane DPP reductions; a lane packs its eight b-bit codes into b bytes, so a
// row's 16 b code bytes leave as one contiguous piece.
template <typename T, int BITS>
__global__ void __launch_bounds__(256)
value_quant_kernel(const void* __restrict__ V, uint8_t* __restrict__ codes,
                   uint16_t* __restrict__ vscale, uint16_t* __restrict__ vzero, long rows) {
  const int c = threadIdx.x & 15, r = threadIdx.x >> 4;
  for (long row = (long)blockIdx.x * 16 + r; row < rows; row += (long)gridDim.x * 16) {
    float x[8];
    load8<T>(V, (size_t)row * 128 + c * 8, x);
    float lo = x[0], hi = x[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) { lo = fminf(lo, x[e]); hi = fmaxf(hi, x[e]); }
    lo = row16_min(lo);
    hi = row16_max(hi);
    uint16_t s16, z16;
    uint32_t q8[8];
    value_codes8<BITS>(x, lo, hi, s16, z16, q8);
    uint8_t* dst = codes + (size_t)row * (16 * BITS) + c * BITS;
    if constexpr (BITS == 8) {
      uint2 w;
      w.x = q8[0] | (q8[1] << 8) | (q8[2] << 16) | (q8[3] << 24);
      w.y = q8[4] | (q8[5] << 8) | (q8[6] << 16) | (q8[7] << 24);
      *reinterpret_cast<uint2*>(dst) = w;
    } else {
      uint32_t word = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) word |= q8[e] << (BITS * e);
      if constexpr (BITS == 4) *reinterpret_cast<uint32_t*>(dst) = word;
      else *reinterpret_cast<uint16_t*>(dst) = (uint16_t)word;
    }
    if (c == 0) { vscale[row] = s16; vzero[row] = z16; }
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
  long blocks = (rows + 15) / 16;
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
