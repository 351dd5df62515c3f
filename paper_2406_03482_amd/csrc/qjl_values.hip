// Value cache quantization (Section 3.2): every token's row of V is normalised
// and rounded to a few-bit integer.  Scheme: zero point = the row's minimum,
// scale = (max - min) / (2^b - 1), both stored as binary16; the code of an
// entry is (v - zero) / scale rounded to the nearest integer (ties to even) and
// clipped to [0, 2^b - 1], taken against the stored zero point and scale, so
// that zero + code * scale is the nearest representable value.  b = 4 here.
//
// The code is an integer decided by floating point: subtract, divide and round
// are IEEE float32 operations in exactly this order (the kernel takes a shortcut
// only where it provably gives the same integer).
#include "qjl_common.hpp"

namespace qjl {
namespace {

// d == 128: sixteen lanes share a row (8 entries each); minimum and maximum by
// 16-lane DPP reductions; a lane packs its eight 4-bit codes into one word, so
// a row's 64 code bytes leave as one contiguous piece.
template <typename T>
__global__ void __launch_bounds__(256)
value_quant4_kernel(const void* __restrict__ V, uint32_t* __restrict__ codes,
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
    const uint16_t s16 = float_to_f16_bits((hi - lo) / 15.0f);
    const uint16_t z16 = float_to_f16_bits(lo);
    const float sc = f16_bits_to_float(s16), z = f16_bits_to_float(z16);
    uint32_t word = 0;
    if (sc > 0.f) {
      // rint((x - z) / sc) without a division per entry: q0 = rint((x - z) * (1/sc)) is right whenever
      // the remainder (x - z) - q0 * sc (exact: one fused multiply-add) is clear of half a step; the
      // rounding of the quotient moves it by < 2^-19 steps, the margin is 2^-18.  The few entries
      // near a tie take the division itself, so every code is the one the definition gives.
      const float inv = 1.0f / sc;
      const float clear = (0.5f - 0x1.0p-18f) * sc;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float t = x[e] - z;
        float q = rintf(t * inv);
        if (!(fabsf(fmaf(-q, sc, t)) < clear)) q = rintf(t / sc);
        q = fminf(fmaxf(q, 0.f), 15.f);
        word |= (uint32_t)q << (4 * e);
      }
    }
    codes[(size_t)row * 16 + c] = word;
    if (c == 0) { vscale[row] = s16; vzero[row] = z16; }
  }
}

}  // namespace

int launch_quantize_values(const qjl_shape& sh, int vbits, const void* V, uint8_t* codes,
                           uint16_t* vscale, uint16_t* vzero, hipStream_t st) {
  if (vbits != 4 || sh.d != 128) return QJL_ERR_UNSUPPORTED;
  const long rows = (long)sh.batch * sh.kv_heads * sh.n;
  long blocks = (rows + 15) / 16;
  const long cap = 32L * device_cu_count();        // grid-stride beyond this
  if (blocks > cap) blocks = cap;
  uint32_t* cw = reinterpret_cast<uint32_t*>(codes);
  switch (sh.dtype) {
    case QJL_F32: hipLaunchKernelGGL(value_quant4_kernel<f32_t>, dim3((unsigned)blocks), dim3(256), 0, st, V, cw, vscale, vzero, rows); break;
    case QJL_F16: hipLaunchKernelGGL(value_quant4_kernel<f16_t>, dim3((unsigned)blocks), dim3(256), 0, st, V, cw, vscale, vzero, rows); break;
    default: hipLaunchKernelGGL(value_quant4_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, st, V, cw, vscale, vzero, rows); break;
  }
  return launch_status();
}

}  // namespace qjl
