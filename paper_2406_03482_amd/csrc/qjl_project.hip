// The query side of Definition 3.1 Eq. (4): SQ = S q, with the query left
// unquantized.  fp32 accumulation.  One workgroup per query vector.
#include "qjl_common.hpp"

namespace qjl {
namespace {

// d == 128: sixteen lanes share one row of S (16 bytes each, so a wave reads
// four whole rows per load), multiply by their slice of q held in registers
// and reduce inside the 16-lane DPP row.  A workgroup handles 128 rows of S
// (blockIdx.y picks which): all eight row passes are requested before anything
// is waited for, so the kernel costs one round trip to L2.
template <typename T>
__global__ void __launch_bounds__(256)
project128_kernel(const void* __restrict__ Q, const void* __restrict__ S, float* __restrict__ SQ,
                  int m) {
  constexpr int kPasses = 8;
  const int row = blockIdx.x;                 // (b, hq) flattened
  const int tid = threadIdx.x;
  const int c = tid & 15;                     // 8-element slice of the row
  const int r = tid >> 4;                     // 0..15: row inside a pass of 16 rows
  const int i0 = blockIdx.y * (16 * kPasses);
  float s[kPasses][8];
#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    const int i = min(i0 + 16 * u + r, m - 1);            // clamp: never read past S
    load8<T>(S, (size_t)i * 128 + c * 8, s[u]);
  }
  float q[8];
  load8<T>(Q, (size_t)row * 128 + c * 8, q);
#pragma unroll
  for (int u = 0; u < kPasses; ++u) {
    float acc = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) acc = fmaf(s[u][t], q[t], acc);
    acc = row16_sum(acc);
    const int i = i0 + 16 * u + r;
    if (c == 0 && i < m) SQ[(size_t)row * m + i] = acc;
  }
}

// Algorithm 1 steps 3-4 for a handful of new keys (d == 128): the same walk over
// S as project128_kernel, but the 128 inner products of a workgroup end as sign
// bits.  Wave w owns projections 32w..32w+31 of the workgroup's 128, four per
// pass (one per 16-lane row), so its ballots assemble exactly one code word.
// Grid: (new key, slice of 128 projections).  Slice 0 also stores the norm.
template <typename T>
__global__ void __launch_bounds__(256)
append128_kernel(const void* __restrict__ K_new, const void* __restrict__ S, uint32_t* __restrict__ bits,
                 uint16_t* __restrict__ norms, int m, int t, int pos, long cap) {
  const int key = blockIdx.x;                 // (b * Hkv + kvh) * t + token
  const int bh = key / t, tok = key - bh * t;
  const size_t row = (size_t)bh * cap + pos + tok;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int c = tid & 15, g = lane >> 4;
  const int i0 = blockIdx.y * 128 + wave * 32;
  float k[8];
  load8<T>(K_new, (size_t)key * 128 + c * 8, k);
  float s[8][8];
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    const int i = min(i0 + 4 * u + g, m - 1);             // clamp: never read past S
    load8<T>(S, (size_t)i * 128 + c * 8, s[u]);
  }
  uint32_t word = 0;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    float acc = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc = fmaf(s[u][e], k[e], acc);
    acc = row16_sum(acc);
    const unsigned long long mask = __ballot(acc >= 0.f);  // sign(0) = +1
#pragma unroll
    for (int gg = 0; gg < 4; ++gg) word |= (uint32_t)((mask >> (16 * gg)) & 1ull) << (4 * u + gg);
  }
  if (lane == 0 && i0 < m) bits[row * (size_t)(m >> 5) + (i0 >> 5)] = word;
  if (blockIdx.y == 0 && wave == 0) {
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) ss = fmaf(k[e], k[e], ss);
    ss = row16_sum(ss);
    if (lane == 0) norms[row] = float_to_f16_bits(sqrtf(ss));
  }
}

// Any d, any m: one thread per projection, scalar loads.
template <typename T>
__global__ void __launch_bounds__(256)
project_generic_kernel(const void* __restrict__ Q, const void* __restrict__ S,
                       float* __restrict__ SQ, int d, int m) {
  const int row = blockIdx.x;
  const int tid = threadIdx.x;
  for (int i = tid; i < m; i += 256) {
    float acc = 0.f;
    for (int t = 0; t < d; ++t)
      acc = fmaf(load1<T>(S, (size_t)i * d + t), load1<T>(Q, (size_t)row * d + t), acc);
    SQ[(size_t)row * m + i] = acc;
  }
}

template <typename T>
int launch_t(int rows, int d, int m, const void* Q, const void* S, float* SQ, hipStream_t st) {
  dim3 grid((unsigned)rows), block(256);
  if (d == 128)
    hipLaunchKernelGGL(project128_kernel<T>, dim3((unsigned)rows, (unsigned)((m + 127) / 128)), block, 0, st,
                       Q, S, SQ, m);
  else
    hipLaunchKernelGGL(project_generic_kernel<T>, grid, block, 0, st, Q, S, SQ, d, m);
  return launch_status();
}

}  // namespace

int launch_append_keys(const qjl_shape& sh, const void* K_new, int t, int pos, const void* S, uint8_t* bits,
                       uint16_t* norms, hipStream_t st) {
  const long keys = (long)sh.batch * sh.kv_heads * t;
  dim3 grid((unsigned)keys, (unsigned)((sh.m + 127) / 128));
  uint32_t* bw = reinterpret_cast<uint32_t*>(bits);
  switch (sh.dtype) {
    case QJL_F32: hipLaunchKernelGGL(append128_kernel<f32_t>, grid, dim3(256), 0, st, K_new, S, bw, norms, sh.m, t, pos, (long)sh.n); break;
    case QJL_F16: hipLaunchKernelGGL(append128_kernel<f16_t>, grid, dim3(256), 0, st, K_new, S, bw, norms, sh.m, t, pos, (long)sh.n); break;
    default: hipLaunchKernelGGL(append128_kernel<bf16_t>, grid, dim3(256), 0, st, K_new, S, bw, norms, sh.m, t, pos, (long)sh.n); break;
  }
  return launch_status();
}

int launch_project(int rows, int d, int m, int dtype, const void* Q, const void* S, float* SQ,
                   hipStream_t st) {
  switch (dtype) {
    case QJL_F32: return launch_t<f32_t>(rows, d, m, Q, S, SQ, st);
    case QJL_F16: return launch_t<f16_t>(rows, d, m, Q, S, SQ, st);
    default: return launch_t<bf16_t>(rows, d, m, Q, S, SQ, st);
  }
}

}  // namespace qjl
