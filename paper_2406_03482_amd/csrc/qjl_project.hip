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

int launch_project(int rows, int d, int m, int dtype, const void* Q, const void* S, float* SQ,
                   hipStream_t st) {
  switch (dtype) {
    case QJL_F32: return launch_t<f32_t>(rows, d, m, Q, S, SQ, st);
    case QJL_F16: return launch_t<f16_t>(rows, d, m, Q, S, SQ, st);
    default: return launch_t<bf16_t>(rows, d, m, Q, S, SQ, st);
  }
}

}  // namespace qjl
