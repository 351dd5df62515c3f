// Outlier channels (Section 4.1, "Outliers"): which channels of a head's keys are
// treated separately, and the stacked sketch that restricts one QJL instance to
// them and a second one to all other channels.
//
// The paper states that the outlier channels are found in the prompt phase and
// that a few fixed channels carry much larger magnitudes (Figure 2 ranks the
// channels by their mean magnitude over the tokens).  Rule used here: per
// (batch, kv head) the `count` channels with the largest mean |k| over the n
// tokens, in decreasing order, ties to the lower channel index.
#include "qjl_common.hpp"

namespace qjl {
namespace {

constexpr int kRowsPerSplit = 2048;   // tokens summed by one workgroup

// sum_j |K[seg, j, t]| over one split of the tokens -> part[seg][split][t], d == 128.
// 16 lanes share a row (16 bytes each); each thread sums its 8 channels over
// every 16th row, then the 16 row groups are added in a fixed order.
template <typename T>
__global__ void __launch_bounds__(256)
abs_sum128_kernel(const void* __restrict__ K, float* __restrict__ part, int n, int nsplit) {
  __shared__ float red[16][128];
  const int tid = threadIdx.x;
  const int c = tid & 15, r = tid >> 4;
  const size_t seg = blockIdx.y;
  const int j0 = blockIdx.x * kRowsPerSplit;
  const int j1 = min(n, j0 + kRowsPerSplit);
  float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  // eight rows requested before the first is used (one load in flight per thread leaves the
  // memory system idle); they are added in row order, as a one-row-at-a-time loop would
  constexpr int kAhead = 8;
  for (int j = j0 + r; j < j1; j += 16 * kAhead) {
    float x[kAhead][8];
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      const int ju = min(j + 16 * u, j1 - 1);           // rows past the split: a row inside it, not added
      load8<T>(K, (seg * (size_t)n + ju) * 128 + c * 8, x[u]);
    }
#pragma unroll
    for (int u = 0; u < kAhead; ++u) {
      if (j + 16 * u < j1) {
#pragma unroll
        for (int e = 0; e < 8; ++e) s[e] += fabsf(x[u][e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) red[r][c * 8 + e] = s[e];
  __syncthreads();
  if (tid < 128) {
    float t = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) t += red[q][tid];
    part[(seg * nsplit + blockIdx.x) * 128 + tid] = t;
  }
}

// Any d: one thread per channel, rows of the split in order.
template <typename T>
__global__ void __launch_bounds__(256)
abs_sum_generic_kernel(const void* __restrict__ K, float* __restrict__ part, int n, int d, int nsplit) {
  const size_t seg = blockIdx.y;
  const int j0 = blockIdx.x * kRowsPerSplit;
  const int j1 = min(n, j0 + kRowsPerSplit);
  for (int t = threadIdx.x; t < d; t += 256) {
    float s = 0.f;
    for (int j = j0; j < j1; ++j) s += fabsf(load1<T>(K, (seg * (size_t)n + j) * d + t));
    part[(seg * nsplit + blockIdx.x) * d + t] = s;
  }
}

// Add the splits (fixed order) and pick the `count` largest sums.  One workgroup
// per (batch, kv head).  The selection is done by the first wave: every lane scans
// the channels lane, lane + 64, ... in increasing order (a strictly larger sum
// replaces the candidate, so the lower index wins a tie inside a lane), then six
// exchange steps keep the larger sum or, for equal sums, the lower index.
__global__ void __launch_bounds__(256)
top_channels_kernel(const float* __restrict__ part, int32_t* __restrict__ channels, int d, int nsplit,
                    int count) {
  extern __shared__ float tot[];                     // [d]
  const size_t seg = blockIdx.x;
  for (int t = threadIdx.x; t < d; t += 256) {
    float s = 0.f;
    for (int q = 0; q < nsplit; ++q) s += part[(seg * nsplit + q) * d + t];
    tot[t] = s;
  }
  __syncthreads();
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    for (int c = 0; c < count; ++c) {
      float bv = -1.f;                                // sums of magnitudes are >= 0 (a NaN sum is never picked)
      int best = 0x7FFFFFFF;
      for (int t = lane; t < d; t += 64) {
        const float v = tot[t];
        if (v > bv) { bv = v; best = t; }
      }
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const float ov = __shfl_xor(bv, off);
        const int ob = __shfl_xor(best, off);
        if (ov > bv || (ov == bv && ob < best)) { bv = ov; best = ob; }
      }
      // every lane now holds the same winner; with nothing left to pick (count > d, or only NaN sums)
      // the serial rule's answer is channel 0
      if (best == 0x7FFFFFFF) best = 0;
      if (lane == 0) {
        channels[seg * count + c] = best;
        tot[best] = -2.f;                             // never picked again
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
  }
}

// S_dual[seg][r][t] = S_in[r][t] outside the segment's outlier channels (rows r < m_in),
//                     S_out[r - m_in][t] on them (rows r >= m_in), zero elsewhere.
template <typename R>
__global__ void __launch_bounds__(256)
dual_sketch_kernel(const R* __restrict__ S_in, const R* __restrict__ S_out,
                   const int32_t* __restrict__ channels, int count, R* __restrict__ S_dual, int m_in,
                   int m_out, int d) {
  extern __shared__ int is_out[];                    // [d]
  const size_t seg = blockIdx.y;
  for (int t = threadIdx.x; t < d; t += 256) is_out[t] = 0;
  __syncthreads();
  if (threadIdx.x < count) {
    const int ch = channels[seg * count + threadIdx.x];
    if (ch >= 0 && ch < d) is_out[ch] = 1;            // entries out of range are ignored
  }
  __syncthreads();
  const int total = (m_in + m_out) * d;
  for (int e = blockIdx.x * 256 + threadIdx.x; e < total; e += gridDim.x * 256) {
    const int r = e / d, t = e - r * d;
    R v = R(0);
    if (r < m_in) { if (!is_out[t]) v = S_in[e]; }
    else if (is_out[t]) v = S_out[e - m_in * d];
    S_dual[seg * (size_t)total + e] = v;
  }
}

int splits_of(int n) { return (n + kRowsPerSplit - 1) / kRowsPerSplit; }

}  // namespace

size_t outlier_workspace_bytes(const qjl_shape& sh) {
  return (size_t)sh.batch * sh.kv_heads * splits_of(sh.n) * sh.d * sizeof(float);
}

int launch_select_outliers(const qjl_shape& sh, const void* K, int count, int32_t* channels,
                           void* workspace, hipStream_t st) {
  const long segs = (long)sh.batch * sh.kv_heads;
  if (segs > 65535) return QJL_ERR_UNSUPPORTED;
  const int nsplit = splits_of(sh.n);
  float* part = static_cast<float*>(workspace);
  dim3 grid((unsigned)nsplit, (unsigned)segs);
  if (sh.d == 128) {
    switch (sh.dtype) {
      case QJL_F32: hipLaunchKernelGGL(abs_sum128_kernel<f32_t>, grid, dim3(256), 0, st, K, part, sh.n, nsplit); break;
      case QJL_F16: hipLaunchKernelGGL(abs_sum128_kernel<f16_t>, grid, dim3(256), 0, st, K, part, sh.n, nsplit); break;
      default: hipLaunchKernelGGL(abs_sum128_kernel<bf16_t>, grid, dim3(256), 0, st, K, part, sh.n, nsplit); break;
    }
  } else {
    switch (sh.dtype) {
      case QJL_F32: hipLaunchKernelGGL(abs_sum_generic_kernel<f32_t>, grid, dim3(256), 0, st, K, part, sh.n, sh.d, nsplit); break;
      case QJL_F16: hipLaunchKernelGGL(abs_sum_generic_kernel<f16_t>, grid, dim3(256), 0, st, K, part, sh.n, sh.d, nsplit); break;
      default: hipLaunchKernelGGL(abs_sum_generic_kernel<bf16_t>, grid, dim3(256), 0, st, K, part, sh.n, sh.d, nsplit); break;
    }
  }
  int rc = launch_status();
  if (rc != QJL_OK) return rc;
  hipLaunchKernelGGL(top_channels_kernel, dim3((unsigned)segs), dim3(256), (size_t)sh.d * sizeof(float), st,
                     part, channels, sh.d, nsplit, count);
  return launch_status();
}

int launch_make_dual_sketch(const qjl_shape& sh, int m_out, const void* S_in, const void* S_out,
                            const int32_t* channels, int count, void* S_dual, hipStream_t st) {
  const long segs = (long)sh.batch * sh.kv_heads;
  if (segs > 65535) return QJL_ERR_UNSUPPORTED;
  const int total = (sh.m + m_out) * sh.d;
  dim3 grid((unsigned)((total + 256 * 8 - 1) / (256 * 8)), (unsigned)segs);
  const size_t lds = (size_t)sh.d * sizeof(int);
  if (sh.dtype == QJL_F32)
    hipLaunchKernelGGL(dual_sketch_kernel<float>, grid, dim3(256), lds, st, static_cast<const float*>(S_in),
                       static_cast<const float*>(S_out), channels, count, static_cast<float*>(S_dual),
                       sh.m, m_out, sh.d);
  else   // 16-bit storage types are copied as raw bits (zero is all-zero bits in both)
    hipLaunchKernelGGL(dual_sketch_kernel<uint16_t>, grid, dim3(256), lds, st,
                       static_cast<const uint16_t*>(S_in), static_cast<const uint16_t*>(S_out), channels,
                       count, static_cast<uint16_t*>(S_dual), sh.m, m_out, sh.d);
  return launch_status();
}

}  // namespace qjl
