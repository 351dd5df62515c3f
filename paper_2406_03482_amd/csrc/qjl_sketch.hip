// Algorithm 1 step 1 / Definition 3.1: the i.i.d. N(0,1) sketch S, drawn on
// the device from a counter-based generator so that it depends on nothing but
// (seed, m, d, dtype).
#include "qjl_common.hpp"

namespace qjl {
namespace {

__device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t counter) {
  uint64_t z = seed + (counter + 1ull) * 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Entry e of the Gaussian sketch: Box-Muller in fp64 from two 53-bit uniforms, rounded to fp32.
__device__ __forceinline__ float gaussian_entry(uint64_t seed, size_t e) {
  uint64_t a = splitmix64_at(seed, 2ull * e);
  uint64_t b = splitmix64_at(seed, 2ull * e + 1ull);
  double u1 = ((double)(a >> 11) + 1.0) * 0x1.0p-53;
  double u2 = (double)(b >> 11) * 0x1.0p-53;
  double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
  return (float)z;
}

template <int DT> __device__ __forceinline__ void store_entry(void* S, size_t e, float f) {
  if (DT == QJL_F32) static_cast<float*>(S)[e] = f;
  else if (DT == QJL_F16) static_cast<uint16_t*>(S)[e] = float_to_f16_bits(f);
  else static_cast<uint16_t*>(S)[e] = float_to_bf16_bits(f);
}

// One thread per entry, rounded to the storage type.
template <int DT>
__global__ void __launch_bounds__(256) sketch_kernel(uint64_t seed, size_t count, void* S) {
  size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= count) return;
  store_entry<DT>(S, e, gaussian_entry(seed, e));
}

// Section 4.1, "Orthogonalized JL transform": the rows of the Gaussian sketch
// are orthogonalised by a QR decomposition.  One workgroup per block of d rows
// (m > d rows cannot all be orthogonal): the block lives in LDS as doubles, row
// i is replaced by the i-th Gram-Schmidt direction of the block's rows and
// scaled back to the length the Gaussian row had, so that every row keeps its
// N(0, I) distribution.  Classical Gram-Schmidt applied twice per row (as
// accurate as Householder QR for this purpose, and every step is a
// workgroup-wide matrix-vector product).  d <= 128.
template <int DT>
__global__ void __launch_bounds__(256) orth_sketch_kernel(uint64_t seed, int m, int d, void* S) {
  extern __shared__ double blk[];                  // [rows][d] block, then coef[128], len[128]
  const int r0 = blockIdx.x * d;
  const int rows = min(d, m - r0);
  double* coef = blk + (size_t)d * d;
  double* len = coef + 128;
  const int tid = threadIdx.x;
  for (int e = tid; e < rows * d; e += 256) blk[e] = (double)gaussian_entry(seed, (size_t)r0 * d + e);
  __syncthreads();
  if (tid < rows) {
    double ss = 0.0;
    for (int t = 0; t < d; ++t) ss += blk[tid * d + t] * blk[tid * d + t];
    len[tid] = sqrt(ss);
  }
  __syncthreads();
  for (int i = 0; i < rows; ++i) {
    double* v = blk + (size_t)i * d;
    for (int pass = 0; pass < 2; ++pass) {
      if (tid < i) {                               // coef_j = <q_j, v>
        double c = 0.0;
        for (int t = 0; t < d; ++t) c += blk[tid * d + t] * v[t];
        coef[tid] = c;
      }
      __syncthreads();
      if (tid < d) {                               // v -= sum_j coef_j q_j
        double x = v[tid];
        for (int j = 0; j < i; ++j) x -= coef[j] * blk[j * d + tid];
        v[tid] = x;
      }
      __syncthreads();
    }
    double ss = 0.0;                               // every thread: the same sum in the same order
    for (int t = 0; t < d; ++t) ss += v[t] * v[t];
    const double inv = 1.0 / sqrt(ss);
    __syncthreads();                               // all have read v
    if (tid < d) v[tid] *= inv;
    __syncthreads();
  }
  for (int e = tid; e < rows * d; e += 256) {
    const int i = e / d;
    store_entry<DT>(S, (size_t)r0 * d + e, (float)(len[i] * blk[e]));
  }
}

}  // namespace

int launch_make_sketch(uint64_t seed, int m, int d, int dtype, void* S, hipStream_t st) {
  size_t count = (size_t)m * (size_t)d;
  dim3 grid((unsigned)((count + 255) / 256)), block(256);
  switch (dtype) {
    case QJL_F32: hipLaunchKernelGGL(sketch_kernel<QJL_F32>, grid, block, 0, st, seed, count, S); break;
    case QJL_F16: hipLaunchKernelGGL(sketch_kernel<QJL_F16>, grid, block, 0, st, seed, count, S); break;
    default: hipLaunchKernelGGL(sketch_kernel<QJL_BF16>, grid, block, 0, st, seed, count, S); break;
  }
  return launch_status();
}

int launch_make_sketch_orthogonal(uint64_t seed, int m, int d, int dtype, void* S, hipStream_t st) {
  if (d > 128) return QJL_ERR_UNSUPPORTED;
  const size_t lds = ((size_t)d * d + 256) * sizeof(double);
  static std::atomic<uint64_t> set32{0}, set16{0}, setb16{0};
  int rc = allow_dynamic_lds(reinterpret_cast<const void*>(&orth_sketch_kernel<QJL_F32>), 160 * 1024, set32);
  if (rc == QJL_OK) rc = allow_dynamic_lds(reinterpret_cast<const void*>(&orth_sketch_kernel<QJL_F16>), 160 * 1024, set16);
  if (rc == QJL_OK) rc = allow_dynamic_lds(reinterpret_cast<const void*>(&orth_sketch_kernel<QJL_BF16>), 160 * 1024, setb16);
  if (rc != QJL_OK) return rc;
  dim3 grid((unsigned)((m + d - 1) / d)), block(256);
  switch (dtype) {
    case QJL_F32: hipLaunchKernelGGL(orth_sketch_kernel<QJL_F32>, grid, block, lds, st, seed, m, d, S); break;
    case QJL_F16: hipLaunchKernelGGL(orth_sketch_kernel<QJL_F16>, grid, block, lds, st, seed, m, d, S); break;
    default: hipLaunchKernelGGL(orth_sketch_kernel<QJL_BF16>, grid, block, lds, st, seed, m, d, S); break;
  }
  return launch_status();
}

}  // namespace qjl
