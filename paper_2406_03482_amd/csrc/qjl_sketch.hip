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

// One thread per entry: Box-Muller in fp64 from two 53-bit uniforms, rounded to
// fp32 and then to the storage type.
template <int DT>
__global__ void __launch_bounds__(256) sketch_kernel(uint64_t seed, size_t count, void* S) {
  size_t e = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= count) return;
  uint64_t a = splitmix64_at(seed, 2ull * e);
  uint64_t b = splitmix64_at(seed, 2ull * e + 1ull);
  double u1 = ((double)(a >> 11) + 1.0) * 0x1.0p-53;
  double u2 = (double)(b >> 11) * 0x1.0p-53;
  double z = sqrt(-2.0 * log(u1)) * cos(6.283185307179586476925286766559 * u2);
  float f = (float)z;
  if (DT == QJL_F32) static_cast<float*>(S)[e] = f;
  else if (DT == QJL_F16) static_cast<uint16_t*>(S)[e] = float_to_f16_bits(f);
  else static_cast<uint16_t*>(S)[e] = float_to_bf16_bits(f);
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

}  // namespace qjl
