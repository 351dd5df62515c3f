// Algorithm 1, EstimateScores before the softmax: Definition 3.1 Eq. (4) for
// every cached key.  HBM-streaming kernel: 34 bytes read per key and KV head,
// one fp32 written per key and query head.  One thread per key; the signed
// sum comes from byte-indexed tables in LDS.
#include "qjl_common.hpp"
#include "qjl_lut.hpp"

namespace qjl {
namespace {

struct scores_args {
  const float* SQ;
  const uint8_t* bits;
  const uint16_t* norms;
  float* out;
  int n, q_heads, kv_heads, groups_per_kv;  // groups_per_kv = G / GT
  int keys_per_block, blocks_per_unit;
  float coef;                               // scale * sqrt(pi/2) / m
};

template <int GT, int MW>
__global__ void __launch_bounds__(256) scores_kernel(scores_args a) {
  extern __shared__ float4 smem4[];
  float* smem = reinterpret_cast<float*>(smem4);
  constexpr int M = MW * 32;
  float* sq = smem;
  float* nib = sq + GT * M;
  float* lut = nib + 4 * M * GT;

  const int tid = threadIdx.x;
  const int unit = blockIdx.x / a.blocks_per_unit;
  const int blk = blockIdx.x - unit * a.blocks_per_unit;
  const int gg = unit % a.groups_per_kv;
  const int bk = unit / a.groups_per_kv;            // b * Hkv + kvh
  const int b = bk / a.kv_heads, kvh = bk - b * a.kv_heads;
  const int G = a.groups_per_kv * GT;
  const size_t hq0 = (size_t)b * a.q_heads + (size_t)kvh * G + (size_t)gg * GT;

  for (int e = tid; e < GT * M; e += 256) sq[e] = a.SQ[hq0 * M + e];
  __syncthreads();
  build_lut<GT>(sq, nib, lut, M, tid, 256);

  const int k_begin = blk * a.keys_per_block;
  const int k_end = min(a.n, k_begin + a.keys_per_block);
  const size_t row0 = (size_t)bk * a.n;
  for (int j = k_begin + tid; j < k_end; j += 256) {
    uint32_t w[MW];
    load_code<MW>(a.bits, row0 + j, w);
    const float nu = f16_bits_to_float(a.norms[row0 + j]);
    const typename vecf<GT>::type s = key_inner<GT, MW>(w, lut);
#pragma unroll
    for (int g = 0; g < GT; ++g) a.out[(hq0 + g) * a.n + j] = a.coef * nu * vget<GT>(s, g);
  }
}

template <int GT, int MW>
int launch_t(const qjl_shape& sh, scores_args a, hipStream_t st) {
  static std::atomic<uint64_t> lds_set{0};
  const size_t lds = lut_lds_floats<GT>(MW * 32) * sizeof(float);
  const int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(&scores_kernel<GT, MW>), lds, lds_set);
  if (rc_lds != QJL_OK) return rc_lds;
  const int G = sh.q_heads / sh.kv_heads;
  a.groups_per_kv = G / GT;
  const long units = (long)sh.batch * sh.kv_heads * a.groups_per_kv;
  // enough workgroups to fill the chip, but at least 2048 keys each so that the
  // table build (about 9*GT*m table writes) stays small against the streaming
  long want = (4L * device_cu_count() + units - 1) / units;
  long kpb = ((long)sh.n + want - 1) / want;
  if (kpb < 2048) kpb = 2048;
  kpb = (kpb + 255) / 256 * 256;
  a.keys_per_block = (int)(kpb > sh.n ? ((sh.n + 255) / 256 * 256) : kpb);
  a.blocks_per_unit = (sh.n + a.keys_per_block - 1) / a.keys_per_block;
  const long total = units * a.blocks_per_unit;
  if (total > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  hipLaunchKernelGGL((scores_kernel<GT, MW>), dim3((unsigned)total), dim3(256), lds, st, a);
  return launch_status();
}

template <int MW>
int launch_m(const qjl_shape& sh, const scores_args& a, hipStream_t st) {
  const int G = sh.q_heads / sh.kv_heads;
  const int m = MW * 32;
  if (G % 4 == 0 && m * 4 <= 1024) return launch_t<4, MW>(sh, a, st);
  if (G % 2 == 0 && m * 2 <= 1024) return launch_t<2, MW>(sh, a, st);
  return launch_t<1, MW>(sh, a, st);
}

}  // namespace

int launch_scores(const qjl_shape& sh, const float* SQ, const uint8_t* bits, const uint16_t* norms,
                  float* out, hipStream_t st) {
  scores_args a;
  a.SQ = SQ; a.bits = bits; a.norms = norms; a.out = out;
  a.n = sh.n; a.q_heads = sh.q_heads; a.kv_heads = sh.kv_heads;
  a.coef = sh.scale * 1.2533141373155002512f / (float)sh.m;
  a.groups_per_kv = 0; a.keys_per_block = 0; a.blocks_per_unit = 0;
  switch (sh.m) {
    case 128: return launch_m<4>(sh, a, st);
    case 256: return launch_m<8>(sh, a, st);
    case 512: return launch_m<16>(sh, a, st);
    default: return QJL_ERR_UNSUPPORTED;
  }
}

}  // namespace qjl
