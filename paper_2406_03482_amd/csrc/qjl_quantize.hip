// Algorithm 1 steps 3-4 / Definition 3.1 Eq. (3): for every key store the packed
// sign bits of S k and the norm ||k||_2.
//
// Two paths:
//  * 16-bit keys with d = 128 and m a multiple of 128: K S^T is a dense
//    contraction and runs on the matrix cores (v_mfma_f32_32x32x16, fp32
//    accumulation).  Each wave keeps its share of S in registers for the whole
//    kernel; key tiles stream HBM -> registers -> LDS once, the norm is taken
//    on the way, and the accumulators are reduced to bits in registers, so the
//    projections never reach memory.
//  * anything else (fp32 keys, other d or m): plain fp32 FMA loops.
#include "qjl_common.hpp"

namespace qjl {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

template <typename T> struct mma;
template <> struct mma<bf16_t> {
  using frag = bf16x8_t;
  static __device__ __forceinline__ f32x16_t run(frag a, frag b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct mma<f16_t> {
  using frag = f16x8_t;
  static __device__ __forceinline__ f32x16_t run(frag a, frag b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
};

constexpr int kTok = 32;        // keys per tile = N of the 32x32 MFMA tile
constexpr int kRowU4 = 17;      // LDS row pitch in 16-byte units: 256 B of key + 16 B pad

// Sixteen accumulators of one lane -> 16 bits, bit v = [acc[v] >= 0].
// v_alignbit shifts the IEEE sign bit of each accumulator in; a sum that
// starts from +0 can only be -0 if it is within rounding of zero.
__device__ __forceinline__ uint32_t nonneg_bits16(const f32x16_t& acc) {
  uint32_t t = 0;
#pragma unroll
  for (int v = 15; v >= 0; --v) t = __builtin_amdgcn_alignbit(t, __float_as_uint(acc[v]), 31);
  return (~t) & 0xFFFFu;
}

// PPW = projections per wave (32, 64 or 128); a workgroup of four waves covers
// 4*PPW projections, blockIdx.y selects which block of 4*PPW out of m.
template <typename T, int PPW>
__global__ void __launch_bounds__(256, 2)
quantize_mfma_kernel(const uint16_t* __restrict__ K, const uint16_t* __restrict__ S,
                     uint32_t* __restrict__ bits, uint16_t* __restrict__ norms, long rows, int m,
                     int num_tiles) {
  using frag = typename mma<T>::frag;
  constexpr int NA = PPW / 32;            // 32x32 MFMA tiles per wave along the projections
  constexpr int WPT = 4 * PPW / 32;       // code words per key written by this workgroup
  constexpr int OPITCH = WPT + 1;         // odd pitch: conflict-free LDS writes
  __shared__ uint4 kbuf[2][kTok * kRowU4];
  __shared__ uint32_t obuf[2][kTok * OPITCH];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int h = lane >> 5;                // which 8 of the 16 k of an MFMA step this lane feeds
  const int j = lane & 31;                // A: row of the S tile, B/D: key of the tile
  const int proj_base = blockIdx.y * (4 * PPW) + wave * PPW;
  const int words_per_row = m >> 5;

  // ---- this wave's rows of S, resident in registers as MFMA A operands.
  // Row rho of tile a is projection  proj_base + ((rho>>2)&1)*PPW/2 + 16a + 4(rho>>3) + (rho&3):
  // with the 32x32 accumulator layout (register v of lane (h, j) is row
  // 8(v/4) + 4h + v%4) lane (h, j) then owns projections
  // proj_base + h*PPW/2 + 16a + v, v = 0..15 -- consecutive code bits of key j.
  frag sfrag[NA][8];
#pragma unroll
  for (int a = 0; a < NA; ++a) {
    const int srow = proj_base + ((j >> 2) & 1) * (PPW / 2) + 16 * a + 4 * (j >> 3) + (j & 3);
    const uint4* sp = reinterpret_cast<const uint4*>(S + (size_t)srow * 128 + 8 * h);
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      uint4 u = sp[2 * s];
      __builtin_memcpy(&sfrag[a][s], &u, 16);
    }
  }

  // ---- loader: thread -> (row lrow + 16u, 16-byte column lcol) of a tile
  const int lrow = tid >> 4, lcol = tid & 15;
  uint4 pre[2];
  auto load_tile = [&](int tile) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      long row = (long)tile * kTok + lrow + 16 * u;
      if (row >= rows) row = rows - 1;    // clamp: stay inside K, results of such rows are dropped
      pre[u] = *reinterpret_cast<const uint4*>(K + (size_t)row * 128 + lcol * 8);
    }
  };
  auto stage_tile = [&](int tile, int buf) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      kbuf[buf][(lrow + 16 * u) * kRowU4 + lcol] = pre[u];
      float x[8];
      unpack2<T>(pre[u].x, x[0], x[1]); unpack2<T>(pre[u].y, x[2], x[3]);
      unpack2<T>(pre[u].z, x[4], x[5]); unpack2<T>(pre[u].w, x[6], x[7]);
      float ss = 0.f;
#pragma unroll
      for (int t = 0; t < 8; ++t) ss = fmaf(x[t], x[t], ss);
      ss = row16_sum(ss);                 // the 16 lanes of a DPP row hold one key
      const long row = (long)tile * kTok + lrow + 16 * u;
      if (lcol == 0 && blockIdx.y == 0 && row < rows) norms[row] = float_to_f16_bits(sqrtf(ss));
    }
  };

  int tile = blockIdx.x;
  if (tile < num_tiles) {
    load_tile(tile);
    stage_tile(tile, 0);
  }
  __syncthreads();

  int buf = 0;
  for (; tile < num_tiles; tile += gridDim.x, buf ^= 1) {
    const int next = tile + gridDim.x;
    const bool has_next = next < num_tiles;
    if (has_next) load_tile(next);

    // B operands: key j, k in [16s + 8h, 16s + 8h + 8)
    frag bfrag[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      uint4 u = kbuf[buf][j * kRowU4 + 2 * s + h];
      __builtin_memcpy(&bfrag[s], &u, 16);
    }
    uint32_t half[NA];
    if constexpr (NA >= 2) {
#pragma unroll
      for (int a = 0; a < NA; a += 2) {
        f32x16_t acc0 = {0}, acc1 = {0};
#pragma unroll
        for (int s = 0; s < 8; ++s) {
          acc0 = mma<T>::run(sfrag[a][s], bfrag[s], acc0);
          acc1 = mma<T>::run(sfrag[a + 1][s], bfrag[s], acc1);
        }
        half[a] = nonneg_bits16(acc0);
        half[a + 1] = nonneg_bits16(acc1);
      }
    } else {
      f32x16_t acc0 = {0};
#pragma unroll
      for (int s = 0; s < 8; ++s) acc0 = mma<T>::run(sfrag[0][s], bfrag[s], acc0);
      half[0] = nonneg_bits16(acc0);
    }
    // lane (h, j) holds PPW/2 consecutive code bits of key j, starting at bit
    // wave*PPW + h*PPW/2 of this workgroup's 4*PPW
    if constexpr (NA >= 2) {
#pragma unroll
      for (int a = 0; a < NA; a += 2)
        obuf[buf][j * OPITCH + wave * (PPW / 32) + h * (PPW / 64) + a / 2] = half[a] | (half[a + 1] << 16);
    } else {
      reinterpret_cast<uint16_t*>(obuf[buf])[(j * OPITCH + wave) * 2 + h] = (uint16_t)half[0];
    }

    if (has_next) stage_tile(next, buf ^ 1);
    __syncthreads();

    // coalesced copy of the tile's code words to HBM
    for (int idx = tid; idx < kTok * WPT; idx += 256) {
      const int tok = idx / WPT, wd = idx - tok * WPT;
      const long row = (long)tile * kTok + tok;
      if (row < rows)
        bits[(size_t)row * words_per_row + blockIdx.y * WPT + wd] = obuf[buf][tok * OPITCH + wd];
    }
  }
}

// ---------------------------------------------------------------- generic fp32-FMA path
constexpr int kGenTok = 8;

template <typename T>
__global__ void __launch_bounds__(256)
quantize_generic_kernel(const void* __restrict__ K, const void* __restrict__ S,
                        uint32_t* __restrict__ bits, uint16_t* __restrict__ norms, long rows, int d,
                        int m) {
  extern __shared__ float4 smem4[];
  float* kf = reinterpret_cast<float*>(smem4);      // [kGenTok][d]
  const int tid = threadIdx.x;
  const long row0 = (long)blockIdx.x * kGenTok;
  const int ntok = (int)min((long)kGenTok, rows - row0);
  for (int e = tid; e < ntok * d; e += 256) kf[e] = load1<T>(K, (size_t)row0 * d + e);
  __syncthreads();
  const int mw = m >> 5;
  for (int idx = tid; idx < ntok * mw; idx += 256) {
    const int tok = idx / mw, wd = idx - tok * mw;
    const float* kr = kf + tok * d;
    uint32_t word = 0;
    for (int i = 0; i < 32; ++i) {
      const size_t srow = (size_t)(wd * 32 + i) * d;
      float acc = 0.f;
      for (int t = 0; t < d; ++t) acc = fmaf(load1<T>(S, srow + t), kr[t], acc);
      word |= (acc >= 0.f ? 1u : 0u) << i;
    }
    bits[(size_t)(row0 + tok) * mw + wd] = word;
  }
  if (tid < ntok) {
    const float* kr = kf + tid * d;
    float ss = 0.f;
    for (int t = 0; t < d; ++t) ss = fmaf(kr[t], kr[t], ss);
    norms[row0 + tid] = float_to_f16_bits(sqrtf(ss));
  }
}

template <typename T, int PPW>
int launch_mfma(const void* K, const void* S, uint8_t* bits, uint16_t* norms, long rows, int m,
                hipStream_t st) {
  const long tiles = (rows + kTok - 1) / kTok;
  if (tiles > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  long gx = 2L * device_cu_count();       // two resident workgroups per CU, each loops over tiles
  if (gx > tiles) gx = tiles;
  dim3 grid((unsigned)gx, (unsigned)(m / (4 * PPW)));
  hipLaunchKernelGGL((quantize_mfma_kernel<T, PPW>), grid, dim3(256), 0, st,
                     static_cast<const uint16_t*>(K), static_cast<const uint16_t*>(S),
                     reinterpret_cast<uint32_t*>(bits), norms, rows, m, (int)tiles);
  return launch_status();
}

template <typename T>
int launch_mfma_m(const void* K, const void* S, uint8_t* bits, uint16_t* norms, long rows, int m,
                  hipStream_t st) {
  if (m % 512 == 0) return launch_mfma<T, 128>(K, S, bits, norms, rows, m, st);
  if (m % 256 == 0) return launch_mfma<T, 64>(K, S, bits, norms, rows, m, st);
  return launch_mfma<T, 32>(K, S, bits, norms, rows, m, st);
}

template <typename T>
int launch_generic(const void* K, const void* S, uint8_t* bits, uint16_t* norms, long rows, int d,
                   int m, hipStream_t st) {
  const long blocks = (rows + kGenTok - 1) / kGenTok;
  if (blocks > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(quantize_generic_kernel<T>, dim3((unsigned)blocks), dim3(256),
                     (size_t)kGenTok * d * sizeof(float), st, K, S,
                     reinterpret_cast<uint32_t*>(bits), norms, rows, d, m);
  return launch_status();
}

}  // namespace

int launch_quantize(const qjl_shape& sh, const void* K, const void* S, uint8_t* bits,
                    uint16_t* norms, hipStream_t st) {
  const long rows = (long)sh.batch * sh.kv_heads * sh.n;
  const bool mfma_ok = sh.d == 128 && sh.m % 128 == 0 && sh.dtype != QJL_F32;
  if (mfma_ok) {
    if (sh.dtype == QJL_BF16) return launch_mfma_m<bf16_t>(K, S, bits, norms, rows, sh.m, st);
    return launch_mfma_m<f16_t>(K, S, bits, norms, rows, sh.m, st);
  }
  switch (sh.dtype) {
    case QJL_F32: return launch_generic<f32_t>(K, S, bits, norms, rows, sh.d, sh.m, st);
    case QJL_F16: return launch_generic<f16_t>(K, S, bits, norms, rows, sh.d, sh.m, st);
    default: return launch_generic<bf16_t>(K, S, bits, norms, rows, sh.d, sh.m, st);
  }
}

}  // namespace qjl
