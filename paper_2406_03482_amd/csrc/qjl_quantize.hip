// Algorithm 1 steps 3-4 / Definition 3.1 Eq. (3): for every key store the packed
// sign bits of S k and the norm ||k||_2.
//
// Three paths:
//  * 16-bit keys with d = 128 and m a multiple of 128: K S^T is a dense
//    contraction and runs on the matrix cores (v_mfma_f32_32x32x16, fp32
//    accumulation); the accumulators are reduced to bits in registers, so the
//    projections never reach memory, and the norm is taken from the same
//    registers that feed the MFMAs.
//      - m <= 512: the sketch lives in LDS, every wave works on key tiles of
//        its own (quantize_slds_kernel);
//      - larger m: each wave keeps its share of S in registers for the whole
//        kernel and the four waves of a workgroup share key tiles staged in
//        LDS (quantize_mfma_kernel).
//  * anything else (fp32 keys, other d or m): plain fp32 FMA loops.
#include <type_traits>

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

typedef float f32x4_t __attribute__((ext_vector_type(4)));
template <typename T> struct mma16;
template <> struct mma16<bf16_t> {
  static __device__ __forceinline__ f32x4_t run(bf16x8_t a, bf16x8_t b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};
template <> struct mma16<f16_t> {
  static __device__ __forceinline__ f32x4_t run(f16x8_t a, f16x8_t b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
};

template <typename T> __device__ __forceinline__ float elem_to_float(uint16_t x);
template <> __device__ __forceinline__ float elem_to_float<bf16_t>(uint16_t x) { return bf16_bits_to_float(x); }
template <> __device__ __forceinline__ float elem_to_float<f16_t>(uint16_t x) { return f16_bits_to_float(x); }

// Outlier channels of a head as a bit mask over its 128 coordinates: entries
// outside [0, 128) are ignored and a channel listed twice counts once -- the
// rule of every quantize path and of the stacked sketch.
struct chan_mask { uint32_t w[4]; };
__device__ __forceinline__ chan_mask make_chan_mask(const int32_t* channels, int count) {
  chan_mask cm = {{0u, 0u, 0u, 0u}};
  for (int t = 0; t < count; ++t) {
    const int c = channels[t];
    if (c >= 0 && c < 128) cm.w[c >> 5] |= 1u << (c & 31);
  }
  return cm;
}
// sums of squares of the eight elements of one 16-byte chunk, split by the chunk's 8 mask bits
template <typename T> __device__ __forceinline__ void sumsq8_split(const uint32_t (&w)[4], uint32_t mb, float& in,
                                                                   float& out) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float a, b;
    unpack2<T>(w[i], a, b);
    const bool oa = (mb >> (2 * i)) & 1u, ob = (mb >> (2 * i + 1)) & 1u;
    out = fmaf(a, oa ? a : 0.f, out);
    in = fmaf(a, oa ? 0.f : a, in);
    out = fmaf(b, ob ? b : 0.f, out);
    in = fmaf(b, ob ? 0.f : b, in);
  }
}

// f(integral_constant<int, I>) for I = 0 .. N-1: indices that are constants to the compiler front end
template <int I, int N, typename F> __device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

constexpr int kTok = 64;        // keys per tile: two N = 32 MFMA sub-tiles
constexpr int kRowU4 = 18;      // LDS row pitch in 16-byte units: 256 B of key + 32 B pad (see kSPitch)

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// sum of squares of the eight 16-bit elements of one 16-byte chunk, fp32 accumulation
// (v_dot2_f32_bf16 / v_dot2_f32_f16: two products and the add per instruction)
template <typename T> __device__ __forceinline__ float sumsq8(const uint4& u);
template <> __device__ __forceinline__ float sumsq8<bf16_t>(const uint4& u) {
  bf16x2_t p[4];
  __builtin_memcpy(p, &u, 16);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) s = __builtin_amdgcn_fdot2_f32_bf16(p[i], p[i], s, false);
  return s;
}
template <> __device__ __forceinline__ float sumsq8<f16_t>(const uint4& u) {
  f16x2_t p[4];
  __builtin_memcpy(p, &u, 16);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) s = __builtin_amdgcn_fdot2(p[i], p[i], s, false);
  return s;
}

template <typename T> __device__ __forceinline__ float sumsq8v(const u32x4& v) {
  uint4 u = make_uint4(v[0], v[1], v[2], v[3]);
  return sumsq8<T>(u);
}

// Sign extraction: v_alignbit(t, acc, 31) shifts the IEEE sign bit of an accumulator
// into t; sixteen of them (v = 15..0) give bit v = sign of acc[v], and the code
// bit is its complement ([acc >= 0]).  A sum that starts from +0 can only be -0
// if it is within rounding of zero.

// PPW = projections per wave (32, 64 or 128); a workgroup of four waves covers
// 4*PPW projections, blockIdx.y selects which block of 4*PPW out of m.
// Per iteration a workgroup turns one tile of 64 keys into 64 code rows:
//   HBM -> registers (issued one tile ahead) -> norm + LDS (padded rows)
//   LDS -> MFMA B operands, S from registers, accumulators -> bits in registers
//   bits -> LDS -> HBM as whole rows (16 bytes per lane, contiguous)
//
// The rows are cut into segments (blockIdx.z): one segment holding every row when
// all keys share one sketch, or one segment per (batch, kv head) when every head
// has a sketch of its own (seg_stride elements apart).  DUAL (Section 4.1,
// outlier channels): the code is that of a stacked sketch whose rows already
// exclude / keep only the head's `count` outlier channels, and two norms are
// stored: of the key without those channels and of those channels alone.
// CW = waves that run MFMAs (4, or 3 for code sizes that are 3 x 128 bits: the
// fourth wave then only helps with loading and takes the norms).
template <typename T, int PPW, bool DUAL, int CW>
__global__ void __launch_bounds__(256, 2)
quantize_mfma_kernel(const uint16_t* __restrict__ K, const uint16_t* __restrict__ S, size_t seg_stride,
                     uint32_t* __restrict__ bits, uint16_t* __restrict__ norms,
                     uint16_t* __restrict__ norms_out, const int32_t* __restrict__ channels, int count,
                     long rows, int m, int num_tiles, int seg0) {
  using frag = typename mma<T>::frag;
  {
    const size_t seg = (size_t)seg0 + blockIdx.z;
    K += seg * (size_t)rows * 128;
    S += seg * seg_stride;
    bits += seg * (size_t)rows * (size_t)(m >> 5);
    norms += seg * (size_t)rows;
    if constexpr (DUAL) {
      norms_out += seg * (size_t)rows;
      channels += seg * (size_t)count;
    }
  }
  constexpr int NA = PPW / 32;            // 32x32 MFMA tiles per wave along the projections
  constexpr int WPT = CW * PPW / 32;      // code words per key written by this workgroup
  __shared__ uint4 kbuf[2][kTok * kRowU4];
  __shared__ uint4 obuf[2][kTok * WPT / 4];
  __shared__ float nsq[2][kTok];           // squared norms of the tile's keys (DUAL: without the outlier channels)
  __shared__ float nsq_out[DUAL ? 2 : 1][kTok];   // DUAL: squared norms of the outlier channels

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int h = lane >> 5;                // which 8 of the 16 k of an MFMA step this lane feeds
  const int j = lane & 31;                // A: row of the S tile, B/D: key of the sub-tile
  const int proj_base = blockIdx.y * (CW * PPW) + wave * PPW;
  const bool computes = CW == 4 || wave < CW;   // uniform per wave
  const int words_per_row = m >> 5;

  // ---- this wave's rows of S, resident in registers as MFMA A operands.
  // Row rho of tile a is projection  proj_base + ((rho>>2)&1)*PPW/2 + 16a + 4(rho>>3) + (rho&3):
  // with the 32x32 accumulator layout (register v of lane (h, j) is row
  // 8(v/4) + 4h + v%4) lane (h, j) then owns projections
  // proj_base + h*PPW/2 + 16a + v, v = 0..15 -- consecutive code bits of key j.
  // PPW == 128 (W16): v_mfma_f32_16x16x32 -- the 32x32x16 form runs at half the rate on this chip.  Eight A
  // tiles of 16 projections x four steps of 32 elements; lane (q16, j16) = (lane >> 4, lane & 15) holds row
  // j16, elements 32s + 8 q16 .. + 7.  Row rho of tile a is projection proj_base + 32 (rho >> 2) + 4a + (rho & 3):
  // accumulator register r of lane (q16, j16) is then projection proj_base + 32 q16 + 4a + r of key j16, so the
  // lane's 32 sign bits (a = 0..7, r = 0..3) are one whole code word, word wave * 4 + q16 of the key's row.
  constexpr bool W16 = PPW == 128;
  const int q16 = lane >> 4, j16 = lane & 15;
  frag sfrag[W16 ? 8 : NA][W16 ? 4 : 8];
  if (computes) {
    if constexpr (W16) {
#pragma unroll
      for (int a = 0; a < 8; ++a) {
        const int srow = proj_base + 32 * (j16 >> 2) + 4 * a + (j16 & 3);
        const uint4* sp = reinterpret_cast<const uint4*>(S + (size_t)srow * 128 + 8 * q16);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          uint4 u = sp[4 * s];
          __builtin_memcpy(&sfrag[a][s], &u, 16);
        }
      }
    } else {
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
    }
  }

  // ---- loader: thread -> (row lrow + 16u, 16-byte column lcol) of a tile, u = 0..3
  const int lrow = tid >> 4, lcol = tid & 15;
  uint4 pre[4];
  // addresses are a uniform 64-bit tile base (scalar ALU) plus a 32-bit lane
  // offset fixed for the whole kernel: no vector ALU work per tile
  const uint32_t koff = (uint32_t)(lrow * 128 + lcol * 8);
  auto load_tile = [&](int tile) {
    const long row0 = (long)tile * kTok;
    if (row0 + kTok <= rows) {            // uniform: whole tile inside K
      const uint16_t* kp = K + (size_t)row0 * 128;
#pragma unroll
      for (int u = 0; u < 4; ++u) pre[u] = *reinterpret_cast<const uint4*>(kp + (koff + (uint32_t)(u * 16 * 128)));
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        long row = row0 + lrow + 16 * u;
        if (row >= rows) row = rows - 1;  // clamp: stay inside K, results of such rows are dropped
        pre[u] = *reinterpret_cast<const uint4*>(K + (size_t)row * 128 + lcol * 8);
      }
    }
  };
  // DUAL: the 8 mask bits of this thread's 16-byte column; the two parts are summed
  // separately (a difference of the whole and the outlier part would cancel)
  uint32_t col_mask = 0;
  if constexpr (DUAL) {
    const chan_mask cm = make_chan_mask(channels, count);
    col_mask = (cm.w[lcol >> 2] >> (8 * (lcol & 3))) & 0xFFu;
  }
  auto stage_tile = [&](int buf) {
    float ss[4], so[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      kbuf[buf][(lrow + 16 * u) * kRowU4 + lcol] = pre[u];
      if (DUAL && col_mask != 0) {
        const uint32_t w[4] = {pre[u].x, pre[u].y, pre[u].z, pre[u].w};
        ss[u] = 0.f;
        sumsq8_split<T>(w, col_mask, ss[u], so[u]);
      } else {
        ss[u] = sumsq8<T>(pre[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) ss[u] = row16_sum(ss[u]);   // the 16 lanes of a DPP row hold one key
    if constexpr (DUAL) {
#pragma unroll
      for (int u = 0; u < 4; ++u) so[u] = row16_sum(so[u]);
    }
    if (lcol == 0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) nsq[buf][lrow + 16 * u] = ss[u];
      if constexpr (DUAL) {
#pragma unroll
        for (int u = 0; u < 4; ++u) nsq_out[buf][lrow + 16 * u] = so[u];
      }
    }
  };

  int tile = blockIdx.x;
  if (tile < num_tiles) {
    load_tile(tile);
    stage_tile(0);
  }
  // All loads issued so far (the S fragments above all) must have landed before
  // the loop: otherwise the loop body carries waits for them that would also
  // wait for each iteration's prefetch of the next tile.
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  int buf = 0;
  for (; tile < num_tiles; tile += gridDim.x, buf ^= 1) {
    const int next = tile + gridDim.x;
    const bool has_next = next < num_tiles;
    if (has_next) load_tile(next);
    // the tile's norms: its squared norms and its keys have been in LDS since the
    // previous iteration's barrier and stay there until this iteration's barrier
    if (blockIdx.y == 0 && wave == 3) {               // one wave, one key per lane: a single square root
      const long trow = (long)tile * kTok + lane;
      if constexpr (DUAL) {
        if (trow < rows) norms_out[trow] = float_to_f16_bits(sqrtf(nsq_out[buf][lane]));
      }
      if (trow < rows) norms[trow] = float_to_f16_bits(sqrtf(nsq[buf][lane]));
    }

    // ---- MFMA phase.  The tile's work is cut into NU units of two accumulator
    // chains (8 MFMAs each).  While unit u accumulates, the sign bits of unit
    // u-1 are extracted (v_alignbit) in the shadow of its MFMAs, and the B
    // operand of step g+2 is fetched from LDS, so the matrix pipe never waits
    // for the vector ALU or for LDS.  sched_barrier keeps that interleaving.
    if constexpr (W16) {
    if (computes) {
      // A unit = one group of 16 keys against the wave's 128 projections: 4 steps x 8 MFMAs on eight
      // independent accumulators.  While unit c accumulates, the sign bits of unit c-1 are shifted into its
      // code word (one v_alignbit per accumulator register, highest bit first), and the B operand of two
      // steps ahead comes from LDS: 1 KB per eight MFMAs.
      auto lds_b16 = [&](int g) {                 // step g = 4c + s: key 16c + j16, elements 32s + 8 q16 .. + 7
        frag f;
        const uint4 u4 = kbuf[buf][(16 * (g >> 2) + j16) * kRowU4 + 4 * (g & 3) + q16];
        __builtin_memcpy(&f, &u4, 16);
        return f;
      };
      frag bq[3];
      bq[0] = lds_b16(0);
      bq[1] = lds_b16(1);
      const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
      f32x4_t acc[2][8];
      uint32_t tb = 0u;
      uint32_t* ocol = reinterpret_cast<uint32_t*>(obuf[buf]) + j16 * WPT + wave * 4 + q16;
      static_for<0, 5>([&](auto uc) {             // round 4 only drains the last unit's bits
        constexpr int u = decltype(uc)::value, par = u & 1;
        static_for<0, 4>([&](auto sc) {
          constexpr int s = decltype(sc)::value, g = u * 4 + s;
          if constexpr (g + 2 < 16) bq[(g + 2) % 3] = lds_b16(g + 2);
          if constexpr (u < 4) {
#pragma unroll
            for (int a = 0; a < 8; ++a)
              acc[par][a] = mma16<T>::run(sfrag[a][s], bq[g % 3], s == 0 ? zero : acc[par][a]);
          }
          if constexpr (u > 0) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
              for (int r = 3; r >= 0; --r)
                tb = __builtin_amdgcn_alignbit(tb, __float_as_uint(acc[par ^ 1][7 - 2 * s - t][r]), 31);
          }
          __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr (u > 0) {
          asm volatile("" : "+v"(tb));             // the bits are taken here, not where they are stored
          ocol[(u - 1) * 16 * WPT] = ~tb;         // bit = [acc >= 0]
          tb = 0u;
        }
      });
    }
    } else if (computes) {
    constexpr int NU = NA >= 2 ? NA : 1;
    auto sub_of = [](int u, int c) { return NA >= 2 ? u / (NA / 2) : c; };
    auto a_of = [](int u, int c) { return NA >= 2 ? 2 * (u % (NA / 2)) + c : 0; };
    auto lds_b = [&](int sub, int s) {          // key sub*32 + j, k in [16s + 8h, 16s + 8h + 8)
      frag f;
      const uint4 u4 = kbuf[buf][(sub * 32 + j) * kRowU4 + 2 * s + h];
      __builtin_memcpy(&f, &u4, 16);
      return f;
    };
    constexpr int kSteps = NU * 8;
    frag bq[3][2];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      bq[g][0] = lds_b(sub_of(g / 8, 0), g % 8);
      if constexpr (NA == 1) bq[g][1] = lds_b(1, g % 8);
    }
    f32x16_t acc[2][2];
    uint32_t tb[2] = {0u, 0u};
    uint32_t half[2 * NU];
#pragma unroll
    for (int u = 0; u <= NU; ++u) {             // round NU only drains the last unit's bits
      const int par = u & 1;
      if (u < NU) {
#pragma unroll
        for (int v = 0; v < 16; ++v) { acc[par][0][v] = 0.f; acc[par][1][v] = 0.f; }
      }
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const int g = u * 8 + s;
        if (g + 2 < kSteps) {
          bq[(g + 2) % 3][0] = lds_b(sub_of((g + 2) / 8, 0), (g + 2) % 8);
          if constexpr (NA == 1) bq[(g + 2) % 3][1] = lds_b(1, (g + 2) % 8);
        }
        if (u < NU) {
          acc[par][0] = mma<T>::run(sfrag[a_of(u, 0)][s], bq[g % 3][0], acc[par][0]);
          acc[par][1] = mma<T>::run(sfrag[a_of(u, 1)][s], bq[g % 3][NA == 1 ? 1 : 0], acc[par][1]);
        }
        if (u > 0) {
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            tb[c] = __builtin_amdgcn_alignbit(tb[c], __float_as_uint(acc[par ^ 1][c][15 - 2 * s]), 31);
            tb[c] = __builtin_amdgcn_alignbit(tb[c], __float_as_uint(acc[par ^ 1][c][14 - 2 * s]), 31);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      if (u > 0) {                              // bit v = [acc[v] >= 0]
        half[2 * (u - 1)] = (~tb[0]) & 0xFFFFu;
        half[2 * (u - 1) + 1] = (~tb[1]) & 0xFFFFu;
        tb[0] = 0u;
        tb[1] = 0u;
      }
    }
    // lane (h, j) holds PPW/2 consecutive code bits of keys j and 32 + j, starting
    // at bit wave*PPW + h*PPW/2 of this workgroup's CW*PPW
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      uint32_t* orow = reinterpret_cast<uint32_t*>(obuf[buf]) + (sub * 32 + j) * WPT;
      if constexpr (NA == 4) {
        *reinterpret_cast<uint2*>(orow + wave * 4 + h * 2) =
            make_uint2(half[4 * sub] | (half[4 * sub + 1] << 16), half[4 * sub + 2] | (half[4 * sub + 3] << 16));
      } else if constexpr (NA == 2) {
        orow[wave * 2 + h] = half[2 * sub] | (half[2 * sub + 1] << 16);
      } else {
        reinterpret_cast<uint16_t*>(orow)[wave * 2 + h] = (uint16_t)half[sub];
      }
    }
    }

    if (has_next) stage_tile(buf ^ 1);
    __syncthreads();

    // whole code rows and the tile's norms go to HBM, 16 contiguous bytes per lane
    constexpr int kChunksPerRow = WPT / 4;
    const long trow0 = (long)tile * kTok;
    const bool full = trow0 + kTok <= rows;           // uniform
    if (tid < kTok * kChunksPerRow) {
      const int tok = tid / kChunksPerRow, part = tid % kChunksPerRow;
      if (full || trow0 + tok < rows) {
        uint32_t* tb0 = bits + (size_t)trow0 * words_per_row;            // uniform
        const uint32_t off = (uint32_t)(tok * words_per_row + blockIdx.y * WPT + part * 4);
        *reinterpret_cast<uint4*>(tb0 + off) = obuf[buf][tid];
      }
    }
  }
}

// ---------------------------------------------------------------- sketch in LDS, keys in registers
// For m <= 512 the whole sketch fits in the CU's LDS (m rows of 256 B + 32 B pad).
// Then the roles swap: S is the MFMA A operand read from LDS, a wave's 64 keys
// are the B operands and stay in its registers.  Keys are fetched as whole
// 128-byte lines one tile ahead and rearranged into the MFMA layout through
// 2 KB of LDS private to the wave.  A wave owns its keys from load to store:
// after the one barrier behind the copy of S no wave ever waits for another,
// and the two waves of a SIMD fill the matrix pipe for each other while one of
// them rearranges keys, takes norms or stores.
// LDS pitch of a sketch row in 16-byte units: 256 B of sketch + 32 B pad.  The LDS
// spreads a 16-lane ds_read_b128 over its banks by address bits 4-7 with bit 8
// folded into bit 4, so a pitch of 18 units gives the sixteen rows of an A
// fragment sixteen different bank groups (4 cycles per wave read); 17 units
// leaves them pairwise on the same group (8 cycles; SQ_LDS_BANK_CONFLICT counted
// 4 cycles per read with it).
constexpr int kSPitch = 18;

// x summed over the four 16-lane rows of a wave, in every lane
// (v_permlane32_swap, v_permlane16_swap: no trip through LDS)
__device__ __forceinline__ float sum_rows4(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);   // {lower half twice, upper half twice}
  const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const uint32_t v = __float_as_uint(y);
  const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);   // {even rows twice, odd rows twice}
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// v_mfma_f32_16x16x32: a unit is 16 projections against four sub-tiles of 16
// keys (four accumulator chains of four MFMAs, 4 registers each), so two sets
// of accumulators fit and the sign bits of unit u-1 are taken between the MFMAs
// of unit u (one v_alignbit per accumulator register).  Lane (q, j) =
// (lane >> 4, lane & 15): A row / key j, elements 32s + 8q .. 32s + 8q + 7 of
// step s; accumulator register v is projection row 4q + v of the unit.  LDS
// row (b, rho) holds projection (rho>>2)*m/4 + 32(b>>3) + 4(7 - (b&7)) + (rho&3):
// shifting one bit per register into a word, units in order, leaves lane (q, j)
// with m/4 consecutive code bits of key j -- m/32 contiguous bytes, stored from
// registers.
template <typename T, int NB, bool DUAL>
__global__ void __launch_bounds__(512, 1)
quantize_slds_kernel(const uint16_t* __restrict__ K, const uint16_t* __restrict__ S, size_t seg_stride,
                       uint32_t* __restrict__ bits, uint16_t* __restrict__ norms,
                       uint16_t* __restrict__ norms_out, const int32_t* __restrict__ channels, int count,
                       long rows, int num_tiles, int seg0) {
  using frag = typename mma<T>::frag;
  constexpr int m = NB * 32;
  constexpr int NU = m / 16;              // units
  constexpr int NW = NB / 4;              // code words a lane holds per key
  extern __shared__ uint4 sbuf[];         // [m][kSPitch]
  {
    const size_t seg = (size_t)seg0 + blockIdx.z;
    K += seg * (size_t)rows * 128;
    S += seg * seg_stride;
    bits += seg * (size_t)rows * (size_t)NB;
    norms += seg * (size_t)rows;
    if constexpr (DUAL) {
      norms_out += seg * (size_t)rows;
      channels += seg * (size_t)count;
    }
  }
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int q = lane >> 4;
  const int j = lane & 15;

  for (int idx = tid; idx < m * 16; idx += 512) {
    const int lr = idx >> 4, c = idx & 15;
    const int b = lr >> 4, rho = lr & 15;
    const int srow = (rho >> 2) * (m / 4) + 32 * (b >> 3) + 4 * (7 - (b & 7)) + (rho & 3);
    sbuf[lr * kSPitch + c] = *reinterpret_cast<const uint4*>(S + (size_t)srow * 128 + c * 8);
  }

  // DUAL: which of this lane's 32 elements are outlier channels.  Bit 8s + e of
  // omask = element 32s + 8q + e; smask (uniform) = steps with any such element.
  uint32_t omask = 0;
  uint32_t smask = 0;
  if constexpr (DUAL) {
    const chan_mask cm = make_chan_mask(channels, count);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if (cm.w[s] != 0) smask |= 1u << s;
      omask |= ((cm.w[s] >> (8 * q)) & 0xFFu) << (8 * s);
    }
  }

  // pre[2*g + p], g = 2*c + kh: keys 16*c + 8*p + (lane >> 3), chunks 8*kh + (lane & 7)
  u32x4 pre[16];
  const int lrow = lane >> 3, lchk = lane & 7;
  const uint32_t koff = (uint32_t)(lrow * 128 + lchk * 8);
  auto load_tile = [&](int wt) {
    const long row0 = (long)wt * kTok;
    if (row0 + kTok <= rows) {            // uniform: whole tile inside K
      const uint16_t* kp = K + (size_t)row0 * 128;
      static_for<0, 16>([&](auto pc) {
        constexpr int p = decltype(pc)::value, g = p >> 1;
        constexpr int key = 16 * (g >> 1) + 8 * (p & 1), kh = g & 1;
        pre[p] = *reinterpret_cast<const u32x4*>(kp + (koff + (uint32_t)(key * 128 + kh * 64)));
      });
    } else {
      static_for<0, 16>([&](auto pc) {
        constexpr int p = decltype(pc)::value, g = p >> 1;
        constexpr int key = 16 * (g >> 1) + 8 * (p & 1), kh = g & 1;
        long row = row0 + key + lrow;
        if (row >= rows) row = rows - 1;  // clamp: stay inside K, results of such rows are dropped
        pre[p] = *reinterpret_cast<const u32x4*>(K + (size_t)row * 128 + kh * 64 + lchk * 8);
      });
    }
  };

  uint32_t* next_tile = reinterpret_cast<uint32_t*>(sbuf + 16);                    // in the padding of sketch row 0
  u32x4* stage = reinterpret_cast<u32x4*>(sbuf + m * kSPitch + wave * 128);        // this wave's 16 keys x 8 chunks
  const int per_wg = (num_tiles + (int)gridDim.x - 1) / (int)gridDim.x;
  const int tile0 = blockIdx.x * per_wg;
  const int ntile = min(per_wg, num_tiles - tile0);      // may be <= 0 for the last workgroups
  if (tid == 0) *next_tile = 8u;
  int wt = wave;                          // index inside the workgroup's range
  if (wt < ntile) load_tile(tile0 + wt);
  __syncthreads();                        // S is in LDS; the only barrier of the kernel
  auto grab_tile = [&]() {
    uint32_t v = 0;
    if (lane == 0) v = atomicAdd(next_tile, 1u);
    return (int)__builtin_amdgcn_readfirstlane(v);
  };
  const int abase = j * kSPitch + q;

  // lane (q, j) holds words q*NW .. q*NW + NW - 1 of the code rows of keys 16*c + j
  uint32_t code[4][NW];
  auto store_codes = [&](int tile) {
    const long r0 = (long)tile * kTok;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const long row = r0 + c * 16 + j;
      if (row < rows) {
        uint32_t* dst = bits + (size_t)row * NB + q * NW;
        if constexpr (NW == 4) {
          *reinterpret_cast<uint4*>(dst) = make_uint4(code[c][0], code[c][1], code[c][2], code[c][3]);
        } else if constexpr (NW == 2) {
          *reinterpret_cast<uint2*>(dst) = make_uint2(code[c][0], code[c][1]);
        } else {
#pragma unroll
          for (int w = 0; w < NW; ++w) dst[w] = code[c][w];
        }
      }
    }
  };

  int done = -1;                          // tile whose code words wait in registers
  while (wt < ntile) {
    // cur[c][s]: key 16*c + j, chunk 4s + q
    u32x4 cur[4][4];
    static_for<0, 8>([&](auto gc) {
      constexpr int g = decltype(gc)::value;
      stage[lrow * 8 + (lchk ^ ((lrow >> 1) & 7))] = pre[2 * g];
      stage[(lrow + 8) * 8 + (lchk ^ (((lrow + 8) >> 1) & 7))] = pre[2 * g + 1];
      __builtin_amdgcn_wave_barrier();
      static_for<0, 2>([&](auto tc) {
        constexpr int t = decltype(tc)::value;
        cur[g >> 1][2 * (g & 1) + t] = stage[j * 8 + ((4 * t + q) ^ ((j >> 1) & 7))];
      });
      __builtin_amdgcn_wave_barrier();
    });
    if (done >= 0) store_codes(done);     // behind the wait for this tile's keys, before the next prefetch
    const int wt_next = grab_tile();
    load_tile(tile0 + min(wt_next, ntile - 1));

    const long row0 = (long)(tile0 + wt) * kTok;
    // ---- norms: a key's elements are split over lanes (0..3, j)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      // DUAL: ss is the inlier part alone; the two parts are summed separately (a
      // difference of the whole and the outlier part would cancel for large outliers)
      float ss = 0.f, so = 0.f;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        if (DUAL && ((smask >> s) & 1u)) {            // uniform
          const uint32_t w[4] = {cur[c][s][0], cur[c][s][1], cur[c][s][2], cur[c][s][3]};
          sumsq8_split<T>(w, (omask >> (8 * s)) & 0xFFu, ss, so);
        } else {
          ss += sumsq8v<T>(cur[c][s]);
        }
      }
      ss = sum_rows4(ss);
      const long row = row0 + c * 16 + j;
      // v_sqrt_f32 (1 ulp) is ample for a value that is then rounded to binary16
      if constexpr (DUAL) {
        so = sum_rows4(so);
        if (q == 0 && row < rows) norms_out[row] = float_to_f16_bits(__builtin_amdgcn_sqrtf(so));
      }
      if (q == 0 && row < rows) norms[row] = float_to_f16_bits(__builtin_amdgcn_sqrtf(ss));
    }

    // ---- MFMA phase
    auto lds_a = [&](int g) {
      frag f;
      const uint4 u4 = sbuf[abase + (g >> 2) * (16 * kSPitch) + 4 * (g & 3)];
      __builtin_memcpy(&f, &u4, 16);
      return f;
    };
    auto key_b = [&](int c, int s) {
      frag f;
      __builtin_memcpy(&f, &cur[c][s], 16);
      return f;
    };
    constexpr int kSteps = NU * 4;
    frag aq[3];
    aq[0] = lds_a(0);
    aq[1] = lds_a(1);
    const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
    f32x4_t acc[2][4];
    uint32_t tb[4] = {0u, 0u, 0u, 0u};
    static_for<0, NU + 1>([&](auto uc) {          // round NU only drains the last unit's bits
      constexpr int u = decltype(uc)::value, par = u & 1;
      static_for<0, 4>([&](auto sc) {
        constexpr int s = decltype(sc)::value, g = u * 4 + s;
        if constexpr (g + 2 < kSteps) aq[(g + 2) % 3] = lds_a(g + 2);
        if constexpr (u < NU) {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            acc[par][c] = mma16<T>::run(aq[g % 3], key_b(c, s), s == 0 ? zero : acc[par][c]);
        }
        if constexpr (u > 0) {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            tb[c] = __builtin_amdgcn_alignbit(tb[c], __float_as_uint(acc[par ^ 1][c][3 - s]), 31);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
      if constexpr (u > 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          asm volatile("" : "+v"(tb[c]));           // the bits are taken here, not where they are stored
          if constexpr ((u - 1) % 8 == 7) {         // bit = [acc >= 0]
            code[c][(u - 1) / 8] = ~tb[c];
            tb[c] = 0u;
          }
        }
      }
    });

    done = tile0 + wt;
    wt = wt_next;
  }
  if (done >= 0) store_codes(done);
}

// ---------------------------------------------------------------- generic fp32-FMA path
constexpr int kGenTok = 8;

template <typename T, bool DUAL>
__global__ void __launch_bounds__(256)
quantize_generic_kernel(const void* __restrict__ K, const void* __restrict__ S, size_t seg_stride,
                        uint32_t* __restrict__ bits, uint16_t* __restrict__ norms,
                        uint16_t* __restrict__ norms_out, const int32_t* __restrict__ channels, int count,
                        long rows, int d, int m, int seg0) {
  extern __shared__ float4 smem4[];
  float* kf = reinterpret_cast<float*>(smem4);      // [kGenTok][d]
  const int tid = threadIdx.x;
  const size_t seg = (size_t)seg0 + blockIdx.y;
  const size_t k0 = seg * (size_t)rows * d;          // first element of the segment's keys
  const size_t s0 = seg * seg_stride;
  const size_t r0 = seg * (size_t)rows;
  const long row0 = (long)blockIdx.x * kGenTok;
  const int ntok = (int)min((long)kGenTok, rows - row0);
  for (int e = tid; e < ntok * d; e += 256) kf[e] = load1<T>(K, k0 + (size_t)row0 * d + e);
  __syncthreads();
  const int mw = m >> 5;
  for (int idx = tid; idx < ntok * mw; idx += 256) {
    const int tok = idx / mw, wd = idx - tok * mw;
    const float* kr = kf + tok * d;
    uint32_t word = 0;
    for (int i = 0; i < 32; ++i) {
      const size_t srow = s0 + (size_t)(wd * 32 + i) * d;
      float acc = 0.f;
      for (int t = 0; t < d; ++t) acc = fmaf(load1<T>(S, srow + t), kr[t], acc);
      word |= (acc >= 0.f ? 1u : 0u) << i;
    }
    bits[(r0 + row0 + tok) * mw + wd] = word;
  }
  if (tid < ntok) {
    const float* kr = kf + tid * d;
    // DUAL: a coordinate is an outlier if the head's list names it (entries outside
    // [0, d) match nothing, a repeated entry matches once); the parts are summed separately
    float ss = 0.f, so = 0.f;
    for (int t = 0; t < d; ++t) {
      bool is_out = false;
      if constexpr (DUAL) {
        for (int u = 0; u < count; ++u) is_out |= channels[seg * (size_t)count + u] == t;
      }
      if (is_out) so = fmaf(kr[t], kr[t], so);
      else ss = fmaf(kr[t], kr[t], ss);
    }
    if constexpr (DUAL) norms_out[r0 + row0 + tid] = float_to_f16_bits(sqrtf(so));
    norms[r0 + row0 + tid] = float_to_f16_bits(sqrtf(ss));
  }
}

struct quant_io {
  const void* K; const void* S; size_t seg_stride;      // seg_stride = 0: one sketch for all rows
  uint8_t* bits; uint16_t* norms; uint16_t* norms_out;  // norms_out / channels: outlier split only
  const int32_t* channels; int count;
  long segments; long rows;                             // rows per segment
  int d, m;                                             // m = all code bits of a key
};

template <typename T, int PPW, bool DUAL, int CW>
int launch_mfma(const quant_io& q, hipStream_t st) {
  const long tiles = (q.rows + kTok - 1) / kTok;
  if (tiles > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  // about two resident workgroups per CU in total, each looping over tiles of its segment
  long gx = (2L * device_cu_count() + q.segments - 1) / q.segments;
  if (gx > tiles) gx = tiles;
  for (long s0 = 0; s0 < q.segments; s0 += 65535) {
    const long nz = q.segments - s0 < 65535 ? q.segments - s0 : 65535;
    dim3 grid((unsigned)gx, (unsigned)(q.m / (CW * PPW)), (unsigned)nz);
    hipLaunchKernelGGL((quantize_mfma_kernel<T, PPW, DUAL, CW>), grid, dim3(256), 0, st,
                       static_cast<const uint16_t*>(q.K), static_cast<const uint16_t*>(q.S), q.seg_stride,
                       reinterpret_cast<uint32_t*>(q.bits), q.norms, q.norms_out, q.channels, q.count,
                       q.rows, q.m, (int)tiles, (int)s0);
  }
  return launch_status();
}

template <typename T, int NB, bool DUAL>
int launch_slds(const quant_io& q, hipStream_t st) {
  const long tiles = (q.rows + kTok - 1) / kTok;
  if (tiles > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  // the sketch (the tile counter sits in its padding), 2 KB per wave to rearrange keys: 160 KiB at m = 512
  constexpr size_t lds = (size_t)NB * 32 * kSPitch * 16 + 8 * 2048;
  static_assert(lds <= 160 * 1024, "the sketch and the staging buffers must fit one CU's LDS");
  static std::atomic<uint64_t> lds_set{0};   // the kernel needs more than the default 64 KB of LDS
  const int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(&quantize_slds_kernel<T, NB, DUAL>), lds, lds_set);
  if (rc_lds != QJL_OK) return rc_lds;
  // one workgroup of eight waves per CU in total, each owning a range of its segment's tiles
  long gx = (device_cu_count() + q.segments - 1) / q.segments;
  if (gx > (tiles + 7) / 8) gx = (tiles + 7) / 8;
  for (long s0 = 0; s0 < q.segments; s0 += 65535) {
    const long nz = q.segments - s0 < 65535 ? q.segments - s0 : 65535;
    dim3 grid((unsigned)gx, 1u, (unsigned)nz);
    hipLaunchKernelGGL((quantize_slds_kernel<T, NB, DUAL>), grid, dim3(512), lds, st,
                       static_cast<const uint16_t*>(q.K), static_cast<const uint16_t*>(q.S), q.seg_stride,
                       reinterpret_cast<uint32_t*>(q.bits), q.norms, q.norms_out, q.channels, q.count,
                       q.rows, (int)tiles, (int)s0);
  }
  return launch_status();
}

template <typename T, bool DUAL>
int launch_mfma_m(const quant_io& q, hipStream_t st) {
  if (q.rows > 0) {
    switch (q.m) {                        // the whole sketch fits in LDS
      case 128: return launch_slds<T, 4, DUAL>(q, st);
      case 256: return launch_slds<T, 8, DUAL>(q, st);
      case 384: return launch_slds<T, 12, DUAL>(q, st);
      case 512: return launch_slds<T, 16, DUAL>(q, st);
      default: break;
    }
  }
  if (q.m % 512 == 0) return launch_mfma<T, 128, DUAL, 4>(q, st);
  if (q.m % 384 == 0) return launch_mfma<T, 128, DUAL, 3>(q, st);   // one pass over the keys instead of three
  if (q.m % 256 == 0) return launch_mfma<T, 64, DUAL, 4>(q, st);
  return launch_mfma<T, 32, DUAL, 4>(q, st);
}

template <typename T, bool DUAL>
int launch_generic(const quant_io& q, hipStream_t st) {
  const long blocks = (q.rows + kGenTok - 1) / kGenTok;
  if (blocks > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  for (long s0 = 0; s0 < q.segments; s0 += 65535) {
    const long ny = q.segments - s0 < 65535 ? q.segments - s0 : 65535;
    hipLaunchKernelGGL((quantize_generic_kernel<T, DUAL>), dim3((unsigned)blocks, (unsigned)ny), dim3(256),
                       (size_t)kGenTok * q.d * sizeof(float), st, q.K, q.S, q.seg_stride,
                       reinterpret_cast<uint32_t*>(q.bits), q.norms, q.norms_out, q.channels, q.count,
                       q.rows, q.d, q.m, (int)s0);
  }
  return launch_status();
}

template <bool DUAL>
int launch_any(const quant_io& q, int dtype, hipStream_t st) {
  const bool mfma_ok = q.d == 128 && q.m % 128 == 0 && dtype != QJL_F32;
  if (mfma_ok) {
    if (dtype == QJL_BF16) return launch_mfma_m<bf16_t, DUAL>(q, st);
    return launch_mfma_m<f16_t, DUAL>(q, st);
  }
  switch (dtype) {
    case QJL_F32: return launch_generic<f32_t, DUAL>(q, st);
    case QJL_F16: return launch_generic<f16_t, DUAL>(q, st);
    default: return launch_generic<bf16_t, DUAL>(q, st);
  }
}

}  // namespace

int launch_quantize(const qjl_shape& sh, const void* K, const void* S, uint8_t* bits,
                    uint16_t* norms, hipStream_t st) {
  quant_io q{K, S, 0, bits, norms, nullptr, nullptr, 0, 1, (long)sh.batch * sh.kv_heads * sh.n, sh.d, sh.m};
  return launch_any<false>(q, sh.dtype, st);
}

// Two-part codes (Section 4.1): S_dual holds one stacked sketch [sh.m + m_out, d] per
// (batch, kv head); channels [B,Hkv,count] lists that head's outlier channels.
int launch_quantize_dual(const qjl_shape& sh, int m_out, const void* K, const void* S_dual,
                         const int32_t* channels, int count, uint8_t* bits, uint16_t* norms_in,
                         uint16_t* norms_out, hipStream_t st) {
  const int mt = sh.m + m_out;
  quant_io q{K, S_dual, (size_t)mt * sh.d, bits, norms_in, norms_out, channels, count,
             (long)sh.batch * sh.kv_heads, (long)sh.n, sh.d, mt};
  return launch_any<true>(q, sh.dtype, st);
}

}  // namespace qjl
