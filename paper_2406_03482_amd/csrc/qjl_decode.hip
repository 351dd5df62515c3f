// One decode step on a quantized key cache: Algorithm 1 EstimateScores
// (Definition 3.1 Eq. (4) for every key, then softmax) followed by the value
// aggregation of Section 2 Eq. (1), fused in one streaming pass.
//
// HBM-bound: per key and KV head the kernel reads m/8 code bytes, a 2-byte
// norm and one row of V, nothing else of size.  The context is cut into
// chunks (one workgroup each).  A workgroup first computes S q for its query
// heads itself (S is small and stays in L2; a kernel of its own for this would
// cost more than the work), turns it into lookup tables, and then streams its
// keys; every wave keeps a running (max, sum, o[d]) and the partial results
// are merged wave -> workgroup -> (a small second kernel) across chunks with
// the usual max/sum-of-exponentials rescaling.
#include "qjl_common.hpp"
#include "qjl_lut.hpp"
#include "qjl_value_codes.hpp"

#include <hip/hip_ext.h>
#include <atomic>
#include <type_traits>

namespace qjl {
namespace {

constexpr int kD = 128;          // head dimension this kernel is written for
constexpr int kPartStride = 132; // floats per partial record: max, sum, 2 pad, o[128]
#ifndef QJL_SMALL_SHARE_1
#define QJL_SMALL_SHARE_1 460
#endif
#ifndef QJL_SMALL_SHARE_G
#define QJL_SMALL_SHARE_G 470
#endif
constexpr long kSmallShareOneHead = QJL_SMALL_SHARE_1;   // per mille of a pair of chunks that the slower XCD takes
constexpr long kSmallShareGroups = QJL_SMALL_SHARE_G;
constexpr int kMaxSplits = 512;  // most chunks a context is ever cut into (combine_kernel keeps that many records' heads in LDS)

// LDS bytes of one workgroup: S q (gt*m floats), 4-bit tables (4*gt*m), byte
// tables (32*gt*m).  Everything else aliases onto tables that are dead by then.
constexpr size_t decode_lds_bytes(int gt, int m) { return (size_t)gt * m * 37 * sizeof(float); }

// Waves per workgroup: small tables let four workgroups share the 160 KiB of a
// CU (four waves each); larger tables mean one or two workgroups per CU, which
// then get eight waves so that every SIMD still has two to switch between.
// (fp32 values need twice the registers per wave, so they stay at four waves.)
// Quantized values (vq): the value pass is bound by the vector ALU, and eight
// waves keep it busier than four (4096 keys x 32 heads: 8.6 against 9.5 us).
constexpr int decode_waves(int gt, int m, int elem_bytes, bool vq = false) {
  return elem_bytes == 4 ? 4 : (decode_lds_bytes(gt, m) <= 40 * 1024 && !vq) ? 4 : 8;
}

struct decode_args {
  const void* Q;          // [B,Hq,128]
  const void* S;          // [m,128], or one [m,128] block per (batch, kv head) if s_head_stride != 0
  const uint8_t* bits;    // [B,Hkv,n,m/8]   (m = all code bits of a key)
  const uint16_t* norms;  // [B,Hkv,n]
  const uint16_t* norms2; // [B,Hkv,n] norm of the outlier part (two-part codes only)
  size_t s_head_stride;   // elements between the sketches of consecutive (batch, kv head) pairs
  const void* V;          // [B,Hkv,n,128], or the codes [B,Hkv,n,16*b bytes] of values quantized to b bits
  const uint16_t* vscale; // [B,Hkv,n] binary16 scale and zero point of a token's values (quantized values only)
  const uint16_t* vzero;
  float* part;            // [B,Hq,nsplit,132]
  float* out;             // [B,Hq,128]
  int n, groups_per_kv;   // n = keys to attend to
  long n_cap;             // rows per (batch, kv head) in the caches (>= n; larger for a cache that is still filling)
  int nsplit, chunk;
  int chunk_big, chunk_small;   // not 0: pairs of uneven chunks, see decode_plan
  unsigned long long* flag;     // (nonce << 32) | parity of the XCD that runs workgroup 0
  uint32_t nonce;               // of this launch, never 0
  float coef2;            // scale * sqrt(pi/2) / m * log2(e); m = bits of the (first) code part
  float coef2b;           // the same for the second part
  // Streaming (Algorithm 1 as a loop): the key of position n - 1 arrives with the call.
  const void* Knew;       // [B,Hkv,1,128], or null
  uint32_t* bits_w;       // the caches again, writable: row n - 1 is written by this call
  uint16_t* norms_w;
  uint16_t* norms2_w;     // two-part codes: the outlier part's norm
  const int32_t* channels;// two-part codes: [B,Hkv,count] outlier channels, to split the new key's norm
  int count;
  // ... and, with quantized values, so does its value row, which is quantized into row n - 1 as well
  const void* Vnew;       // [B,Hkv,1,128] (type T), or null
  uint8_t* vcodes_w;      // the value caches, writable
  uint16_t* vscale_w;
  uint16_t* vzero_w;
  // Streaming with the position in device memory (a generation loop captured in a graph): n above is then
  // the capacity the chunks were planned for, and the kernel attends over rows 0 .. *pos_dev.
  const int32_t* pos_dev; // or null
};

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// The value cache is read exactly once per call and is far larger than any
// cache: its loads are marked non-temporal, so that the lines neither stay in
// L2 nor are written into the 256 MB last-level cache on their way through.
// (4 x 32 heads x 32768 keys: 199 -> 177 us per step, 0.76 -> 0.86 of 8 TB/s;
// grouped-query shapes of 304 MB on rotating copies: 0.63 -> 0.70.)
// 16 bytes of V -> 8 floats (16-bit types) ...
template <typename T> struct vtile {
  static constexpr int kRegs = 1;  // uint4 per 8 elements
  uint4 r;
  __device__ __forceinline__ void load(const void* V, uint32_t elem) {
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(static_cast<const uint16_t*>(V) + elem));
    r = make_uint4(t[0], t[1], t[2], t[3]);
  }
  __device__ __forceinline__ void get(float (&x)[8]) const {
    unpack2<T>(r.x, x[0], x[1]); unpack2<T>(r.y, x[2], x[3]);
    unpack2<T>(r.z, x[4], x[5]); unpack2<T>(r.w, x[6], x[7]);
  }
};
// ... or 32 bytes (fp32).
template <> struct vtile<f32_t> {
  float4 a, b;
  __device__ __forceinline__ void load(const void* V, uint32_t elem) {
    const f32x4_t* p = reinterpret_cast<const f32x4_t*>(static_cast<const float*>(V) + elem);
    const f32x4_t t0 = __builtin_nontemporal_load(p), t1 = __builtin_nontemporal_load(p + 1);
    a = make_float4(t0[0], t0[1], t0[2], t0[3]); b = make_float4(t1[0], t1[1], t1[2], t1[3]);
  }
  __device__ __forceinline__ void get(float (&x)[8]) const {
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
};

// The query side of Eq. (4), S q, for the GT heads of a workgroup, computed by
// the workgroup itself: sixteen lanes share a row of S (16 bytes each for the
// 16-bit types, so one load instruction covers four rows), multiply it with
// their slice of q and add up inside the 16-lane DPP row.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
template <typename T> struct slice8 {   // eight consecutive elements, as stored
  u32x4_t r;
  __device__ __forceinline__ void load(const void* base, size_t elem) {
    r = *reinterpret_cast<const u32x4_t*>(static_cast<const uint16_t*>(base) + elem);
  }
  __device__ __forceinline__ void get(float (&x)[8]) const {
    unpack2<T>(r[0], x[0], x[1]); unpack2<T>(r[1], x[2], x[3]);
    unpack2<T>(r[2], x[4], x[5]); unpack2<T>(r[3], x[6], x[7]);
  }
};
template <> struct slice8<f32_t> {
  f32x4_t a, b;
  __device__ __forceinline__ void load(const void* base, size_t elem) {
    const f32x4_t* p = reinterpret_cast<const f32x4_t*>(static_cast<const float*>(base) + elem);
    a = p[0]; b = p[1];
  }
  __device__ __forceinline__ void get(float (&x)[8]) const {
    x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3]; x[4] = b[0]; x[5] = b[1]; x[6] = b[2]; x[7] = b[3];
  }
};
__device__ __forceinline__ float dot8(const slice8<bf16_t>& s, const slice8<bf16_t>& q) {
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    bf16x2_t x, y;
    uint32_t sx = s.r[i], qx = q.r[i];
    __builtin_memcpy(&x, &sx, 4); __builtin_memcpy(&y, &qx, 4);
    acc = __builtin_amdgcn_fdot2_f32_bf16(x, y, acc, false);
  }
  return acc;
}
__device__ __forceinline__ float dot8(const slice8<f16_t>& s, const slice8<f16_t>& q) {
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f16x2_t x, y;
    uint32_t sx = s.r[i], qx = q.r[i];
    __builtin_memcpy(&x, &sx, 4); __builtin_memcpy(&y, &qx, 4);
    acc = __builtin_amdgcn_fdot2(x, y, acc, false);
  }
  return acc;
}
__device__ __forceinline__ float dot8(const slice8<f32_t>& s, const slice8<f32_t>& q) {
  float acc = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) acc = fmaf(s.a[i], q.a[i], acc);
#pragma unroll
  for (int i = 0; i < 4; ++i) acc = fmaf(s.b[i], q.b[i], acc);
  return acc;
}

// MW = 32-bit words of a key's code.  MWB = 0: one QJL instance.  MWB > 0: the
// last MWB words belong to a second, independent instance (Section 4.1: outlier
// channels) with its own norm; a.S then points to per-head sketches whose rows
// are already restricted to the coordinates of each instance, so S q needs no
// special case, and the two partial inner products are weighted separately.
// ... or b bytes: eight b-bit codes of a quantized value row (Section 3.2), b = 2, 4
// or 8.  The codes come out as floats proportional to 0 .. 2^b - 1; scale and zero
// point are applied per row.  Every code is first moved into a byte of its own.
// Eight-bit codes: one v_cvt_f32_ubyteN per code, written as asm because the
// compiler otherwise extracts every code with its own bit-field instruction.
// Two- and four-bit codes: a byte that holds a code c <= 15 is, read as an 8-bit float (1-4-3), exactly c * 2^-9
// (subnormal c/8 * 2^-6 below 8, (1 + (c-8)/8) * 2^-6 from 8 on), and v_cvt_pk_f32_fp8 converts two such bytes per
// instruction: four conversions instead of eight.  The factor 2^9 goes into the weight of the row, once per key.
constexpr float kSmallCodeUnit = 0x1.0p-9f;
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void bytes_to_floats(uint32_t even, uint32_t odd, float (&x)[8]) {
  const f32x2_t a = __builtin_amdgcn_cvt_pk_f32_fp8((int)even, false), b = __builtin_amdgcn_cvt_pk_f32_fp8((int)even, true);
  const f32x2_t c = __builtin_amdgcn_cvt_pk_f32_fp8((int)odd, false), d = __builtin_amdgcn_cvt_pk_f32_fp8((int)odd, true);
  x[0] = a[0]; x[2] = a[1]; x[4] = b[0]; x[6] = b[1];
  x[1] = c[0]; x[3] = c[1]; x[5] = d[0]; x[7] = d[1];
}
template <int BITS> struct vtile_q;
template <> struct vtile_q<4> {
  uint32_t r;
  __device__ __forceinline__ void load(const void* V, uint32_t byte_off) {
    r = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(static_cast<const char*>(V) + byte_off));
  }
  __device__ __forceinline__ void get(float (&x)[8]) const {
    bytes_to_floats(r & 0x0F0F0F0Fu, (r >> 4) & 0x0F0F0F0Fu, x);
  }
};
template <> struct vtile_q<2> {
  uint32_t r;
  __device__ __forceinline__ void load(const void* V, uint32_t byte_off) {
    r = __builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(static_cast<const char*>(V) + byte_off));
  }
  __device__ __forceinline__ void get(float (&x)[8]) const {
    uint32_t t = (r | (r << 8)) & 0x00FF00FFu;      // the two code bytes, a byte apart
    t = (t | (t << 4)) & 0x0F0F0F0Fu;               // byte i: codes 2i (low two bits) and 2i + 1
    bytes_to_floats(t & 0x03030303u, (t >> 2) & 0x03030303u, x);
  }
};
template <> struct vtile_q<8> {
  uint2 r;
  __device__ __forceinline__ void load(const void* V, uint32_t byte_off) {
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    const u32x2_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(static_cast<const char*>(V) + byte_off));
    r = make_uint2(t[0], t[1]);
  }
  __device__ __forceinline__ void get(float (&x)[8]) const {
    asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(x[0]) : "v"(r.x));
    asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(x[1]) : "v"(r.x));
    asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(x[2]) : "v"(r.x));
    asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(x[3]) : "v"(r.x));
    asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(x[4]) : "v"(r.y));
    asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(x[5]) : "v"(r.y));
    asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(x[6]) : "v"(r.y));
    asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(x[7]) : "v"(r.y));
  }
};

// VB > 0: the values are stored as VB-bit codes with a binary16 scale and zero point
// per token (Section 3.2).  o = sum_j p_j (zero_j + scale_j c_j): the weight
// that goes to the value pass is p_j scale_j, and sum_j p_j zero_j, the same for
// every channel, is carried next to the softmax denominator.
// UN: uneven pairs of chunks shared out by XCD parity (a kernel of its own: the steps it adds to the prologue
// are not free for short contexts -- as a run-time branch they cost 4096 keys x 32 heads 9.3 -> 10.7 us).
template <typename T, int GT, int MW, int MWB, int VB, bool AP, bool UN = false>
__global__ void __launch_bounds__(decode_waves(GT, MW * 32, T::bytes, VB > 0) * 64,
                                  (T::bytes == 4 || GT == 4) ? 1 : (decode_waves(GT, MW * 32, 2, VB > 0) == 4 && GT == 1) ? 4 : 2)
decode_kernel(decode_args a) {
  constexpr int kNW = decode_waves(GT, MW * 32, T::bytes, VB > 0);
  constexpr int MWA = MW - MWB;                        // words of the first instance
  extern __shared__ float4 smem4[];
  float* smem = reinterpret_cast<float*>(smem4);
  constexpr int M = MW * 32;
  float* sq = smem;
  float* nib = sq + GT * M;
  float* lut = nib + 4 * M * GT;
  // the 4-bit tables are dead once the byte tables exist; their space then
  // holds the per-wave probability buffers.  The wave-merge records reuse the
  // byte tables after the last key has been scored.
  // AP: the projections of the new key (M floats), its squared norm, then its
  // code words and its norm as stored -- behind everything else
  // (two-part codes: two squared norms and two stored norms; quantized values: the
  // new value row's codes as floats, its scale and zero point, its packed codes)
  float* sk = lut + 32 * M * GT;
  uint32_t* newcode = reinterpret_cast<uint32_t*>(sk + M + 2);
  float* newval = reinterpret_cast<float*>(newcode + MW + 2);   // [128] codes, then scale and zero point (binary16 bits), then 16 * VB bytes
  uint32_t* newval_u = reinterpret_cast<uint32_t*>(newval + kD);
  float* pbuf_all = nib;                              // [kNW][64*GT]
  float* merge = lut;                                 // [kNW][GT][132]
  static_assert(kNW * 64 <= 4 * M, "probability buffers must fit the 4-bit tables");
  static_assert(kNW * kPartStride <= 32 * M, "merge records must fit the byte tables");

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: keeps block indices in SGPRs
  // grid: x = (batch, kv head), y = group of GT query heads, z = chunk of the context.
  // Query heads of one kv head are consecutive, so the first head of this
  // workgroup is ((b * Hkv + kvh) * groups + group) * GT: no division needed.
  // With x fastest, workgroups are dealt to the eight XCDs by (batch, kv head):
  // for head counts that are multiples of 8 all chunks and all query-head groups
  // of a kv head run on one XCD and share its L2 (the head's sketch, and for
  // grouped queries its codes and values).
  int split = blockIdx.z;
  int bk = blockIdx.x;                                // b * Hkv + kvh
  int grp = blockIdx.y;
  // Uneven pairs of chunks (see below, where the chunk is chosen): workgroup 8a + c of the launch order takes
  // (batch, kv head) 4 (a mod gx/4) + c/2, so that the two workgroups that share a pair of chunks are
  // neighbours in that order and run on XCDs of different parity; the query-head groups of a kv head still
  // share an XCD.
  int pair_slot = 0, place_parity = 0;
  if constexpr (UN) {
    const unsigned L = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const unsigned cx = L & 7u, aa = L >> 3;
    const unsigned q4 = gridDim.x >> 2;
    const unsigned t = aa / q4;
    bk = (int)(4u * (aa - t * q4) + (cx >> 1));
    const unsigned t2 = t / gridDim.y;
    grp = (int)(t - t2 * gridDim.y);
    pair_slot = (int)t2;
    place_parity = (int)(cx & 1u);
  }
  const size_t hq0 = ((size_t)bk * a.groups_per_kv + grp) * GT;

  int n = a.n;
  if constexpr (AP) {
    if (a.pos_dev != nullptr) n = min(max(*a.pos_dev, 0), a.n - 1) + 1;   // uniform: a scalar load
  }
  int k_begin = split * a.chunk;
  int k_end = min(n, k_begin + a.chunk);
  if constexpr (AP) {
    // chunks planned for the capacity that lie wholly behind the newest row: an empty record (weight 0 in
    // the merge) and nothing else
    if (k_begin >= n) {                               // uniform; never the first chunk
      for (int idx = threadIdx.x; idx < GT * kD; idx += kNW * 64) {
        const int g = idx >> 7, ch = idx & 127;
        float* rec = a.part + ((hq0 + g) * a.nsplit + split) * kPartStride;
        rec[4 + ch] = 0.f;
        if (ch == 0) { rec[0] = -INFINITY; rec[1] = 0.f; rec[2] = 0.f; }
      }
      return;
    }
  }
  const size_t row0 = (size_t)bk * a.n_cap;         // first row of this (batch, kv head) in the caches
  float* pbuf = pbuf_all + wave * 64 * GT;
  int r = lane >> 4;                                  // row of a 4-row V pass
  const int c = lane & 15;                            // 8-channel slice

  // ---- the rows of S and the queries first: loads come back in issue order, and
  // S q (then the tables) is the first thing that has to be ready
  // LPR = 4 lanes share a row of S: a lane holds four 8-element slices of the row
  // (slices c, c+4, c+8, c+12, so that a quad still reads 64 contiguous bytes)
  // and two DPP steps finish the row's sum.  (Sixteen lanes per row with one
  // slice each and four DPP steps is the same arithmetic in four times as many
  // dependent reduction steps: with four query heads per workgroup it took 2.5 us
  // of the prologue, against 0.8 us for one head in this form.)  The four query
  // slices per head take 16 registers per head; the four-head group has a CU to
  // itself (its tables fill the LDS), so it may use up to 256 registers.  Only
  // fp32 slices of four heads (32 bytes each) would not fit: they keep sixteen
  // lanes per row.
  constexpr int LPR = (GT == 4 && T::bytes == 4) ? 16 : 4;
  constexpr int SPL = 16 / LPR;                        // slices per lane and row
  constexpr int kRowsPerPass = kNW * 64 / LPR;
  constexpr int kPasses = M / kRowsPerPass;
  static_assert(M % kRowsPerPass == 0, "whole passes over S");
  slice8<T> qs[GT][SPL], srow[kPasses][SPL];
  slice8<T> ks[SPL];                                  // AP: this lane's slices of the new key
  float vnew[8];                                      // AP with quantized values: entries 8c .. 8c+7 of the new value row
  constexpr bool APV = AP && VB > 0;
  // AP: the new key is row n - 1; the workgroups whose chunk holds that row
  // quantize it themselves (same S, same walk as for the queries), use its code
  // from LDS and, the first group of query heads only, write it to the caches.
  const int pos = n - 1;
  const bool has_new = AP && pos >= k_begin && pos < k_end;   // uniform
  {
    const int c16 = tid & (LPR - 1), r16 = tid / LPR;
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
      for (int i = 0; i < SPL; ++i) qs[g][i].load(a.Q, (hq0 + g) * kD + (c16 + LPR * i) * 8);
    if constexpr (AP) {
#pragma unroll
      for (int i = 0; i < SPL; ++i) ks[i].load(a.Knew, (size_t)bk * kD + (c16 + LPR * i) * 8);
    }
    if constexpr (APV) load8<T>(a.Vnew, (size_t)bk * kD + (lane & 15) * 8, vnew);
    const size_t s0 = (size_t)bk * a.s_head_stride;
#pragma unroll
    for (int u = 0; u < kPasses; ++u)
#pragma unroll
      for (int i = 0; i < SPL; ++i)
        srow[u][i].load(a.S, s0 + (size_t)(u * kRowsPerPass + r16) * kD + (c16 + LPR * i) * 8);
  }
  __builtin_amdgcn_sched_barrier(0);
  // ---- which chunk of its pair this workgroup takes.  The odd-numbered XCDs of this chip stream 5-12 %
  // slower than the even ones (every workgroup stamped with its end time and XCC_ID: same buffers or
  // rotating ones, eager or from a graph), and workgroups are dealt to the XCDs in turn -- but from a
  // starting point that differs between launches (eager launches start at XCD 0, the same kernel replayed
  // from a graph was seen to start at XCD 7).  So the launch agrees on it at run time: workgroup 0 publishes
  // the parity of its own XCC_ID under this launch's nonce, every wave waits for that word (behind the loads
  // of S and q that it has just issued) and a workgroup whose place in the order puts it on an odd XCD takes
  // the small chunk.  The chunks and their records are the same whoever takes them, so the result does not
  // depend on the outcome.  A word that already carries the nonce (a graph replayed) is used as it is: the
  // same for every workgroup, which is all that correctness needs.  Workgroup 0 is dispatched first and waits
  // for nobody, so the wait ends; should it not (20000 polls), the wave poisons its record with a NaN.
  float poison = 0.f;
  if constexpr (UN) {
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && tid == 0) {
      const unsigned long long cur = __hip_atomic_load(a.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((uint32_t)(cur >> 32) != a.nonce) {
        unsigned xcc;
        asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
        __hip_atomic_store(a.flag, ((unsigned long long)a.nonce << 32) | (xcc & 1u), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    unsigned word = 0xFFFFFFFFu;                       // bit 0: parity of workgroup 0's XCD; all ones: no answer
    if (lane == 0) {
      for (int it = 0; it < 20000; ++it) {
        const unsigned long long v = __hip_atomic_load(a.flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if ((uint32_t)(v >> 32) == a.nonce) { word = (uint32_t)v & 1u; break; }
        __builtin_amdgcn_s_sleep(4);
      }
    }
    word = __builtin_amdgcn_readfirstlane(word);
    if (word == 0xFFFFFFFFu) { poison = __builtin_nanf(""); word = 0; }
    const int slow = (place_parity ^ (int)word) & 1;
    const int both = a.chunk_big + a.chunk_small;
    split = 2 * pair_slot + slow;
    k_begin = pair_slot * both + (slow ? a.chunk_big : 0);
    k_end = min(n, k_begin + (slow ? a.chunk_small : a.chunk_big));
  }
  // ---- then the first block of this wave: its HBM reads are in flight while
  // the tables are built.  Rows past the chunk end are clamped (never out of
  // bounds); their weight is 0.
  int k0 = k_begin + wave * 64;
  uint32_t wcur[MW];
  uint16_t ncur = 0;   // norm of this lane's key, still as binary16: converting it where it is
                       // loaded would make the wave wait for the load (and every older one) there
  uint16_t ncur2 = 0;  // norm of the second code part
  uint16_t vscur = 0, vzcur = 0;   // scale and zero point of this lane's key's values
  // V rows in flight per lane: 16 (a whole 64-key block ahead), or 8 where the
  // four-head group needs the registers for its accumulators and tables
  constexpr int VD = GT == 4 ? 8 : 16;
  constexpr bool VQ = VB > 0;
  using VT = typename std::conditional<VQ, vtile_q<VQ ? VB : 4>, vtile<T>>::type;
  VT v[VD];
  // V loads requested before the tables are built: enough to keep HBM busy
  // meanwhile, few enough that the rows of S (requested just before them, and
  // on the critical path) are not held up behind them.  Eight for one or two
  // query heads (4096 keys x 32 heads: 9.9 us against 10.1 with four, 14 with
  // twelve); four where more work sits between the loads and the tables (four
  // heads; the new key's projection of a streaming step: 10.9 us against 14.6).
  constexpr int VP = (GT == 4 || AP) ? 4 : 8;
  // row (4i + r) of the block starting at key kb: uniform base pointer + a
  // 32-bit lane offset, the row clamped to the last key of the chunk
  auto issue_v = [&](int slot, int i, int kb, int last_row) {   // row pass i of block kb -> v[slot]
    const int rr = min(4 * i + r, last_row);
    if constexpr (VQ) {
      const char* base = static_cast<const char*>(a.V) + (row0 + kb) * (size_t)(kD * VB / 8);
      v[slot].load(base, (uint32_t)(rr * (kD * VB / 8) + c * VB));
    } else {
      const char* base = static_cast<const char*>(a.V) + (row0 + kb) * (size_t)(kD * T::bytes);
      v[slot].load(base, (uint32_t)(rr * kD + c * 8));
    }
  };
  // No branch around these loads (a wave whose first block lies past the chunk
  // end reads the chunk's last key instead and never uses it): with straight-line
  // code the wait for S q below does not have to wait for them as well.
  const int kf = min(k0, k_end - 1);
  {
    const int j = min(kf + lane, k_end - 1);
    load_code<MW>(a.bits, row0 + j, wcur);
    ncur = a.norms[row0 + j];
    if constexpr (MWB > 0) ncur2 = a.norms2[row0 + j];
    if constexpr (VQ) { vscur = a.vscale[row0 + j]; vzcur = a.vzero[row0 + j]; }
#pragma unroll
    for (int i = 0; i < VP; ++i) {
      issue_v(i, i, kf, k_end - 1 - kf);
      __builtin_amdgcn_sched_barrier(0);   // issue order = use order (see the second half below)
    }
  }

  __builtin_amdgcn_sched_barrier(0);
  {
    const int c16 = tid & (LPR - 1), r16 = tid / LPR;
    auto row_dot = [&](const slice8<T> (&x)[SPL], const slice8<T> (&y)[SPL]) {   // sum over the row's LPR lanes
      float t = dot8(x[0], y[0]);
#pragma unroll
      for (int i = 1; i < SPL; ++i) t += dot8(x[i], y[i]);
      if constexpr (LPR == 16) return row16_sum(t);
      t += QJL_DPP_F(t, 0xB1);   // quad_perm [1,0,3,2]
      t += QJL_DPP_F(t, 0x4E);   // quad_perm [2,3,0,1]
      return t;
    };
#pragma unroll
    for (int u = 0; u < kPasses; ++u) {
#pragma unroll
      for (int g = 0; g < GT; ++g) {
        const float t = row_dot(srow[u], qs[g]);
        if (c16 == 0) sq[g * M + u * kRowsPerPass + r16] = t;
      }
      if constexpr (AP) {                             // every workgroup: no branch inside this stretch of code
        const float t = row_dot(srow[u], ks);
        if (c16 == 0) sk[u * kRowsPerPass + r16] = t;
      }
    }
    if constexpr (AP) {
      if constexpr (MWB > 0) {
        // Section 4.1: the inlier code goes with the norm of the key without its head's outlier channels, the
        // outlier code with the norm of those channels (out-of-range entries ignored, repeats count once)
        uint32_t cm[4] = {0u, 0u, 0u, 0u};
        for (int t = 0; t < a.count; ++t) {
          const int ch = a.channels[(size_t)bk * a.count + t];
          if (ch >= 0 && ch < kD) cm[ch >> 5] |= 1u << (ch & 31);
        }
        float kin = 0.f, kout = 0.f;
#pragma unroll
        for (int i = 0; i < SPL; ++i) {
          const int e0 = (c16 + LPR * i) * 8;            // first element of this slice
          const uint32_t mb = (cm[e0 >> 5] >> (e0 & 31)) & 0xFFu;
          float x[8];
          ks[i].get(x);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const bool o = (mb >> e) & 1u;
            kout = fmaf(x[e], o ? x[e] : 0.f, kout);
            kin = fmaf(x[e], o ? 0.f : x[e], kin);
          }
        }
        if constexpr (LPR == 16) { kin = row16_sum(kin); kout = row16_sum(kout); }
        else {
          kin += QJL_DPP_F(kin, 0xB1); kin += QJL_DPP_F(kin, 0x4E);
          kout += QJL_DPP_F(kout, 0xB1); kout += QJL_DPP_F(kout, 0x4E);
        }
        if (tid == 0) { sk[M] = kin; sk[M + 1] = kout; }
      } else {
        const float kk = row_dot(ks, ks);
        if (tid == 0) sk[M] = kk;
      }
    }
  }
  __syncthreads();
  if constexpr (AP) {
    if (has_new) {                                    // bit i of the code = [(S k)_i >= 0]: one ballot per 64 projections
#pragma unroll
      for (int i0 = 0; i0 < M; i0 += kNW * 64) {
        const int i = i0 + tid;                       // more threads than projections for small m
        const uint64_t bal = __ballot(i < M && sk[min(i, M - 1)] >= 0.f);
        if ((lane & 31) == 0 && i < M) {
          const uint32_t word = (uint32_t)(bal >> (lane & 32));
          newcode[i >> 5] = word;
        }
      }
      if (tid == 0) {
        newcode[MW] = float_to_f16_bits(sqrtf(sk[M]));
        if constexpr (MWB > 0) newcode[MW + 1] = float_to_f16_bits(sqrtf(sk[M + 1]));
      }
      if constexpr (APV) {
        // Section 3.2 for the new token's value row: the same arithmetic as the bulk quantizer, by the first
        // sixteen lanes; the codes stay in LDS for this step's own use and go to the cache at the end
        if (tid < 16) {
          float lo = vnew[0], hi = vnew[0];
#pragma unroll
          for (int e = 1; e < 8; ++e) { lo = fminf(lo, vnew[e]); hi = fmaxf(hi, vnew[e]); }
          lo = row16_min(lo);
          hi = row16_max(hi);
          uint16_t s16, z16;
          uint32_t q8[8];
          value_codes8<VB>(vnew, lo, hi, s16, z16, q8);
#pragma unroll
          for (int e = 0; e < 8; ++e) newval[tid * 8 + e] = (float)q8[e] * (VB == 8 ? 1.f : kSmallCodeUnit);
          if (tid == 0) { newval_u[0] = s16; newval_u[1] = z16; }
          if constexpr (VB == 8) {
            newval_u[2 + 2 * tid] = q8[0] | (q8[1] << 8) | (q8[2] << 16) | (q8[3] << 24);
            newval_u[3 + 2 * tid] = q8[4] | (q8[5] << 8) | (q8[6] << 16) | (q8[7] << 24);
          } else {
            uint32_t word = 0;
#pragma unroll
            for (int e = 0; e < 8; ++e) word |= q8[e] << (VB * e);
            newval_u[2 + tid] = word;                   // VB == 2: the low 16 bits
          }
        }
      }
    }
  }
  build_lut<GT>(sq, nib, lut, M, tid, kNW * 64);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = VP; i < VD; ++i) {
    issue_v(i, i, kf, k_end - 1 - kf);
    // Loads return in issue order and the loop below consumes the rows in index
    // order; left alone the scheduler may issue these in any order, and the wait
    // for row VP inside the loop then has to cover the whole queue, every block.
    __builtin_amdgcn_sched_barrier(0);
  }
  // lut_build ends with a barrier: nobody reads `nib` any more.

  using PV = typename vecf<GT>::type;
  float m_run[GT], l_lane[GT], z_lane[GT];            // z: sum of p * zero point (quantized values)
  PV acc[8];                                          // acc[e] holds channel 8c+e of all GT heads
#pragma unroll
  for (int g = 0; g < GT; ++g) { m_run[g] = -INFINITY; l_lane[g] = 0.f; z_lane[g] = 0.f; }
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;

  for (; k0 < k_end; k0 += kNW * 64) {
    const int kn = k0 + kNW * 64;
    const bool have_next = kn < k_end;
    int new_pass = -1, new_r = 0;                     // APV: the row pass and row group of the new token in this block
    if constexpr (APV) {
      if (has_new && pos >= k0 && pos < k0 + 64) { new_pass = (pos - k0) >> 2; new_r = (pos - k0) & 3; }
    }
    if constexpr (AP) {                               // the lane of the new key takes its code from LDS
      if (has_new && pos >= k0 && pos < k0 + 64) {    // uniform
        if (k0 + lane == pos) {
#pragma unroll
          for (int w = 0; w < MW; ++w) wcur[w] = newcode[w];
          ncur = (uint16_t)newcode[MW];
          if constexpr (MWB > 0) ncur2 = (uint16_t)newcode[MW + 1];
          if constexpr (APV) { vscur = (uint16_t)newval_u[0]; vzcur = (uint16_t)newval_u[1]; }
        }
      }
    }
    // ---- scores of this block: lane <-> key
    const PV s = key_inner<GT, MW, 0, MWA>(wcur, lut);
    PV s2 = 0.f;
    if constexpr (MWB > 0) s2 = key_inner<GT, MW, MWA, MW>(wcur, lut);
    const bool valid = (k0 + lane) < k_end;
    const float nu = f16_bits_to_float(ncur) * a.coef2;
    const float nu2 = MWB > 0 ? f16_bits_to_float(ncur2) * a.coef2b : 0.f;
    // (codes of 2 and 4 bits reach the value pass as c * 2^-9)
    const float vs = VQ ? f16_bits_to_float(vscur) * (VB == 8 ? 1.f : 1.f / kSmallCodeUnit) : 1.f;
    const float vz = VQ ? f16_bits_to_float(vzcur) : 0.f;
    // the code registers are free again: fetch the next block's codes and norm
    // into them now, the value pass below hides the latency
    if (have_next) {
      const int j = min(kn + lane, k_end - 1);
      load_code<MW>(a.bits, row0 + j, wcur);
      ncur = a.norms[row0 + j];
      if constexpr (MWB > 0) ncur2 = a.norms2[row0 + j];
      if constexpr (VQ) { vscur = a.vscale[row0 + j]; vzcur = a.vzero[row0 + j]; }
    }
    PV alpha, p;
#pragma unroll
    for (int g = 0; g < GT; ++g) {
      float sv = vget<GT>(s, g) * nu;                                       // log2 domain
      if constexpr (MWB > 0) sv = fmaf(vget<GT>(s2, g), nu2, sv);
      const float sg = valid ? sv : -INFINITY;
      const float m_new = fmaxf(m_run[g], wave_max(sg));
      const float al = __builtin_amdgcn_exp2f(m_run[g] - m_new);
      const float pg = __builtin_amdgcn_exp2f(sg - m_new);
      vset<GT>(alpha, g, al);
      vset<GT>(p, g, VQ ? pg * vs : pg);
      l_lane[g] = l_lane[g] * al + pg;
      if constexpr (VQ) z_lane[g] = z_lane[g] * al + pg * vz;
      m_run[g] = m_new;
    }
    // key (4i + r) of the block goes to slot r*16 + i, so that a V lane reads
    // its 16 weights from consecutive slots
    reinterpret_cast<PV*>(pbuf)[(lane & 3) * 16 + (lane >> 2)] = p;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ---- o = o * alpha + sum_j p_j v_j; each V register is refilled with the
    // next block's row as soon as it has been consumed.
    // Straight-line on purpose (no branch on have_next): when there is no next
    // block every lane re-reads row 0 of the current one, a single cached line.
    const int kb_next = have_next ? kn : k0;
    const int lim_next = have_next ? k_end - 1 - kn : 0;
    // Groups of two and four heads: the two waves of a SIMD both keep the vector ALU busy most of the time.
    // The one that is in its value pass -- the pass that issues the loads -- goes first (measured: 8192 keys
    // x 16 x 8 kv heads 55.9 -> 54.9 us, with 4-bit values 43.6 -> 40.8 us, with 384-bit codes as well,
    // two heads at a time, 52.4 -> 48.9 us; one-head groups do not change).
    if constexpr (GT >= 2) __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] *= alpha;
    const PV* pw = reinterpret_cast<const PV*>(pbuf) + r * 16;
    PV pv_next = pw[0];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const PV pv = pv_next;
      if (i + 1 < 16) pv_next = pw[i + 1];            // hide the LDS latency behind this row's FMAs
      float x[8];
      v[i % VD].get(x);
      if constexpr (APV) {                              // the new token's row: its codes are in LDS, not yet in the cache
        if (new_pass == i) {                            // uniform; -1 in every block but the one that holds row pos
#pragma unroll
          for (int e = 0; e < 8; ++e) x[e] = (lane >> 4) == new_r ? newval[c * 8 + e] : x[e];
        }
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += pv * x[e];
      // The refill overwrites the registers just read.  Tie its address (through r)
      // to the accumulators: otherwise the compiler may move the load above the last
      // read, give it fresh registers and copy them back at the loop end -- a copy
      // that has to wait for the whole queue of loads, every block.
#pragma unroll
      for (int e = 0; e < 8; ++e) asm volatile("" : "+v"(r), "+v"(acc[e]));
      if (i + VD < 16) issue_v(i % VD, i + VD, k0, k_end - 1 - k0);   // later row of this block
      else issue_v(i % VD, i + VD - 16, kb_next, lim_next);          // first rows of the next block
      // keep each refill right behind the last use of its registers: hoisting
      // all sixteen would need a second set of V registers
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (GT >= 2) __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }

  __syncthreads();   // every wave is done with the tables: their space now takes the merge records
  // ---- wave result: sum over lanes / over the four row groups
#pragma unroll
  for (int g = 0; g < GT; ++g) {
    const float l = wave_sum(l_lane[g]);
    const float zsum = VQ ? wave_sum(z_lane[g]) : 0.f;
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x = vget<GT>(acc[e], g);
      x += __shfl_xor(x, 16);
      x += __shfl_xor(x, 32);
      o[e] = x;
    }
    float* rec = merge + (wave * GT + g) * kPartStride;
    if (lane < 16) {
#pragma unroll
      for (int e = 0; e < 8; ++e) rec[4 + c * 8 + e] = o[e];
    }
    if (lane == 0) {
      rec[0] = m_run[g];
      if constexpr (UN) rec[1] = l + poison; else rec[1] = l;
      rec[2] = zsum;
    }
  }
  __syncthreads();

  // ---- workgroup result: merge the waves
  for (int idx = tid; idx < GT * kD; idx += kNW * 64) {
    const int g = idx >> 7, ch = idx & 127;
    float mx = -INFINITY;
#pragma unroll
    for (int w = 0; w < kNW; ++w) mx = fmaxf(mx, merge[(w * GT + g) * kPartStride]);
    float L = 0.f, O = 0.f, Z = 0.f;
#pragma unroll
    for (int w = 0; w < kNW; ++w) {
      const float* rec = merge + (w * GT + g) * kPartStride;
      const float f = __builtin_amdgcn_exp2f(rec[0] - mx);
      L = fmaf(rec[1], f, L);
      if constexpr (VQ) Z = fmaf(rec[2], f, Z);
      O = fmaf(rec[4 + ch], f, O);
    }
    if (a.nsplit == 1) {
      a.out[(hq0 + g) * kD + ch] = (O + Z) / L;
    } else {
      float* rec = a.part + ((hq0 + g) * a.nsplit + split) * kPartStride;
      rec[4 + ch] = O;
      if (ch == 0) { rec[0] = mx; rec[1] = L; rec[2] = Z; }
    }
  }
  if constexpr (AP) {                                   // the new key's row of the caches, last: no store ahead of the loop's loads
    if (has_new && grp == 0) {
      if (tid < MW) a.bits_w[(row0 + pos) * MW + tid] = newcode[tid];
      if (tid == 0) a.norms_w[row0 + pos] = (uint16_t)newcode[MW];
      if constexpr (MWB > 0) { if (tid == 0) a.norms2_w[row0 + pos] = (uint16_t)newcode[MW + 1]; }
      if constexpr (APV) {
        uint8_t* dst = a.vcodes_w + (row0 + pos) * (size_t)(16 * VB);
        if (tid < 16) {
          if constexpr (VB == 8) *reinterpret_cast<uint2*>(dst + 8 * tid) = make_uint2(newval_u[2 + 2 * tid], newval_u[3 + 2 * tid]);
          else if constexpr (VB == 4) *reinterpret_cast<uint32_t*>(dst + 4 * tid) = newval_u[2 + tid];
          else *reinterpret_cast<uint16_t*>(dst + 2 * tid) = (uint16_t)newval_u[2 + tid];
        }
        if (tid == 0) { a.vscale_w[row0 + pos] = (uint16_t)newval_u[0]; a.vzero_w[row0 + pos] = (uint16_t)newval_u[1]; }
      }
    }
  }
}

// Merge the per-chunk records of one query head: out = sum_s o_s 2^(m_s - M) / sum_s l_s 2^(m_s - M).
// A kernel of its own: the kernel boundary makes the records of all workgroups
// visible without device-wide fences inside the streaming kernel.
// 256 threads: thread (half, ch) sums the chunks s = half, half + 2, ... for
// channel ch.  Every load of a pass is issued before the first use, so a head
// with up to 16 chunks costs a single round trip to memory.
__global__ void __launch_bounds__(2 * kD) combine_kernel(const float* __restrict__ part,
                                                         float* __restrict__ out, int nsplit) {
  __shared__ float s_m[kMaxSplits], s_l[kMaxSplits], s_z[kMaxSplits];   // per chunk: running max, sum, zero-point sum
  __shared__ float s_o[kD], s_lsum, s_zsum;
  const size_t head = blockIdx.x;
  const int tid = threadIdx.x;
  const float* base = part + head * (size_t)nsplit * kPartStride;
  const int ch = tid & (kD - 1), half = tid >> 7;
  constexpr int kB = 8;                  // chunks per thread and pass
  float O = 0.f, L = 0.f, Zc = 0.f, mx = -INFINITY;
  for (int s0 = 0; s0 < nsplit; s0 += 2 * kB) {
    float o[kB];
#pragma unroll
    for (int u = 0; u < kB; ++u) {
      const int s2 = s0 + half + 2 * u;
      o[u] = s2 < nsplit ? base[(size_t)s2 * kPartStride + 4 + ch] : 0.f;
    }
    if (s0 == 0) {                       // first pass also fetches every chunk's (max, sum)
      for (int s2 = tid; s2 < nsplit; s2 += 2 * kD) {
        s_m[s2] = base[(size_t)s2 * kPartStride];
        s_l[s2] = base[(size_t)s2 * kPartStride + 1];
        s_z[s2] = base[(size_t)s2 * kPartStride + 2];   // 0 unless the values are quantized
      }
      __syncthreads();
      for (int s2 = 0; s2 < nsplit; ++s2) mx = fmaxf(mx, s_m[s2]);
    }
#pragma unroll
    for (int u = 0; u < kB; ++u) {
      const int s2 = s0 + half + 2 * u;
      if (s2 < nsplit) {
        const float f = __builtin_amdgcn_exp2f(s_m[s2] - mx);
        O = fmaf(o[u], f, O);
        L = fmaf(s_l[s2], f, L);
        Zc = fmaf(s_z[s2], f, Zc);
      }
    }
  }
  if (half == 1) {
    s_o[ch] = O;
    if (ch == 0) { s_lsum = L; s_zsum = Zc; }
  }
  __syncthreads();
  if (half == 0) out[head * kD + ch] = (O + s_o[ch] + Zc + s_zsum) / (L + s_lsum);
}

template <typename T, int GT, int MW, int MWB, int VB, bool AP, bool UN = false>
int launch_t(const qjl_shape& sh, const decode_plan& plan, decode_args a, hipStream_t st,
             hipEvent_t ev0, hipEvent_t ev1) {
  static std::atomic<uint64_t> lds_set{0};             // per kernel instantiation: devices whose limit is raised
  constexpr int kNW = decode_waves(GT, MW * 32, T::bytes, VB > 0);
  // AP: projections of the new key + two squared norms, its code + two norms, then (quantized values) the new
  // value row: 128 codes as floats, scale, zero point, up to 128 packed bytes
  const size_t lds = decode_lds_bytes(GT, MW * 32) +
                     (AP ? (MW * 32 + 2 + MW + 2 + (VB > 0 ? kD + 2 + 32 : 0) + 2) * sizeof(float) : 0);
  int rc_lds = allow_dynamic_lds(reinterpret_cast<const void*>(&decode_kernel<T, GT, MW, MWB, VB, AP, UN>), lds, lds_set);
  if (rc_lds != QJL_OK) return rc_lds;
  const long pairs = (long)sh.batch * sh.kv_heads;
  if (a.groups_per_kv > 65535 || plan.nsplit > 65535 || pairs > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  const dim3 grid((unsigned)pairs, (unsigned)a.groups_per_kv, (unsigned)plan.nsplit);
  if (ev0 || ev1)   // the events take the kernel's own start and stop timestamps
    hipExtLaunchKernelGGL((decode_kernel<T, GT, MW, MWB, VB, AP, UN>), grid, dim3(kNW * 64), (uint32_t)lds, st,
                          ev0, ev1, 0u, a);
  else
    hipLaunchKernelGGL((decode_kernel<T, GT, MW, MWB, VB, AP, UN>), grid, dim3(kNW * 64), lds, st, a);
  return launch_status();
}

template <typename T, int MW, int MWB, int VB = 0, bool AP = false>
int launch_g(const qjl_shape& sh, const decode_plan& plan, const decode_args& a, hipStream_t st,
             hipEvent_t ev0, hipEvent_t ev1) {
  // uneven pairs of chunks: 16-bit types, one-part codes, unquantized values, not the streaming step (two-part
  // codes measured no gain: 185.3 us either way for 4 x 32 heads x 32768 keys on 384 bits)
  if constexpr (T::bytes == 2 && MWB == 0 && VB == 0 && !AP) {
    if (a.chunk_small != 0) {
      switch (plan.gt) {
        case 4: if constexpr (MW * 32 * 4 <= 1024) return launch_t<T, 4, MW, MWB, VB, AP, true>(sh, plan, a, st, ev0, ev1); else return QJL_ERR_UNSUPPORTED;
        case 2: if constexpr (MW * 32 * 2 <= 1024) return launch_t<T, 2, MW, MWB, VB, AP, true>(sh, plan, a, st, ev0, ev1); else return QJL_ERR_UNSUPPORTED;
        default: return launch_t<T, 1, MW, MWB, VB, AP, true>(sh, plan, a, st, ev0, ev1);
      }
    }
  }
  switch (plan.gt) {
    case 4: if constexpr (MW * 32 * 4 <= 1024) return launch_t<T, 4, MW, MWB, VB, AP>(sh, plan, a, st, ev0, ev1); else return QJL_ERR_UNSUPPORTED;
    case 2: if constexpr (MW * 32 * 2 <= 1024) return launch_t<T, 2, MW, MWB, VB, AP>(sh, plan, a, st, ev0, ev1); else return QJL_ERR_UNSUPPORTED;
    default: return launch_t<T, 1, MW, MWB, VB, AP>(sh, plan, a, st, ev0, ev1);
  }
}

// The instantiations that exist for a code of MW words whose last MWB belong to a second quantizer:
//   one-part codes: plain, streaming (AP), quantized values (2, 4, 8 bits)
//   two-part codes: plain, quantized values, quantized values + streaming (the generation step at the
//   paper's operating point)
// Quantized values and streaming take 16-bit queries and sketches.
template <typename T, int MW, int MWB>
int launch_v(const qjl_shape& sh, int vbits, bool ap, const decode_plan& plan, const decode_args& a, hipStream_t st,
             hipEvent_t ev0, hipEvent_t ev1) {
  if (vbits == 0 && !ap) return launch_g<T, MW, MWB>(sh, plan, a, st, ev0, ev1);
  if constexpr (T::bytes == 2) {
    if (vbits == 0) {                                 // streaming on unquantized values: one-part codes
      if constexpr (MWB == 0) return launch_g<T, MW, 0, 0, true>(sh, plan, a, st, ev0, ev1);
      else return QJL_ERR_UNSUPPORTED;
    }
    if (!ap) {
      switch (vbits) {
        case 2: return launch_g<T, MW, MWB, 2>(sh, plan, a, st, ev0, ev1);
        case 4: return launch_g<T, MW, MWB, 4>(sh, plan, a, st, ev0, ev1);
        case 8: return launch_g<T, MW, MWB, 8>(sh, plan, a, st, ev0, ev1);
        default: return QJL_ERR_UNSUPPORTED;
      }
    }
    if constexpr (MWB > 0) {                          // streaming into quantized values: two-part codes
      switch (vbits) {
        case 2: return launch_g<T, MW, MWB, 2, true>(sh, plan, a, st, ev0, ev1);
        case 4: return launch_g<T, MW, MWB, 4, true>(sh, plan, a, st, ev0, ev1);
        case 8: return launch_g<T, MW, MWB, 8, true>(sh, plan, a, st, ev0, ev1);
        default: return QJL_ERR_UNSUPPORTED;
      }
    }
  }
  return QJL_ERR_UNSUPPORTED;
}

// m = bits of the (first) code part, m_out = bits of the second part (0: none)
template <typename T>
int launch_m(const qjl_shape& sh, int m_out, int vbits, const decode_plan& plan, const decode_args& a, hipStream_t st,
             hipEvent_t ev0, hipEvent_t ev1) {
  const bool ap = a.Knew != nullptr;
  if (a.vscale == nullptr) vbits = 0;
  if (m_out == 0) {
    switch (sh.m) {
      case 128: return launch_v<T, 4, 0>(sh, vbits, ap, plan, a, st, ev0, ev1);
      case 256: return launch_v<T, 8, 0>(sh, vbits, ap, plan, a, st, ev0, ev1);
      case 512: return launch_v<T, 16, 0>(sh, vbits, ap, plan, a, st, ev0, ev1);
      default: return QJL_ERR_UNSUPPORTED;
    }
  }
  if (m_out == 128 && sh.m == 128) return launch_v<T, 8, 4>(sh, vbits, ap, plan, a, st, ev0, ev1);
  if (m_out == 128 && sh.m == 256) return launch_v<T, 12, 4>(sh, vbits, ap, plan, a, st, ev0, ev1);
  // larger two-part codes: unquantized values, no streaming
  if (vbits == 0 && !ap) {
    if (m_out == 128 && sh.m == 512) return launch_g<T, 20, 4>(sh, plan, a, st, ev0, ev1);
    if (m_out == 256 && sh.m == 256) return launch_g<T, 16, 8>(sh, plan, a, st, ev0, ev1);
  }
  return QJL_ERR_UNSUPPORTED;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace

// Compute units of the current device.  The only thing the library remembers
// between calls are such device attributes, per device ordinal, in atomics:
// a value is written once and two threads that race write the same value.
int device_cu_count() {
  static std::atomic<int> cached[64];
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) {
    (void)hipGetLastError();
    return 256;  // MI355X; used when no device is visible (host-only callers)
  }
  const bool slot = dev >= 0 && dev < 64;
  if (slot) {
    cus = cached[dev].load(std::memory_order_relaxed);
    if (cus > 0) return cus;
  }
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) {
    if (slot) cached[dev].store(cus, std::memory_order_relaxed);
    return cus;
  }
  (void)hipGetLastError();
  return 256;
}

// Kernels with more than 64 KB of dynamic LDS need their limit raised once per
// device.  `done` has one bit per device ordinal; setting the attribute twice
// is harmless, so two threads that race both set it.
int allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hip_status(hipErrorInvalidDevice);
  const bool slot = dev >= 0 && dev < 64;
  if (slot && ((done.load(std::memory_order_acquire) >> dev) & 1u)) return QJL_OK;
  hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return hip_status(e);
  if (slot) done.fetch_or(uint64_t{1} << dev, std::memory_order_release);
  return QJL_OK;
}

// How the context is cut up.  One "unit" is a (batch, kv head, group of GT
// query heads); it gets nsplit workgroups of `chunk` keys each.
// force_splits > 0 fixes the number of chunks (tests and tuning); it is clamped
// like the automatic choice.  The workspace is sized from the split count before
// the chunk length is rounded up to whole 64-key blocks: that count never
// decreases when n grows, so the workspace for a cache's capacity covers every
// shorter context (the rounded count is not monotonic in n).
bool plan_decode(const qjl_shape& sh, int m_out, decode_plan* plan, int force_splits) {
  if (sh.d != kD) return false;
  if (sh.n > (1 << 30)) return false;               // key indices and chunk bounds are 32-bit in the kernel
  if (m_out == 0) {
    if (sh.m != 128 && sh.m != 256 && sh.m != 512) return false;
  } else if (!((m_out == 128 && (sh.m == 128 || sh.m == 256 || sh.m == 512)) || (m_out == 256 && sh.m == 256))) {
    return false;
  }
  const int mt = sh.m + m_out;                      // all code bits of a key
  const int G = sh.q_heads / sh.kv_heads;
  int gt = 1;
  if (G % 4 == 0 && mt * 4 <= 1024) gt = 4;
  else if (G % 2 == 0 && mt * 2 <= 1024) gt = 2;
  const long units = (long)sh.batch * sh.kv_heads * (G / gt);
  const size_t lds = decode_lds_bytes(gt, mt);
  const long occ = (160 * 1024) / (long)lds;        // workgroups a CU can hold, by LDS
  // One workgroup per CU: what a workgroup does before its first key (its
  // share of S through L2, S q, the tables: about 3 us) is paid once per
  // workgroup, and with more workgroups per CU it is paid more often for
  // shorter chunks (32 units of 4096 keys: 10.1 us with 8 chunks each, 11.1
  // with 16, 14.5 with 32; of 16384 keys: 27 / 30 / 33 us).  Two per CU where
  // each still gets a long stream (>= 4096 keys): there a second workgroup hides
  // latency that the first cannot (long contexts with 4-bit values: 89 us
  // against 109).
  const long cus = device_cu_count();
  long per_cu = 1;
  if (occ >= 2 && (long)sh.n / ((2 * cus + units - 1) / units) >= 4096) per_cu = 2;
  const long slots = cus * per_cu;
  long nsplit = (slots + units - 1) / units;
  const long min_chunk = 64L * decode_waves(gt, mt, sh.dtype == QJL_F32 ? 4 : 2);  // one 64-key block per wave
  long max_split = ((long)sh.n + min_chunk - 1) / min_chunk;
  if (force_splits > 0) nsplit = force_splits;
  if (nsplit > max_split) nsplit = max_split;
  if (nsplit > kMaxSplits) nsplit = kMaxSplits;
  if (nsplit < 1) nsplit = 1;
  const long records = nsplit;                      // upper bound of the rounded count below
  long chunk = ((long)sh.n + nsplit - 1) / nsplit;
  chunk = (chunk + 63) / 64 * 64;
  nsplit = ((long)sh.n + chunk - 1) / chunk;
  plan->gt = gt;
  plan->nsplit = (int)nsplit;
  plan->chunk = (int)chunk;
  // Uneven pairs of chunks for long streams: 2 * chunk keys are cut 54 : 46 (53 : 47 for groups of heads),
  // the odd-numbered XCDs take the small halves (see the kernel).  Needs an even number of chunks, whole
  // groups of four (batch, kv head) pairs for the renumbering, and a last small chunk that is not empty.
  plan->chunk_big = 0;
  plan->chunk_small = 0;
  const long pairs = (long)sh.batch * sh.kv_heads;
  if (nsplit % 2 == 0 && pairs % 4 == 0 && chunk >= 2048) {
    const long both = 2 * chunk;
    const long small = (both * (gt == 1 ? kSmallShareOneHead : kSmallShareGroups) / 1000 + 32) / 64 * 64;
    const long big = both - small;
    if (small >= min_chunk && (nsplit / 2 - 1) * both + big < (long)sh.n) {
      plan->chunk_big = (int)big;
      plan->chunk_small = (int)small;
    }
  }
  size_t off = 0;
  plan->off_part = off;
  off = align_up(off + (size_t)sh.batch * sh.q_heads * records * kPartStride * sizeof(float), 256);
  plan->off_flag = off;
  off += 256;
  plan->total = off;
  return true;
}

int launch_decode(const qjl_shape& sh, int m_out, const decode_plan& plan, const void* Q, const void* S,
                  const uint8_t* bits, const uint16_t* norms, const uint16_t* norms_out, const void* V,
                  const uint16_t* vscale, const uint16_t* vzero, int vbits, long n_cap, float* out, void* workspace,
                  hipStream_t st, hipEvent_t ev_before, hipEvent_t ev_after, const void* K_new, uint8_t* bits_w,
                  uint16_t* norms_w, const decode_new_token* nt) {
  char* ws = static_cast<char*>(workspace);
  int rc = QJL_OK;
  decode_args a;
  a.Q = Q; a.S = S; a.bits = bits; a.norms = norms; a.V = V;
  a.norms2 = norms_out;
  a.vscale = vscale; a.vzero = vzero;
  a.Knew = K_new; a.bits_w = reinterpret_cast<uint32_t*>(bits_w); a.norms_w = norms_w;
  a.norms2_w = nt ? nt->norms_out_w : nullptr;
  a.channels = nt ? nt->channels : nullptr;
  a.count = nt ? nt->count : 0;
  a.Vnew = nt ? nt->V_new : nullptr;
  a.vcodes_w = nt ? nt->vcodes_w : nullptr;
  a.vscale_w = nt ? nt->vscale_w : nullptr;
  a.vzero_w = nt ? nt->vzero_w : nullptr;
  a.pos_dev = nt ? nt->pos_dev : nullptr;
  a.s_head_stride = m_out > 0 ? (size_t)(sh.m + m_out) * kD : 0;
  a.coef2b = m_out > 0 ? sh.scale * 1.2533141373155002512f / (float)m_out * 1.4426950408889634074f : 0.f;
  a.part = reinterpret_cast<float*>(ws + plan.off_part);
  a.out = out;
  a.n = sh.n;
  a.n_cap = n_cap > 0 ? n_cap : sh.n;
  a.groups_per_kv = (sh.q_heads / sh.kv_heads) / plan.gt;
  a.nsplit = plan.nsplit; a.chunk = plan.chunk;
  // uneven pairs of chunks: not for the streaming step (its newest row and the chunks planned for a capacity
  // keep the plain cut)
  // ... nor for quantized values: there the vector ALU sets the pace, the same on every XCD, and uneven
  // chunks are only uneven (4 x 32 heads x 32768 keys with 4-bit values: 71.9 -> 73.8 us with them)
  const bool uneven = K_new == nullptr && !(vbits > 0 && vscale != nullptr) && m_out == 0 && sh.dtype != QJL_F32;
  a.chunk_big = uneven ? plan.chunk_big : 0;
  a.chunk_small = uneven ? plan.chunk_small : 0;
  a.flag = reinterpret_cast<unsigned long long*>(ws + plan.off_flag);
  static std::atomic<uint32_t> launches{0};            // a number per launch, never 0: names the launch in the flag word
  uint32_t nonce = launches.fetch_add(1, std::memory_order_relaxed) + 1;
  if (nonce == 0) nonce = launches.fetch_add(1, std::memory_order_relaxed) + 1;
  a.nonce = nonce;
  a.coef2 = sh.scale * 1.2533141373155002512f / (float)sh.m * 1.4426950408889634074f;
  switch (sh.dtype) {
    case QJL_F32: rc = launch_m<f32_t>(sh, m_out, vbits, plan, a, st, ev_before, ev_after); break;
    case QJL_F16: rc = launch_m<f16_t>(sh, m_out, vbits, plan, a, st, ev_before, ev_after); break;
    default: rc = launch_m<bf16_t>(sh, m_out, vbits, plan, a, st, ev_before, ev_after); break;
  }
  if (rc != QJL_OK || plan.nsplit == 1) return rc;
  // kernel 3: merge the chunks
  hipLaunchKernelGGL(combine_kernel, dim3((unsigned)(sh.batch * sh.q_heads)), dim3(2 * kD), 0, st,
                     a.part, out, plan.nsplit);
  return launch_status();
}

}  // namespace qjl
