// Shared device/host helpers of the QJL library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "qjl.h"

namespace qjl {

constexpr int kWave = 64;

// ---------------------------------------------------------------- storage types
// Tag types for the three storage formats of K, Q, V and S.
struct f32_t { using raw = float;    static constexpr int bytes = 4; };
struct f16_t { using raw = uint16_t; static constexpr int bytes = 2; };
struct bf16_t { using raw = uint16_t; static constexpr int bytes = 2; };

__device__ __forceinline__ float bf16_bits_to_float(uint32_t lo16) { return __uint_as_float(lo16 << 16); }
__device__ __forceinline__ float f16_bits_to_float(uint16_t h) {
  _Float16 x;
  __builtin_memcpy(&x, &h, 2);
  return (float)x;
}
__device__ __forceinline__ uint16_t float_to_f16_bits(float f) {  // RNE
  _Float16 x = (_Float16)f;
  uint16_t h;
  __builtin_memcpy(&h, &x, 2);
  return h;
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {  // RNE (finite inputs)
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// Unpack the two 16-bit elements of one dword (element 2i in the low half).
template <typename T> __device__ __forceinline__ void unpack2(uint32_t w, float& a, float& b);
template <> __device__ __forceinline__ void unpack2<bf16_t>(uint32_t w, float& a, float& b) {
  a = __uint_as_float(w << 16);
  b = __uint_as_float(w & 0xFFFF0000u);
}
template <> __device__ __forceinline__ void unpack2<f16_t>(uint32_t w, float& a, float& b) {
  a = f16_bits_to_float((uint16_t)(w & 0xFFFFu));
  b = f16_bits_to_float((uint16_t)(w >> 16));
}

// Load `8` consecutive elements starting at element index `e` (e % 8 == 0 for
// 16-bit types so that the access is one 16-byte load) as floats.
template <typename T> __device__ __forceinline__ void load8(const void* base, size_t e, float (&x)[8]);
template <> __device__ __forceinline__ void load8<f32_t>(const void* base, size_t e, float (&x)[8]) {
  const float4* p = reinterpret_cast<const float4*>(static_cast<const float*>(base) + e);
  float4 a = p[0], b = p[1];
  x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
template <> __device__ __forceinline__ void load8<bf16_t>(const void* base, size_t e, float (&x)[8]) {
  uint4 r = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + e);
  unpack2<bf16_t>(r.x, x[0], x[1]); unpack2<bf16_t>(r.y, x[2], x[3]);
  unpack2<bf16_t>(r.z, x[4], x[5]); unpack2<bf16_t>(r.w, x[6], x[7]);
}
template <> __device__ __forceinline__ void load8<f16_t>(const void* base, size_t e, float (&x)[8]) {
  uint4 r = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(base) + e);
  unpack2<f16_t>(r.x, x[0], x[1]); unpack2<f16_t>(r.y, x[2], x[3]);
  unpack2<f16_t>(r.z, x[4], x[5]); unpack2<f16_t>(r.w, x[6], x[7]);
}

// One element, any alignment.
template <typename T> __device__ __forceinline__ float load1(const void* base, size_t e);
template <> __device__ __forceinline__ float load1<f32_t>(const void* base, size_t e) {
  return static_cast<const float*>(base)[e];
}
template <> __device__ __forceinline__ float load1<bf16_t>(const void* base, size_t e) {
  return bf16_bits_to_float(static_cast<const uint16_t*>(base)[e]);
}
template <> __device__ __forceinline__ float load1<f16_t>(const void* base, size_t e) {
  return f16_bits_to_float(static_cast<const uint16_t*>(base)[e]);
}

// ---------------------------------------------------------------- wavefront reductions (DPP)
// A DPP "row" is 16 lanes.  After the four steps every lane of a row holds the
// row's reduction; the four row results are then merged through readlane.
#define QJL_DPP_F(v, ctrl) \
  __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), (ctrl), 0xF, 0xF, true))

__device__ __forceinline__ float row16_sum(float v) {
  v += QJL_DPP_F(v, 0xB1);   // quad_perm [1,0,3,2]
  v += QJL_DPP_F(v, 0x4E);   // quad_perm [2,3,0,1]
  v += QJL_DPP_F(v, 0x141);  // row_half_mirror
  v += QJL_DPP_F(v, 0x140);  // row_mirror
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, QJL_DPP_F(v, 0xB1));
  v = fmaxf(v, QJL_DPP_F(v, 0x4E));
  v = fmaxf(v, QJL_DPP_F(v, 0x141));
  v = fmaxf(v, QJL_DPP_F(v, 0x140));
  return v;
}
__device__ __forceinline__ float row16_min(float v) {
  v = fminf(v, QJL_DPP_F(v, 0xB1));
  v = fminf(v, QJL_DPP_F(v, 0x4E));
  v = fminf(v, QJL_DPP_F(v, 0x141));
  v = fminf(v, QJL_DPP_F(v, 0x140));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  v = row16_sum(v);
  float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ float wave_max(float v) {
  v = row16_max(v);
  float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// ---------------------------------------------------------------- host side
inline int hip_status(hipError_t e) {
  if (e == hipSuccess) return QJL_OK;
  (void)hipGetLastError();  // clear the sticky error so later calls start clean
  return QJL_ERR_HIP;
}
inline int launch_status() { return hip_status(hipGetLastError()); }

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Launchers implemented one per source file; all validation is done by the
// caller in qjl_api.hip.
int launch_make_sketch(uint64_t seed, int m, int d, int dtype, void* S, hipStream_t st);
int launch_make_sketch_orthogonal(uint64_t seed, int m, int d, int dtype, void* S, hipStream_t st);
int launch_quantize(const qjl_shape& sh, const void* K, const void* S, uint8_t* bits,
                    uint16_t* norms, hipStream_t st);
int launch_quantize_dual(const qjl_shape& sh, int m_out, const void* K, const void* S_dual,
                         const int32_t* channels, int count, uint8_t* bits, uint16_t* norms_in,
                         uint16_t* norms_out, hipStream_t st);
size_t outlier_workspace_bytes(const qjl_shape& sh);
int launch_select_outliers(const qjl_shape& sh, const void* K, int count, int32_t* channels,
                           void* workspace, hipStream_t st);
int launch_make_dual_sketch(const qjl_shape& sh, int m_out, const void* S_in, const void* S_out,
                            const int32_t* channels, int count, void* S_dual, hipStream_t st);
int launch_quantize_values(const qjl_shape& sh, int vbits, const void* V, uint8_t* codes,
                           uint16_t* vscale, uint16_t* vzero, hipStream_t st);
int launch_project(int rows, int d, int m, int dtype, const void* Q, const void* S, float* SQ,
                   hipStream_t st);
int launch_scores(const qjl_shape& sh, const float* SQ, const uint8_t* bits,
                  const uint16_t* norms, float* out, hipStream_t st);

struct decode_plan {
  int gt;            // query heads handled together by one workgroup (divides G)
  int nsplit;        // context chunks per (batch, kv head, head group)
  int chunk;         // keys per chunk (multiple of 64)
  // Not 0: the chunks come in pairs of chunk_big + chunk_small = 2 * chunk keys (both multiples of 64), and
  // of the two workgroups that share a pair the one that runs on an odd-numbered XCD takes the small one.
  int chunk_big, chunk_small;
  size_t off_part;   // byte offset of the per-chunk records inside the workspace
  size_t off_flag;   // byte offset of the 8-byte word through which the workgroups of a launch agree on that
  size_t total;      // bytes
};
// m_out = 0: one code per key (sh.m bits, one shared sketch S[m,d]).  m_out > 0: a key's
// code is sh.m + m_out bits of two independent instances with a norm each, and S
// holds one stacked sketch [sh.m + m_out, d] per (batch, kv head).  vscale != nullptr: V holds
// vbits-bit value codes (2, 4 or 8) with a binary16 scale and zero point per token.
bool plan_decode(const qjl_shape& sh, int m_out, decode_plan* plan, int force_splits = 0);
// What a generation step on two-part codes and quantized values needs beyond K_new / bits_w / norms_w:
// where the outlier part's norm and the new token's value row go, and the head's outlier channels.
struct decode_new_token {
  uint16_t* norms_out_w;
  const int32_t* channels;   // [B,Hkv,count]
  int count;
  const void* V_new;         // [B,Hkv,1,d]
  uint8_t* vcodes_w;
  uint16_t* vscale_w;
  uint16_t* vzero_w;
  // not null: the position of the new token is read from device memory by the kernel (sh.n is then the
  // capacity the plan was made for); values outside [0, sh.n) are clamped into it
  const int32_t* pos_dev = nullptr;
};
int launch_decode(const qjl_shape& sh, int m_out, const decode_plan& plan, const void* Q, const void* S,
                  const uint8_t* bits, const uint16_t* norms, const uint16_t* norms_out, const void* V,
                  const uint16_t* vscale, const uint16_t* vzero, int vbits, long n_cap, float* out, void* workspace,
                  hipStream_t st, hipEvent_t ev_before, hipEvent_t ev_after, const void* K_new = nullptr,
                  uint8_t* bits_w = nullptr, uint16_t* norms_w = nullptr, const decode_new_token* nt = nullptr);
// K_new != nullptr (16-bit types, m_out = 0, no value codes): K_new[B,Hkv,1,d] is the key of position sh.n - 1;
// it is quantized inside the attention kernel, attended to, and written to row sh.n - 1 of bits_w / norms_w
// (the same arrays as bits / norms).
// n_cap: rows per (batch, kv head) in bits / norms / V (0: exactly sh.n, the number of keys attended to).
int launch_append_keys(const qjl_shape& sh, const void* K_new, int t, int pos, const void* S, uint8_t* bits,
                       uint16_t* norms, hipStream_t st);
int device_cu_count();
int allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done);

}  // namespace qjl
