// extern "C" entry points: argument validation and dispatch only.
#include "qjl_common.hpp"

using namespace qjl;

namespace {

bool dtype_ok(int dt) { return dt == QJL_F32 || dt == QJL_F16 || dt == QJL_BF16; }

// Fields every call relies on.
int check_shape(const qjl_shape* sh) {
  if (!sh) return QJL_ERR_INVALID_ARG;
  if (sh->batch < 1 || sh->q_heads < 1 || sh->kv_heads < 1 || sh->n < 1 || sh->d < 1 || sh->m < 1)
    return QJL_ERR_INVALID_ARG;
  if (sh->q_heads % sh->kv_heads != 0) return QJL_ERR_INVALID_ARG;
  if (!dtype_ok(sh->dtype)) return QJL_ERR_INVALID_ARG;
  if (!(sh->scale == sh->scale)) return QJL_ERR_INVALID_ARG;  // NaN
  // index arithmetic inside the kernels is 64-bit, but tile and head counts are int: at most 2^40 cached
  // keys and 2^31 - 1 query heads in all (the products are formed with overflow checks: each factor may be
  // anything up to INT_MAX)
  long rows = (long)sh->batch * sh->kv_heads;            // < 2^62
  if (__builtin_mul_overflow(rows, (long)sh->n, &rows) || rows > (1L << 40)) return QJL_ERR_UNSUPPORTED;
  if ((long)sh->batch * sh->q_heads > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  return QJL_OK;
}

bool ptr_ok(const void* p) { return p != nullptr && aligned16(p); }

// ---- scratch of qjl_decode_attention_noalloc: the per-chunk softmax records, in
// a device array that exists from the moment the library is loaded on a GPU
// until the process ends (every GPU holds its own copy at its own address).
constexpr size_t kScratchBytes = size_t{4} << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// Device address of `scratch` on the current device.  In host code the array's
// name is only a handle for hipGetSymbolAddress, never an address: the pointer
// obtained here is what kernels, copies and fills receive.  Looked up once per
// device ordinal (with that device current) and remembered.
int scratch_of_current_device(void** out) {
  static std::atomic<void*> known[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hip_status(hipErrorInvalidDevice);
  const bool slot = dev >= 0 && dev < 64;
  void* ptr = slot ? known[dev].load(std::memory_order_acquire) : nullptr;
  if (ptr == nullptr) {
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_status(e);
    if (ptr == nullptr) return QJL_ERR_HIP;
    if (slot) known[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return QJL_OK;
}

}  // namespace

extern "C" {

int qjl_version(void) { return 100; }

const char* qjl_status_string(int status) {
  switch (status) {
    case QJL_OK: return "ok";
    case QJL_ERR_INVALID_ARG: return "invalid argument";
    case QJL_ERR_UNSUPPORTED: return "shape not supported by this build";
    case QJL_ERR_WORKSPACE: return "workspace missing or too small";
    case QJL_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int qjl_make_sketch(uint64_t seed, int m, int d, int dtype, void* S, void* stream) {
  if (m < 1 || d < 1 || !dtype_ok(dtype) || !ptr_ok(S)) return QJL_ERR_INVALID_ARG;
  if ((long)m * d > (1L << 31)) return QJL_ERR_UNSUPPORTED;
  return launch_make_sketch(seed, m, d, dtype, S, static_cast<hipStream_t>(stream));
}

int qjl_make_sketch_orthogonal(uint64_t seed, int m, int d, int dtype, void* S, void* stream) {
  if (m < 1 || d < 1 || !dtype_ok(dtype) || !ptr_ok(S)) return QJL_ERR_INVALID_ARG;
  if ((long)m * d > (1L << 31)) return QJL_ERR_UNSUPPORTED;
  return launch_make_sketch_orthogonal(seed, m, d, dtype, S, static_cast<hipStream_t>(stream));
}

int qjl_quantize_keys(const qjl_shape* shape, const void* K, const void* S, uint8_t* bits,
                      uint16_t* norms, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(K) || !ptr_ok(S) || !ptr_ok(bits) || !ptr_ok(norms)) return QJL_ERR_INVALID_ARG;
  if (shape->m % 32 != 0 || shape->d > 1024) return QJL_ERR_UNSUPPORTED;
  return launch_quantize(*shape, K, S, bits, norms, static_cast<hipStream_t>(stream));
}

int qjl_project_query(const qjl_shape* shape, const void* Q, const void* S, float* SQ,
                      void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(Q) || !ptr_ok(S) || !ptr_ok(SQ)) return QJL_ERR_INVALID_ARG;
  if ((long)shape->batch * shape->q_heads > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  return launch_project(shape->batch * shape->q_heads, shape->d, shape->m, shape->dtype, Q, S, SQ,
                        static_cast<hipStream_t>(stream));
}

int qjl_scores(const qjl_shape* shape, const float* SQ, const uint8_t* bits, const uint16_t* norms,
               float* out, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(SQ) || !ptr_ok(bits) || !ptr_ok(norms) || !ptr_ok(out)) return QJL_ERR_INVALID_ARG;
  if (shape->m != 128 && shape->m != 256 && shape->m != 512) return QJL_ERR_UNSUPPORTED;
  return launch_scores(*shape, SQ, bits, norms, out, static_cast<hipStream_t>(stream));
}

size_t qjl_decode_workspace_bytes(const qjl_shape* shape) {
  if (check_shape(shape) != QJL_OK) return 0;
  decode_plan plan;
  if (!plan_decode(*shape, 0, &plan)) return 0;
  return plan.total;
}

size_t qjl_decode_plan(const qjl_shape* shape, int m_out, int splits, int32_t* plan_out) {
  if (check_shape(shape) != QJL_OK || m_out < 0 || splits < 0) return 0;
  decode_plan plan;
  if (!plan_decode(*shape, m_out, &plan, splits)) return 0;
  if (plan_out) {
    plan_out[0] = plan.gt;
    plan_out[1] = plan.nsplit;
    plan_out[2] = plan.chunk;
  }
  return plan.total;
}

int qjl_decode_attention(const qjl_shape* shape, const void* Q, const void* S, const uint8_t* bits,
                         const uint16_t* norms, const void* V, float* out, void* workspace,
                         size_t workspace_bytes, void* stream) {
  return qjl_decode_attention_timed(shape, Q, S, bits, norms, V, out, workspace, workspace_bytes,
                                    stream, nullptr, nullptr);
}

int qjl_decode_attention_splits(const qjl_shape* shape, int splits, const void* Q, const void* S,
                                const uint8_t* bits, const uint16_t* norms, const void* V, float* out,
                                void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(Q) || !ptr_ok(S) || !ptr_ok(bits) || !ptr_ok(norms) || !ptr_ok(V) || !ptr_ok(out) || splits < 1)
    return QJL_ERR_INVALID_ARG;
  decode_plan plan;
  if (!plan_decode(*shape, 0, &plan, splits)) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < plan.total) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return QJL_ERR_INVALID_ARG;
  return launch_decode(*shape, 0, plan, Q, S, bits, norms, nullptr, V, nullptr, nullptr, 0, 0, out, workspace,
                       static_cast<hipStream_t>(stream), nullptr, nullptr);
}

int qjl_decode_attention_timed(const qjl_shape* shape, const void* Q, const void* S,
                               const uint8_t* bits, const uint16_t* norms, const void* V,
                               float* out, void* workspace, size_t workspace_bytes, void* stream,
                               void* event_before, void* event_after) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(Q) || !ptr_ok(S) || !ptr_ok(bits) || !ptr_ok(norms) || !ptr_ok(V) || !ptr_ok(out))
    return QJL_ERR_INVALID_ARG;
  decode_plan plan;
  if (!plan_decode(*shape, 0, &plan)) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < plan.total) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return QJL_ERR_INVALID_ARG;
  return launch_decode(*shape, 0, plan, Q, S, bits, norms, nullptr, V, nullptr, nullptr, 0, 0, out, workspace,
                       static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(event_before),
                       static_cast<hipEvent_t>(event_after));
}

size_t qjl_decode_noalloc_max_bytes(void) { return kScratchBytes; }

int qjl_decode_attention_noalloc(const qjl_shape* shape, const void* Q, const void* S, const uint8_t* bits,
                                 const uint16_t* norms, const void* V, float* out, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(Q) || !ptr_ok(S) || !ptr_ok(bits) || !ptr_ok(norms) || !ptr_ok(V) || !ptr_ok(out))
    return QJL_ERR_INVALID_ARG;
  decode_plan plan;
  if (!plan_decode(*shape, 0, &plan)) return QJL_ERR_UNSUPPORTED;
  if (plan.total > kScratchBytes) return QJL_ERR_WORKSPACE;   // the shape needs more records than the array holds
  void* ws = nullptr;
  rc = scratch_of_current_device(&ws);
  if (rc != QJL_OK) return rc;
  // nothing to clear: every record that the merge kernel reads is written by this call's attention kernel first
  return launch_decode(*shape, 0, plan, Q, S, bits, norms, nullptr, V, nullptr, nullptr, 0, 0, out, ws,
                       static_cast<hipStream_t>(stream), nullptr, nullptr);
}

size_t qjl_outlier_workspace_bytes(const qjl_shape* shape) {
  if (check_shape(shape) != QJL_OK) return 0;
  return outlier_workspace_bytes(*shape);
}

int qjl_select_outliers(const qjl_shape* shape, const void* K, int count, int32_t* channels,
                        void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(K) || channels == nullptr) return QJL_ERR_INVALID_ARG;
  if (count < 1 || count > 16 || count > shape->d) return QJL_ERR_INVALID_ARG;
  if (shape->d > 8192) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < outlier_workspace_bytes(*shape)) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 15u) != 0) return QJL_ERR_INVALID_ARG;
  return launch_select_outliers(*shape, K, count, channels, workspace, static_cast<hipStream_t>(stream));
}

int qjl_make_dual_sketch(const qjl_shape* shape, int m_out, const void* S_in, const void* S_out,
                         const int32_t* channels, int count, void* S_dual, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(S_in) || !ptr_ok(S_out) || !ptr_ok(S_dual) || (channels == nullptr && count > 0))
    return QJL_ERR_INVALID_ARG;
  if (m_out < 1 || count < 0 || count > 16 || count > shape->d) return QJL_ERR_INVALID_ARG;
  if ((long)(shape->m + m_out) * shape->d > (1L << 30) || shape->d > 8192) return QJL_ERR_UNSUPPORTED;
  return launch_make_dual_sketch(*shape, m_out, S_in, S_out, channels, count, S_dual,
                                 static_cast<hipStream_t>(stream));
}

int qjl_quantize_keys_dual(const qjl_shape* shape, int m_out, const void* K, const void* S_dual,
                           const int32_t* channels, int count, uint8_t* bits, uint16_t* norms_in,
                           uint16_t* norms_out, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(K) || !ptr_ok(S_dual) || !ptr_ok(bits) || !ptr_ok(norms_in) || !ptr_ok(norms_out) ||
      (channels == nullptr && count > 0))
    return QJL_ERR_INVALID_ARG;
  if (m_out < 1 || count < 0 || count > 16 || count > shape->d) return QJL_ERR_INVALID_ARG;
  if ((shape->m + m_out) % 32 != 0 || shape->d > 1024) return QJL_ERR_UNSUPPORTED;
  return launch_quantize_dual(*shape, m_out, K, S_dual, channels, count, bits, norms_in, norms_out,
                              static_cast<hipStream_t>(stream));
}

size_t qjl_decode_dual_workspace_bytes(const qjl_shape* shape, int m_out) {
  if (check_shape(shape) != QJL_OK || m_out < 1) return 0;
  decode_plan plan;
  if (!plan_decode(*shape, m_out, &plan)) return 0;
  return plan.total;
}

int qjl_decode_attention_dual(const qjl_shape* shape, int m_out, const void* Q, const void* S_dual,
                              const uint8_t* bits, const uint16_t* norms_in,
                              const uint16_t* norms_out, const void* V, float* out, void* workspace,
                              size_t workspace_bytes, void* stream, void* event_before,
                              void* event_after) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(Q) || !ptr_ok(S_dual) || !ptr_ok(bits) || !ptr_ok(norms_in) || !ptr_ok(norms_out) ||
      !ptr_ok(V) || !ptr_ok(out))
    return QJL_ERR_INVALID_ARG;
  if (m_out < 1) return QJL_ERR_INVALID_ARG;
  decode_plan plan;
  if (!plan_decode(*shape, m_out, &plan)) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < plan.total) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return QJL_ERR_INVALID_ARG;
  return launch_decode(*shape, m_out, plan, Q, S_dual, bits, norms_in, norms_out, V, nullptr, nullptr, 0, 0, out,
                       workspace,
                       static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(event_before),
                       static_cast<hipEvent_t>(event_after));
}

int qjl_quantize_values(const qjl_shape* shape, int vbits, const void* V, uint8_t* vcodes,
                        uint16_t* vscale, uint16_t* vzero, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(V) || !ptr_ok(vcodes) || !ptr_ok(vscale) || !ptr_ok(vzero)) return QJL_ERR_INVALID_ARG;
  if (vbits < 1 || vbits > 8) return QJL_ERR_INVALID_ARG;
  return launch_quantize_values(*shape, vbits, V, vcodes, vscale, vzero, static_cast<hipStream_t>(stream));
}

int qjl_decode_attention_vq(const qjl_shape* shape, int vbits, const void* Q, const void* S,
                            const uint8_t* bits, const uint16_t* norms, const uint8_t* vcodes,
                            const uint16_t* vscale, const uint16_t* vzero, float* out, void* workspace,
                            size_t workspace_bytes, void* stream, void* event_before,
                            void* event_after) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(Q) || !ptr_ok(S) || !ptr_ok(bits) || !ptr_ok(norms) || !ptr_ok(vcodes) || !ptr_ok(vscale) ||
      !ptr_ok(vzero) || !ptr_ok(out))
    return QJL_ERR_INVALID_ARG;
  if (vbits < 1 || vbits > 8) return QJL_ERR_INVALID_ARG;
  if ((vbits != 2 && vbits != 4 && vbits != 8) || shape->dtype == QJL_F32) return QJL_ERR_UNSUPPORTED;
  decode_plan plan;
  if (!plan_decode(*shape, 0, &plan)) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < plan.total) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return QJL_ERR_INVALID_ARG;
  return launch_decode(*shape, 0, plan, Q, S, bits, norms, nullptr, vcodes, vscale, vzero, vbits, 0, out, workspace,
                       static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(event_before),
                       static_cast<hipEvent_t>(event_after));
}

int qjl_decode_attention_dual_vq(const qjl_shape* shape, int m_out, int vbits, const void* Q, const void* S_dual,
                                 const uint8_t* bits, const uint16_t* norms_in, const uint16_t* norms_out,
                                 const uint8_t* vcodes, const uint16_t* vscale, const uint16_t* vzero, float* out,
                                 void* workspace, size_t workspace_bytes, void* stream, void* event_before,
                                 void* event_after) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(Q) || !ptr_ok(S_dual) || !ptr_ok(bits) || !ptr_ok(norms_in) || !ptr_ok(norms_out) || !ptr_ok(vcodes) ||
      !ptr_ok(vscale) || !ptr_ok(vzero) || !ptr_ok(out))
    return QJL_ERR_INVALID_ARG;
  if (m_out < 1 || vbits < 1 || vbits > 8) return QJL_ERR_INVALID_ARG;
  if ((vbits != 2 && vbits != 4 && vbits != 8) || shape->dtype == QJL_F32) return QJL_ERR_UNSUPPORTED;
  if (m_out != 128 || (shape->m != 128 && shape->m != 256)) return QJL_ERR_UNSUPPORTED;
  decode_plan plan;
  if (!plan_decode(*shape, m_out, &plan)) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < plan.total) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return QJL_ERR_INVALID_ARG;
  return launch_decode(*shape, m_out, plan, Q, S_dual, bits, norms_in, norms_out, vcodes, vscale, vzero, vbits, 0, out,
                       workspace, static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(event_before),
                       static_cast<hipEvent_t>(event_after));
}

int qjl_generation_step(const qjl_shape* shape, int m_out, int vbits, int pos, const void* K_new, const void* V_new,
                        const void* Q, const void* S_dual, const int32_t* channels, int count, uint8_t* bits,
                        uint16_t* norms_in, uint16_t* norms_out, uint8_t* vcodes, uint16_t* vscale, uint16_t* vzero,
                        float* out, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(K_new) || !ptr_ok(V_new) || !ptr_ok(Q) || !ptr_ok(S_dual) || !ptr_ok(bits) || !ptr_ok(norms_in) ||
      !ptr_ok(norms_out) || !ptr_ok(vcodes) || !ptr_ok(vscale) || !ptr_ok(vzero) || !ptr_ok(out) ||
      (channels == nullptr && count > 0))
    return QJL_ERR_INVALID_ARG;
  if (m_out < 1 || vbits < 1 || vbits > 8 || count < 0 || count > 16) return QJL_ERR_INVALID_ARG;
  if (pos < 0 || pos >= shape->n) return QJL_ERR_INVALID_ARG;
  if ((vbits != 2 && vbits != 4 && vbits != 8) || shape->dtype == QJL_F32) return QJL_ERR_UNSUPPORTED;
  if (m_out != 128 || (shape->m != 128 && shape->m != 256)) return QJL_ERR_UNSUPPORTED;
  qjl_shape now = *shape;                          // attention covers rows 0..pos of caches with shape->n rows
  now.n = pos + 1;
  decode_plan plan;
  if (!plan_decode(now, m_out, &plan)) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < plan.total) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return QJL_ERR_INVALID_ARG;
  const decode_new_token nt{norms_out, channels, count, V_new, vcodes, vscale, vzero};
  return launch_decode(now, m_out, plan, Q, S_dual, bits, norms_in, norms_out, vcodes, vscale, vzero, vbits, shape->n,
                       out, workspace, static_cast<hipStream_t>(stream), nullptr, nullptr, K_new, bits, norms_in, &nt);
}

int qjl_generation_step_devpos(const qjl_shape* shape, int m_out, int vbits, const int32_t* pos_dev,
                               const void* K_new, const void* V_new, const void* Q, const void* S_dual,
                               const int32_t* channels, int count, uint8_t* bits, uint16_t* norms_in,
                               uint16_t* norms_out, uint8_t* vcodes, uint16_t* vscale, uint16_t* vzero, float* out,
                               void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(pos_dev) || !ptr_ok(K_new) || !ptr_ok(V_new) || !ptr_ok(Q) || !ptr_ok(S_dual) || !ptr_ok(bits) ||
      !ptr_ok(norms_in) || !ptr_ok(norms_out) || !ptr_ok(vcodes) || !ptr_ok(vscale) || !ptr_ok(vzero) || !ptr_ok(out) ||
      (channels == nullptr && count > 0))
    return QJL_ERR_INVALID_ARG;
  if (m_out < 1 || vbits < 1 || vbits > 8 || count < 0 || count > 16) return QJL_ERR_INVALID_ARG;
  if ((vbits != 2 && vbits != 4 && vbits != 8) || shape->dtype == QJL_F32) return QJL_ERR_UNSUPPORTED;
  if (m_out != 128 || (shape->m != 128 && shape->m != 256)) return QJL_ERR_UNSUPPORTED;
  decode_plan plan;                                // the chunks are those of the capacity, whatever the position
  if (!plan_decode(*shape, m_out, &plan)) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < plan.total) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return QJL_ERR_INVALID_ARG;
  decode_new_token nt{norms_out, channels, count, V_new, vcodes, vscale, vzero};
  nt.pos_dev = pos_dev;
  return launch_decode(*shape, m_out, plan, Q, S_dual, bits, norms_in, norms_out, vcodes, vscale, vzero, vbits,
                       shape->n, out, workspace, static_cast<hipStream_t>(stream), nullptr, nullptr, K_new, bits,
                       norms_in, &nt);
}

int qjl_append_keys(const qjl_shape* shape, int pos, int count, const void* K_new, const void* S,
                    uint8_t* bits, uint16_t* norms, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(K_new) || !ptr_ok(S) || !ptr_ok(bits) || !ptr_ok(norms)) return QJL_ERR_INVALID_ARG;
  if (pos < 0 || count < 1 || (long)pos + count > shape->n) return QJL_ERR_INVALID_ARG;
  if (shape->d != 128 || shape->m % 32 != 0) return QJL_ERR_UNSUPPORTED;
  if ((long)shape->batch * shape->kv_heads * count > 0x7FFFFFFFL) return QJL_ERR_UNSUPPORTED;
  return launch_append_keys(*shape, K_new, count, pos, S, bits, norms, static_cast<hipStream_t>(stream));
}

int qjl_decode_step(const qjl_shape* shape, int pos, const void* K_new, const void* Q, const void* S,
                    uint8_t* bits, uint16_t* norms, const void* V, float* out, void* workspace,
                    size_t workspace_bytes, void* stream) {
  int rc = check_shape(shape);
  if (rc != QJL_OK) return rc;
  if (!ptr_ok(K_new) || !ptr_ok(Q) || !ptr_ok(S) || !ptr_ok(bits) || !ptr_ok(norms) || !ptr_ok(V) || !ptr_ok(out))
    return QJL_ERR_INVALID_ARG;
  if (pos < 0 || pos >= shape->n) return QJL_ERR_INVALID_ARG;
  qjl_shape now = *shape;                          // attention covers rows 0..pos of caches with shape->n rows
  now.n = pos + 1;
  decode_plan plan;
  if (!plan_decode(now, 0, &plan)) return QJL_ERR_UNSUPPORTED;
  if (workspace == nullptr || workspace_bytes < plan.total) return QJL_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return QJL_ERR_INVALID_ARG;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (shape->dtype != QJL_F32)                     // 16-bit types: the attention kernel quantizes the new key itself
    return launch_decode(now, 0, plan, Q, S, bits, norms, nullptr, V, nullptr, nullptr, 0, shape->n, out, workspace,
                         st, nullptr, nullptr, K_new, bits, norms);
  rc = launch_append_keys(*shape, K_new, 1, pos, S, bits, norms, st);
  if (rc != QJL_OK) return rc;
  return launch_decode(now, 0, plan, Q, S, bits, norms, nullptr, V, nullptr, nullptr, 0, shape->n, out, workspace, st,
                       nullptr, nullptr);
}

}  // extern "C"
