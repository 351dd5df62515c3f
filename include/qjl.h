/*
 * qjl.h -- C ABI of the MI355X (gfx950) QJL key-cache library.
 *
 * QJL (arXiv 2406.03482) compresses the key cache of an attention layer to one
 * sign bit per random projection plus one norm per key, and estimates
 * query-key inner products from that code:
 *
 *   Definition 3.1, Eq. (3)   H_S(k) = sign(S k)                 S in R^{m x d}, i.i.d. N(0,1)
 *   Definition 3.1, Eq. (4)   Prod_QJL(q,k) = sqrt(pi/2)/m * ||k||_2 * <S q, H_S(k)>
 *   Algorithm 1               per key store H_S(k) and nu = ||k||_2; EstimateScores = softmax of Eq. (4)
 *   Section 2, Eq. (1)-(2)    o = sum_j softmax(.)_j v_j
 *
 * General rules for every call
 *   - All data pointers are DEVICE pointers owned by the caller; the library
 *     allocates nothing.  Between calls it remembers only attributes of the
 *     devices it has run on (compute-unit count, "LDS limit of this kernel
 *     already raised"), per device ordinal, in atomics, and a count of the
 *     attention launches it has made (a launch's number names it in a word
 *     of the caller's workspace through which the workgroups of that launch
 *     agree on how they share their chunks): calls from several host threads
 *     and on several devices are safe, and no result depends on that memory.
 *     No environment variable is read.  Tensors are dense,
 *     row-major, with exactly the shapes stated below.  Pointers must be
 *     16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without waiting.
 *   - The return value is a status code; nothing throws or aborts.  Invalid
 *     arguments are rejected on the host before anything is launched.
 *   - Head mapping (grouped-query attention): query head h uses the keys and
 *     values of KV head h / (q_heads / kv_heads).
 *   - Code layout (fixed, shared by all calls): projection i of a key is bit
 *     i%8 of byte i/8 (equivalently bit i%32 of little-endian 32-bit word
 *     i/32); bit 1 means (S k)_i >= 0, i.e. sign +1 (sign(0) := +1).
 *     Norms are IEEE binary16, round-to-nearest-even of the fp32 norm; a
 *     norm above 65504 becomes infinity and the softmax over such a row NaN.
 */
#ifndef QJL_H_
#define QJL_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  QJL_OK = 0,
  QJL_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, misaligned pointer, bad dtype tag */
  QJL_ERR_UNSUPPORTED = -2, /* a valid shape this build has no kernel for (see each call) */
  QJL_ERR_WORKSPACE = -3,   /* workspace missing or smaller than qjl_decode_workspace_bytes() */
  QJL_ERR_HIP = -4          /* the HIP runtime reported an error at launch */
};

/* Storage type of K, Q, V and S (the paper's kernels take bf16, fp16 and fp32). */
enum { QJL_F32 = 0, QJL_F16 = 1, QJL_BF16 = 2 };

typedef struct {
  int32_t batch;    /* B   >= 1; B * Hq < 2^31 and B * Hkv * n <= 2^40, else QJL_ERR_UNSUPPORTED */
  int32_t q_heads;  /* Hq  >= 1, a multiple of kv_heads */
  int32_t kv_heads; /* Hkv >= 1 */
  int32_t n;        /* number of cached keys per (batch, kv head), >= 1; the decode calls take up to 2^30 */
  int32_t d;        /* head dimension; this build: 128 */
  int32_t m;        /* sketch dimension; this build: 128, 256 or 512 */
  int32_t dtype;    /* QJL_F32 / QJL_F16 / QJL_BF16: type of K, Q, V and S */
  float scale;      /* multiplies Eq. (4) before the softmax; 1.0f is Eq. (2) as printed */
} qjl_shape;

/* Library version (major*10000 + minor*100 + patch). Host only. */
int qjl_version(void);

/* Human-readable text for a status code (static storage). Host only. */
const char* qjl_status_string(int status);

/*
 * Algorithm 1 step 1 / Definition 3.1: fill S[m,d] (device, row-major, type
 * `dtype`) with i.i.d. N(0,1) samples that depend only on (seed, m, d, dtype):
 * entry e = i*d+j takes outputs 2e and 2e+1 of the SplitMix64 stream `seed`,
 * U1 = ((a>>11)+1)/2^53, U2 = (b>>11)/2^53, z = sqrt(-2 ln U1) cos(2 pi U2) in
 * fp64, rounded to fp32 and then (for 16-bit types) to `dtype`, both RNE.
 * The same S must be passed to the key and to the query side.
 * Requires m >= 1, d >= 1.
 */
int qjl_make_sketch(uint64_t seed, int m, int d, int dtype, void* S, void* stream);

/*
 * Section 4.1, "Orthogonalized JL transform": the sketch of qjl_make_sketch
 * (same seed, same Gaussian draws) with its rows orthogonalised by QR.  Rows
 * are taken in blocks of d (m > d rows cannot all be orthogonal); inside a
 * block row i becomes the i-th Gram-Schmidt direction of the block's rows,
 * scaled back to the length the Gaussian row had, so that each row is still
 * N(0, I) by itself.  float64 arithmetic, rounded to float32 and then to
 * `dtype`.  d <= 128.  A drop-in replacement for the sketch in every other
 * call.
 */
int qjl_make_sketch_orthogonal(uint64_t seed, int m, int d, int dtype, void* S, void* stream);

/*
 * Algorithm 1 steps 3-4 for all keys at once (Definition 3.1 Eq. (3)):
 *   bits [B,Hkv,n,m/8] (uint8)  <- packed sign(S k)
 *   norms[B,Hkv,n]     (binary16 bit patterns) <- ||k||_2
 * K is [B,Hkv,n,d] and S is [m,d], both of type shape->dtype.  q_heads and
 * scale are ignored.  bf16/fp16 inputs run on the matrix cores with fp32
 * accumulation; fp32 inputs run an fp32 FMA path.  A sign decision can differ
 * from exact arithmetic only when |(S k)_i| is within fp32 rounding of zero
 * (< 1e-5 * ||s_i|| * ||k||).
 */
int qjl_quantize_keys(const qjl_shape* shape, const void* K, const void* S,
                      uint8_t* bits, uint16_t* norms, void* stream);

/*
 * The query side of Eq. (4): SQ[B,Hq,m] (fp32) <- S q for Q[B,Hq,d] of type
 * shape->dtype.  The query is NOT quantized.  kv_heads, n and scale are
 * ignored (kv_heads must still divide q_heads).
 */
int qjl_project_query(const qjl_shape* shape, const void* Q, const void* S,
                      float* SQ, void* stream);

/*
 * Algorithm 1, EstimateScores before the softmax (Eq. (4) for every key):
 *   out[B,Hq,n] (fp32) <- scale * sqrt(pi/2)/m * norms[j] * <SQ[h], sign bits of key j>
 * SQ is [B,Hq,m] fp32 (from qjl_project_query), bits/norms as written by
 * qjl_quantize_keys.  dtype and d are ignored.
 */
int qjl_scores(const qjl_shape* shape, const float* SQ, const uint8_t* bits,
               const uint16_t* norms, float* out, void* stream);

/*
 * Bytes of device scratch qjl_decode_attention needs for this shape
 * (per-chunk softmax partials).  Returns 0
 * for an invalid or unsupported shape.  Host only.
 */
size_t qjl_decode_workspace_bytes(const qjl_shape* shape);

/*
 * One decode step on a quantized key cache (Algorithm 1 EstimateScores, then
 * Eq. (1)):  out[B,Hq,d] (fp32) <- sum_j softmax_j(scale * Prod_QJL(q_h, k_j)) * V[j,:]
 * Q is [B,Hq,d], V is [B,Hkv,n,d], S is [m,d], all of type shape->dtype;
 * bits/norms as written by qjl_quantize_keys.  The context is split into
 * chunks that are processed in parallel and merged with a running
 * max / sum-of-exponentials combine; the result does not depend on the split
 * beyond fp32 rounding.  `workspace` is caller-owned device memory of at
 * least qjl_decode_workspace_bytes(shape) bytes, 256-byte aligned; its
 * contents on entry are irrelevant and undefined on exit.  Two calls that
 * share a workspace must be ordered on the same stream.
 */
int qjl_decode_attention(const qjl_shape* shape, const void* Q, const void* S,
                         const uint8_t* bits, const uint16_t* norms, const void* V,
                         float* out, void* workspace, size_t workspace_bytes,
                         void* stream);

/*
 * For tests and tuning: how qjl_decode_attention (m_out = 0) or
 * qjl_decode_attention_dual (m_out > 0) would cut the context of this shape.
 * splits = 0: the library's own choice; splits > 0: that many chunks, clamped
 * to at most 512 and to at least one 64-key block per wave.  plan_out (host,
 * may be NULL) receives {query heads per workgroup, chunks, keys per chunk}.
 * Returns the workspace bytes of that plan (0: invalid or unsupported shape).
 * The bytes never decrease when shape->n grows.  Host only.
 */
size_t qjl_decode_plan(const qjl_shape* shape, int m_out, int splits, int32_t* plan_out);

/*
 * For tests and tuning: qjl_decode_attention with the number of context chunks
 * fixed by the caller (splits >= 1, clamped as in qjl_decode_plan; workspace
 * of at least qjl_decode_plan(shape, 0, splits, NULL) bytes).  The result
 * equals qjl_decode_attention's up to fp32 rounding (Eq. (1)-(2) do not depend
 * on how the sum over j is cut).
 */
int qjl_decode_attention_splits(const qjl_shape* shape, int splits, const void* Q, const void* S,
                                const uint8_t* bits, const uint16_t* norms, const void* V, float* out,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * qjl_decode_attention, plus kernel timing without a profiler: the two
 * caller-owned events (hipEvent_t passed as void*, created with timing
 * enabled; either may be NULL) receive the start and the stop timestamp of
 * the attention kernel itself (S q, Algorithm 1 EstimateScores, Eq. (1)), the
 * way a profiler sees that dispatch; the chunk-merge kernel after it is
 * outside the interval.
 * hipEventElapsedTime(before, after) is valid once `after` has completed.
 * Everything else is exactly qjl_decode_attention.
 */
int qjl_decode_attention_timed(const qjl_shape* shape, const void* Q, const void* S,
                               const uint8_t* bits, const uint16_t* norms, const void* V,
                               float* out, void* workspace, size_t workspace_bytes,
                               void* stream, void* event_before, void* event_after);

/*
 * For callers that cannot allocate device memory or carry a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): qjl_decode_attention without the workspace arguments.  The
 * per-chunk records live in a device array inside the library, 4 MiB
 * (qjl_decode_noalloc_max_bytes(), 7943 (query head, chunk) records) that every
 * GPU the library runs on holds until the process ends.  The call allocates and
 * frees nothing and calls no allocating routine.  A shape whose
 * qjl_decode_workspace_bytes() exceeds the array is rejected with
 * QJL_ERR_WORKSPACE (all of this build's benchmark shapes fit: the largest
 * needs 1.1 MB).  Every call on a GPU uses that GPU's one array, whose contents
 * are whatever the last call left (nothing needs clearing: each call writes
 * every record before it reads it): two calls that overlap in time on one GPU
 * -- different streams, or different threads -- race and must be ordered by the
 * caller.  Inputs, outputs, result and every other rule as in
 * qjl_decode_attention.
 */
size_t qjl_decode_noalloc_max_bytes(void);
int qjl_decode_attention_noalloc(const qjl_shape* shape, const void* Q, const void* S,
                                 const uint8_t* bits, const uint16_t* norms, const void* V,
                                 float* out, void* stream);

/* ------------------------------------------------------------------------
 * Outlier channels (Section 4.1, "Outliers"; end of Section 1): certain fixed
 * channels of the keys of a head are much larger than the rest; they are
 * identified in the prompt phase and two independent copies of the quantizer
 * are applied to the outlier and to the inlier coordinates, the outlier copy
 * with more bits per coordinate.  The paper fixes no selection rule, sizes or
 * layout; the calls below use:
 *   - per (batch, kv head) the `count` channels with the largest mean |k| over
 *     the n tokens, in decreasing order, ties to the lower channel index;
 *   - inlier copy: the key with those coordinates set to zero, sketch
 *     S_in[m,d]; outlier copy: only those coordinates (in place), sketch
 *     S_out[m_out,d]; a binary16 norm of each part; the query is split the
 *     same way and the two Eq. (4) estimates are added;
 *   - a cache row is the m/8 bytes of the inlier code followed by the
 *     m_out/8 bytes of the outlier code.
 * In these calls shape->m is the inlier sketch size.
 * ---------------------------------------------------------------------- */

/* Bytes of device scratch qjl_select_outliers needs (partial sums).  Host only. */
size_t qjl_outlier_workspace_bytes(const qjl_shape* shape);

/*
 * channels[B,Hkv,count] (int32, device) <- for every (batch, kv head) the
 * `count` channels of K[B,Hkv,n,d] with the largest sum_j |K[j,t]| (fp32
 * accumulation in a fixed order), largest first, ties to the lower index.
 * 1 <= count <= min(d, 16).  workspace: caller-owned device memory of at least
 * qjl_outlier_workspace_bytes(shape) bytes; asynchronous on `stream`.
 */
int qjl_select_outliers(const qjl_shape* shape, const void* K, int count, int32_t* channels,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * S_dual[B,Hkv,m+m_out,d] (device, shape->dtype) <- per (batch, kv head) the
 * stacked sketch: rows [0,m) are S_in[m,d] with that head's outlier columns
 * set to zero, rows [m,m+m_out) are S_out[m_out,d] with every other column set
 * to zero.  sign(S_dual k) is then the inlier code followed by the outlier
 * code, and S_dual q the two query projections.  Channel entries outside
 * [0,d) are ignored; count == 0 (channels may then be NULL) leaves S_in whole
 * and the outlier rows zero.
 */
int qjl_make_dual_sketch(const qjl_shape* shape, int m_out, const void* S_in, const void* S_out,
                         const int32_t* channels, int count, void* S_dual, void* stream);

/*
 * Algorithm 1 steps 3-4, twice per key: bits[B,Hkv,n,(m+m_out)/8] <- packed
 * sign(S_dual k) (same bit order as qjl_quantize_keys), norms_in[B,Hkv,n] <-
 * ||k without its head's outlier channels||, norms_out[B,Hkv,n] <- ||those
 * channels of k||, both binary16 (each summed over its own coordinates).
 * (m+m_out) % 32 == 0.  Channel entries outside [0,d) are ignored and a
 * channel listed twice counts once, as in qjl_make_dual_sketch.  A norm above
 * 65504 is stored as binary16 infinity, and a decode step over such a row
 * yields NaN: keys must be scaled to stay below that.
 */
int qjl_quantize_keys_dual(const qjl_shape* shape, int m_out, const void* K, const void* S_dual,
                           const int32_t* channels, int count, uint8_t* bits, uint16_t* norms_in,
                           uint16_t* norms_out, void* stream);

/* Workspace of qjl_decode_attention_dual; 0 for unsupported shapes.  Host only. */
size_t qjl_decode_dual_workspace_bytes(const qjl_shape* shape, int m_out);

/*
 * qjl_decode_attention on a cache written by qjl_quantize_keys_dual:
 *   score_j = scale * sqrt(pi/2) * ( norms_in[j]/m * <S_in q_in, inlier bits_j>
 *                                  + norms_out[j]/m_out * <S_out q_out, outlier bits_j> )
 * then softmax and Eq. (1).  S_dual as written by qjl_make_dual_sketch.
 * Supported: d == 128 and (m, m_out) in {(128,128), (256,128), (512,128),
 * (256,256)}.  Workspace rules as for
 * qjl_decode_attention; event_before / event_after (may be NULL) as in
 * qjl_decode_attention_timed.
 */
int qjl_decode_attention_dual(const qjl_shape* shape, int m_out, const void* Q, const void* S_dual,
                              const uint8_t* bits, const uint16_t* norms_in,
                              const uint16_t* norms_out, const void* V, float* out, void* workspace,
                              size_t workspace_bytes, void* stream, void* event_before,
                              void* event_after);

/* ------------------------------------------------------------------------
 * Value cache (Section 3.2): "normalizing each token's entries and then
 * rounding each entry to a few-bit integer".  Scheme used: per (batch, kv
 * head, token) zero point = the row's minimum, scale = (max - min)/(2^b - 1),
 * both stored as binary16; code = (v - zero)/scale rounded to nearest (ties to
 * even), clipped to [0, 2^b - 1], taken in float32 against the stored zero
 * point and scale; element t of a row occupies bits [b*t, b*t + b) of the
 * row's d*b/8 bytes (LSB first); a value reads back as zero + code * scale.
 * ---------------------------------------------------------------------- */

/*
 * vcodes[B,Hkv,n,d*vbits/8], vscale[B,Hkv,n], vzero[B,Hkv,n] (binary16) <-
 * V[B,Hkv,n,d] of type shape->dtype.  Supported: vbits in {2, 4, 8}, d == 128.
 */
int qjl_quantize_values(const qjl_shape* shape, int vbits, const void* V, uint8_t* vcodes,
                        uint16_t* vscale, uint16_t* vzero, void* stream);

/*
 * qjl_decode_attention with the values taken from a cache written by
 * qjl_quantize_values: out[B,Hq,d] <- sum_j softmax_j(...) * (vzero[j] + vscale[j] * code[j,:]).
 * Supported: vbits in {2, 4, 8}, d == 128, 16-bit shape->dtype (type of Q and S).
 * Workspace: qjl_decode_workspace_bytes(shape); events as in qjl_decode_attention_timed.
 */
int qjl_decode_attention_vq(const qjl_shape* shape, int vbits, const void* Q, const void* S,
                            const uint8_t* bits, const uint16_t* norms, const uint8_t* vcodes,
                            const uint16_t* vscale, const uint16_t* vzero, float* out,
                            void* workspace, size_t workspace_bytes, void* stream,
                            void* event_before, void* event_after);

/* ------------------------------------------------------------------------
 * Streaming (Algorithm 1's loop over the token stream): a key is quantized
 * when it arrives and appended to the cache; the estimator runs over the keys
 * stored so far.  In these calls shape->n is the capacity of the caches
 * (rows per (batch, kv head) of bits, norms and V).
 * ---------------------------------------------------------------------- */

/*
 * Algorithm 1 steps 3-4 for `count` new tokens: K_new[B,Hkv,count,d] ->
 * rows pos..pos+count-1 of bits[B,Hkv,n,m/8] and norms[B,Hkv,n]; other rows are
 * not touched.  0 <= pos, pos + count <= n.  d == 128.
 */
int qjl_append_keys(const qjl_shape* shape, int pos, int count, const void* K_new, const void* S,
                    uint8_t* bits, uint16_t* norms, void* stream);

/*
 * One generation step: K_new[B,Hkv,1,d] is quantized into row `pos` of the
 * caches, then out[B,Hq,d] <- attention of Q[B,Hq,d] over rows 0..pos
 * (Algorithm 1 EstimateScores + Eq. (1)).  Row `pos` of V[B,Hkv,n,d] must
 * already hold the new token's value.  Workspace:
 * qjl_decode_workspace_bytes(shape), taken at the capacity, covers every pos.  For 16-bit types the
 * key is quantized inside the attention kernel (one launch less than
 * qjl_append_keys + qjl_decode_attention); the cache row is written by that
 * kernel and is complete when the call's work on `stream` is.
 */
int qjl_decode_step(const qjl_shape* shape, int pos, const void* K_new, const void* Q, const void* S,
                    uint8_t* bits, uint16_t* norms, const void* V, float* out, void* workspace,
                    size_t workspace_bytes, void* stream);

/* ------------------------------------------------------------------------
 * The paper's operating point as one path: two-part key codes (Section 4.1,
 * used "in all experiments"), token-wise quantized values (Section 3.2) and a
 * cache that grows with the token stream (Algorithm 1).  m + m_out = 384 with
 * 4-bit values is 3 bits per cached number for the keys and 4.25 for the
 * values.  Supported: d == 128, m in {128, 256}, m_out == 128, vbits in
 * {2, 4, 8}, 16-bit shape->dtype.
 * ---------------------------------------------------------------------- */

/*
 * qjl_decode_attention_dual with the values taken from a cache written by
 * qjl_quantize_values:
 *   out[B,Hq,d] <- sum_j softmax_j(score_j) * (vzero[j] + vscale[j] * code[j,:])
 * with score_j the sum of the two Eq. (4) estimates as in
 * qjl_decode_attention_dual.  Workspace: qjl_decode_dual_workspace_bytes(shape,
 * m_out); events as in qjl_decode_attention_timed.
 */
int qjl_decode_attention_dual_vq(const qjl_shape* shape, int m_out, int vbits, const void* Q,
                                 const void* S_dual, const uint8_t* bits, const uint16_t* norms_in,
                                 const uint16_t* norms_out, const uint8_t* vcodes,
                                 const uint16_t* vscale, const uint16_t* vzero, float* out,
                                 void* workspace, size_t workspace_bytes, void* stream,
                                 void* event_before, void* event_after);

/*
 * One generation step (the body of Algorithm 1's loop) on such caches of
 * capacity shape->n rows per (batch, kv head).  The new token's key
 * K_new[B,Hkv,1,d] is quantized by the two quantizers of Section 4.1 --
 * sign(S_dual k) and the norms of k without / on its head's outlier channels
 * (channels[B,Hkv,count], as in qjl_quantize_keys_dual) -- and its value row
 * V_new[B,Hkv,1,d] token-wise as in qjl_quantize_values; both are written to row
 * `pos` of bits / norms_in / norms_out / vcodes / vscale / vzero.  Then
 *   out[B,Hq,d] <- attention of Q[B,Hq,d] over rows 0..pos,
 * the new token included with its code and its value as stored.  One launch of
 * the attention kernel (+ the chunk merge): the new row is quantized inside it,
 * used from on-chip memory, and written to the caches by that kernel; it is
 * complete when the call's work on `stream` is.  0 <= pos < shape->n.
 * Workspace: qjl_decode_dual_workspace_bytes(shape, m_out), taken at the
 * capacity, covers every pos.
 */
int qjl_generation_step(const qjl_shape* shape, int m_out, int vbits, int pos, const void* K_new,
                        const void* V_new, const void* Q, const void* S_dual,
                        const int32_t* channels, int count, uint8_t* bits, uint16_t* norms_in,
                        uint16_t* norms_out, uint8_t* vcodes, uint16_t* vscale, uint16_t* vzero,
                        float* out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same generation step (Algorithm 1's loop body at the operating point of
 * Section 4.1 + Section 3.2) with the position read from device memory by the
 * kernel: a step recorded once into a HIP graph can be replayed for a whole
 * generation, the caller advancing *pos_dev (device int32) between replays by
 * work of its own on the same stream.  shape->n is the capacity of the caches.
 * The context is always cut into the chunks planned for the capacity, so a step
 * far below the capacity leaves most workgroups without keys (they write an
 * empty record); qjl_generation_step, which plans for pos + 1, is the faster
 * call outside graphs.  A value of *pos_dev outside [0, shape->n) cannot be
 * reported from inside the kernel: it is clamped into that range.  Everything
 * else -- arguments, supported combinations, workspace (taken at the capacity),
 * results bit for bit up to the order in which chunks are summed -- as
 * qjl_generation_step.
 */
int qjl_generation_step_devpos(const qjl_shape* shape, int m_out, int vbits, const int32_t* pos_dev,
                               const void* K_new, const void* V_new, const void* Q, const void* S_dual,
                               const int32_t* channels, int count, uint8_t* bits, uint16_t* norms_in,
                               uint16_t* norms_out, uint8_t* vcodes, uint16_t* vscale, uint16_t* vzero,
                               float* out, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QJL_H_ */
