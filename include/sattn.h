/*
 * sattn.h -- C ABI of the MI355X (gfx950) fused sigmoid-attention library.
 *
 * The library computes, per (batch, head), with Q, K, V of shape [N, d]:
 *
 *     S = Q K^T / sqrt(d)                     (paper: Appendix F.1 table, "Forward")
 *     T = S + bias - slope_h * |i - j|        (bias: Section 2 boxed equation, b = -log n in
 *                                              practice, Appendix E; ALiBi: Appendix F.4)
 *     P = sigmoid(T), P_ij = 0 if causal and j > i   (mask keeps the diagonal, Appendix G.1)
 *     O = P V                                 (Algorithm 1)
 *
 * and the recompute-based backward of Algorithm 2, which needs only Q, K, V, dO:
 *
 *     dV = P^T dO,  dP = dO V^T,  dS = P (1 - P) dP,
 *     dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d).
 *
 * (The paper's table prints sqrt(d) in the last two; with S scaled by 1/sqrt(d) the chain
 * rule gives 1/sqrt(d), which is what is implemented.)  No row maximum, row sum or
 * log-sum-exp is kept between the passes.  A softmax flash-attention pair built on the
 * same tiling is exported for on-chip comparison (Appendix F.1 table, left half).
 *
 * Conventions for every entry point
 *  - All tensor pointers are DEVICE pointers.  The caller owns every buffer; the library
 *    never allocates, frees or keeps device memory.
 *  - Tensors are [B, H, N, d] with the last dimension contiguous.  A NULL strides pointer
 *    means fully contiguous [B, H, N, d]; otherwise strides are in ELEMENTS and must be
 *    multiples of 8 (bf16) or 4 (f32) so that rows stay 16-byte aligned.  Base pointers
 *    must be 16-byte aligned.
 *  - d must be 64 or 128.  N >= 1 need not be a multiple of any tile size.
 *  - SATTN_BF16: inputs/outputs bf16, logits, sigmoid and accumulation in fp32, P and dS
 *    rounded to bf16 before the second matrix product.  SATTN_F32: everything fp32.
 *  - bias is the scalar b in natural-log units (callers pass -log(N)); alibi_slopes is a
 *    device pointer to H floats or NULL; causal is 0 or 1.
 *  - Calls are asynchronous on `stream` (a hipStream_t; NULL = default stream) and launch on
 *    the calling thread's current device, which must be the device of the stream and of the
 *    buffers.  No hidden synchronisation.  The entry points of this header may be called
 *    from several threads at once; the only process-wide state they read is the forced tile
 *    shape of sattn_bench.h (measurements only, see there).
 *  - Return 0 on success, a negative SATTN_ERR_* otherwise.  Argument errors (every code but
 *    SATTN_ERR_LAUNCH) are found before anything is launched: nothing is written.  An entry
 *    point that launches several kernels (the backward passes, the softmax backward with its
 *    pre-pass, the bias gradient) returns SATTN_ERR_LAUNCH as soon as the runtime rejects one
 *    of them; kernels launched before that one have run, so outputs may be partly written.
 *
 * Measurement and comparison aids (compiler-scheduled twins of the sigmoid kernels, the
 * matrix-rate probe, the tile-shape setters, device information) are declared in
 * sattn_bench.h, not here.
 */
#ifndef SATTN_H_
#define SATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SATTN_BF16 = 0, SATTN_F32 = 1 } sattn_dtype;

typedef struct {
  int64_t batch; /* elements between consecutive batches */
  int64_t head;  /* elements between consecutive heads   */
  int64_t seq;   /* elements between consecutive tokens  */
} sattn_strides;

enum {
  SATTN_OK = 0,
  SATTN_ERR_NULL = -1,        /* a required pointer is NULL */
  SATTN_ERR_SHAPE = -2,       /* B, H or N not positive, too large for 32-bit tile indexing, or
                                 (N + 256) * seq stride * element size exceeds 4 GiB - 1 */
  SATTN_ERR_UNSUPPORTED = -3, /* d not in {64,128} or unknown dtype */
  SATTN_ERR_ALIGN = -4,       /* pointer or stride breaks the 16-byte rule */
  SATTN_ERR_WORKSPACE = -5,   /* workspace NULL or smaller than *_workspace_bytes() */
  SATTN_ERR_LAUNCH = -6,      /* the HIP runtime rejected the launch */
  SATTN_ERR_TOO_LARGE = -7    /* softmax_attn_bwd_noalloc: more padded query rows than its scratch holds */
};

/* Forward pass of sigmoid attention (Algorithm 1): writes O only. */
int sigmoid_attn_fwd(const void* q, const void* k, const void* v, void* o,
                     int B, int H, int N, int d, sattn_dtype dtype,
                     float bias, int causal, const float* alibi_slopes,
                     const sattn_strides* sq, const sattn_strides* sk,
                     const sattn_strides* sv, const sattn_strides* so,
                     void* stream);

/* Backward pass of sigmoid attention (Algorithm 2): reads Q, K, V, dO; writes dQ, dK, dV.
 * P is recomputed on chip; neither O nor any per-row statistic is read.  No gradient is
 * produced for bias or alibi_slopes.  `workspace` must hold at least
 * sigmoid_attn_bwd_workspace_bytes() bytes (may be NULL when that is 0); its contents on
 * entry are ignored. */
int sigmoid_attn_bwd(const void* q, const void* k, const void* v, const void* dout,
                     void* dq, void* dk, void* dv,
                     int B, int H, int N, int d, sattn_dtype dtype,
                     float bias, int causal, const float* alibi_slopes,
                     const sattn_strides* sq, const sattn_strides* sk,
                     const sattn_strides* sv, const sattn_strides* sdout,
                     const sattn_strides* sdq, const sattn_strides* sdk,
                     const sattn_strides* sdv,
                     void* workspace, size_t workspace_bytes, void* stream);

size_t sigmoid_attn_bwd_workspace_bytes(int B, int H, int N, int d, sattn_dtype dtype);

/* The two halves of sigmoid_attn_bwd as separate launches (Algorithm 2 split by output
 * owner): *_dkdv keeps a key block on chip and streams query blocks (dK_j, dV_j of
 * Algorithm 2's outer loop); *_dq keeps a query block on chip and streams key blocks, so
 * dQ_i never round-trips through HBM.  Calling both equals sigmoid_attn_bwd. */
int sigmoid_attn_bwd_dkdv(const void* q, const void* k, const void* v, const void* dout,
                          void* dk, void* dv,
                          int B, int H, int N, int d, sattn_dtype dtype,
                          float bias, int causal, const float* alibi_slopes,
                          const sattn_strides* sq, const sattn_strides* sk,
                          const sattn_strides* sv, const sattn_strides* sdout,
                          const sattn_strides* sdk, const sattn_strides* sdv,
                          void* stream);
int sigmoid_attn_bwd_dq(const void* q, const void* k, const void* v, const void* dout,
                        void* dq,
                        int B, int H, int N, int d, sattn_dtype dtype,
                        float bias, int causal, const float* alibi_slopes,
                        const sattn_strides* sq, const sattn_strides* sk,
                        const sattn_strides* sv, const sattn_strides* sdout,
                        const sattn_strides* sdq,
                        void* stream);

/* Softmax flash attention with the same tiling, for comparison (Appendix F.1 table, left
 * half).  lse is [B, H, N] fp32, contiguous, natural-log units: lse_i = log sum_j exp(T_ij)
 * with T = S - slope_h |i-j| (no bias: a constant shift cancels). */
int softmax_attn_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
                     int B, int H, int N, int d, sattn_dtype dtype,
                     int causal, const float* alibi_slopes,
                     const sattn_strides* sq, const sattn_strides* sk,
                     const sattn_strides* sv, const sattn_strides* so,
                     void* stream);

/* Softmax backward: dS = P (dP - rowsum(dO o O)); reads O and lse from the forward.
 * The workspace holds two fp32 vectors per query row (the rowsum D and the rescaled log-sum-exp),
 * rows padded to a multiple of 64: softmax_attn_bwd_workspace_bytes() says how much. */
int softmax_attn_bwd(const void* q, const void* k, const void* v, const void* o,
                     const float* lse, const void* dout,
                     void* dq, void* dk, void* dv,
                     int B, int H, int N, int d, sattn_dtype dtype,
                     int causal, const float* alibi_slopes,
                     const sattn_strides* sq, const sattn_strides* sk,
                     const sattn_strides* sv, const sattn_strides* so,
                     const sattn_strides* sdout,
                     const sattn_strides* sdq, const sattn_strides* sdk,
                     const sattn_strides* sdv,
                     void* workspace, size_t workspace_bytes, void* stream);

size_t softmax_attn_bwd_workspace_bytes(int B, int H, int N, int d, sattn_dtype dtype);

/* softmax_attn_bwd for callers that cannot allocate device memory or pass a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments, results and errors as softmax_attn_bwd without `workspace`; the two fp32 per
 * padded query row live in a fixed 8 MiB array inside the library's device image (one copy per
 * GPU, held until the process ends) whose address is looked up on the first call on each device.
 * Limit: B * H * roundup(N, 64) <= softmax_attn_bwd_noalloc_max_rows() (2^20), else
 * SATTN_ERR_TOO_LARGE and nothing is launched.  No hipMalloc / hipFree / allocating library
 * routine is called.  All calls on one GPU share that GPU's array: calls that may overlap on one
 * GPU (different streams or threads) race on it and must be ordered by the caller; calls on
 * one stream are ordered by the stream.  Nothing needs clearing between calls (the pre-pass
 * rewrites every entry that the call reads). */
int softmax_attn_bwd_noalloc(const void* q, const void* k, const void* v, const void* o,
                             const float* lse, const void* dout,
                             void* dq, void* dk, void* dv,
                             int B, int H, int N, int d, sattn_dtype dtype,
                             int causal, const float* alibi_slopes,
                             const sattn_strides* sq, const sattn_strides* sk,
                             const sattn_strides* sv, const sattn_strides* so,
                             const sattn_strides* sdout,
                             const sattn_strides* sdq, const sattn_strides* sdk,
                             const sattn_strides* sdv, void* stream);
size_t softmax_attn_bwd_noalloc_max_rows(void);

/* Hybrid-norm (Section 5.5, Appendix G.6: x + norm(attention output), a LayerNorm without
 * learnable affine parameters; RMSNorm is the other norm the paper's models use).  Token (b, n)
 * of a [B,H,N,d] bf16 tensor (any batch/head/token strides, NULL = contiguous) is normalised
 * over its H*d features:  LayerNorm  y = (x - mean) / sqrt(var + eps)  (population variance),
 * RMSNorm  y = x / sqrt(mean(x^2) + eps).  Statistics are fp32; `stats` (device, [B,N,2] fp32,
 * 8-byte aligned) receives mean (0 for RMSNorm) and 1/sqrt(. + eps) per token in the forward
 * call and is read by the backward call, which returns dx for L = sum(y * dy) from x, dy and
 * those statistics.  One read and one write of the tensor (two reads in the backward).  bf16
 * only, d in {64,128}, H*d <= 8192 (SATTN_ERR_SHAPE beyond).  The residual add and any affine
 * parameters are the caller's. */
typedef enum { SATTN_NORM_LAYER = 0, SATTN_NORM_RMS = 1 } sattn_norm_kind;
int sattn_headconcat_norm_fwd(const void* x, void* y, float* stats, int B, int H, int N, int d,
                              sattn_dtype dtype, int kind, float eps,
                              const sattn_strides* sx, const sattn_strides* sy, void* stream);
int sattn_headconcat_norm_bwd(const void* x, const void* dy, const float* stats, void* dx,
                              int B, int H, int N, int d, sattn_dtype dtype, int kind,
                              const sattn_strides* sx, const sattn_strides* sdy,
                              const sattn_strides* sdx, void* stream);

/* Forward tile shape (Appendix F.5: the block shape of the forward kernel is a tuning
 * parameter; the paper's second variant halves B_c for d = 64).  Here the tuned quantities are
 * the query rows per workgroup and per wave and, for 4-wave workgroups at d = 128, the depth of
 * the V ring in LDS: 4 or 8 waves of 32 query rows (two waves per SIMD), or, at d = 128 on long
 * key loops, 4 waves of 64 query rows (one wave per SIMD, half the LDS traffic per MFMA).  The
 * bf16 forward entry points (sigmoid, softmax, variable-length, ...) choose them per problem
 * from d, B*H*N, the mask and the number of compute units.  sattn_fwd_waves returns that
 * choice as 4, 8, or 64 for the four 64-row waves (the softmax comparison kernel and
 * non-causal ALiBi run the 8-wave shape where 64 is returned); sattn_fwd_v_slots returns the V
 * ring depth (3; 2: two 4-wave workgroups per compute unit); both return a negative error code
 * for bad arguments.  The outputs are bit-identical for all shapes: the arithmetic of a query
 * row does not depend on which rows share its workgroup. */
int sattn_fwd_waves(int B, int H, int N, int d, int causal);
int sattn_fwd_v_slots(int B, int H, int N, int d, int causal);

/* Human-readable text for an SATTN_ERR_* code (static storage). */
const char* sattn_strerror(int code);

/* Shared key/value heads (Section 5.1, multi-query attention: one K/V head for all query
 * heads; any Hkv that divides H is accepted).  Query head h attends to K/V head
 * h / (H / Hkv).  q, o, dout, dq are [B, H, N, d]; k, v, dk, dv are [B, Hkv, N, d] (strides as
 * usual, NULL = contiguous with that head count).  dK/dV of a shared head is the sum over its
 * query heads, accumulated in fp32 inside one workgroup (no atomics, no workspace).  bf16 or
 * fp32; SATTN_ERR_SHAPE if Hkv does not divide H.  Otherwise as sigmoid_attn_fwd /
 * sigmoid_attn_bwd. */
int sigmoid_attn_mqa_fwd(const void* q, const void* k, const void* v, void* o,
                         int B, int H, int Hkv, int N, int d, sattn_dtype dtype,
                         float bias, int causal, const float* alibi_slopes,
                         const sattn_strides* sq, const sattn_strides* sk,
                         const sattn_strides* sv, const sattn_strides* so, void* stream);
int sigmoid_attn_mqa_bwd(const void* q, const void* k, const void* v, const void* dout,
                         void* dq, void* dk, void* dv,
                         int B, int H, int Hkv, int N, int d, sattn_dtype dtype,
                         float bias, int causal, const float* alibi_slopes,
                         const sattn_strides* sq, const sattn_strides* sk,
                         const sattn_strides* sv, const sattn_strides* sdout,
                         const sattn_strides* sdq, const sattn_strides* sdk,
                         const sattn_strides* sdv, void* stream);

/* sigmoid_attn_mqa_bwd for problems with few K/V heads (Section 5.1 trains with one): there the
 * dK/dV pass, one workgroup per K/V head and 128 keys, leaves compute units idle or unevenly
 * loaded, and this form splits the query heads of a group over 2, 4, ... workgroups that write
 * fp32 partial dK, dV to `workspace` (device memory, 16-byte aligned, at least
 * sigmoid_attn_mqa_bwd_workspace_bytes(...) bytes, contents undefined before and after), added
 * up and rounded to bf16 once by a second kernel.  ..._workspace_bytes returns 0 where the
 * library would not split (enough K/V heads, fp32, invalid arguments): the call then equals
 * sigmoid_attn_mqa_bwd and workspace may be NULL.  The results differ from sigmoid_attn_mqa_bwd's
 * only in the order of the fp32 sums over the query heads.  SATTN_ERR_WORKSPACE if the
 * workspace is NULL or too small where one is needed. */
size_t sigmoid_attn_mqa_bwd_workspace_bytes(int B, int H, int Hkv, int N, int d, sattn_dtype dtype, int causal);
int sigmoid_attn_mqa_bwd_split(const void* q, const void* k, const void* v, const void* dout,
                               void* dq, void* dk, void* dv,
                               int B, int H, int Hkv, int N, int d, sattn_dtype dtype,
                               float bias, int causal, const float* alibi_slopes,
                               const sattn_strides* sq, const sattn_strides* sk,
                               const sattn_strides* sv, const sattn_strides* sdout,
                               const sattn_strides* sdq, const sattn_strides* sdk,
                               const sattn_strides* sdv, void* workspace, size_t workspace_bytes,
                               void* stream);

/* Different numbers of queries and keys (the definition of Section 2 with Q of n_q rows and
 * K, V of n_k rows; the paper's models only use n_q = n_k).  q, o, dout, dq are [B,H,Nq,d];
 * k, v, dk, dv are [B,H,Nk,d].  Plain sigmoid attention only (bf16 or fp32): no causal mask, no ALiBi
 * (both are defined by positions that the two sides would have to share), one K/V head per
 * query head; `bias` is the caller's (the paper's rule gives -ln(Nk)).  Otherwise as
 * sigmoid_attn_fwd / sigmoid_attn_bwd. */
int sigmoid_attn_cross_fwd(const void* q, const void* k, const void* v, void* o,
                           int B, int H, int Nq, int Nk, int d, sattn_dtype dtype, float bias,
                           const sattn_strides* sq, const sattn_strides* sk,
                           const sattn_strides* sv, const sattn_strides* so, void* stream);
int sigmoid_attn_cross_bwd(const void* q, const void* k, const void* v, const void* dout,
                           void* dq, void* dk, void* dv,
                           int B, int H, int Nq, int Nk, int d, sattn_dtype dtype, float bias,
                           const sattn_strides* sq, const sattn_strides* sk,
                           const sattn_strides* sv, const sattn_strides* sdout,
                           const sattn_strides* sdq, const sattn_strides* sdk,
                           const sattn_strides* sdv, void* stream);

/* The same with the queries placed at the END of the key sequence: query i sits at position
 * i + Nk - Nq (the keys and values of a prefix are already there and Nq new tokens attend to
 * them).  That placement is this library's reading, the paper's models only have Nq = Nk; it
 * gives the causal mask (Appendix E.1: key j is kept for query i iff j <= i + Nk - Nq) and
 * ALiBi (Section 5.3: distance |i + Nk - Nq - j|) a meaning when the two counts differ; with
 * Nq = Nk the calls equal sigmoid_attn_fwd / sigmoid_attn_bwd, with Nq > Nk the first Nq - Nk
 * queries see no key (their outputs and gradients are zero).  causal and alibi_slopes as in
 * sigmoid_attn_fwd.  fp32 takes any pair of counts; bf16 with the causal mask needs Nk - Nq to
 * be a multiple of 32 (SATTN_ERR_UNSUPPORTED otherwise).  One K/V head per query head. */
int sigmoid_attn_cross_aligned_fwd(const void* q, const void* k, const void* v, void* o,
                                   int B, int H, int Nq, int Nk, int d, sattn_dtype dtype, float bias,
                                   int causal, const float* alibi_slopes,
                                   const sattn_strides* sq, const sattn_strides* sk,
                                   const sattn_strides* sv, const sattn_strides* so, void* stream);
int sigmoid_attn_cross_aligned_bwd(const void* q, const void* k, const void* v, const void* dout,
                                   void* dq, void* dk, void* dv,
                                   int B, int H, int Nq, int Nk, int d, sattn_dtype dtype, float bias,
                                   int causal, const float* alibi_slopes,
                                   const sattn_strides* sq, const sattn_strides* sk,
                                   const sattn_strides* sv, const sattn_strides* sdout,
                                   const sattn_strides* sdq, const sattn_strides* sdk,
                                   const sattn_strides* sdv, void* stream);

/* Backward with the gradient of a learnable bias (Section 5.4 and Appendix G.4 train with a
 * learnable scalar b, one per layer; Appendix F.1 backward table: T = S + b, so dL/db is the
 * sum of dS over the pairs the bias enters).  Same as sigmoid_attn_bwd (bf16 or fp32), and the
 * dQ pass also writes db_rows[b][h][i] = sum_j dS_ij (device pointer, contiguous [B,H,N] fp32,
 * required: the gradient of a bias per query row).  If db is not NULL (device pointer, B*H
 * fp32), a second small kernel sums each head's rows in a fixed order into db[b*H+h]; the
 * scalar gradient of a bias shared by a layer is the sum of those B*H numbers.  Errors as
 * sigmoid_attn_bwd; SATTN_ERR_NULL for db_rows == NULL. */
int sigmoid_attn_bwd_bias_grad(const void* q, const void* k, const void* v, const void* dout,
                               void* dq, void* dk, void* dv, float* db_rows, float* db,
                               int B, int H, int N, int d, sattn_dtype dtype,
                               float bias, int causal, const float* alibi_slopes,
                               const sattn_strides* sq, const sattn_strides* sk,
                               const sattn_strides* sv, const sattn_strides* sdout,
                               const sattn_strides* sdq, const sattn_strides* sdk,
                               const sattn_strides* sdv, void* stream);

/* Variable-length batches (Appendix G.4, training details of the speech models: dynamic
 * batching, and every sample's own length gives its bias b = -ln(n), a non-trainable bias
 * vector for the minibatch): the B
 * sequences are packed along the token axis of [tokens, H, d] tensors; sequence s owns tokens
 * cu_seqlens[s] .. cu_seqlens[s+1]-1 (device pointer to B+1 non-decreasing int32 offsets,
 * cu_seqlens[0] >= 0) and attends only to itself.  max_seqlen bounds every length (tokens of
 * a longer sequence beyond it are not written).  bias_per_seq is a device pointer to B floats
 * or NULL (then `bias` applies to every sequence).  Strides: `batch` is ignored, `head` and
 * `seq` (token) as usual; NULL = contiguous [tokens, H, d].  bf16 or fp32.  Same error codes and
 * stream semantics as the dense entry points; the offsets themselves are not validated. */
int sigmoid_attn_varlen_fwd(const void* q, const void* k, const void* v, void* o,
                            const int32_t* cu_seqlens, const float* bias_per_seq,
                            int B, int H, int max_seqlen, int d, sattn_dtype dtype,
                            float bias, int causal, const float* alibi_slopes,
                            const sattn_strides* sq, const sattn_strides* sk,
                            const sattn_strides* sv, const sattn_strides* so,
                            void* stream);
int sigmoid_attn_varlen_bwd(const void* q, const void* k, const void* v, const void* dout,
                            void* dq, void* dk, void* dv,
                            const int32_t* cu_seqlens, const float* bias_per_seq,
                            int B, int H, int max_seqlen, int d, sattn_dtype dtype,
                            float bias, int causal, const float* alibi_slopes,
                            const sattn_strides* sq, const sattn_strides* sk,
                            const sattn_strides* sv, const sattn_strides* sdout,
                            const sattn_strides* sdq, const sattn_strides* sdk,
                            const sattn_strides* sdv, void* stream);

/* Variable-length batches with the gradient of a learnable bias: sigmoid_attn_varlen_bwd, and
 * the dQ pass also writes db_rows[h][t] = sum_j dS_tj for every packed token t that the pass
 * covers (device pointer, contiguous [H, total_tokens] fp32, required; tokens of a sequence
 * beyond max_seqlen are not written).  If db is not NULL (device pointer, B*H fp32), a second
 * small kernel sums each sequence's rows in a fixed order into db[b*H + h]: with a bias per
 * sequence (Appendix G.4) that is the gradient of that sequence's bias, per head.  total_tokens
 * is the first dimension of the packed tensors.  Errors as sigmoid_attn_varlen_bwd and
 * sigmoid_attn_bwd_bias_grad. */
int sigmoid_attn_varlen_bwd_bias_grad(const void* q, const void* k, const void* v, const void* dout,
                                      void* dq, void* dk, void* dv, float* db_rows, float* db,
                                      const int32_t* cu_seqlens, const float* bias_per_seq,
                                      int B, int H, int max_seqlen, int64_t total_tokens, int d,
                                      sattn_dtype dtype, float bias, int causal,
                                      const float* alibi_slopes,
                                      const sattn_strides* sq, const sattn_strides* sk,
                                      const sattn_strides* sv, const sattn_strides* sdout,
                                      const sattn_strides* sdq, const sattn_strides* sdk,
                                      const sattn_strides* sdv, void* stream);

/* Library version: major*10000 + minor*100 + patch. */
int sattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SATTN_H_ */
