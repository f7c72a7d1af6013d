/*
 * sattn_bench.h -- measurement and comparison aids of the sigmoid-attention library.
 *
 * Nothing here is part of the product contract of sattn.h: these entry points exist so that
 * the kernels can be timed like for like against the softmax comparison kernels, so that
 * the benchmark can report the matrix rate the device sustains, and so that a tile shape
 * can be forced for a sweep.  Same conventions as sattn.h (device pointers, element
 * strides, asynchronous on `stream`, negative SATTN_ERR_* on error).
 */
#ifndef SATTN_BENCH_H_
#define SATTN_BENCH_H_

#include "sattn.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Force the forward tile shape for measurements (Appendix F.5: the block shape is a tuning
 * parameter): waves in {4, 8, 32, 64, 65, 66}, v_slots in {2, 3}; 0 = back to the automatic choice; a
 * forced v_slots only applies where that shape exists, a forced 64 / 65 / 66 only for the pinned
 * sigmoid kernel at d = 128 (other kernels then run a 4-wave shape).  32 = the automatic choice
 * among the shapes with 32 query rows per wave (4 or 8 waves), which is the choice every kernel
 * without a 64-row form gets: it lets the sigmoid forward be timed in the shape the softmax
 * forward runs.  64 = four waves of 64 query rows.  65 = the same with Q multiplied by the logit scale and rounded to bf16 once, and
 * the bias applied as a factor, which removes the scale-and-bias fma in front of every exp2: a
 * measurement variant, NOT bit-identical to the other shapes and never chosen automatically (its
 * logit error grows with |q||k|: one more bf16 rounding on an operand).  66 = as 64 with one
 * query block per workgroup also under the causal mask (64 deals a head's blocks out in pairs,
 * longest with shortest, where their number is even).  The value is
 * process-wide (an atomic that every forward launch reads): set it from one thread while no
 * other thread launches, or launches in flight on other threads may take either shape.  Apart
 * from 65, results do not depend on it. */
int sattn_set_fwd_waves(int waves);
int sattn_set_fwd_v_slots(int v_slots);

/* Force (1) or forbid (2) the one-grid form of the sigmoid backward, in which the dK/dV and
 * the dQ workgroups of Algorithm 2's two output owners share one launch; 0 = back to the
 * automatic choice; 3 = forbid it and also keep one block per workgroup in the causal passes
 * (which otherwise deal a long head's blocks out in pairs, longest with shortest).  Only sigmoid_attn_bwd / sigmoid_attn_varlen_bwd have that form (both
 * passes, self-attention, one K/V head per query head, no bias gradient).  Results do not
 * depend on it.  Process-wide like the setters above.  Returns 0 or SATTN_ERR_UNSUPPORTED. */
int sattn_set_bwd_merged(int mode);
/* 1 if sigmoid_attn_bwd on a bf16 self-attention problem of this size would run its two
 * passes as one grid, 0 if as two launches; SATTN_ERR_SHAPE for non-positive sizes. */
int sattn_bwd_merged(int B, int H, int N, int causal);

/* Comparison aids (Section 4 and Appendix F.2 compare the sigmoid kernels with softmax kernels
 * built the same way).  Same arguments, results and error behaviour as sigmoid_attn_fwd /
 * sigmoid_attn_bwd / softmax_attn_fwd / softmax_attn_bwd; the kernels run every pipeline step
 * in the compiler-scheduled form instead of the hand-pinned instruction stream (of the softmax
 * backward only the dQ pass has a hand-pinned form; its dK/dV pass is compiler-scheduled in
 * softmax_attn_bwd too).  They exist so that sigmoid and softmax can be timed like for like at
 * both levels of tuning; not meant for production. */
int sigmoid_attn_fwd_compiler_scheduled(const void* q, const void* k, const void* v, void* o,
                                        int B, int H, int N, int d, sattn_dtype dtype,
                                        float bias, int causal, const float* alibi_slopes,
                                        const sattn_strides* sq, const sattn_strides* sk,
                                        const sattn_strides* sv, const sattn_strides* so,
                                        void* stream);
int softmax_attn_fwd_compiler_scheduled(const void* q, const void* k, const void* v, void* o, float* lse,
                                        int B, int H, int N, int d, sattn_dtype dtype,
                                        int causal, const float* alibi_slopes,
                                        const sattn_strides* sq, const sattn_strides* sk,
                                        const sattn_strides* sv, const sattn_strides* so,
                                        void* stream);
int sigmoid_attn_bwd_compiler_scheduled(const void* q, const void* k, const void* v, const void* dout,
                                        void* dq, void* dk, void* dv,
                                        int B, int H, int N, int d, sattn_dtype dtype,
                                        float bias, int causal, const float* alibi_slopes,
                                        const sattn_strides* sq, const sattn_strides* sk,
                                        const sattn_strides* sv, const sattn_strides* sdout,
                                        const sattn_strides* sdq, const sattn_strides* sdk,
                                        const sattn_strides* sdv,
                                        void* workspace, size_t workspace_bytes, void* stream);
int softmax_attn_bwd_compiler_scheduled(const void* q, const void* k, const void* v, const void* o,
                                        const float* lse, const void* dout,
                                        void* dq, void* dk, void* dv,
                                        int B, int H, int N, int d, sattn_dtype dtype,
                                        int causal, const float* alibi_slopes,
                                        const sattn_strides* sq, const sattn_strides* sk,
                                        const sattn_strides* sv, const sattn_strides* so,
                                        const sattn_strides* sdout, const sattn_strides* sdq,
                                        const sattn_strides* sdk, const sattn_strides* sdv,
                                        void* workspace, size_t workspace_bytes, void* stream);

/* Measurement aid (Appendix F.2 reports kernel times; here they are also quoted as a fraction
 * of the matrix-unit rate): launches `blocks` workgroups of 4 waves that each issue iters*8
 * independent register-resident 32x32x16 bf16 MFMAs (32768 flop each) and nothing else,
 * asynchronously on `stream`.  The
 * caller times the launch; blocks*4*iters*8*32768 flop / time is the matrix rate this device
 * sustains at its actual clock.  `sink` is a device pointer to blocks*256 floats that
 * receives one value per lane (keeps the loop alive).  Returns 0 or SATTN_ERR_*. */
int sattn_mfma_bf16_probe(int blocks, int iters, float* sink, void* stream);

/* Measurement aid: the engine clock a kernel actually runs at, and where a workgroup's time
 * goes.  While a device buffer of 8 * capacity int64 is set (NULL = off; process-wide like the
 * tile-shape setters, same threading rule), every bf16 attention kernel launched by this
 * library has workgroup w < capacity write out[8w] = core cycles and out[8w+1] = ticks of the
 * constant-rate counter (hipDeviceAttributeWallClockRate, in kHz) it spent in the kernel;
 * sum(cycles) / sum(ticks) * tick rate is the clock under that kernel's load, which on this part
 * lies well below the nominal peak clock that the 2.5 PFLOP/s figure assumes.  out[8w+2..5] are
 * the ticks since the kernel's start at which wave 0 of the workgroup issued its first tile
 * product, entered its steady-state loop, left it, and began to store its outputs; out[8w+6]
 * the tiles it ran in that loop and out[8w+7] the tiles of the workgroup.  Workgroups that exit
 * at once (blocks beyond a sequence's length) write nothing: clear the buffer first.  8-byte
 * aligned. */
int sattn_set_clock_probe(void* device_buffer, int capacity);
/* Rate of that constant-rate counter on the current device in kHz, or SATTN_ERR_LAUNCH. */
int sattn_wall_clock_khz(void);

/* Measurement aid: compute units and nominal peak engine clock (kHz) of the current device, as
 * the runtime reports them (host pointers).  SATTN_ERR_LAUNCH if there is no usable device. */
int sattn_device_info(int* compute_units, int* clock_khz);

#ifdef __cplusplus
}
#endif
#endif /* SATTN_BENCH_H_ */
