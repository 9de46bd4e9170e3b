/*
 * agentx_debug.h - test-only entry points of libagentx.so: they expose single kernels and the
 * intermediates of the last forward so that GPU tests can localise a mismatch against the CPU
 * oracle.  Not part of the serving API; they synchronise the device.
 */
#ifndef AGENTX_DEBUG_H
#define AGENTX_DEBUG_H

#include "agentx.h"

#ifdef __cplusplus
extern "C" {
#endif

/* C = A[M,K] * W[N,K]^T through the library's GEMM dispatcher (the projection / MLP / LM-head
 * contraction of the decoder).  All pointers are device memory.  dtype AX_F32: A, W, W2 fp32;
 * AX_BF16: W, W2 bf16 and A fp16 (the activation type of bf16-weight models).  epilogue: 0 store
 * float C[M,N]; 1 float C[M,N] += ; 2 SwiGLU, C (activation type) = silu(A W^T) * (A W2^T).
 * AX_BF16 needs K % 64 == 0 and N % 16 == 0.  Synchronises. */
ax_status ax_dbg_gemm(int dtype, int epilogue, const void *A, const void *W, const void *W2, void *C,
                      int M, int N, int K, void *hip_stream);

/* The residual GEMM as a bf16-weight decoder layer runs it (O and down projections): x[M,N] (float,
 * updated in place) += A[M,K] W[N,K]^T, then a16[M,N] = fp16(x * gain[n]) and per-row partial sums
 * of x^2: ssq[m * (*n_parts) + p], p < *n_parts (written by the call; at most N / 8), whose sum
 * over p is sum_n x[m,n]^2.  A fp16, W and gain bf16, all device memory; ssq must hold M * N / 8
 * floats.  K % 64 == 0, N % 16 == 0, and N % 32 == 0 with more than 16 rows (N is a model width there).
 * split_ws / split_ws_bytes: device scratch for K-slice partial products (the launcher
 * cuts K only when scratch is given and it pays); 0 bytes = never.  Synchronises. */
ax_status ax_dbg_gemm_residual(const void *A, const void *W, const void *gain, float *x, void *a16, float *ssq,
                               int *n_parts, int M, int N, int K, void *split_ws, size_t split_ws_bytes,
                               void *hip_stream);

/* Times `iters` back-to-back launches of the same GEMM with HIP events on hip_stream and writes the
 * average microseconds per launch to *avg_us.  Launch i reads its weights at W + (i % w_count) *
 * w_stride_bytes (same for W2), so that a set of weight copies larger than the caches can be
 * cycled through (w_count = 1: always the same weights).  Arguments otherwise as ax_dbg_gemm. */
ax_status ax_dbg_gemm_time(int dtype, int epilogue, const void *A, const void *W, const void *W2, void *C,
                           int M, int N, int K, int iters, size_t w_stride_bytes, int w_count,
                           float *avg_us, void *hip_stream);

/* Plain device-to-device copy kernel (16-byte words, grid-stride) of `bytes` bytes (a multiple of
 * 16): the kernel of known traffic that hardware-counter readings are scaled against. */
ax_status ax_dbg_copy(void *dst, const void *src, size_t bytes, void *hip_stream);

/* What the machine delivers, measured beside the nominal peaks the roofline fractions are quoted
 * against.  buf: device memory of `bytes` bytes (a multiple of 16; use a few hundred MiB so that no
 * cache holds it).  Runs 2 untimed and `reps` timed launches each of (i) a read-only stream over buf,
 * (ii) the plain copy kernel from the first half of buf to the second, (iii) a register-resident
 * fp16 MFMA loop (32x32x16, fp32 accumulate) on every compute unit; HIP events on hip_stream.
 * Writes GB/s read, GB/s copied (read + written bytes) and TFLOP/s.  Synchronises. */
ax_status ax_dbg_peaks(void *buf, size_t bytes, int reps, float *read_gbs, float *copy_gbs,
                       float *mfma_f16_tflops, void *hip_stream);

/* What one compute unit can pull.  256 workgroups of 512 threads (one per compute unit of an otherwise idle MI355X)
 * each read a region of their own with many more loads in flight than the memory pipeline keeps outstanding: a 64 KB
 * region 256 times (served by the L2 of the workgroup's XCD from the second pass on), then a region of bytes / 256 once
 * (from HBM, all compute units pulling together; whatever of buf the 256 MB memory-side cache still holds from the caller's own
 * last pass over it comes from there - use a buffer of 1 GiB or more).  buf: device memory of `bytes` bytes, at least 256 MiB and a multiple of
 * 4096, read only.  Writes GB/s PER COMPUTE UNIT for both.  Synchronises. */
ax_status ax_dbg_cu_fill(void *buf, size_t bytes, float *l2_gbs_per_cu, float *hbm_gbs_per_cu, void *hip_stream);

/* The two ways to order the dependent phases of a step, timed: `rounds` back-to-back launches of an
 * empty kernel of `blocks` workgroups of 512 threads on hip_stream (microseconds per kernel boundary),
 * and one launch of the same shape that crosses a barrier over all its workgroups `rounds` times
 * (microseconds per barrier; two-level counters, device-scope atomics, fences on both sides).  blocks: a
 * multiple of 8, at most 256 (one workgroup per compute unit, so that all are resident on an otherwise
 * idle device); buf: at least 4096 bytes of device memory, overwritten.  Every wait of the barrier kernel
 * is bounded: AX_ERR_DEVICE if a workgroup gave up.  Synchronises. */
ax_status ax_dbg_phase_order(void *buf, size_t bytes, int blocks, int rounds, float *boundary_us,
                             float *barrier_us, void *hip_stream);

/* Copies a workspace buffer as left by the last ax_extend* call to host memory (synchronises).
 * which: 0 residual stream x float[rows][d_model]; 1 qkv float[rows][(Hq+2Hkv)*hd] (pre-rotary,
 * last layer); 2 q after rotary, act[rows][Hq*hd]; 3 attention output act[rows][Hq*hd];
 * 4 SwiGLU activations act[rows][d_ff]; 5 LM-head input, where act is float for AX_F32 models
 * and fp16 for AX_BF16 models.  AX_F32: buffer 5 is rmsnorm(x) * gain of the n_out output rows.
 * AX_BF16: buffer 1 is unused and buffer 5 is fp16(x * final gain) of all rows (the division by
 * the rms happens inside the LM-head GEMM).
 * Copies min(bytes, buffer size) bytes. */
ax_status ax_dbg_read(ax_model *model, int which, void *host_dst, size_t bytes);

/* The workspace of a model is cut into regions (rotary tables, descriptor slots, residual stream, activations,
 * norm partial sums, fp32 q/k/v of fp32 models, q, attention output, SwiGLU activations, attention slice records, GEMM
 * slabs, logits chunk, argmax scratch, argmax output, result words, packed weights - in this order), each followed by
 * 256 guard bytes that ax_model_create fills with a pattern and nothing may write.  Synchronises the device, reads
 * the guards back and writes the index of the first region whose guard was touched (an overrun of that region), or
 * -1 if all are intact. */
ax_status ax_dbg_check_guards(ax_model *model, int *first_bad);

/* ax_verify replays one captured HIP graph per (draft count, key-slice count); enable = 0 makes it
 * enqueue the same launches one by one instead (the reference a test compares the replays with). */
ax_status ax_dbg_use_graphs(ax_model *model, int enable);

/* Per-kernel timing with HIP events on the caller's stream.  While enabled, every launch of the
 * classes below inside ax_extend* / ax_verify is bracketed by a pair of events (this perturbs
 * the step a little, so enable it only for steps whose total time is not reported).
 * Classes: 0 QKV projection, 1 attention (split + combine), 2 O projection, 3 SwiGLU gate/up,
 * 4 down projection, 5 LM head, 6 an empty bracket (once per layer of a bf16-weight model): what a
 * pair of events measures around nothing, to be subtracted.  ax_dbg_profile_read synchronises, adds up the elapsed
 * milliseconds and the launch count of each class since the last read and clears them. */
#define AX_DBG_PROFILE_CLASSES 7
ax_status ax_dbg_profile(ax_model *model, int enable);
ax_status ax_dbg_profile_read(ax_model *model, double *ms_by_class, int64_t *launches_by_class);

#ifdef __cplusplus
}
#endif
#endif /* AGENTX_DEBUG_H */
