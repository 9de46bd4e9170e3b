// Internal interface between the C-ABI host code and the HIP kernels (gfx950 only).
// Every launcher only enqueues work on `stream`; shapes are validated by the caller.
#pragma once

#include <hip/hip_runtime.h>
#include <cstdint>

#include "kv_geom.h"

namespace ax {

// F32: fp32 weights, activations and KV.  BF16: bf16 weights; activations and KV are fp16
// ("the activation type" below), products on the fp16 MFMA with fp32 accumulation.
enum DType { F32 = 0, BF16 = 1 };

// Device views of the per-call descriptor (one packed int32 buffer uploaded per call).
struct StepView {
    const int* row_tok;     // [n_rows] token id
    const int* row_pos;     // [n_rows] absolute position
    const int* row_seq;     // [n_rows] sequence index within the call
    const int* row_slot;    // [n_rows] KV slot the row is written to: block id * 16 + position % 16
    const int* seq_P;       // [n_seq] cached length before the call
    const int* seq_T;       // [n_seq] new rows
    const int* seq_row0;    // [n_seq] first row
    const int* seq_bt;      // [n_seq] offset of the sequence's block table inside bt
    const int* bt;          // concatenated block tables
    const int* out_rows;    // [n_out] rows that go through the LM head
    const int* tile_info;   // [n_tiles + n_tiles_shared][8] attention q-tile groups over stacked rows (t, g):
                            // sequence, first stacked row, P, T, first row of the sequence, block-table offset,
                            // key limit (0 = the rows' causal bound), first key
                            // (a group = tile_nq tiles of 32 rows; 32-byte aligned records)
    int n_rows, n_seq, n_out, n_tiles, tile_nq;
    // shared-prefix pass (calls with several sequences whose block tables start alike): groups of
    // shared_nq tiles over ALL rows of the call against keys [0, shared_len); 0 groups = no such pass
    int n_tiles_shared, shared_nq, shared_len, shared_splits;
};

enum Epilogue { EPI_STORE_F32 = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_QKV = 3 };

// Rotary + KV-append part of the QKV epilogue (bf16-weight models).
struct RopeArgs {
    KVGeom kv;
    int layer, n_q_heads;
    void* q_out;                      // fp16 [n_rows, Hq, hd]
    const int *row_pos;               // [n_rows] absolute position
    const int *row_slot;              // [n_rows] KV slot of the row: block id * 16 + position % 16
    const float *cos, *sin;           // [max_pos][hd/2]
};

// Split activations.  An fp16 value keeps 11 significant bits; the rounding of the five activation tensors a
// layer hands from kernel to kernel is what separates the logits of a deep, wide decoder from the exact ones
// (measured: ~1B x 16 layers 5e-3, ~3B x 28 layers 1.3e-2, ~8B x 32 layers 2.7e-2 max-abs).  A model created
// with split activations stores every such tensor as TWO fp16 values per element, hi = fp16(v) and
// lo = fp16(v - hi) (together ~22 bits), the second tensor `*_lo_off` elements behind the first, and every
// consumer multiplies both parts against the SAME weight fragment (two MFMAs per fragment: no extra weight
// traffic, twice the matrix-core work and activation traffic).  An offset of 0 means "not split".
//
// One GEMM of a bf16-weight model: C = A[M,K] * W[N,K]^T, A fp16, W bf16.
struct GemmArgs {
    const void* A;                    // fp16 [rows, K]
    long long a_lo_off;               // split activations: the lo parts of A lie this many elements behind A (0 = none)
    long long c_lo_off;               // ... and the lo parts of C16 (and of rope.q_out) this many elements behind it
    const int* a_rows;                // optional gather: A row of output row m is a_rows[m]
    const void *W, *W2;               // [N, K] packed by launch_pack_weights (fp16, MFMA operand order); W2 only for EPI_SWIGLU
    int M, N, K;
    // deferred RMSNorm of the A rows: ssq[row][nparts] partial sums of x^2 over d_norm columns;
    // the accumulators are scaled by 1 / sqrt(sum / d_norm + eps).  NULL = no scaling.
    const float* ssq;
    int nparts, d_norm;
    float eps;
    float* Cf;                        // EPI_STORE_F32: out [M,N]; EPI_RESIDUAL: x [M,N], updated in place
    void* C16;                        // EPI_SWIGLU: fp16 out [M,N]; EPI_RESIDUAL: fp16(x * gain_next) [M,N]
    const void* gain_next;            // EPI_RESIDUAL: bf16 [N] gain of the next norm, NULL = plain residual add
    float* ssq_out;                   // EPI_RESIDUAL: [M][parts] partial sums of x^2, parts = what launch_gemm_bf16 returns
    RopeArgs rope;                    // EPI_QKV
    // EPI_RESIDUAL on the tile kernels with few output tiles: K may be cut into ksplit slices (chosen by
    // the launcher) whose fp32 partial products go to split_ws [ksplit][M][N]; a second kernel
    // adds them up and runs the residual epilogue.  split_ws == NULL: never split.
    float* split_ws;
    size_t split_ws_bytes;
    int ksplit;
};
constexpr int SPLITK_MAX = 8;
// EPI_RESIDUAL with gain_next: returns the number of partial sums of x^2 per row the launch leaves in
// ssq_out (rows are that many floats apart): the consumer of the pending norm passes it as nparts.
// It depends on which kernel ran (a few per row after a K-split reduce kernel, N / 32 or N / 8-16
// from kernels that finish a column block on their own).  Other epilogues return 0.
// EPI_QKV above 64 rows writes its raw products to split_ws first: -1, and nothing launched, if one [M, N] fp32
// slab does not fit there.
int launch_gemm_bf16(Epilogue epi, const GemmArgs& g, hipStream_t s);
// Repacks a row-major bf16 [N, K] matrix (N % 16 == 0, K % 32 == 0) into what every bf16-model GEMM
// kernel reads: fp16 values in 16-row panels, 32-k chunks in MFMA operand order; src and dst must not overlap.
// `bad` (device int, may be NULL) is set to 1 if some weight does not survive the narrowing (not finite in fp16).
void launch_pack_weights(const void* src, void* dst, int N, int K, hipStream_t s, int* bad = nullptr);
// bf16-weight models: x[r,:] = emb[tok], a[r,:] = fp16(x * gain), ssq[r][0] = sum x^2, ssq[r][1..nparts) = 0
// a_lo_off != 0: also the lo parts fp16(x * gain - a), that many elements behind a
void launch_embed_norm(const void* emb, const int* row_tok, const void* gain, float* x, void* a, long long a_lo_off,
                       float* ssq, int nparts, int n_rows, int d, hipStream_t s);

// x[r, :] = emb[row_tok[r], :] widened to fp32
void launch_embed(DType dt, const void* emb, const int* row_tok, float* x, int n_rows, int d,
                  hipStream_t s);
// h[i, :] = rmsnorm(x[rows ? rows[i] : i, :]) * gain, written in the activation type
void launch_rmsnorm(DType dt, const float* x, const void* gain, void* h, const int* rows,
                    int n_rows, int d, float eps, hipStream_t s);
// C = A[M,K] * W[N,K]^T with fp32 accumulation.  A is of the activation type, W of the weight
// type.  EPI_STORE_F32: C float [M,N].  EPI_RESIDUAL: C float [M,N] += .
// EPI_SWIGLU: C (activation type) [M,N] = silu(A*W^T) * (A*W2^T).
void launch_gemm(DType dt, Epilogue epi, const void* A, const void* W, const void* W2, void* C,
                 int M, int N, int K, hipStream_t s);
// rotary on q and k heads of qkv (fp32 [n_rows, (Hq+2Hkv)*hd]); q -> q_out [n_rows, Hq, hd]
// (activation type), k and v -> pages of `layer`.
void launch_rope_kv(DType dt, const float* qkv, void* q_out, KVGeom kv, int layer,
                    const StepView& sv, const float* rope_cos, const float* rope_sin,
                    int n_q_heads, hipStream_t s);
// Causal attention of the new rows over the paged cache (which already holds the new rows).
// out [n_rows, Hq, hd] in the activation type.  `partials` is fp32 scratch for the split-KV
// path (bf16 only); n_splits >= 1.
// q_lo_off / out_lo_off: split activations (see GemmArgs): lo parts of q read, lo parts of out written (0 = none).
void launch_attention(DType dt, const void* q, void* out, KVGeom kv, int layer,
                      const StepView& sv, int n_q_heads, float* partials, int n_splits,
                      hipStream_t s, long long q_lo_off = 0, long long out_lo_off = 0);
// Floats of `partials` launch_attention needs for n_tiles q tiles (of 32 rows) and n_splits splits.
size_t attention_partial_floats(int n_tiles, int n_kv_heads, int head_dim, int n_splits);
// out[r] = argmax of logits[r, 0..V), lowest index on ties.  scratch: 2*rows*ARGMAX_PARTS ints.
constexpr int ARGMAX_PARTS = 64;
void launch_argmax(const float* logits, int rows, int V, int* out, int* scratch, hipStream_t s);
// Greedy acceptance per sequence of a verify call: the sequence's rows are [pending, drafts],
// g[row] the greedy token after each row.  result[2s] = a (longest prefix of the drafts equal to
// g), result[2s + 1] = g[row0 + a].
void launch_accept(const int* g, const StepView& sv, int* result, hipStream_t s);
// The same two steps fused for verify calls whose rows fit one LM-head pass: launch_argmax_partials
// is stage 1 alone (per row ARGMAX_PARTS (value, id) candidates into scratch), launch_argmax_accept
// finishes every row of a sequence (g[row], as launch_argmax would write it), votes, and writes
// (a, next token) to result and - when result_host is given: pinned host memory the device can
// address - straight to the host, so no copy has to follow.  At most ACCEPT_MAX_ROWS rows per sequence.
constexpr int ACCEPT_MAX_ROWS = 1024;
void launch_argmax_partials(const float* logits, int rows, int V, int* scratch, hipStream_t s);
void launch_argmax_accept(const int* scratch, int rows, int* g, const StepView& sv, int* result, int* result_host,
                          hipStream_t s);
// Plain copy of n16 16-byte words (calibration kernel for hardware counters).
void launch_plain_copy(void* dst, const void* src, size_t n16, hipStream_t s);
void launch_read_stream(const void* src, size_t n16, void* sink, hipStream_t s);   // read-only stream; sink: 4 writable bytes, never written
double launch_mfma_loop(int iters, void* sink, hipStream_t s);                    // register-resident fp16 MFMA loop; returns its flops
void launch_cu_fill(const void* src, size_t words_per_block, int blocks, int passes, void* sink, hipStream_t s);   // block b reads words [b, b + 1) * words_per_block, `passes` times; sink never written
void launch_grid_barrier(void* ctr, int* err, int blocks, int rounds, hipStream_t s);   // ctr: 3072 zeroed bytes; blocks: a multiple of 8, all resident
void launch_boundary(void* sink, int blocks, hipStream_t s);                          // an empty kernel of `blocks` x 512 threads; sink never written
// Copy one KV block (all layers, K and V, all heads) src -> dst: copy on write.
void launch_block_copy(DType dt, KVGeom kv, int n_layers, int src, int dst, hipStream_t s);

// Gather (to_image) or scatter the blocks `ids[0..n_seq_blocks)` of a sequence between the pool and
// an image buffer (device-accessible memory) that holds them back to back in logical order.
// last_fill: tokens in the last block (export zero-fills the slots beyond).
void launch_kv_image(bool to_image, DType dt, KVGeom kv, int n_layers, const int* ids, int n_seq_blocks,
                     void* image, int last_fill, hipStream_t s);

}  // namespace ax
