/*
 * fedattn.h - C ABI of the FedAttn attention library for AMD MI355X (gfx950).
 *
 * Federated Attention runs the self-attention of a stack of M Transformer blocks
 * over a global sequence that is partitioned among N participants (Section IV-A:
 * disjoint ordered index sets L_n; here contiguous segments given by offsets).
 * In a local block every participant attends only to its own tokens (Phase I,
 * local self-attention); in every H-th block the participants' K and V are
 * aggregated into a global KV matrix and each participant's queries attend to it
 * (Phase II, global self-attention; Algorithm 1).  Decoding reuses the per-block
 * KV caches kept from prefill (Section IV-C).
 *
 * Conventions for every entry point
 *  - "device" pointers are HIP device memory on the current device; "host"
 *    pointers are ordinary host memory, read before the call returns.
 *  - Tensors are token-major and contiguous: q,out [tokens, Hq, D];
 *    k,v [tokens, Hkv, D].  Element type is params->dtype.  Device tensor
 *    pointers must be 16-byte aligned.
 *  - The caller owns every buffer.  The library allocates no device memory and
 *    keeps nothing between calls that a result depends on (it remembers, per
 *    device, the compute-unit count and which kernel attributes it has set).
 *    Kernels are enqueued on `stream` (a hipStream_t cast to void*, NULL =
 *    default stream) and the call returns without waiting for them.
 *  - Every failure is a return code; fedattn_last_error() gives the reason as
 *    text (thread-local).  Nothing is enqueued when a call fails validation.
 *  - Query head h reads KV head h / (Hq/Hkv) (grouped-query attention).
 *  - Softmax runs on scores scaled by softmax_scale (0 selects 1/sqrt(D),
 *    Section III-B), accumulates in fp32 and writes out in params->dtype.
 *  - A query with no visible key gets a zero output row.
 */
#ifndef FEDATTN_H
#define FEDATTN_H

#include <stddef.h>
#include <stdint.h>

/* The entry points below are the library's only exported symbols. */
#define FEDATTN_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

#define FEDATTN_MAX_PARTICIPANTS 128

typedef enum {
  FEDATTN_OK = 0,
  FEDATTN_EINVAL = 1,       /* bad argument: null/misaligned pointer, bad offsets, bad sizes */
  FEDATTN_EUNSUPPORTED = 2, /* valid request the kernels do not cover */
  FEDATTN_EWORKSPACE = 3,   /* workspace missing or smaller than fedattn_workspace_bytes() */
  FEDATTN_ELAUNCH = 4       /* HIP reported an error when enqueuing */
} fedattn_status;

typedef enum { FEDATTN_BF16 = 0, FEDATTN_F32 = 1 } fedattn_dtype;

typedef enum { FEDATTN_OP_PREFILL = 0, FEDATTN_OP_DECODE = 1, FEDATTN_OP_PREFILL_SYNC_LOCAL_KV = 2 } fedattn_op;

typedef struct fedattn_params {
  int32_t n_participants; /* N, 1..FEDATTN_MAX_PARTICIPANTS */
  int32_t n_q_heads;      /* Hq */
  int32_t n_kv_heads;     /* Hkv, divides Hq */
  int32_t head_dim;       /* D: multiple of 8, at most 256 (bf16 with D = 64 or 128 runs on MFMA) */
  int32_t sync_interval;  /* H of Algorithm 1; <= 0: no block ever synchronises */
  int32_t causal;         /* 1: decoder (a token sees itself and earlier tokens); 0: encoder */
  int32_t dtype;          /* fedattn_dtype of q, k, v, out */
  float softmax_scale;    /* 0: 1/sqrt(D) */
} fedattn_params;

/* Algorithm 1: with blocks numbered m = H t + h (1-based), block m runs global
 * attention iff h = H.  For the 0-based block_idx used here that is
 * H >= 1 && (block_idx + 1) % H == 0.  Returns 1 (sync block) or 0 (local). */
FEDATTN_API int fedattn_is_sync_block(int32_t sync_interval, int32_t block_idx);

/* Bytes of device workspace the given op needs (16-byte aligned start).
 *   FEDATTN_OP_PREFILL: `tokens` = total tokens; needed only when a keep-list is
 *     passed (chunk_tokens > 0); 0 otherwise.
 *   FEDATTN_OP_DECODE:  `tokens` = total cache capacity; chunk_tokens ignored.
 *   FEDATTN_OP_PREFILL_SYNC_LOCAL_KV: `tokens` = total tokens; room for one aggregated copy of K
 *     and V (used only when the participants' matrices do not lie back to back) plus the
 *     keep-list's share (chunk_tokens > 0).
 * Returns 0 on invalid params. */
FEDATTN_API size_t fedattn_workspace_bytes(const fedattn_params* params, int32_t op, int32_t tokens,
                               int32_t chunk_tokens);

/*
 * Attention of one Transformer block over all participants' tokens (prefill).
 *   Local block (Phase I, o_n = Attention(q_n, k_n, v_n)): query i sees keys of
 *   its own segment only.  Sync block (Phase II, o_n = Attention(q_n, K, V)):
 *   query i sees the aggregated KV of all participants in the order of the
 *   global sequence.  With causal = 1 a query sees key j only if j <= i.
 *   Sparse KV exchange (adaptive KV aggregation): when keep_chunks is given,
 *   a sync block sees a remote participant's rows only in the chunks flagged 1;
 *   a participant's own rows are always complete.
 *   Arithmetic: fp32 inputs in fp32 throughout.  bf16 inputs with D = 64 or 128: both products
 *   on bf16 MFMA with fp32 accumulation, softmax in fp32, the weights rounded to bf16 for the
 *   second product (the row sum is taken over the rounded weights); when the softmax scale does
 *   not exceed 1/sqrt(D) it is folded into the query operand (q * scale * log2(e), rounded to
 *   bf16), otherwise applied to the fp32 scores.  Other bf16 shapes: fp32 arithmetic on the
 *   bf16 values.
 *
 *   block_idx      0-based block index; with sync_override = -1 the block is a sync
 *                  block iff fedattn_is_sync_block(params->sync_interval, block_idx).
 *   q,k,v,out      device; q,out [total,Hq,D], k,v [total,Hkv,D]; k,v hold the
 *                  aggregated (global-order) matrices, see fedattn_aggregate_kv.
 *   seg_offsets    host int32[N+1], non-decreasing, [0] = 0, [N] = total tokens.
 *                  Empty segments are legal.
 *   keep_chunks    device uint8[sum_n ceil(len_n / chunk_tokens)] or NULL (dense).
 *                  Chunk c of participant n covers tokens
 *                  seg_offsets[n] + c*chunk_tokens ... (clipped to the segment);
 *                  flags are stored participant after participant.  Read only in
 *                  sync blocks.  chunk_tokens must be positive when keep_chunks is
 *                  given (1 = token-granular exchange).  On the MFMA path (bf16,
 *                  D = 64 or 128) chunks that are multiples of 64 are visited where
 *                  they are; finer chunks have their kept rows packed into the
 *                  workspace first (a K,V-sized copy).  One block per call.
 *   sync_override  -1: rule above; 0: force local; 1: force sync (variable sync
 *                  schedules H_t).
 *   workspace      device, >= fedattn_workspace_bytes(PREFILL); may be NULL when
 *                  keep_chunks is NULL.
 */
FEDATTN_API fedattn_status fedattn_prefill(const fedattn_params* params, int32_t block_idx, const void* q,
                               const void* k, const void* v, void* out,
                               const int32_t* seg_offsets, const uint8_t* keep_chunks,
                               int32_t chunk_tokens, int32_t sync_override, void* workspace,
                               size_t workspace_bytes, void* stream);

/*
 * A sync block straight from the participants' own matrices: Phase II of Algorithm 1,
 * [K V] = sum_n Pi_n [k_n v_n] followed by o_n = Attention(q_n, K, V), in one call.  The sum
 * places row r of participant n at global row seg_offsets[n] + r; when the N matrices already
 * lie back to back in participant order in device memory (k_local[n] = base + seg_offsets[n]
 * rows, likewise v_local), that IS the aggregated matrix and the attention reads it in place:
 * no copy, no extra launch.  Otherwise the matrices are first aggregated into the workspace
 * (fedattn_aggregate_kv) and the attention reads the copy.  Always a sync block (the caller
 * decides which blocks are, e.g. with fedattn_is_sync_block); results equal
 * fedattn_aggregate_kv + fedattn_prefill with sync_override = 1.
 *   q,out          device [total,Hq,D].
 *   k_local,v_local host arrays of N device pointers, entry n -> [len_n,Hkv,D], 16-byte aligned
 *                   (entries of empty segments are ignored).
 *   keep_chunks, chunk_tokens  as in fedattn_prefill (sparse KV exchange).
 *   workspace      device, >= fedattn_workspace_bytes(PREFILL_SYNC_LOCAL_KV); when the matrices
 *                  lie back to back only the keep-list's share is used (the copy's share may
 *                  be left out, and the workspace may be NULL without a keep-list).
 */
FEDATTN_API fedattn_status fedattn_prefill_sync_local_kv(const fedattn_params* params, const void* q,
                                             const void* const* k_local, const void* const* v_local, void* out,
                                             const int32_t* seg_offsets, const uint8_t* keep_chunks,
                                             int32_t chunk_tokens, void* workspace, size_t workspace_bytes,
                                             void* stream);

/*
 * The same for n_blocks consecutive blocks block_idx0 .. block_idx0+n_blocks-1 in
 * one launch.  Block b reads q + b*q_block_stride elements etc. (strides in
 * elements, multiples of 8); every block uses the same segment layout; dense
 * exchange only.  Semantics per block are exactly those of fedattn_prefill.  For
 * workloads whose per-block work is too small to fill the GPU.
 */
FEDATTN_API fedattn_status fedattn_prefill_blocks(const fedattn_params* params, int32_t block_idx0,
                                      int32_t n_blocks, const void* q, const void* k,
                                      const void* v, void* out, int64_t q_block_stride,
                                      int64_t kv_block_stride, const int32_t* seg_offsets,
                                      void* stream);

/*
 * One decoding step of one block (Section IV-C): one new query per participant
 * over the block's KV cache.  The caller has already appended the step's own
 * k,v, so a query sees itself; everything cached is in the past (no mask).
 *   Local block: participant n's query sees rows [0, seg_lens[n]) of its own
 *   cache segment.  Sync block: it also sees rows [0, remote_lens[m]) of every
 *   other participant m's segment (the aggregated cache).
 *
 *   q,out          device [N,Hq,D].
 *   k_cache,v_cache device [capacity_total,Hkv,D].
 *   seg_offsets    host int32[N+1]: capacity layout ([0] = 0, [N] = capacity_total).
 *   seg_lens       host int32[N]: valid rows of each segment, <= its capacity.
 *   remote_lens    host int32[N] or NULL (= seg_lens): rows of segment m that the
 *                  other participants see in a sync block (e.g. the prompt length
 *                  when generated tokens are not exchanged).
 *   workspace      device, >= fedattn_workspace_bytes(DECODE); holds split-KV partials and
 *                  chunk counters while the call's kernels run.  What it contains on entry
 *                  does not matter; calls that share a workspace must be ordered (same stream).
 */
FEDATTN_API fedattn_status fedattn_decode(const fedattn_params* params, int32_t block_idx, const void* q,
                              const void* k_cache, const void* v_cache, void* out,
                              const int32_t* seg_offsets, const int32_t* seg_lens,
                              const int32_t* remote_lens, int32_t sync_override, void* workspace,
                              size_t workspace_bytes, void* stream);

/*
 * The same for n_blocks consecutive blocks block_idx0 .. block_idx0+n_blocks-1 of one
 * decoding step in one host call: block b reads q + b*q_block_stride and the caches
 * + b*cache_block_stride (strides in elements, multiples of 8) and writes
 * out + b*q_block_stride; all blocks share the segment layout and lengths.  The
 * blocks are enqueued one after the other (each with its own launches, as the blocks
 * of a model depend on each other); results equal n_blocks calls of fedattn_decode.
 * The workspace is reused from block to block in stream order.
 */
FEDATTN_API fedattn_status fedattn_decode_blocks(const fedattn_params* params, int32_t block_idx0, int32_t n_blocks,
                                     const void* q, const void* k_cache, const void* v_cache, void* out,
                                     int64_t q_block_stride, int64_t cache_block_stride,
                                     const int32_t* seg_offsets, const int32_t* seg_lens,
                                     const int32_t* remote_lens, int32_t sync_override, void* workspace,
                                     size_t workspace_bytes, void* stream);

/*
 * fedattn_decode_blocks for callers that hold the queries of all n_blocks blocks before the
 * first one runs (the blocks of a model do not: the query of block m + 1 comes out of block
 * m; this entry point serves measurements of the kernels without launch effects and callers
 * with independent layers): same arguments and results, but the blocks of one kind (local /
 * sync, Algorithm 1) share launches.  Every block in flight works in its own slice of the
 * workspace: a launch takes as many blocks as the workspace has slices of
 * fedattn_workspace_bytes(DECODE) rounded up to 256 bytes (at least one, at most 64).
 * No order is kept between the blocks; q, the caches and out of different blocks must not
 * overlap.
 */
FEDATTN_API fedattn_status fedattn_decode_blocks_fused(const fedattn_params* params, int32_t block_idx0,
                                           int32_t n_blocks, const void* q, const void* k_cache,
                                           const void* v_cache, void* out, int64_t q_block_stride,
                                           int64_t cache_block_stride, const int32_t* seg_offsets,
                                           const int32_t* seg_lens, const int32_t* remote_lens,
                                           int32_t sync_override, void* workspace, size_t workspace_bytes,
                                           void* stream);

/*
 * fedattn_decode for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments (without the workspace) and bit-identical results; the split-KV partials and chunk
 * counters live in an array of FEDATTN_STATIC_SCRATCH_BYTES that is part of the library's
 * device code (every GPU the library runs on holds its own copy until the process ends).  The
 * call allocates and frees nothing.  Problems whose fedattn_workspace_bytes(DECODE) exceeds
 * the array are rejected with FEDATTN_EWORKSPACE.  All calls on one GPU share that GPU's array:
 * calls that may overlap (different streams, different threads) race and must be ordered by the
 * caller; what a previous call left in the array does not matter.  The array's address is
 * looked up at the first call on each device: make that call outside a graph capture.
 */
#define FEDATTN_STATIC_SCRATCH_BYTES (16u << 20)
FEDATTN_API fedattn_status fedattn_decode_static(const fedattn_params* params, int32_t block_idx, const void* q,
                                     const void* k_cache, const void* v_cache, void* out,
                                     const int32_t* seg_offsets, const int32_t* seg_lens,
                                     const int32_t* remote_lens, int32_t sync_override, void* stream);

/*
 * KV aggregation of a sync block (Phase II): [K V] = sum_n Pi_n [k_n v_n], i.e.
 * row r of participant n's local k_n, v_n lands at global row seg_offsets[n] + r.
 *   k_local,v_local host arrays of N device pointers, entry n -> [len_n,Hkv,D]
 *                   (entries of empty segments may be NULL).
 *   k_global,v_global device [total,Hkv,D], written completely.
 * A pure copy; on one GPU a caller that already keeps the participants' K,V
 * back to back in global order can skip it.
 */
FEDATTN_API fedattn_status fedattn_aggregate_kv(const fedattn_params* params, const void* const* k_local,
                                    const void* const* v_local, const int32_t* seg_offsets,
                                    void* k_global, void* v_global, void* stream);

/*
 * Element-wise pieces of the decoder block around the attention operator, for the end-to-end
 * configuration (a block is attention and a feed-forward network, each with a residual
 * connection and a normalisation: Section III-B; the local forward of Section IV-B):
 *   x += W_O Attention(RoPE(RMSNorm(x) W_QKV));  x += W_down (silu(gate) * up),
 *   [gate up] = RMSNorm(x) W_gate_up.
 * The matrix products are plain GEMMs and stay with the caller; these passes are the rest.  Residual stream x in fp32, every other tensor bf16, all device pointers, 16-byte
 * aligned, contiguous rows.
 *
 * fedattn_rmsnorm: out[r] = bf16(x[r] / sqrt(mean_j x[r][j]^2 + eps)), unit gain;
 *   x fp32 [rows, d_model], out bf16 [rows, d_model]; d_model a multiple of 4.
 * fedattn_rope_split_qkv: splits the fused projection qkv bf16 [tokens, (Hq + 2 Hkv) D]
 *   (q heads, then k heads, then v heads) into q [tokens,Hq,D], k,v [tokens,Hkv,D] and
 *   applies the rotary embedding to q and k: element i < D/2 is paired with i + D/2 and the
 *   pair is rotated by pos * theta^(-2i/D).  pos: device int32[tokens], or NULL for
 *   pos[t] = t (the index in the global sequence).  D a multiple of 8.
 * fedattn_swiglu: out[r][f] = bf16(silu(gate_up[r][f]) * gate_up[r][hidden + f]);
 *   gate_up bf16 [rows, 2 hidden], out bf16 [rows, hidden]; hidden a multiple of 8.
 * fedattn_residual_add: x[i] += y[i]; x fp32, y bf16, n elements (a multiple of 4).
 * fedattn_residual_add_rmsnorm: fedattn_residual_add(x, y) followed by fedattn_rmsnorm(x, out) in
 *   one pass over the residual stream (the update that closes one half of a block and the
 *   normalisation that opens the next); same results as the two calls.  x fp32 [rows, d_model]
 *   updated in place, y bf16 [rows, d_model], out bf16 [rows, d_model].
 */
FEDATTN_API fedattn_status fedattn_rmsnorm(const float* x, void* out, int64_t rows, int32_t d_model, float eps, void* stream);
FEDATTN_API fedattn_status fedattn_rope_split_qkv(const void* qkv, const int32_t* pos, void* q, void* k, void* v, int64_t tokens,
                                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float theta,
                                      void* stream);
FEDATTN_API fedattn_status fedattn_swiglu(const void* gate_up, void* out, int64_t rows, int32_t hidden, void* stream);
FEDATTN_API fedattn_status fedattn_residual_add(float* x, const void* y, int64_t n, void* stream);
FEDATTN_API fedattn_status fedattn_residual_add_rmsnorm(float* x, const void* y, void* out, int64_t rows, int32_t d_model,
                                            float eps, void* stream);

/*
 * Measurement aids (no part of the method): the rates the GPU reaches on the bare resources the
 * attention kernels are bound by, for benchmarks that report a fraction of a measured peak beside
 * the fraction of the published one.  Each call enqueues ONE kernel; the caller times it.
 * fedattn_probe_stream: one workgroup per CU reads `bytes` bytes at src (device, 16-byte aligned;
 *   rounded down to whole tiles per workgroup) through LDS rings with the direct HBM -> LDS loads of
 *   the decode kernel and does nothing else.  pattern 0: contiguous shares.  pattern 1: the decode
 *   kernel's access pattern on a [rows, 8 KV heads, 128] bf16 cache (256-byte pieces at a 2 KB
 *   stride, from a K array in the first half of the buffer and a V array in the second).  sink:
 *   device, one float per workgroup (never written in practice).  Returns the bytes read, -1 on error.
 * fedattn_probe_mfma: every SIMD runs two wavefronts that issue `iters` x 8 v_mfma_f32_32x32x16_bf16
 *   on register operands.  sink: device, 512 floats per CU.  Returns the FLOPs performed, -1 on error.
 */
FEDATTN_API int64_t fedattn_probe_stream(const void* src, int64_t bytes, int32_t pattern, void* sink, void* stream);
FEDATTN_API int64_t fedattn_probe_mfma(void* sink, int32_t iters, void* stream);

/* Reason of the calling thread's most recent failure ("" if none). */
FEDATTN_API const char* fedattn_last_error(void);

/* Library version string. */
FEDATTN_API const char* fedattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FEDATTN_H */
