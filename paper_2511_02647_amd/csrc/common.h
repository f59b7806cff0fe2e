// Shared declarations of the FedAttn HIP library (gfx950 only): kernel argument
// blocks, launcher prototypes and small device helpers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "fedattn.h"

namespace fedattn {

constexpr int kMaxP = FEDATTN_MAX_PARTICIPANTS;
constexpr int kKvTile = 64;    // KV rows per MFMA prefill tile; also the keep-list tile
constexpr int kWaveRows = 32;  // query rows per wave in the MFMA prefill kernel
constexpr int kMaxOrderedTiles = 512;
constexpr int kMaxFusedBlocks = 64;    // blocks of one fused decode launch  // query tiles of a launch that assigns them through an explicit order

// Segment layout of the global sequence, passed by value in the kernel arguments
// (read with scalar loads; no device copy of host arrays is needed).
struct SegLayout {
  int32_t n;                    // N participants
  int32_t seg_off[kMaxP + 1];   // token offsets, seg_off[N] = total
  int32_t tile_cum[kMaxP + 1];  // cumulative count of query tiles (tiles never straddle segments)
  int32_t chunk_cum[kMaxP + 1]; // cumulative count of keep-list chunks
  int32_t pair_cum[kMaxP + 1];  // cumulative count of query-tile pairs, tiles paired inside each segment
};

struct PrefillArgs {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  int64_t q_block_stride;   // elements between consecutive blocks (batched launch)
  int64_t kv_block_stride;
  const uint8_t* keep_chunks;   // device, or nullptr
  const void* k_list;           // K, V the kept-tile list refers to: k, v themselves when the keep chunks
  const void* v_list;           // are whole tiles, else the packed copies of the kept rows (workspace)
  const int2* kept_tiles;       // device (workspace): (first row, valid rows) of kept 64-row tiles
  const int32_t* kept_cum;      // device (workspace): kept tiles of participants < n, [N+1]
  int32_t chunk_tokens;
  int32_t total;
  int32_t Hq, Hkv, D;
  int32_t block_idx0;
  int32_t sync_interval;
  int32_t sync_override;    // -1 rule, 0 local, 1 sync
  int32_t causal;
  int32_t heads_per_wg;     // MFMA kernel: query heads of one KV group handled by one workgroup
  int32_t q_tile_rows;      // MFMA kernel: query rows per workgroup
  int32_t n_q_tiles;
  int32_t n_cus;            // compute units of the device (launch shape heuristics)
  float scale;              // softmax scale
  int32_t n_ordered;        // > 0: one workgroup per query tile, workgroup p takes tile_order[p] (MFMA kernel)
  int32_t warm_kv;          // MFMA kernel: every workgroup pulls the K, V rows of its own query rows into L2 first
  int32_t one_tile_heavy_first;  // MFMA kernel, causal launch of several rounds of workgroups: one query tile per
                                 // workgroup, heaviest first (seg.pair_cum then counts tiles in seg_order's order)
  SegLayout seg;
  uint16_t tile_order[kMaxOrderedTiles];
  uint8_t seg_order[kMaxP];      // participants by decreasing length (local blocks of a heavy-first launch)
};

static_assert(sizeof(PrefillArgs) <= 4096, "kernel arguments are limited to 4 KB");

struct DecodeArgs {
  const void* q;
  const void* k_cache;
  const void* v_cache;
  void* out;
  float* part_o;            // [Hkv, n_chunks, cols, D] fp32: sum_j p_j v_j with p_j = 2^(s_j - m), unnormalised
  float* part_ml;           // [Hkv, n_chunks, cols, 2] (m in log2 domain, l)
  int32_t* counters;        // [Hkv, N] chunks counted in per (KV head, segment); zero before and after a launch
  int32_t fuse_combine;     // local block with at most 16 query columns: the last chunk of a segment merges
  int32_t N, Hq, Hkv, D;
  int32_t is_sync;
  int32_t chunk_rows;       // cache rows per workgroup
  int32_t n_chunks;         // total chunks over all segments
  int32_t cols;             // query columns per partial row block: G (local) or N*G (sync)
  int32_t has_remote;       // remote_lens given
  float scale;
  // several blocks in one launch (grid z, or y for the combine): block z is block_list[z]
  // blocks of block_stride bytes away from q/out and the caches, and works in its own slice
  // of the workspace (slice_bytes apart, partials and counters laid out alike in every slice)
  int64_t q_block_bytes;
  int64_t cache_block_bytes;
  int64_t slice_bytes;
  uint16_t block_list[kMaxFusedBlocks];
  int32_t seg_off[kMaxP + 1];
  int32_t seg_lens[kMaxP];
  int32_t remote_lens[kMaxP];
  int32_t chunk_cum[kMaxP + 1];
};

struct AggregateArgs {
  const void* k_local[kMaxP];
  const void* v_local[kMaxP];
  void* k_global;
  void* v_global;
  int32_t seg_off[kMaxP + 1];
  int32_t n;
  int32_t row_bytes;        // Hkv * D * element size, multiple of 16
};

// Host-side launchers (one per kernel family); each returns the hipError_t of the launch.
hipError_t launch_prefill_generic(const PrefillArgs& a, int n_blocks, int dtype, hipStream_t s);
hipError_t launch_prefill_mfma(const PrefillArgs& a, int n_blocks, hipStream_t s);
hipError_t launch_build_kept_tiles(const PrefillArgs& a, int2* kept_tiles, int32_t* kept_cum,
                                   hipStream_t s);
hipError_t launch_pack_kept_rows(const PrefillArgs& a, int32_t* kept_rows, int32_t* src_index, void* k_packed,
                                 void* v_packed, int2* kept_tiles, int32_t* kept_cum, hipStream_t s);
hipError_t launch_decode(const DecodeArgs& a, int dtype, int n_z, hipStream_t s);
hipError_t launch_decode_zero_counters(int32_t* counters, int n, int slices, int64_t slice_bytes, hipStream_t s);
hipError_t launch_aggregate(const AggregateArgs& a, hipStream_t s);
hipError_t launch_rmsnorm(const float* x, void* out, int64_t rows, int d_model, float eps, hipStream_t s);
hipError_t launch_residual_add_rmsnorm(float* x, const void* y, void* out, int64_t rows, int d_model, float eps,
                                       hipStream_t s);
hipError_t launch_rope_split(const void* qkv, const int32_t* pos, void* q, void* k, void* v, int64_t tokens, int Hq,
                             int Hkv, int D, float theta, hipStream_t s);
hipError_t launch_swiglu(const void* gate_up, void* out, int64_t rows, int F, hipStream_t s);
hipError_t launch_residual_add(float* x, const void* y, int64_t n, hipStream_t s);
hipError_t launch_stream_probe(const void* src, int64_t bytes, int n_wgs, int pattern, float* sink, hipStream_t s);
hipError_t launch_mfma_probe(float* sink, int n_wgs, int iters, hipStream_t s);

// A kernel's dynamic-LDS limit is a per-device attribute: set it the first time the kernel is
// launched on a device (`done` holds one bit per device; setting it twice is harmless).
inline hipError_t set_max_dynamic_lds_once(std::atomic<uint64_t>& done, const void* kernel, int bytes) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = (dev >= 0 && dev < 64) ? (1ull << dev) : 0;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && bit) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// Algorithm 1: block m = Ht + h (1-based) is the global-attention block iff h = H.
__host__ __device__ inline bool sync_block_rule(int32_t H, int32_t block_idx) {
  return H >= 1 && ((block_idx + 1) % H) == 0;
}

#if defined(__HIPCC__)
typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ inline float bf16_bits_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round-to-nearest-even float -> bf16 (hardware conversion on gfx950)
__device__ inline uint16_t f32_to_bf16_bits(float f) {
  bf16_t b = (bf16_t)f;
  return __builtin_bit_cast(uint16_t, b);
}

__device__ inline float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
#endif

}  // namespace fedattn
