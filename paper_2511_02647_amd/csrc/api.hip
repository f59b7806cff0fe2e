// C ABI of the FedAttn library: argument validation, the sync-block rule of
// Algorithm 1, kernel selection and launch.  No device memory is allocated here
// and nothing is kept between calls.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "common.h"

using namespace fedattn;

namespace {

thread_local char g_err[512] = "";

fedattn_status fail(fedattn_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

fedattn_status check_params(const fedattn_params* p) {
  if (!p) return fail(FEDATTN_EINVAL, "params is NULL");
  if (p->n_participants < 1 || p->n_participants > FEDATTN_MAX_PARTICIPANTS)
    return fail(FEDATTN_EINVAL, "n_participants %d outside 1..%d", p->n_participants, FEDATTN_MAX_PARTICIPANTS);
  if (p->n_q_heads < 1 || p->n_kv_heads < 1 || p->n_q_heads % p->n_kv_heads != 0)
    return fail(FEDATTN_EINVAL, "n_q_heads %d must be a positive multiple of n_kv_heads %d", p->n_q_heads,
                p->n_kv_heads);
  if (p->head_dim < 8 || p->head_dim > 256 || p->head_dim % 8 != 0)
    return fail(FEDATTN_EINVAL, "head_dim %d must be a multiple of 8 in 8..256", p->head_dim);
  if (p->dtype != FEDATTN_BF16 && p->dtype != FEDATTN_F32) return fail(FEDATTN_EINVAL, "unknown dtype %d", p->dtype);
  if (!(p->softmax_scale >= 0.f) || !isfinite(p->softmax_scale))
    return fail(FEDATTN_EINVAL, "softmax_scale must be finite and >= 0");
  if (p->causal != 0 && p->causal != 1) return fail(FEDATTN_EINVAL, "causal must be 0 or 1");
  return FEDATTN_OK;
}

float resolve_scale(const fedattn_params* p) {
  return p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
}

fedattn_status check_offsets(const fedattn_params* p, const int32_t* seg) {
  if (!seg) return fail(FEDATTN_EINVAL, "seg_offsets is NULL");
  if (seg[0] != 0) return fail(FEDATTN_EINVAL, "seg_offsets[0] must be 0");
  for (int n = 0; n < p->n_participants; ++n)
    if (seg[n + 1] < seg[n]) return fail(FEDATTN_EINVAL, "seg_offsets decreases at participant %d", n);
  return FEDATTN_OK;
}

bool use_mfma_prefill(const fedattn_params* p) {
  return p->dtype == FEDATTN_BF16 && (p->head_dim == 64 || p->head_dim == 128);
}

// keep chunks that are not whole 64-row tiles: the MFMA path packs the kept rows first
bool needs_row_packing(int chunk_tokens) { return chunk_tokens > 0 && chunk_tokens % kKvTile != 0; }

// Decode splits every participant's cache segment into chunks of `rows` cache rows (a
// multiple of the 64-row tile), one workgroup per (chunk, KV head).  The split aims at
// one workgroup per CU of the current device: about n_cus / Hkv chunks over all segments.
// The CU count is looked up once per device.
int device_cus() {
  constexpr int kMaxDevices = 64;
  static std::atomic<int> cus[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  const bool cached = dev >= 0 && dev < kMaxDevices;
  if (cached) {
    const int c = cus[dev].load(std::memory_order_relaxed);
    if (c > 0) return c;
  }
  int n = 0;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
  if (cached) cus[dev].store(n, std::memory_order_relaxed);
  return n;
}

int decode_target_chunks(int Hkv) {
  const int t = device_cus() / Hkv;
  return t < 1 ? 1 : t;
}

int decode_chunk_rows(int64_t total_rows, int Hkv) {
  const int64_t target = decode_target_chunks(Hkv);
  int64_t rows = (total_rows + target - 1) / target;
  rows = (rows + kKvTile - 1) / kKvTile * kKvTile;
  return (int)(rows < kKvTile ? kKvTile : rows);
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// prefill workspace: [kept_cum: (kMaxP+1) int32, padded][kept_tiles: int2 per 64-row tile]
// and, for keep chunks finer than a tile on the MFMA path:
// [kept_rows: kMaxP int32][src_index: int32 per token][packed K][packed V]
constexpr size_t kKeptCumBytes = 1024;
constexpr size_t kKeptRowsBytes = 512;
struct PrefillWs {
  size_t tiles_off, rows_off, index_off, k_off, v_off, total;
};
PrefillWs prefill_ws_layout(const fedattn_params* p, int32_t tokens, int32_t chunk_tokens) {
  PrefillWs w;
  const size_t max_tiles = (size_t)tokens / kKvTile + (size_t)p->n_participants + 1;
  w.tiles_off = kKeptCumBytes;
  w.rows_off = w.tiles_off + align_up(max_tiles * sizeof(int2), 256);
  w.index_off = w.k_off = w.v_off = w.total = w.rows_off;
  if (use_mfma_prefill(p) && needs_row_packing(chunk_tokens)) {
    const size_t kv_bytes = (size_t)tokens * (size_t)p->n_kv_heads * (size_t)p->head_dim * 2;
    w.index_off = w.rows_off + kKeptRowsBytes;
    w.k_off = w.index_off + align_up((size_t)tokens * 4, 256);
    w.v_off = w.k_off + align_up(kv_bytes, 256);
    w.total = w.v_off + align_up(kv_bytes, 256);
  }
  return w;
}

// chunk counters of the fused combine, one per (KV head, participant), at the end of the workspace
size_t decode_counter_bytes(const fedattn_params* p) {
  return align_up((size_t)p->n_kv_heads * (size_t)p->n_participants * 4, 256);
}

size_t decode_ws_bytes(const fedattn_params* p, int32_t capacity) {
  if (!(p->dtype == FEDATTN_BF16 && (p->head_dim == 64 || p->head_dim == 128))) return 16;
  const size_t G = (size_t)(p->n_q_heads / p->n_kv_heads);
  const size_t N = (size_t)p->n_participants;
  // chunks <= sum_n (rows_n / chunk_rows + 1) <= target + N
  (void)capacity;
  const size_t chunks = (size_t)decode_target_chunks(p->n_kv_heads) + N;
  const size_t rows = (size_t)p->n_kv_heads * chunks * G * N;  // sync blocks: N*G query columns per chunk
  return align_up(rows * (size_t)p->head_dim * 4, 256) + align_up(rows * 8, 256) + decode_counter_bytes(p);
}

// fedattn_prefill_sync_local_kv, participants' K/V not back to back: room for one aggregated copy each
size_t local_kv_copy_bytes(const fedattn_params* p, int32_t tokens) {
  return align_up((size_t)tokens * (size_t)p->n_kv_heads * (size_t)p->head_dim * (p->dtype == FEDATTN_BF16 ? 2 : 4), 256);
}

fedattn_status run_prefill(const fedattn_params* p, int32_t block_idx0, int32_t n_blocks, const void* q,
                           const void* k, const void* v, void* out, int64_t q_stride, int64_t kv_stride,
                           const int32_t* seg, const uint8_t* keep_chunks, int32_t chunk_tokens,
                           int32_t sync_override, void* workspace, size_t workspace_bytes, void* stream) {
  fedattn_status st = check_params(p);
  if (st != FEDATTN_OK) return st;
  st = check_offsets(p, seg);
  if (st != FEDATTN_OK) return st;
  if (block_idx0 < 0 || n_blocks < 0) return fail(FEDATTN_EINVAL, "negative block index or count");
  if (sync_override < -1 || sync_override > 1) return fail(FEDATTN_EINVAL, "sync_override must be -1, 0 or 1");
  const int N = p->n_participants;
  const int32_t total = seg[N];
  if (total == 0 || n_blocks == 0) return FEDATTN_OK;
  if (!q || !k || !v || !out) return fail(FEDATTN_EINVAL, "q, k, v and out must not be NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return fail(FEDATTN_EINVAL, "q, k, v and out must be 16-byte aligned");
  if (n_blocks > 1 && (q_stride % 8 != 0 || kv_stride % 8 != 0 || q_stride < 0 || kv_stride < 0))
    return fail(FEDATTN_EINVAL, "block strides must be non-negative multiples of 8 elements");
  if (n_blocks > 65535) return fail(FEDATTN_EINVAL, "at most 65535 blocks per launch");
  const bool has_keep = keep_chunks != nullptr;
  if (has_keep && chunk_tokens <= 0) return fail(FEDATTN_EINVAL, "chunk_tokens must be positive with a keep-list");

  PrefillArgs a;
  memset(&a, 0, sizeof(a));
  a.q = q; a.k = k; a.v = v; a.out = out;
  a.q_block_stride = q_stride;
  a.kv_block_stride = kv_stride;
  a.keep_chunks = keep_chunks;
  a.chunk_tokens = has_keep ? chunk_tokens : 1;
  a.total = total;
  a.Hq = p->n_q_heads; a.Hkv = p->n_kv_heads; a.D = p->head_dim;
  a.block_idx0 = block_idx0;
  a.sync_interval = p->sync_interval;
  a.sync_override = sync_override;
  a.causal = p->causal;
  a.scale = resolve_scale(p);
  a.seg.n = N;

  const bool mfma = use_mfma_prefill(p);
  a.k_list = k;
  a.v_list = v;
  const int G = a.Hq / a.Hkv;
  a.heads_per_wg = (G % 4 == 0) ? 4 : ((G % 2 == 0) ? 2 : 1);
  a.q_tile_rows = kWaveRows * (4 / a.heads_per_wg);
  int64_t tiles = 0, chunks = 0, pairs = 0;
  for (int n = 0; n <= N; ++n) {
    a.seg.seg_off[n] = seg[n];
    a.seg.tile_cum[n] = (int32_t)tiles;
    a.seg.chunk_cum[n] = (int32_t)chunks;
    a.seg.pair_cum[n] = (int32_t)pairs;
    if (n < N) {
      const int64_t len = seg[n + 1] - seg[n];
      const int64_t tn = (len + a.q_tile_rows - 1) / a.q_tile_rows;
      tiles += tn;
      pairs += (tn + 1) / 2;
      if (has_keep) chunks += (len + chunk_tokens - 1) / chunk_tokens;
    }
  }
  a.n_q_tiles = (int32_t)tiles;
  a.n_cus = device_cus();
  if (tiles * a.Hkv * (G / a.heads_per_wg) > 0x7fffffffLL) return fail(FEDATTN_EUNSUPPORTED, "too many query tiles");

  hipStream_t s = reinterpret_cast<hipStream_t>(stream);
  // a block reads the keep-list only if it is a sync block
  bool any_sync = sync_override == 1;
  if (sync_override == -1)
    for (int b = 0; b < n_blocks && !any_sync; ++b) any_sync = sync_block_rule(p->sync_interval, block_idx0 + b);
  if (!has_keep || !any_sync) a.keep_chunks = nullptr;

  if (mfma) {
    if (a.keep_chunks) {
      if (n_blocks != 1) return fail(FEDATTN_EUNSUPPORTED, "a keep-list applies to one block per call");
      const PrefillWs w = prefill_ws_layout(p, total, chunk_tokens);
      if (!workspace || workspace_bytes < w.total)
        return fail(FEDATTN_EWORKSPACE, "prefill with a keep-list needs %zu workspace bytes, got %zu", w.total,
                    workspace_bytes);
      if (!aligned16(workspace)) return fail(FEDATTN_EINVAL, "workspace must be 16-byte aligned");
      unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
      int32_t* kept_cum = reinterpret_cast<int32_t*>(ws);
      int2* kept_tiles = reinterpret_cast<int2*>(ws + w.tiles_off);
      a.kept_cum = kept_cum;
      a.kept_tiles = kept_tiles;
      hipError_t e;
      if (needs_row_packing(chunk_tokens)) {
        a.k_list = ws + w.k_off;
        a.v_list = ws + w.v_off;
        e = launch_pack_kept_rows(a, reinterpret_cast<int32_t*>(ws + w.rows_off),
                                  reinterpret_cast<int32_t*>(ws + w.index_off), ws + w.k_off, ws + w.v_off,
                                  kept_tiles, kept_cum, s);
      } else {
        e = launch_build_kept_tiles(a, kept_tiles, kept_cum, s);
      }
      if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "keep-list compaction: %s", hipGetErrorString(e));
    }
    hipError_t e = launch_prefill_mfma(a, n_blocks, s);
    if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "prefill (mfma): %s", hipGetErrorString(e));
  } else {
    hipError_t e = launch_prefill_generic(a, n_blocks, p->dtype, s);
    if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "prefill (general): %s", hipGetErrorString(e));
  }
  return FEDATTN_OK;
}

}  // namespace

extern "C" {

int fedattn_is_sync_block(int32_t sync_interval, int32_t block_idx) {
  return sync_block_rule(sync_interval, block_idx) ? 1 : 0;
}

size_t fedattn_workspace_bytes(const fedattn_params* params, int32_t op, int32_t tokens, int32_t chunk_tokens) {
  if (check_params(params) != FEDATTN_OK || tokens < 0) return 0;
  if (op == FEDATTN_OP_PREFILL) return chunk_tokens > 0 ? prefill_ws_layout(params, tokens, chunk_tokens).total : 0;
  if (op == FEDATTN_OP_DECODE) return decode_ws_bytes(params, tokens);
  if (op == FEDATTN_OP_PREFILL_SYNC_LOCAL_KV)
    return 2 * local_kv_copy_bytes(params, tokens) + (chunk_tokens > 0 ? prefill_ws_layout(params, tokens, chunk_tokens).total : 0);
  fail(FEDATTN_EINVAL, "unknown op %d", op);
  return 0;
}

fedattn_status fedattn_prefill(const fedattn_params* params, int32_t block_idx, const void* q, const void* k,
                               const void* v, void* out, const int32_t* seg_offsets, const uint8_t* keep_chunks,
                               int32_t chunk_tokens, int32_t sync_override, void* workspace,
                               size_t workspace_bytes, void* stream) {
  return run_prefill(params, block_idx, 1, q, k, v, out, 0, 0, seg_offsets, keep_chunks, chunk_tokens,
                     sync_override, workspace, workspace_bytes, stream);
}

fedattn_status fedattn_prefill_sync_local_kv(const fedattn_params* params, const void* q, const void* const* k_local,
                                             const void* const* v_local, void* out, const int32_t* seg_offsets,
                                             const uint8_t* keep_chunks, int32_t chunk_tokens, void* workspace,
                                             size_t workspace_bytes, void* stream) {
  fedattn_status st = check_params(params);
  if (st != FEDATTN_OK) return st;
  st = check_offsets(params, seg_offsets);
  if (st != FEDATTN_OK) return st;
  if (!k_local || !v_local) return fail(FEDATTN_EINVAL, "k_local and v_local must not be NULL");
  const int N = params->n_participants;
  const int32_t total = seg_offsets[N];
  if (total == 0) return FEDATTN_OK;
  const int64_t row_bytes = (int64_t)params->n_kv_heads * params->head_dim * (params->dtype == FEDATTN_BF16 ? 2 : 4);
  // Sum_n Pi_n [k_n v_n] puts row r of participant n at global row seg_offsets[n] + r.  If every
  // participant's matrices already start that many rows behind one common base address, the
  // aggregated matrices exist as they are and the attention reads them in place.
  const unsigned char* k_base = nullptr;
  const unsigned char* v_base = nullptr;
  bool in_place = true;
  for (int n = 0; n < N; ++n) {
    if (seg_offsets[n + 1] == seg_offsets[n]) continue;
    if (!k_local[n] || !v_local[n]) return fail(FEDATTN_EINVAL, "local K/V of participant %d is NULL", n);
    if (!aligned16(k_local[n]) || !aligned16(v_local[n]))
      return fail(FEDATTN_EINVAL, "local K/V of participant %d is not 16-byte aligned", n);
    const unsigned char* kb = reinterpret_cast<const unsigned char*>(k_local[n]) - (int64_t)seg_offsets[n] * row_bytes;
    const unsigned char* vb = reinterpret_cast<const unsigned char*>(v_local[n]) - (int64_t)seg_offsets[n] * row_bytes;
    if (!k_base) {
      k_base = kb;
      v_base = vb;
    } else if (kb != k_base || vb != v_base) {
      in_place = false;
    }
  }
  unsigned char* ws = reinterpret_cast<unsigned char*>(workspace);
  size_t ws_left = workspace ? workspace_bytes : 0;
  if (!in_place) {
    const size_t copy = local_kv_copy_bytes(params, total);
    if (!workspace || workspace_bytes < 2 * copy)
      return fail(FEDATTN_EWORKSPACE,
                  "the participants' K/V do not lie back to back: aggregating them needs %zu workspace bytes, got %zu",
                  2 * copy, workspace_bytes);
    if (!aligned16(workspace)) return fail(FEDATTN_EINVAL, "workspace must be 16-byte aligned");
    if (keep_chunks && chunk_tokens > 0 &&
        workspace_bytes < 2 * copy + prefill_ws_layout(params, total, chunk_tokens).total)
      return fail(FEDATTN_EWORKSPACE, "workspace too small for the aggregated copy and the keep-list (%zu bytes needed)",
                  2 * copy + prefill_ws_layout(params, total, chunk_tokens).total);
    k_base = ws;
    v_base = ws + copy;
    ws += 2 * copy;
    ws_left -= 2 * copy;
  }
  // q, out and the keep-list arguments are validated by the prefill path; when they pass,
  // nothing there can fail short of a launch error, so the copy is enqueued only for valid calls
  if (!q || !out || !aligned16(q) || !aligned16(out)) return fail(FEDATTN_EINVAL, "q and out must be non-NULL and 16-byte aligned");
  if (keep_chunks && chunk_tokens <= 0) return fail(FEDATTN_EINVAL, "chunk_tokens must be positive with a keep-list");
  if (!in_place) {
    st = fedattn_aggregate_kv(params, k_local, v_local, seg_offsets, const_cast<unsigned char*>(k_base),
                              const_cast<unsigned char*>(v_base), stream);
    if (st != FEDATTN_OK) return st;
  }
  return run_prefill(params, 0, 1, q, k_base, v_base, out, 0, 0, seg_offsets, keep_chunks, chunk_tokens, 1,
                     ws_left ? ws : nullptr, ws_left, stream);
}

fedattn_status fedattn_prefill_blocks(const fedattn_params* params, int32_t block_idx0, int32_t n_blocks,
                                      const void* q, const void* k, const void* v, void* out,
                                      int64_t q_block_stride, int64_t kv_block_stride,
                                      const int32_t* seg_offsets, void* stream) {
  return run_prefill(params, block_idx0, n_blocks, q, k, v, out, q_block_stride, kv_block_stride, seg_offsets,
                     nullptr, 0, -1, nullptr, 0, stream);
}

// Everything about a decode call that can be checked without the workspace or the device.
static fedattn_status check_decode_args(const fedattn_params* params, int32_t block_idx0, int32_t n_blocks, const void* q,
                                        const void* k_cache, const void* v_cache, void* out, int64_t q_block_stride,
                                        int64_t cache_block_stride, const int32_t* seg_offsets, const int32_t* seg_lens,
                                        const int32_t* remote_lens, int32_t sync_override) {
  fedattn_status st = check_params(params);
  if (st != FEDATTN_OK) return st;
  st = check_offsets(params, seg_offsets);
  if (st != FEDATTN_OK) return st;
  if (!seg_lens) return fail(FEDATTN_EINVAL, "seg_lens is NULL");
  if (block_idx0 < 0 || n_blocks < 0) return fail(FEDATTN_EINVAL, "negative block index or count");
  if (sync_override < -1 || sync_override > 1) return fail(FEDATTN_EINVAL, "sync_override must be -1, 0 or 1");
  const int N = params->n_participants;
  for (int n = 0; n < N; ++n) {
    const int cap = seg_offsets[n + 1] - seg_offsets[n];
    if (seg_lens[n] < 0 || seg_lens[n] > cap)
      return fail(FEDATTN_EINVAL, "seg_lens[%d] = %d outside 0..capacity %d", n, seg_lens[n], cap);
    if (remote_lens && (remote_lens[n] < 0 || remote_lens[n] > cap))
      return fail(FEDATTN_EINVAL, "remote_lens[%d] = %d outside 0..capacity %d", n, remote_lens[n], cap);
  }
  if (n_blocks == 0) return FEDATTN_OK;
  if (!q || !out) return fail(FEDATTN_EINVAL, "q and out must not be NULL");
  const int32_t capacity = seg_offsets[N];
  if (capacity > 0 && (!k_cache || !v_cache)) return fail(FEDATTN_EINVAL, "k_cache and v_cache must not be NULL");
  if (!aligned16(q) || !aligned16(out) || !aligned16(k_cache) || !aligned16(v_cache))
    return fail(FEDATTN_EINVAL, "q, out, k_cache and v_cache must be 16-byte aligned");
  if (n_blocks > 1 && (q_block_stride % 8 != 0 || cache_block_stride % 8 != 0 || q_block_stride < 0 ||
                       cache_block_stride < 0))
    return fail(FEDATTN_EINVAL, "block strides must be non-negative multiples of 8 elements");

  return FEDATTN_OK;
}

// fused: blocks of one kind (local / sync) share launches, as many per launch as the workspace
// has slices for; otherwise one launch (pair) per block in block order
static fedattn_status run_decode(bool fused, const fedattn_params* params, int32_t block_idx0, int32_t n_blocks,
                                 const void* q, const void* k_cache, const void* v_cache, void* out,
                                 int64_t q_block_stride, int64_t cache_block_stride,
                                 const int32_t* seg_offsets, const int32_t* seg_lens,
                                 const int32_t* remote_lens, int32_t sync_override, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  fedattn_status st = check_decode_args(params, block_idx0, n_blocks, q, k_cache, v_cache, out, q_block_stride,
                                        cache_block_stride, seg_offsets, seg_lens, remote_lens, sync_override);
  if (st != FEDATTN_OK) return st;
  if (n_blocks == 0) return FEDATTN_OK;
  const int N = params->n_participants;
  const int32_t capacity = seg_offsets[N];

  const bool mfma = params->dtype == FEDATTN_BF16 && (params->head_dim == 64 || params->head_dim == 128);
  const size_t esize = params->dtype == FEDATTN_BF16 ? 2 : 4;
  DecodeArgs args[2];  // [0] local block, [1] sync block: the split differs, the layout does not
  bool built[2] = {false, false};
  int32_t* counters = nullptr;
  int slices = 1;            // blocks in flight at once, each in its own slice of the workspace
  size_t slice_bytes = 0;
  if (mfma) {
    const size_t need = decode_ws_bytes(params, capacity);
    if (!workspace || workspace_bytes < need)
      return fail(FEDATTN_EWORKSPACE, "decode needs %zu workspace bytes, got %zu", need, workspace_bytes);
    if (!aligned16(workspace)) return fail(FEDATTN_EINVAL, "workspace must be 16-byte aligned");
    slice_bytes = align_up(need, 256);
    if (fused) {
      if (n_blocks > 65535) return fail(FEDATTN_EINVAL, "at most 65535 blocks per fused call");
      const size_t fit = 1 + (workspace_bytes - need) / slice_bytes;
      slices = (int)(fit < (size_t)kMaxFusedBlocks ? fit : (size_t)kMaxFusedBlocks);
      if (slices > n_blocks) slices = n_blocks;
    }
    // local blocks count their chunks in at the end of their slice; the counters start at
    // zero and every launch leaves them at zero for the next one
    counters = reinterpret_cast<int32_t*>(reinterpret_cast<unsigned char*>(workspace) + need - decode_counter_bytes(params));
  }
  fused = fused && mfma;
  const auto block_is_sync = [&](int b) {
    return sync_override >= 0 ? sync_override != 0 : sync_block_rule(params->sync_interval, block_idx0 + b);
  };
  const auto prepare = [&](bool sync) -> fedattn_status {
    DecodeArgs& a = args[sync ? 1 : 0];
    if (!built[sync ? 1 : 0]) {
      memset(&a, 0, sizeof(a));
      a.N = N; a.Hq = params->n_q_heads; a.Hkv = params->n_kv_heads; a.D = params->head_dim;
      a.is_sync = sync ? 1 : 0;
      a.has_remote = (sync && remote_lens) ? 1 : 0;
      a.scale = resolve_scale(params);
      const int G = a.Hq / a.Hkv;
      a.cols = sync ? N * G : G;
      int64_t total_rows = 0;
      for (int n = 0; n < N; ++n) {
        const int rem = a.has_remote ? remote_lens[n] : seg_lens[n];
        total_rows += sync ? (seg_lens[n] > rem ? seg_lens[n] : rem) : seg_lens[n];
      }
      a.chunk_rows = decode_chunk_rows(total_rows, a.Hkv);
      int64_t chunks = 0;
      for (int n = 0; n <= N; ++n) {
        a.seg_off[n] = seg_offsets[n];
        a.chunk_cum[n] = (int32_t)chunks;
        if (n < N) {
          a.seg_lens[n] = seg_lens[n];
          a.remote_lens[n] = remote_lens ? remote_lens[n] : seg_lens[n];
          const int rem = a.has_remote ? a.remote_lens[n] : seg_lens[n];
          const int rows = sync ? (seg_lens[n] > rem ? seg_lens[n] : rem) : seg_lens[n];
          chunks += (rows + a.chunk_rows - 1) / a.chunk_rows;
        }
      }
      a.n_chunks = (int32_t)chunks;
      if (mfma) {
        const size_t need = decode_ws_bytes(params, capacity) - decode_counter_bytes(params);
        const size_t rows = (size_t)a.Hkv * (size_t)a.n_chunks * (size_t)a.cols;
        const size_t o_bytes = align_up(rows * (size_t)a.D * 4, 256);
        if (o_bytes + rows * 8 > need)
          return fail(FEDATTN_EWORKSPACE, "decode partials (%zu bytes) exceed the workspace", o_bytes + rows * 8);
        a.part_o = reinterpret_cast<float*>(workspace);
        a.part_ml = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(workspace) + o_bytes);
        a.counters = counters;
        // fused combine: the workgroups of a segment write its output rows, so every segment
        // needs one (an empty segment's zero rows come from the separate combine kernel)
        bool all_have_rows = true;
        for (int n = 0; n < N; ++n) all_have_rows = all_have_rows && seg_lens[n] > 0;
        a.fuse_combine = (!sync && a.cols <= 16 && all_have_rows) ? 1 : 0;
      }
      a.q_block_bytes = q_block_stride * (int64_t)esize;
      a.cache_block_bytes = cache_block_stride * (int64_t)esize;
      a.slice_bytes = (int64_t)slice_bytes;
      built[sync ? 1 : 0] = true;
    }
    return FEDATTN_OK;
  };
  // everything that can fail validation is decided before the first launch
  for (int b = 0; b < n_blocks && !(built[0] && built[1]); ++b) {
    st = prepare(block_is_sync(b));
    if (st != FEDATTN_OK) return st;
  }
  if (mfma) {
    hipError_t e = launch_decode_zero_counters(counters, params->n_kv_heads * N, slices, (int64_t)slice_bytes,
                                               reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "decode (counters): %s", hipGetErrorString(e));
  }
  if (fused) {
    for (int kind = 0; kind < 2; ++kind) {
      int first = 0;
      while (first < n_blocks) {
        int cnt = 0;
        DecodeArgs& a = args[kind];
        int b = first;
        for (; b < n_blocks && cnt < slices; ++b) {
          if ((block_is_sync(b) ? 1 : 0) != kind) continue;
          if (cnt == 0) {
            st = prepare(kind == 1);
            if (st != FEDATTN_OK) return st;
          }
          a.block_list[cnt++] = (uint16_t)b;
        }
        first = b;
        if (cnt == 0) continue;
        a.q = q; a.out = out; a.k_cache = k_cache; a.v_cache = v_cache;
        hipError_t e = launch_decode(a, params->dtype, cnt, reinterpret_cast<hipStream_t>(stream));
        if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "decode (fused, %d blocks): %s", cnt, hipGetErrorString(e));
      }
    }
    return FEDATTN_OK;
  }
  for (int b = 0; b < n_blocks; ++b) {
    const bool sync = block_is_sync(b);
    st = prepare(sync);
    if (st != FEDATTN_OK) return st;
    DecodeArgs& a = args[sync ? 1 : 0];
    a.q = reinterpret_cast<const unsigned char*>(q) + (size_t)b * (size_t)q_block_stride * esize;
    a.out = reinterpret_cast<unsigned char*>(out) + (size_t)b * (size_t)q_block_stride * esize;
    a.k_cache = reinterpret_cast<const unsigned char*>(k_cache) + (size_t)b * (size_t)cache_block_stride * esize;
    a.v_cache = reinterpret_cast<const unsigned char*>(v_cache) + (size_t)b * (size_t)cache_block_stride * esize;
    hipError_t e = launch_decode(a, params->dtype, 1, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "decode (block %d): %s", block_idx0 + b, hipGetErrorString(e));
  }
  return FEDATTN_OK;
}

fedattn_status fedattn_decode_blocks(const fedattn_params* params, int32_t block_idx0, int32_t n_blocks,
                                     const void* q, const void* k_cache, const void* v_cache, void* out,
                                     int64_t q_block_stride, int64_t cache_block_stride,
                                     const int32_t* seg_offsets, const int32_t* seg_lens,
                                     const int32_t* remote_lens, int32_t sync_override, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  return run_decode(false, params, block_idx0, n_blocks, q, k_cache, v_cache, out, q_block_stride, cache_block_stride,
                    seg_offsets, seg_lens, remote_lens, sync_override, workspace, workspace_bytes, stream);
}

fedattn_status fedattn_decode_blocks_fused(const fedattn_params* params, int32_t block_idx0, int32_t n_blocks,
                                           const void* q, const void* k_cache, const void* v_cache, void* out,
                                           int64_t q_block_stride, int64_t cache_block_stride,
                                           const int32_t* seg_offsets, const int32_t* seg_lens,
                                           const int32_t* remote_lens, int32_t sync_override, void* workspace,
                                           size_t workspace_bytes, void* stream) {
  return run_decode(true, params, block_idx0, n_blocks, q, k_cache, v_cache, out, q_block_stride, cache_block_stride,
                    seg_offsets, seg_lens, remote_lens, sync_override, workspace, workspace_bytes, stream);
}

fedattn_status fedattn_decode(const fedattn_params* params, int32_t block_idx, const void* q, const void* k_cache,
                              const void* v_cache, void* out, const int32_t* seg_offsets, const int32_t* seg_lens,
                              const int32_t* remote_lens, int32_t sync_override, void* workspace,
                              size_t workspace_bytes, void* stream) {
  return fedattn_decode_blocks(params, block_idx, 1, q, k_cache, v_cache, out, 0, 0, seg_offsets, seg_lens,
                               remote_lens, sync_override, workspace, workspace_bytes, stream);
}

// ---- decode for callers that cannot allocate ---------------------------------------------
// The split-KV partials and chunk counters of fedattn_decode live in this array instead of a
// caller's workspace.  Every device the library runs on holds its own copy at its own address;
// in host code the array's name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[FEDATTN_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxScratchDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxScratchDevices];  // device address of `scratch`, per device; NULL until looked up

// Device address of the current device's copy of `scratch` (looked up once per device).
fedattn_status static_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxScratchDevices)
    return fail(FEDATTN_EUNSUPPORTED, "device %d outside 0..%d", dev, kMaxScratchDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr)
      return fail(FEDATTN_ELAUNCH, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return FEDATTN_OK;
}
}  // namespace

fedattn_status fedattn_decode_static(const fedattn_params* params, int32_t block_idx, const void* q,
                                     const void* k_cache, const void* v_cache, void* out,
                                     const int32_t* seg_offsets, const int32_t* seg_lens,
                                     const int32_t* remote_lens, int32_t sync_override, void* stream) {
  fedattn_status st = check_decode_args(params, block_idx, 1, q, k_cache, v_cache, out, 0, 0, seg_offsets, seg_lens,
                                        remote_lens, sync_override);
  if (st != FEDATTN_OK) return st;
  const size_t need = decode_ws_bytes(params, seg_offsets[params->n_participants]);
  if (need > (size_t)FEDATTN_STATIC_SCRATCH_BYTES)
    return fail(FEDATTN_EWORKSPACE,
                "fedattn_decode_static: this problem needs %zu bytes of scratch, the built-in array holds %zu; "
                "use fedattn_decode with a workspace",
                need, (size_t)FEDATTN_STATIC_SCRATCH_BYTES);
  void* ptr = nullptr;
  st = static_scratch(&ptr);
  if (st != FEDATTN_OK) return st;
  return run_decode(false, params, block_idx, 1, q, k_cache, v_cache, out, 0, 0, seg_offsets, seg_lens, remote_lens,
                    sync_override, ptr, (size_t)FEDATTN_STATIC_SCRATCH_BYTES, stream);
}

fedattn_status fedattn_aggregate_kv(const fedattn_params* params, const void* const* k_local,
                                    const void* const* v_local, const int32_t* seg_offsets, void* k_global,
                                    void* v_global, void* stream) {
  fedattn_status st = check_params(params);
  if (st != FEDATTN_OK) return st;
  st = check_offsets(params, seg_offsets);
  if (st != FEDATTN_OK) return st;
  if (!k_local || !v_local) return fail(FEDATTN_EINVAL, "k_local and v_local must not be NULL");
  const int N = params->n_participants;
  if (seg_offsets[N] == 0) return FEDATTN_OK;
  if (!k_global || !v_global || !aligned16(k_global) || !aligned16(v_global))
    return fail(FEDATTN_EINVAL, "k_global and v_global must be non-NULL and 16-byte aligned");
  AggregateArgs a;
  memset(&a, 0, sizeof(a));
  a.n = N;
  a.row_bytes = params->n_kv_heads * params->head_dim * (params->dtype == FEDATTN_BF16 ? 2 : 4);
  a.k_global = k_global;
  a.v_global = v_global;
  for (int n = 0; n <= N; ++n) a.seg_off[n] = seg_offsets[n];
  for (int n = 0; n < N; ++n) {
    a.k_local[n] = k_local[n];
    a.v_local[n] = v_local[n];
    if (seg_offsets[n + 1] > seg_offsets[n]) {
      if (!k_local[n] || !v_local[n]) return fail(FEDATTN_EINVAL, "local K/V of participant %d is NULL", n);
      if (!aligned16(k_local[n]) || !aligned16(v_local[n]))
        return fail(FEDATTN_EINVAL, "local K/V of participant %d is not 16-byte aligned", n);
    }
  }
  hipError_t e = launch_aggregate(a, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "aggregate: %s", hipGetErrorString(e));
  return FEDATTN_OK;
}

// ---- element-wise pieces of the decoder block around the attention ----------------------
namespace {
constexpr int64_t kMaxGrid = 0x7fffffffLL;
}

fedattn_status fedattn_rmsnorm(const float* x, void* out, int64_t rows, int32_t d_model, float eps, void* stream) {
  if (rows < 0 || d_model <= 0 || d_model % 4 != 0) return fail(FEDATTN_EINVAL, "rmsnorm: rows >= 0, d_model a positive multiple of 4");
  if (!(eps >= 0.f)) return fail(FEDATTN_EINVAL, "rmsnorm: eps must be non-negative");
  if (rows == 0) return FEDATTN_OK;
  if (!x || !out || !aligned16(x) || !aligned16(out)) return fail(FEDATTN_EINVAL, "rmsnorm: x and out must be non-NULL and 16-byte aligned");
  if ((rows + 3) / 4 > kMaxGrid) return fail(FEDATTN_EUNSUPPORTED, "rmsnorm: too many rows");
  hipError_t e = launch_rmsnorm(x, out, rows, d_model, eps, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "rmsnorm: %s", hipGetErrorString(e));
  return FEDATTN_OK;
}

fedattn_status fedattn_residual_add_rmsnorm(float* x, const void* y, void* out, int64_t rows, int32_t d_model, float eps,
                                            void* stream) {
  if (rows < 0 || d_model <= 0 || d_model % 4 != 0)
    return fail(FEDATTN_EINVAL, "residual_add_rmsnorm: rows >= 0, d_model a positive multiple of 4");
  if (!(eps >= 0.f)) return fail(FEDATTN_EINVAL, "residual_add_rmsnorm: eps must be non-negative");
  if (rows == 0) return FEDATTN_OK;
  if (!x || !y || !out || !aligned16(x) || !aligned16(y) || !aligned16(out))
    return fail(FEDATTN_EINVAL, "residual_add_rmsnorm: x, y and out must be non-NULL and 16-byte aligned");
  if ((rows + 3) / 4 > kMaxGrid) return fail(FEDATTN_EUNSUPPORTED, "residual_add_rmsnorm: too many rows");
  hipError_t e = launch_residual_add_rmsnorm(x, y, out, rows, d_model, eps, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "residual_add_rmsnorm: %s", hipGetErrorString(e));
  return FEDATTN_OK;
}

fedattn_status fedattn_rope_split_qkv(const void* qkv, const int32_t* pos, void* q, void* k, void* v, int64_t tokens,
                                      int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float theta,
                                      void* stream) {
  if (tokens < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || head_dim <= 0 || head_dim % 8 != 0)
    return fail(FEDATTN_EINVAL, "rope: tokens >= 0, positive head counts, head_dim a positive multiple of 8");
  if (!(theta > 1.f)) return fail(FEDATTN_EINVAL, "rope: theta must exceed 1");
  if (tokens == 0) return FEDATTN_OK;
  if (!qkv || !q || !k || !v || !aligned16(qkv) || !aligned16(q) || !aligned16(k) || !aligned16(v))
    return fail(FEDATTN_EINVAL, "rope: qkv, q, k and v must be non-NULL and 16-byte aligned");
  if (tokens * (head_dim / 8) / 256 + 1 > kMaxGrid) return fail(FEDATTN_EUNSUPPORTED, "rope: too many tokens");
  hipError_t e = launch_rope_split(qkv, pos, q, k, v, tokens, n_q_heads, n_kv_heads, head_dim, theta,
                                   reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "rope: %s", hipGetErrorString(e));
  return FEDATTN_OK;
}

fedattn_status fedattn_swiglu(const void* gate_up, void* out, int64_t rows, int32_t hidden, void* stream) {
  if (rows < 0 || hidden <= 0 || hidden % 8 != 0) return fail(FEDATTN_EINVAL, "swiglu: rows >= 0, hidden a positive multiple of 8");
  if (rows == 0) return FEDATTN_OK;
  if (!gate_up || !out || !aligned16(gate_up) || !aligned16(out)) return fail(FEDATTN_EINVAL, "swiglu: gate_up and out must be non-NULL and 16-byte aligned");
  if (rows * (hidden / 8) / 256 + 1 > kMaxGrid) return fail(FEDATTN_EUNSUPPORTED, "swiglu: too many elements");
  hipError_t e = launch_swiglu(gate_up, out, rows, hidden, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "swiglu: %s", hipGetErrorString(e));
  return FEDATTN_OK;
}

fedattn_status fedattn_residual_add(float* x, const void* y, int64_t n, void* stream) {
  if (n < 0 || n % 4 != 0) return fail(FEDATTN_EINVAL, "residual_add: n must be a non-negative multiple of 4");
  if (n == 0) return FEDATTN_OK;
  if (!x || !y || !aligned16(x) || !aligned16(y)) return fail(FEDATTN_EINVAL, "residual_add: x and y must be non-NULL and 16-byte aligned");
  if (n / 4 / 256 + 1 > kMaxGrid) return fail(FEDATTN_EUNSUPPORTED, "residual_add: too many elements");
  hipError_t e = launch_residual_add(x, y, n, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) return fail(FEDATTN_ELAUNCH, "residual_add: %s", hipGetErrorString(e));
  return FEDATTN_OK;
}

// ---- measurement aids ---------------------------------------------------------------------
int64_t fedattn_probe_stream(const void* src, int64_t bytes, int32_t pattern, void* sink, void* stream) {
  if (!src || !sink || !aligned16(src) || bytes <= 0 || (pattern != 0 && pattern != 1)) {
    fail(FEDATTN_EINVAL, "probe_stream: src and sink non-NULL, src 16-byte aligned, bytes > 0, pattern 0 or 1");
    return -1;
  }
  const int n_wgs = device_cus() / 8 * 8;
  const int64_t unit = pattern == 0 ? (int64_t)n_wgs * 32768 : (int64_t)n_wgs * 64 * 256 * 2;
  const int64_t moved = bytes / unit * unit;
  if (moved == 0) {
    fail(FEDATTN_EINVAL, "probe_stream: at least %lld bytes", (long long)unit);
    return -1;
  }
  hipError_t e = launch_stream_probe(src, moved, n_wgs, pattern, reinterpret_cast<float*>(sink), reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) {
    fail(FEDATTN_ELAUNCH, "probe_stream: %s", hipGetErrorString(e));
    return -1;
  }
  return moved;
}

int64_t fedattn_probe_mfma(void* sink, int32_t iters, void* stream) {
  if (!sink || iters <= 0) {
    fail(FEDATTN_EINVAL, "probe_mfma: sink non-NULL, iters > 0");
    return -1;
  }
  const int n_wgs = device_cus();
  hipError_t e = launch_mfma_probe(reinterpret_cast<float*>(sink), n_wgs, iters, reinterpret_cast<hipStream_t>(stream));
  if (e != hipSuccess) {
    fail(FEDATTN_ELAUNCH, "probe_mfma: %s", hipGetErrorString(e));
    return -1;
  }
  return (int64_t)n_wgs * 8 /* wavefronts */ * iters * 8 /* MFMAs */ * (2LL * 32 * 32 * 16);
}

const char* fedattn_last_error(void) { return g_err; }

const char* fedattn_version(void) { return "fedattn-gfx950 0.1"; }

}  // extern "C"
