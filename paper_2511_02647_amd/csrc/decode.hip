// Decode attention (Section IV-C): one new query per participant over the block's
// KV cache; bandwidth-bound, so the cache is streamed exactly once.
//
// Split-KV: a workgroup takes one chunk of one participant's cache segment for
// one KV head and ALL query rows that may see it - the G query heads of that
// participant in a local block, the N*G rows of all participants in a sync block
// (the aggregated cache is read once for everybody).  The chunk streams through a
// 3-stage LDS ring of 64-row K/V tiles filled by direct HBM -> LDS loads (two
// tiles in flight per workgroup, one workgroup per CU).  Every wavefront works on
// every tile: wavefront w takes tile rows 16w..16w+15 against all query columns,
// S^T[kv][q] = K Q^T on v_mfma_f32_16x16x32_bf16 and O^T[d][q] += V^T P^T on
// v_mfma_f32_16x16x16_bf16, whose k-slots are exactly the 4 rows per lane that the
// first product leaves in a lane, with V^T operands from transposing LDS reads.  Each
// wavefront keeps its own online softmax per query column; the wavefronts are merged
// at the end and a second small kernel merges the chunks:
//   o = sum_c O_c 2^(m_c - m) / sum_c l_c 2^(m_c - m).
#include "common.h"
#include "mfma_tile.h"

namespace fedattn {

namespace {

// Three stages of 64-row K/V tiles (96 KB per workgroup, two tiles in flight while one is
// worked on): measured against four stages (three in flight), the deeper ring only lengthens
// the queue in front of the memory system; a block-step of 16 x 1152 rows takes 17.4 instead
// of 18.0 us.
constexpr int kDecodeStages = 3;

template <int D>
constexpr int decode_smem_bytes() { return kDecodeStages * 2 * KvTile<D, 0>::TILEB; }

// value of x maximised / summed over the 4 lanes (lane%16 + 16 k) that share a query column
__device__ inline float max_over_kgroups(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];
  return max_across_halves(fmaxf(__uint_as_float(a), __uint_as_float(b)));
}
__device__ inline float sum_over_kgroups(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];
  return sum_across_halves(__uint_as_float(a) + __uint_as_float(b));
}

// COLSPLIT = false (at most 16 query columns, e.g. the G heads of one participant in a
// local block): 4 wavefronts, wavefront w takes tile rows 16w..16w+15; they are merged
// through LDS at the end.  COLSPLIT = true (up to 64 query columns, sync blocks): 8
// wavefronts (two per SIMD, so that one's LDS and MFMA latencies hide behind the other);
// wavefront w takes query columns 16 (w mod 4).. against tile rows 32 (w / 4)..+31.  Its two
// 16-row sub-tiles fill the 8 k-slots per lane of one v_mfma_f32_16x16x32_bf16 in the second
// product (slot e < 4: row 4 kg + e of the first sub-tile, e >= 4: of the second), which
// halves its MFMA count.  The two row halves of a column block are merged through LDS.
template <int D, bool COLSPLIT>
__global__ __launch_bounds__(COLSPLIT ? 512 : 256, 1) void decode_stream_kernel(DecodeArgs a) {
  constexpr int NW = COLSPLIT ? 8 : 4;
  using TL = KvTile<D, 0, NW>;
  constexpr int KS = D / 32;                 // k-steps of S^T (16x16x32)
  constexpr int DT = D / 16;                 // 16-row tiles of O^T along head_dim
  constexpr int CPR = TL::CPR, ROWB = TL::ROWB, TILEB = TL::TILEB, IPW = TL::IPW;
  constexpr int RSUB = COLSPLIT ? 2 : 1;     // 16-row sub-tiles a wavefront processes per tile
  constexpr int QCOLS = COLSPLIT ? 64 : 16;  // query columns per workgroup
  constexpr int OPAD = D + 4;                // floats per row of the merge buffer
  // stage s: K tile at s*2*TILEB, V tile at s*2*TILEB + TILEB; after the stream the
  // ring is reused as the merge buffer (row split only)
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  __shared__ float m_s[4][16];
  __shared__ float l_s[4][16];
  const lds_cptr lds0 = (lds_cptr)(lds_void_ptr)smem;
  const uint32_t lds_base = lds_addr_of(smem);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15;
  const int kg = lane >> 4;

  // block of a fused launch: its q/out, caches and workspace slice
  const int bz = blockIdx.z;
  const int64_t blk = a.block_list[bz];
  const unsigned char* q_ptr = reinterpret_cast<const unsigned char*>(a.q) + blk * a.q_block_bytes;
  unsigned char* out_ptr = reinterpret_cast<unsigned char*>(a.out) + blk * a.q_block_bytes;
  const unsigned char* k_ptr = reinterpret_cast<const unsigned char*>(a.k_cache) + blk * a.cache_block_bytes;
  const unsigned char* v_ptr = reinterpret_cast<const unsigned char*>(a.v_cache) + blk * a.cache_block_bytes;
  float* part_o = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(a.part_o) + bz * a.slice_bytes);
  float* part_ml = reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(a.part_ml) + bz * a.slice_bytes);
  int32_t* counters = reinterpret_cast<int32_t*>(reinterpret_cast<unsigned char*>(a.counters) + bz * a.slice_bytes);

  const int Hq = a.Hq, Hkv = a.Hkv;
  const int G = Hq / Hkv;
  const int g = blockIdx.x % Hkv;
  const int gc = blockIdx.x / Hkv;  // chunk index over all segments
  const int rh = COLSPLIT ? wave >> 2 : 0;   // row half of the tile (column split only)
  const int cb = blockIdx.y * QCOLS + (COLSPLIT ? 16 * (wave & 3) : 0);  // first query column of this wavefront

  // The segment tables sit in the kernel-argument buffer; a walk over them would take one
  // scalar-cache miss after another before the first cache row is requested.  Every lane
  // fetches the entries of segments `lane` and `lane + 64` at once, the chunk's segment is
  // found with ballots and its entries are read out of the lanes that hold them.
  const int N = a.N;
  const int ck_lo = a.chunk_cum[lane + 1], ck_hi = a.chunk_cum[lane + 65];
  const int sl_lo = a.seg_lens[lane], sl_hi = a.seg_lens[lane + 64];
  const int rl_lo = a.remote_lens[lane], rl_hi = a.remote_lens[lane + 64];
  const int so_lo = a.seg_off[lane], so_hi = a.seg_off[lane + 64];
  int m = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane < N && gc >= ck_lo));
  if (N > 64) m += __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane + 64 < N && gc >= ck_hi));
  auto pick = [&](int lo, int hi, int idx) __attribute__((always_inline)) {
    return idx < 64 ? __builtin_amdgcn_readlane(lo, idx) : __builtin_amdgcn_readlane(hi, idx - 64);
  };
  const int chunk0 = m == 0 ? 0 : pick(ck_lo, ck_hi, m - 1);  // first chunk of segment m
  const int n_seg_chunks = pick(ck_lo, ck_hi, m) - chunk0;
  const int c = gc - chunk0;
  const int own_len = pick(sl_lo, sl_hi, m);
  const int rem_len = a.has_remote ? pick(rl_lo, rl_hi, m) : own_len;
  const int seg_row0 = pick(so_lo, so_hi, m);
  const bool sync = a.is_sync != 0;
  const int rows_end = sync ? max(own_len, rem_len) : own_len;
  const int min_limit = sync ? min(own_len, rem_len) : own_len;
  const int r_lo = c * a.chunk_rows;
  const int r_hi = min(r_lo + a.chunk_rows, rows_end);
  const int nt = (r_hi - r_lo + kKvTile - 1) / kKvTile;
  const int row_elems = Hkv * D;

  const uint16_t* kbase = reinterpret_cast<const uint16_t*>(k_ptr) + ((int64_t)(seg_row0 + r_lo) * Hkv + g) * D;
  const uint16_t* vbase = reinterpret_cast<const uint16_t*>(v_ptr) + ((int64_t)(seg_row0 + r_lo) * Hkv + g) * D;

  TL tile_io;
  tile_io.init(lane, wave, row_elems);

  // this lane's query column -> (participant, head); columns past the end are zero
  // rows: local block, column = head inside the KV group; sync block, column =
  // participant * G + head inside the group.  The loads are written out (like the tile
  // loads) so that the compiler's own wait for them does not drain the tile ring; they
  // are issued before any tile load, so the first tile wait below covers them.
  const int col = cb + l16;
  const bool col_ok = col < a.cols;
  const bool wave_has_cols = cb < a.cols;  // wave-uniform
  const int col_part = col_ok ? (sync ? col / G : m) : 0;
  const int col_head = col_ok ? g * G + (sync ? col % G : col) : 0;
  const int limit = col_ok ? (col_part == m ? own_len : rem_len) : 0;  // visible rows of this segment
  u32x4 qw[KS];  // B operand of S^T: Q[col][32 st + 8 kg .. +8]
  {
    const uint16_t* qrow = reinterpret_cast<const uint16_t*>(q_ptr) + ((int64_t)col_part * Hq + col_head) * D + 8 * kg;
#pragma unroll
    for (int st = 0; st < KS; ++st)
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(qw[st]) : "v"(qrow + 32 * st) : "memory");
  }

  auto issue = [&](int t) __attribute__((always_inline)) {
    const int len = min(kKvTile, r_hi - r_lo - kKvTile * t);
    const uint32_t stage = lds_base + (t % kDecodeStages) * 2 * TILEB;
    // every cache row is read once: the local-block kernel streams them past the caches (19.2
    // against 20.7 us per block-step at 16 x 1152 rows; no gain in the column-split kernel)
    tile_io.template dma<false, !COLSPLIT>(kbase + (int64_t)t * kKvTile * row_elems, stage, len);
    tile_io.template dma<true, !COLSPLIT>(vbase + (int64_t)t * kKvTile * row_elems, stage + TILEB, len);
  };
#pragma unroll
  for (int t = 0; t < kDecodeStages - 1; ++t)
    if (t < nt) issue(t);

  // LDS -> A operand of S^T: lane (row l16 of a 16-row sub-tile, k-group kg) reads chunk
  // 4 st + kg; the sub-tile's first row goes in the address as a multiple of 16 rows,
  // which leaves the swizzle term unchanged
  int k_off[KS];
#pragma unroll
  for (int st = 0; st < KS; ++st) k_off[st] = l16 * ROWB + (((4 * st + kg) ^ (l16 & (CPR - 1))) * 16);
  // LDS -> A operand of O^T: transposing 8-byte reads; lane i = 4 e + c of a 16-lane group
  // supplies the address of V[sub-tile row 4 kg + e][16 dt + 4 c ..] and receives
  // V[sub-tile rows 4 kg + 0..3][16 dt + i]
  int v_off[DT];
  {
    const int vrow = 4 * kg + (l16 >> 2);
    const int fv = TL::v_swizzle(vrow);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) v_off[dt] = vrow * ROWB + (((2 * dt + ((l16 & 3) >> 1)) ^ fv) * 16) + (l16 & 1) * 8;
  }

  f32x4 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = a.scale * kLog2e;

  for (int t = 0; t < nt; ++t) {
    // this wavefront's part of tile t has landed once at most the loads of the tiles
    // issued after it are outstanding (the query loads are older still)
    const int after = min(nt, t + kDecodeStages - 1) - (t + 1);
    if (after >= 2)
      wait_vmcnt<2 * 2 * IPW>();
    else if (after == 1)
      wait_vmcnt<2 * IPW>();
    else
      wait_vmcnt<0>();
    __syncthreads();  // tile t is complete in LDS, and everyone is done with tile t-1
#pragma unroll
    for (int st = 0; st < KS; ++st) asm volatile("" : "+v"(qw[st]));  // the query loads have landed by now
    if (t + kDecodeStages - 1 < nt) issue(t + kDecodeStages - 1);  // into the stage tile t-1 used
    if (COLSPLIT && !wave_has_cols) continue;

    const int kb = (t % kDecodeStages) * 2 * TILEB;
    // ---- S^T: element e of s[rs] = sub-tile row 4 kg + e, query column l16 --------------------
    f32x4 s[RSUB];
#pragma unroll
    for (int rs = 0; rs < RSUB; ++rs) {
      s[rs] = f32x4{0.f, 0.f, 0.f, 0.f};
      const int sub = (COLSPLIT ? 2 * rh + rs : wave) * 16 * ROWB;
#pragma unroll
      for (int st = 0; st < KS; ++st) {
        const bf16x8 kf = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(lds0 + (kb + sub + k_off[st])));
        s[rs] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, __builtin_bit_cast(bf16x8, qw[st]), s[rs], 0, 0, 0);
      }
    }
    if (r_lo + kKvTile * (t + 1) > min_limit) {
#pragma unroll
      for (int rs = 0; rs < RSUB; ++rs) {
        const int row0 = r_lo + kKvTile * t + 16 * (COLSPLIT ? 2 * rh + rs : wave) + 4 * kg;  // cache row of element 0
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (row0 + e >= limit) s[rs][e] = -INFINITY;
      }
    }

    // ---- online softmax of the query column (log2 domain, lazy rescale) -----------------------
    float mx = -INFINITY;
#pragma unroll
    for (int rs = 0; rs < RSUB; ++rs) mx = fmaxf(mx, fmaxf(fmaxf(s[rs][0], s[rs][1]), fmaxf(s[rs][2], s[rs][3])));
    const float m_cand = max_over_kgroups(mx) * sc;
    if (__builtin_amdgcn_ballot_w64(m_cand > m_run + kRescaleThreshold) != 0) {
      const float m_new = fmaxf(m_run, m_cand);
      const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    s16x4 pb[RSUB];
#pragma unroll
    for (int rs = 0; rs < RSUB; ++rs) {
      float p[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) p[e] = __builtin_amdgcn_exp2f(fmaf(s[rs][e], sc, -m_use));
      l_run += (p[0] + p[1]) + (p[2] + p[3]);
      const bf16x4 pv4 = {(bf16_t)p[0], (bf16_t)p[1], (bf16_t)p[2], (bf16_t)p[3]};
      pb[rs] = __builtin_bit_cast(s16x4, pv4);
    }

    // ---- O^T[d][q] += V^T P^T -----------------------------------------------------------------
    if constexpr (COLSPLIT) {
      // both sub-tiles in one 16x16x32 MFMA: k-slot 8 kg + e = row 4 kg + (e mod 4) of sub-tile e / 4
      const int sub = 2 * rh * 16 * ROWB;
      const s16x8 pp = __builtin_shufflevector(pb[0], pb[1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(lds0 + (kb + TILEB + sub + v_off[dt])));
        const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(lds0 + (kb + TILEB + sub + 16 * ROWB + v_off[dt])));
        const s16x8 vv = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
        o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, vv), __builtin_bit_cast(bf16x8, pp),
                                                        o[dt], 0, 0, 0);
      }
    } else {
      // k-slot 4 kg + e of the 16x16x16 MFMA = sub-tile row 4 kg + e
      const int sub = wave * 16 * ROWB;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const s16x4 vf = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(lds0 + (kb + TILEB + sub + v_off[dt])));
        o[dt] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(vf, pb[0], o[dt], 0, 0, 0);
      }
    }
  }

  l_run = sum_over_kgroups(l_run);
  if constexpr (COLSPLIT) {
    // ---- merge the two row halves of a column block: half 1 hands (m, l, O) to half 0 -------
    __syncthreads();  // every wavefront is done with the tile ring
    f32x4* xo = reinterpret_cast<f32x4*>(smem) + (wave & 3) * (DT * 64) + lane;         // [DT][64 lanes]
    float* xml = reinterpret_cast<float*>(smem + 4 * DT * 64 * 16) + (wave & 3) * 128 + lane;  // m, l per lane
    if (rh == 1) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) xo[dt * 64] = o[dt];
      xml[0] = m_run;
      xml[64] = l_run;
    }
    __syncthreads();
    if (rh == 0) {
      const float m1 = xml[0], l1 = xml[64];
      const float mm = fmaxf(m_run, m1);
      const float mu = (mm == -INFINITY) ? 0.f : mm;
      const float f0 = __builtin_amdgcn_exp2f(m_run - mu), f1 = __builtin_amdgcn_exp2f(m1 - mu);
      m_run = mm;
      l_run = l_run * f0 + l1 * f1;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] = o[dt] * f0 + xo[dt * 64] * f1;
    }
    // half 0 owns the merged 16 columns: write the partial straight from registers
    if (rh == 0 && col_ok) {
      const int64_t prow = ((int64_t)g * a.n_chunks + gc) * a.cols + col;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4*>(part_o + prow * D + 16 * dt + 4 * kg) = o[dt];
      if (kg == 0) {
        part_ml[prow * 2] = m_run;
        part_ml[prow * 2 + 1] = l_run;
      }
    }
  } else {
    // ---- merge the 4 wavefronts (each saw a quarter of the rows) ----------------------------
    if (kg == 0) m_s[wave][l16] = m_run;
    __syncthreads();  // also: every wavefront is done with the tile ring
    const float mm = fmaxf(fmaxf(m_s[0][l16], m_s[1][l16]), fmaxf(m_s[2][l16], m_s[3][l16]));
    const float mu = (mm == -INFINITY) ? 0.f : mm;
    const float f = __builtin_amdgcn_exp2f(m_run - mu);
    if (kg == 0) l_s[wave][l16] = l_run * f;
    float* o_s = reinterpret_cast<float*>(smem) + wave * (16 * OPAD);  // one region per wavefront
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) *reinterpret_cast<f32x4*>(o_s + l16 * OPAD + 16 * dt + 4 * kg) = o[dt] * f;
    __syncthreads();
    const int n_cols = min(QCOLS, a.cols - blockIdx.y * QCOLS);
    const int col0 = blockIdx.y * QCOLS;
    const int64_t prow0 = ((int64_t)g * a.n_chunks + gc) * a.cols + col0;
    const float* o_all = reinterpret_cast<const float*>(smem);
    // local block with the combine fused in: query column cl is head g G + cl of participant m
    uint16_t* out_rows = reinterpret_cast<uint16_t*>(out_ptr) + ((int64_t)m * Hq + g * G + col0) * D;
    if (a.fuse_combine && n_seg_chunks == 1) {
      // the segment's only chunk: normalise and write the output rows, no partials
      for (int idx = tid; idx < n_cols * (D / 4); idx += 256) {
        const int cl = idx / (D / 4), d4 = idx % (D / 4);
        const float* src = o_all + cl * OPAD + 4 * d4;
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(src);
        const f32x4 v1 = *reinterpret_cast<const f32x4*>(src + 16 * OPAD);
        const f32x4 v2 = *reinterpret_cast<const f32x4*>(src + 32 * OPAD);
        const f32x4 v3 = *reinterpret_cast<const f32x4*>(src + 48 * OPAD);
        const float den = l_s[0][cl] + l_s[1][cl] + l_s[2][cl] + l_s[3][cl];
        const f32x4 val = ((v0 + v1) + (v2 + v3)) * (den > 0.f ? 1.f / den : 0.f);
        const bf16x4 w = {(bf16_t)val[0], (bf16_t)val[1], (bf16_t)val[2], (bf16_t)val[3]};
        *reinterpret_cast<u32x2*>(out_rows + cl * D + 4 * d4) = __builtin_bit_cast(u32x2, w);
      }
      return;
    }
    if (!a.fuse_combine) {
      for (int idx = tid; idx < n_cols * (D / 4); idx += 256) {
        const int cl = idx / (D / 4), d4 = idx % (D / 4);
        const float* src = o_all + cl * OPAD + 4 * d4;
        const f32x4 v0 = *reinterpret_cast<const f32x4*>(src);
        const f32x4 v1 = *reinterpret_cast<const f32x4*>(src + 16 * OPAD);
        const f32x4 v2 = *reinterpret_cast<const f32x4*>(src + 32 * OPAD);
        const f32x4 v3 = *reinterpret_cast<const f32x4*>(src + 48 * OPAD);
        *reinterpret_cast<f32x4*>(part_o + (prow0 + cl) * D + 4 * d4) = (v0 + v1) + (v2 + v3);
      }
      if (tid < n_cols) {
        part_ml[(prow0 + tid) * 2] = fmaxf(fmaxf(m_s[0][tid], m_s[1][tid]), fmaxf(m_s[2][tid], m_s[3][tid]));
        part_ml[(prow0 + tid) * 2 + 1] = l_s[0][tid] + l_s[1][tid] + l_s[2][tid] + l_s[3][tid];
      }
      return;
    }

    // ---- fused combine: the workgroup that finishes a segment's last chunk merges them ------
    // The partials travel between workgroups inside one launch, so they are written and read
    // with device-scope atomic accesses (coherent at the device whatever caches sit in
    // between) rather than with plain accesses plus cache-wide write-back and invalidate
    // fences, which cost far more than the few KB exchanged here.  A workgroup counts itself
    // in only after all its partial stores have completed (vmcnt = 0 in every wavefront,
    // then the barrier); the workgroup that finds all other chunks counted in merges and
    // leaves the counter at zero for the next launch.
    for (int idx = tid; idx < n_cols * (D / 4); idx += 256) {
      const int cl = idx / (D / 4), d4 = idx % (D / 4);
      const float* src = o_all + cl * OPAD + 4 * d4;
      const f32x4 v0 = *reinterpret_cast<const f32x4*>(src);
      const f32x4 v1 = *reinterpret_cast<const f32x4*>(src + 16 * OPAD);
      const f32x4 v2 = *reinterpret_cast<const f32x4*>(src + 32 * OPAD);
      const f32x4 v3 = *reinterpret_cast<const f32x4*>(src + 48 * OPAD);
      const f32x4 sum = (v0 + v1) + (v2 + v3);
      float* dst = part_o + (prow0 + cl) * D + 4 * d4;
#pragma unroll
      for (int e = 0; e < 4; ++e) __hip_atomic_store(dst + e, sum[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid < n_cols) {
      __hip_atomic_store(part_ml + (prow0 + tid) * 2,
                         fmaxf(fmaxf(m_s[0][tid], m_s[1][tid]), fmaxf(m_s[2][tid], m_s[3][tid])), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(part_ml + (prow0 + tid) * 2 + 1, l_s[0][tid] + l_s[1][tid] + l_s[2][tid] + l_s[3][tid],
                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __shared__ int last_s;
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    wait_vmcnt<0>();
    __atomic_signal_fence(__ATOMIC_SEQ_CST);
    __syncthreads();
    if (tid == 0) {
      int* cnt = counters + g * N + m;  // at most 16 columns: one workgroup per chunk
      const int seen = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      const int last = seen == n_seg_chunks - 1;
      if (last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      last_s = last;
    }
    __syncthreads();
    if (!last_s) return;
    const int64_t crow0 = ((int64_t)g * a.n_chunks + chunk0) * a.cols + col0;  // chunk 0 of the segment, column 0
    const int64_t cstride = a.cols;                                            // partial rows between chunks
    for (int idx = tid; idx < n_cols * (D / 4); idx += 256) {
      const int cl = idx / (D / 4), d4 = idx % (D / 4);
      const float* ml = part_ml + (crow0 + cl) * 2;
      float mm = -INFINITY;
      for (int cc = 0; cc < n_seg_chunks; ++cc)
        mm = fmaxf(mm, __hip_atomic_load(ml + cc * cstride * 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      const float mu = (mm == -INFINITY) ? 0.f : mm;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      float den = 0.f;
      const float* po = part_o + (crow0 + cl) * D + 4 * d4;
      for (int cc = 0; cc < n_seg_chunks; ++cc) {
        const float mc = __hip_atomic_load(ml + cc * cstride * 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float lc = __hip_atomic_load(ml + cc * cstride * 2 + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float w = __builtin_amdgcn_exp2f(mc - mu);
        den = fmaf(lc, w, den);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          acc[e] = fmaf(__hip_atomic_load(po + cc * cstride * D + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT), w, acc[e]);
      }
      const f32x4 val = acc * (den > 0.f ? 1.f / den : 0.f);
      const bf16x4 w4 = {(bf16_t)val[0], (bf16_t)val[1], (bf16_t)val[2], (bf16_t)val[3]};
      *reinterpret_cast<u32x2*>(out_rows + cl * D + 4 * d4) = __builtin_bit_cast(u32x2, w4);
    }
  }
}

// Zeroes the chunk counters of the fused combine (a kernel rather than a memset so that
// callers may capture the calls in a graph).
__global__ void decode_zero_counters_kernel(int32_t* counters, int n, int64_t slice_bytes) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;  // grid y: workspace slice
  if (i < n) reinterpret_cast<int32_t*>(reinterpret_cast<unsigned char*>(counters) + blockIdx.y * slice_bytes)[i] = 0;
}

// Merges the chunk partials of one (participant, query head) and writes the output row:
//   o = sum_c O_c 2^(m_c - m) / sum_c l_c 2^(m_c - m),  m = max_c m_c.
// D/4 x 4 threads: thread (cg, d4) sums 4 head-dim elements over the chunks c = cg (mod 4),
// all its loads in flight at once (the kernel is a chain of memory round trips: (m, l) of
// every chunk, then the partial O rows, then the store); the 4 chunk groups meet in LDS.
template <typename T>
__global__ __launch_bounds__(256) void decode_combine_kernel(DecodeArgs a) {
  constexpr int CG = 4;
  __shared__ float m_s[256];
  __shared__ float w_s[256];
  __shared__ float l_s[256];
  __shared__ f32x4 acc_s[CG][64];
  const int n = blockIdx.x / a.Hq;
  const int h = blockIdx.x % a.Hq;
  const int G = a.Hq / a.Hkv;
  const int g = h / G, hh = h % G;
  const int c0 = a.is_sync ? 0 : a.chunk_cum[n];
  const int c1 = a.is_sync ? a.n_chunks : a.chunk_cum[n + 1];
  const int col = a.is_sync ? n * G + hh : hh;
  const int64_t base = (int64_t)g * a.n_chunks;
  const int tid = threadIdx.x;
  const int D = a.D, D4 = D / 4;
  const int d4 = tid % D4, cg = tid / D4;  // blockDim = D4 * CG
  // block of a fused launch
  const int bz = blockIdx.y;
  unsigned char* out_ptr = reinterpret_cast<unsigned char*>(a.out) + (int64_t)a.block_list[bz] * a.q_block_bytes;
  const float* part_o = reinterpret_cast<const float*>(reinterpret_cast<const unsigned char*>(a.part_o) + bz * a.slice_bytes);
  const float* part_ml = reinterpret_cast<const float*>(reinterpret_cast<const unsigned char*>(a.part_ml) + bz * a.slice_bytes);
  const int64_t cstride = a.cols;          // partial rows between consecutive chunks

  if (c1 - c0 <= 16 * CG) {
    // Few chunks (the usual case): one round trip.  Every thread requests its partial O rows
    // and one chunk's (m, l) before anything is known about the weights.
    const int nb = c1 - c0;
    const float* po = part_o + ((base + c0) * cstride + col) * D + 4 * d4;
    f32x4 part[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int i = cg + CG * u;
      part[u] = i < nb ? *reinterpret_cast<const f32x4*>(po + i * cstride * D) : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    float m_i = -INFINITY, l_i = 0.f;
    if (tid < nb) {
      const f32x2 ml = *reinterpret_cast<const f32x2*>(part_ml + ((base + c0 + tid) * cstride + col) * 2);
      m_i = ml[0];
      l_i = ml[1];
    }
    float mm = wave_max(m_i);
    if ((tid & 63) == 0) m_s[tid >> 6] = mm;
    __syncthreads();
    mm = -INFINITY;
    for (int w = 0; w < (int)((blockDim.x + 63) >> 6); ++w) mm = fmaxf(mm, m_s[w]);
    const float mu = (mm == -INFINITY) ? 0.f : mm;
    if (tid < nb) {
      w_s[tid] = __builtin_amdgcn_exp2f(m_i - mu);
      l_s[tid] = l_i;
    }
    __syncthreads();
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const int i = cg + CG * u;
      if (i < nb) acc += part[u] * w_s[i];
    }
    acc_s[cg][d4] = acc;
    if (tid == 0) {
      float den = 0.f;
      for (int i = 0; i < nb; ++i) den = fmaf(l_s[i], w_s[i], den);
      m_s[8] = den;
    }
    __syncthreads();
    if (cg == 0) {
      const float dn = m_s[8];
      const f32x4 sum = (acc_s[0][d4] + acc_s[1][d4]) + (acc_s[2][d4] + acc_s[3][d4]);
      const f32x4 val = sum * (dn > 0.f ? 1.f / dn : 0.f);
      T* out = reinterpret_cast<T*>(out_ptr) + ((int64_t)n * a.Hq + h) * D + 4 * d4;
      if constexpr (sizeof(T) == 2) {
        const bf16x4 w4 = {(bf16_t)val[0], (bf16_t)val[1], (bf16_t)val[2], (bf16_t)val[3]};
        *reinterpret_cast<u32x2*>(out) = __builtin_bit_cast(u32x2, w4);
      } else {
        *reinterpret_cast<f32x4*>(out) = val;
      }
    }
    return;
  }

  // row maximum over all chunks
  float mm = -INFINITY;
  for (int cc = c0 + tid; cc < c1; cc += blockDim.x) mm = fmaxf(mm, part_ml[((base + cc) * cstride + col) * 2]);
  mm = wave_max(mm);
  if ((tid & 63) == 0) m_s[tid >> 6] = mm;
  __syncthreads();
  mm = -INFINITY;
  for (int w = 0; w < (int)((blockDim.x + 63) >> 6); ++w) mm = fmaxf(mm, m_s[w]);
  const float mu = (mm == -INFINITY) ? 0.f : mm;

  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  float den = 0.f;
  for (int cb = c0; cb < c1; cb += 256) {
    const int nb = min(256, c1 - cb);
    __syncthreads();
    for (int i = tid; i < nb; i += blockDim.x) {
      const float* ml = part_ml + ((base + cb + i) * cstride + col) * 2;
      w_s[i] = __builtin_amdgcn_exp2f(ml[0] - mu);
      l_s[i] = ml[1];
    }
    __syncthreads();
    const float* po = part_o + ((base + cb) * cstride + col) * D + 4 * d4;
#pragma unroll 8
    for (int i = cg; i < nb; i += CG) acc += *reinterpret_cast<const f32x4*>(po + i * cstride * D) * w_s[i];
    if (tid == 0)
      for (int i = 0; i < nb; ++i) den = fmaf(l_s[i], w_s[i], den);
  }
  acc_s[cg][d4] = acc;
  if (tid == 0) m_s[8] = den;
  __syncthreads();
  if (cg == 0) {
    const float dn = m_s[8];
    const f32x4 sum = (acc_s[0][d4] + acc_s[1][d4]) + (acc_s[2][d4] + acc_s[3][d4]);
    const f32x4 val = sum * (dn > 0.f ? 1.f / dn : 0.f);
    T* out = reinterpret_cast<T*>(out_ptr) + ((int64_t)n * a.Hq + h) * D + 4 * d4;
    if constexpr (sizeof(T) == 2) {
      const bf16x4 w4 = {(bf16_t)val[0], (bf16_t)val[1], (bf16_t)val[2], (bf16_t)val[3]};
      *reinterpret_cast<u32x2*>(out) = __builtin_bit_cast(u32x2, w4);
    } else {
      *reinterpret_cast<f32x4*>(out) = val;
    }
  }
}

// General decode kernel (plain ALU, fp32 arithmetic, any head_dim up to 256, fp32 or
// bf16 storage): one wavefront per (participant, query head), no split.
template <typename T>
__device__ inline float ld(const T* p) {
  if constexpr (sizeof(T) == 2)
    return bf16_bits_to_f32(*p);
  else
    return *p;
}

template <typename T>
__global__ __launch_bounds__(64) void decode_rows_kernel(DecodeArgs a) {
  __shared__ float qs[256];
  __shared__ float ps[64];
  const int lane = threadIdx.x;
  const int n = blockIdx.x / a.Hq, h = blockIdx.x % a.Hq;
  const int g = h / (a.Hq / a.Hkv);
  const int D = a.D;
  const T* q = reinterpret_cast<const T*>(a.q) + ((int64_t)n * a.Hq + h) * D;
  const T* kc = reinterpret_cast<const T*>(a.k_cache);
  const T* vc = reinterpret_cast<const T*>(a.v_cache);
  for (int d = lane; d < D; d += 64) qs[d] = ld(q + d);
  __syncthreads();

  float m_run = -INFINITY, l_run = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int m = 0; m < a.N; ++m) {
    int len;
    if (m == n) len = a.seg_lens[m];
    else if (!a.is_sync) len = 0;
    else len = a.has_remote ? a.remote_lens[m] : a.seg_lens[m];
    for (int base = 0; base < len; base += 64) {
      const int r = base + lane;
      float s = -INFINITY;
      if (r < len) {
        const T* krow = kc + ((int64_t)(a.seg_off[m] + r) * a.Hkv + g) * D;
        float dot = 0.f;
        for (int d = 0; d < D; ++d) dot = fmaf(qs[d], ld(krow + d), dot);
        s = a.scale * dot;
      }
      const float m_new = fmaxf(m_run, wave_max(s));
      const float alpha = expf(m_run - m_new);
      const float p = expf(s - m_new);
      ps[lane] = p;
      l_run = l_run * alpha + wave_sum(p);
      m_run = m_new;
#pragma unroll
      for (int dd = 0; dd < 4; ++dd) acc[dd] *= alpha;
      __syncthreads();
      const int cnt = min(64, len - base);
      for (int jj = 0; jj < cnt; ++jj) {
        const float pj = ps[jj];
        const T* vrow = vc + ((int64_t)(a.seg_off[m] + base + jj) * a.Hkv + g) * D;
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
          const int d = lane + 64 * dd;
          if (d < D) acc[dd] = fmaf(pj, ld(vrow + d), acc[dd]);
        }
      }
      __syncthreads();
    }
  }
  const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
  T* out = reinterpret_cast<T*>(a.out) + ((int64_t)n * a.Hq + h) * D;
#pragma unroll
  for (int dd = 0; dd < 4; ++dd) {
    const int d = lane + 64 * dd;
    if (d < D) {
      if constexpr (sizeof(T) == 2)
        out[d] = f32_to_bf16_bits(acc[dd] * inv);
      else
        out[d] = acc[dd] * inv;
    }
  }
}

template <int D, bool COLSPLIT>
hipError_t launch_stream_mode(const DecodeArgs& a, int n_z, hipStream_t s) {
  static std::atomic<uint64_t> attr_done{0};
  hipError_t e0 = set_max_dynamic_lds_once(attr_done, reinterpret_cast<const void*>(&decode_stream_kernel<D, COLSPLIT>),
                                           decode_smem_bytes<D>());
  if (e0 != hipSuccess) return e0;
  const int qcols = COLSPLIT ? 64 : 16;
  dim3 grid((unsigned)(a.n_chunks * a.Hkv), (unsigned)((a.cols + qcols - 1) / qcols), (unsigned)n_z);
  hipLaunchKernelGGL((decode_stream_kernel<D, COLSPLIT>), grid, dim3(COLSPLIT ? 512 : 256), decode_smem_bytes<D>(), s, a);
  return hipGetLastError();
}

template <int D>
hipError_t launch_stream(const DecodeArgs& a, int n_z, hipStream_t s) {
  return a.cols <= 16 ? launch_stream_mode<D, false>(a, n_z, s) : launch_stream_mode<D, true>(a, n_z, s);
}

}  // namespace

// n_z > 1: the blocks a.block_list[0 .. n_z) in one launch (MFMA path only)
hipError_t launch_decode(const DecodeArgs& a, int dtype, int n_z, hipStream_t s) {
  if (a.N == 0 || n_z == 0) return hipSuccess;
  const bool mfma = dtype == FEDATTN_BF16 && (a.D == 64 || a.D == 128);
  if (!mfma) {
    if (n_z != 1) return hipErrorInvalidValue;
    dim3 grid((unsigned)(a.N * a.Hq));
    if (dtype == FEDATTN_F32)
      hipLaunchKernelGGL(decode_rows_kernel<float>, grid, dim3(64), 0, s, a);
    else
      hipLaunchKernelGGL(decode_rows_kernel<uint16_t>, grid, dim3(64), 0, s, a);
    return hipGetLastError();
  }
  if (a.n_chunks > 0) {
    hipError_t e = a.D == 128 ? launch_stream<128>(a, n_z, s) : launch_stream<64>(a, n_z, s);
    if (e != hipSuccess) return e;
  }
  if (a.fuse_combine) return hipSuccess;
  hipLaunchKernelGGL(decode_combine_kernel<uint16_t>, dim3((unsigned)(a.N * a.Hq), (unsigned)n_z), dim3(a.D), 0,
                     s, a);
  return hipGetLastError();
}

hipError_t launch_decode_zero_counters(int32_t* counters, int n, int slices, int64_t slice_bytes, hipStream_t s) {
  hipLaunchKernelGGL(decode_zero_counters_kernel, dim3((unsigned)((n + 255) / 256), (unsigned)slices), dim3(256), 0, s,
                     counters, n, slice_bytes);
  return hipGetLastError();
}

}  // namespace fedattn
