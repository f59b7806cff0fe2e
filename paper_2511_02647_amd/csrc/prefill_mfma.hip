// bf16 prefill attention on the gfx950 matrix cores: varlen, segment-aware,
// flash-style tiling with fp32 online softmax in registers.
//
// One workgroup = 4 wavefronts.  Each wavefront owns 32 query rows of one query
// head; the 4 wavefronts of a workgroup share one KV head (GQA head sharing: with
// a group of 4 query heads they are the 4 heads of the group on the same 32 rows,
// so every wave has the same KV range and nobody idles on the causal diagonal).
// KV tiles of 64 rows are staged through LDS once per workgroup.
//
// Both products run transposed so that the softmax row statistics stay inside a
// lane: S^T = K Q^T puts one query row in one lane (32 of the tile's 64 scores in
// its registers, the other 32 in lane^32), and O^T += V^T P^T consumes P^T straight
// from those registers as the MFMA B operand.  V is transposed on its way into LDS.
//
// Which KV tiles a query tile walks (Phase I / Phase II attention, causal mask of
// Section III-B, sparse KV exchange):
//   local block:  own segment, up to the diagonal;
//   sync block:   the global sequence from token 0 up to the diagonal;
//   sparse sync:  the kept 64-row tiles of the remote participants, then the own
//                 segment up to the diagonal.
// Tiles entirely above the diagonal or in other participants' segments of a local
// block are never visited; only diagonal and ragged tiles apply an element mask.
#include <type_traits>

#include "common.h"

namespace fedattn {

namespace {

constexpr float kLog2e = 1.4426950408889634f;

__device__ inline uint32_t pack_lo(uint32_t a, uint32_t b) {  // (a.lo16, b.lo16)
  return (a & 0xFFFFu) | (b << 16);
}
__device__ inline uint32_t pack_hi(uint32_t a, uint32_t b) {  // (a.hi16, b.hi16)
  return (a >> 16) | (b & 0xFFFF0000u);
}

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(1))) void* global_void_ptr;

constexpr float kRescaleThreshold = 8.f;  // log2 units a row maximum may lag behind before O is rescaled

template <int D>
struct PrefillTiling {
  static constexpr int KSTEPS = D / 16;             // MFMA k-steps of S^T = K Q^T
  static constexpr int DT = D / 32;                 // 32-row tiles of O^T along head_dim
  static constexpr int CPR = D / 8;                 // 16-byte chunks per K/V row
  static constexpr int ROWB = D * 2;                // LDS bytes per K/V row (unpadded; chunks XOR-swizzled)
  static constexpr int TILEB = kKvTile * ROWB;      // one K or V stage
  static constexpr int NINST = TILEB / 1024;        // direct-to-LDS load instructions per tile (1 KB each)
  static constexpr int IPW = NINST / 4;             // per wavefront
};

// One direct-to-LDS load: every lane fetches 16 bytes from base + off (bytes) and the
// wavefront's 1 KB lands at LDS byte address lds_addr (+16 per lane).
__device__ inline void lds_dma_16(const void* base, uint32_t off, uint32_t lds_addr) {
  // the base and the LDS address are the same in every lane; say so to the compiler
  const uint64_t b = (uint64_t)(uintptr_t)base;
  const uint64_t bs = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
                      (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  base = (const void*)(uintptr_t)bs;
  lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr);
  asm volatile(
      "s_mov_b32 m0, %0\n\t"
      "s_nop 0\n\t"
      "global_load_lds_dwordx4 %1, %2"
      :
      : "s"(lds_addr), "v"(off), "s"(base)
      : "memory", "m0");
}

__device__ inline uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(lds_void_ptr)p;
}

// Both halves of a wavefront's 32-lane rows: returns (value of lane%32, value of
// lane%32 + 32) in every lane (v_permlane32_swap: no LDS round trip).
__device__ inline void both_halves(float x, float& lo, float& hi) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const unsigned a = r[0], b = r[1];
  lo = __uint_as_float(a);
  hi = __uint_as_float(b);
}
__device__ inline float max_across_halves(float x) {
  float lo, hi;
  both_halves(x, lo, hi);
  return fmaxf(lo, hi);
}
__device__ inline float sum_across_halves(float x) {
  float lo, hi;
  both_halves(x, lo, hi);
  return lo + hi;
}

// scheduling hints: instruction classes of __builtin_amdgcn_sched_group_barrier
#define SGB_MFMA 0x008
#define SGB_DS_READ 0x100

// Waits until this wavefront's direct-to-LDS loads have landed (vmcnt(0) only).
__device__ inline void wait_lds_dma() { __builtin_amdgcn_s_waitcnt(0x0F70); }

#ifndef FEDATTN_PREFILL_OCC
#define FEDATTN_PREFILL_OCC 2
#endif

template <int D>
__global__ __launch_bounds__(256, FEDATTN_PREFILL_OCC) void prefill_mfma_kernel(PrefillArgs a) {
  using TL = PrefillTiling<D>;
  constexpr int KSTEPS = TL::KSTEPS, DT = TL::DT, CPR = TL::CPR, ROWB = TL::ROWB, TILEB = TL::TILEB;
  constexpr int IPW = TL::IPW;
  // K and V tiles are double-buffered: tile j lives in stage j&1.
  // Layout: K stage 0, K stage 1, V stage 0, V stage 1 (TILEB bytes each).
  __shared__ __attribute__((aligned(1024))) unsigned char kv_lds[4 * TILEB];
  typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;
  const lds_cptr lds0 = (lds_cptr)(lds_void_ptr)kv_lds;
  const uint32_t lds_base = lds_addr_of(kv_lds);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;
  const int hf = lane >> 5;

  const int Hq = a.Hq, Hkv = a.Hkv;
  const int G = Hq / Hkv;
  const int HS = a.heads_per_wg;
  const int HG = G / HS;
  const int BM = a.q_tile_rows;
  const int N = a.seg.n;
  const int T = a.n_q_tiles;

  // workgroup -> (kv head, head subgroup, query tile pair); kv head fastest so that the
  // workgroups of one KV head land on one XCD (8 XCDs, round-robin dispatch) and its
  // K/V stay in that XCD's L2; heaviest work first.
  const int id = blockIdx.x;
  const int g = id % Hkv;
  const int rest = id / Hkv;
  const int hsub = rest % HG;
  const int p = rest / HG;
  const int block = blockIdx.y;

  const bool is_sync = a.sync_override >= 0 ? (a.sync_override != 0)
                                            : sync_block_rule(a.sync_interval, a.block_idx0 + block);
  const bool causal = a.causal != 0;
  const bool sparse = is_sync && a.keep_chunks != nullptr;

  // Causal work grows along the sequence (sync block) or along each segment (local
  // block); a workgroup takes a heavy query tile and then its light mirror image so
  // that all workgroups carry the same load.
  int tile_a = -1, tile_b = -1;  // heavy tile, then its light partner (or none)
  if (!causal) {
    if (p >= T) return;
    tile_a = T - 1 - p;
  } else if (is_sync) {
    if (p >= (T + 1) / 2) return;
    tile_a = T - 1 - p;
    if (p < T - 1 - p) tile_b = p;
  } else {
    if (p >= a.seg.pair_cum[N]) return;
    int n = 0;
    while (p >= a.seg.pair_cum[n + 1]) ++n;
    const int pi = p - a.seg.pair_cum[n];
    const int t0 = a.seg.tile_cum[n], tn = a.seg.tile_cum[n + 1] - t0;
    tile_a = t0 + tn - 1 - pi;
    if (pi < tn - 1 - pi) tile_b = t0 + pi;
  }

  const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + (int64_t)block * a.q_block_stride;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(a.k) + (int64_t)block * a.kv_block_stride + g * D;
  const uint16_t* vp = reinterpret_cast<const uint16_t*>(a.v) + (int64_t)block * a.kv_block_stride + g * D;
  uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + (int64_t)block * a.q_block_stride;
  const float sc = a.scale * kLog2e;
  const int row_elems = Hkv * D;  // elements between consecutive KV rows in HBM

  // ---- per-lane constants of the tile traffic ---------------------------------------
  // HBM -> LDS: one load instruction moves 64 x 16 bytes to 1 KB of consecutive LDS
  // (lane l lands at +16 l).  LDS slot (row, cp) receives chunk cp ^ f(row) of the row:
  // f = row mod CPR for K (conflict-free 16-byte reads down 16 rows), f = 2 (row mod 8)
  // for V (conflict-free 8-byte transposing reads across 4 rows).
  int dma_row[IPW];        // tile row this lane fetches in its wave's i-th instruction
  int dma_kcol[IPW];       // element offset of the K chunk inside the row
  int dma_vcol[IPW];       // element offset of the V chunk inside the row
  uint32_t dma_koff[IPW];  // byte offset from the tile's first row (full tiles)
  uint32_t dma_voff[IPW];
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int sidx = (wave * IPW + i) * 64 + lane;
    const int row = sidx / CPR, cp = sidx % CPR;
    dma_row[i] = row;
    dma_kcol[i] = (cp ^ (row & (CPR - 1))) * 8;
    dma_vcol[i] = (cp ^ ((2 * (row & 7)) & (CPR - 1))) * 8;
    dma_koff[i] = (uint32_t)(row * row_elems + dma_kcol[i]) * 2u;
    dma_voff[i] = (uint32_t)(row * row_elems + dma_vcol[i]) * 2u;
  }
  // LDS -> MFMA A operand of S^T: lane (kv row 32 aa + l32, half hf) reads chunk
  // 2 st + hf of its row; k_off[st] is its swizzled byte offset (aa goes in the
  // instruction's immediate offset).
  int k_off[KSTEPS];
#pragma unroll
  for (int st = 0; st < KSTEPS; ++st) k_off[st] = l32 * ROWB + (((2 * st + hf) ^ (l32 & (CPR - 1))) * 16);
  // LDS -> MFMA A operand of O^T (V^T): transposing 8-byte reads.  In each group of 16
  // lanes, lane i = 4 e + c supplies the address of V[rows + e][d0 + 4 c ..] and
  // receives V[rows + 0..3][d0 + i]; d0 = 32 dt + 16 (group & 1), rows = base + 4 hf.
  int v_off[DT];
  {
    const int i16 = lane & 15, e = i16 >> 2, c = i16 & 3, dsel = (lane >> 4) & 1;
    const int vrow = 4 * hf + e;
    const int fv = (2 * (vrow & 7)) & (CPR - 1);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      v_off[dt] = vrow * ROWB + (((4 * dt + 2 * dsel + (c >> 1)) ^ fv) * 16) + (c & 1) * 8;
  }

  for (int part = 0; part < 2; ++part) {
    const int tile = part == 0 ? tile_a : tile_b;
    if (tile < 0) break;

    int n = 0;
    while (tile >= a.seg.tile_cum[n + 1]) ++n;
    const int seg_lo = a.seg.seg_off[n];
    const int seg_hi = a.seg.seg_off[n + 1];
    const int q0 = seg_lo + (tile - a.seg.tile_cum[n]) * BM;
    const int head = g * G + hsub * HS + (wave % HS);
    const int row0w = q0 + kWaveRows * (wave / HS);
    const int my_row = row0w + l32;
    const int row_ld = min(my_row, seg_hi - 1);
    const int i_last = min(q0 + BM, seg_hi) - 1;

    // KV tile schedule of this query tile: two runs of the kept-tile list, then a
    // dense range.
    int la_n = 0, lb0 = 0, lb_n = 0;
    if (sparse) {
      la_n = a.kept_cum[n];
      if (!causal) {
        lb0 = a.kept_cum[n + 1];
        lb_n = a.kept_cum[N] - lb0;
      }
    }
    const int n_list = la_n + lb_n;
    const int dlo = (is_sync && !sparse) ? 0 : seg_lo;
    const int dhi = causal ? i_last + 1 : ((is_sync && !sparse) ? a.total : seg_hi);
    const int n_dense = (dhi - dlo + kKvTile - 1) / kKvTile;
    const int nt = n_list + n_dense;

    auto tile_desc = [&](int it, int& kv0, int& len, bool& causal_tile) __attribute__((always_inline)) {
      if (it < n_list) {
        const int idx = it < la_n ? it : lb0 + (it - la_n);
        const int2 t = a.kept_tiles[idx];
        kv0 = __builtin_amdgcn_readfirstlane(t.x);
        len = __builtin_amdgcn_readfirstlane(t.y);
        causal_tile = false;
      } else {
        kv0 = dlo + kKvTile * (it - n_list);
        len = min(kKvTile, dhi - kv0);
        causal_tile = causal;
      }
    };

    // HBM -> LDS, no registers in between (the load instruction is written out so that
    // the compiler does not serialise it against unrelated LDS reads; completion is
    // awaited explicitly with wait_lds_dma() before the barrier that publishes the tile).
    // Rows past the tile's valid length re-read its last valid row (they are masked out
    // of the scores).
    auto dma_tile = [&](const uint16_t* src, uint32_t lds_base, const uint32_t (&off)[IPW],
                        const int (&col)[IPW], int kv0, int len) __attribute__((always_inline)) {
      const uint16_t* base = src + (int64_t)kv0 * row_elems;
      if (len == kKvTile) {
#pragma unroll
        for (int i = 0; i < IPW; ++i) lds_dma_16(base, off[i], lds_base + (wave * IPW + i) * 1024);
      } else {
#pragma unroll
        for (int i = 0; i < IPW; ++i) {
          const uint32_t o2 = (uint32_t)(min(dma_row[i], len - 1) * row_elems + col[i]) * 2u;
          lds_dma_16(base, o2, lds_base + (wave * IPW + i) * 1024);
        }
      }
    };

    // Q fragments (B operand of S^T): lane (q row = l32, half hf) holds
    // Q[row][16*step + 8*hf .. +8].
    bf16x8 qf[KSTEPS];
    {
      const uint16_t* qrow = qp + ((int64_t)row_ld * Hq + head) * D + 8 * hf;
#pragma unroll
      for (int st = 0; st < KSTEPS; ++st)
        qf[st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + 16 * st));
    }

    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
    float m_run = -INFINITY;  // row maximum the accumulators refer to, log2 domain
    float l_run = 0.f;        // this lane's share of the row sum

    // S^T[kv][q] = K Q^T from the K stage at LDS byte offset kb; register e of s[aa]
    // holds kv row 32*aa + 8*(e/4) + 4*hf + (e%4) of the tile, query row l32.
    auto compute_s = [&](int kb, f32x16 (&s)[2]) __attribute__((always_inline)) {
#pragma unroll
      for (int e = 0; e < 16; ++e) { s[0][e] = 0.f; s[1][e] = 0.f; }
      bf16x8 kf[KSTEPS][2];
#pragma unroll
      for (int st = 0; st < KSTEPS; ++st) {
        const lds_cptr ptr = lds0 + (k_off[st] + kb);
#pragma unroll
        for (int aa = 0; aa < 2; ++aa)
          kf[st][aa] = __builtin_bit_cast(
              bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(ptr + 32 * aa * ROWB));
      }
#pragma unroll
      for (int st = 0; st < KSTEPS; ++st)
#pragma unroll
        for (int aa = 0; aa < 2; ++aa) s[aa] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[st][aa], qf[st], s[aa], 0, 0, 0);
      // keep the LDS reads kLookS k-steps ahead of the MFMAs that consume them
      constexpr int kLookS = 3;
      __builtin_amdgcn_sched_group_barrier(SGB_DS_READ, 2 * kLookS, 0);
#pragma unroll
      for (int st = 0; st < KSTEPS - kLookS; ++st) {
        __builtin_amdgcn_sched_group_barrier(SGB_MFMA, 2, 0);
        __builtin_amdgcn_sched_group_barrier(SGB_DS_READ, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(SGB_MFMA, 2 * kLookS, 0);
    };
    // O^T[d][q] += V^T P^T from the V stage at LDS byte offset vb; k-step kk covers tile
    // rows 16 kk + {4hf..4hf+3, 8+4hf..8+4hf+3}, the order in which P^T sits in the
    // lane's registers.  k-step major, so that the first MFMAs need only the first
    // quarter of P.
    auto compute_pv = [&](int vb, const bf16x8 (&pb)[4]) __attribute__((always_inline)) {
      bf16x8 vf[4][DT];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const lds_cptr ptr = lds0 + (v_off[dt] + vb) + 16 * kk * ROWB;
          const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)ptr);
          const s16x4 hi =
              __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(ptr + 8 * ROWB));
          vf[kk][dt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
          o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk][dt], pb[kk], o[dt], 0, 0, 0);
      constexpr int kLookV = 4;        // MFMAs of lookahead
      constexpr int NM = 4 * DT;       // MFMAs in this product
      __builtin_amdgcn_sched_group_barrier(SGB_DS_READ, 2 * kLookV, 0);
#pragma unroll
      for (int i = 0; i < NM - kLookV; ++i) {
        __builtin_amdgcn_sched_group_barrier(SGB_MFMA, 1, 0);
        __builtin_amdgcn_sched_group_barrier(SGB_DS_READ, 2, 0);
      }
      __builtin_amdgcn_sched_group_barrier(SGB_MFMA, kLookV, 0);
    };

    // ---- prologue: K and V tile 0 into stage 0 -----------------------------------------
    __syncthreads();  // the previous query tile of this workgroup is done with LDS
    {
      int kv0, len;
      bool ct;
      tile_desc(0, kv0, len, ct);
      dma_tile(kp, lds_base, dma_koff, dma_kcol, kv0, len);
      dma_tile(vp, lds_base + 2 * TILEB, dma_voff, dma_vcol, kv0, len);
    }
    wait_lds_dma();
    __syncthreads();

    // ---- main loop: tile j is computed from stage j&1 while tile j+1 streams into the
    // other stage; the two wavefronts that share a SIMD overlap one's matrix work with
    // the other's softmax ------------------------------------------------------------------
    for (int j = 0; j < nt; ++j) {
      const int st_cur = (j & 1) * TILEB;
      const int st_nxt = TILEB - st_cur;
      int kv0, len;
      bool causal_tile;
      tile_desc(j, kv0, len, causal_tile);
      if (j + 1 < nt) {
        int kv1, len1;
        bool ct1;
        tile_desc(j + 1, kv1, len1, ct1);
        dma_tile(kp, lds_base + st_nxt, dma_koff, dma_kcol, kv1, len1);
        dma_tile(vp, lds_base + 2 * TILEB + st_nxt, dma_voff, dma_vcol, kv1, len1);
      }

      f32x16 s_cur[2];
      compute_s(st_cur, s_cur);

      if (len < kKvTile || (causal_tile && kv0 + kKvTile - 1 > row0w)) {
        // valid kv rows of this tile for this lane's query: [0, lim)
        int lim = len;
        if (causal_tile) lim = min(lim, my_row - kv0 + 1);
        const int limh = lim - 4 * hf;
#pragma unroll
        for (int aa = 0; aa < 2; ++aa)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (32 * aa + 8 * (e >> 2) + (e & 3) >= limh) s_cur[aa][e] = -INFINITY;
      }

      float mx0 = fmaxf(s_cur[0][0], s_cur[1][0]);
      float mx1 = fmaxf(s_cur[0][1], s_cur[1][1]);
#pragma unroll
      for (int e = 2; e < 16; e += 2) {
        mx0 = fmaxf(fmaxf(mx0, s_cur[0][e]), s_cur[1][e]);
        mx1 = fmaxf(fmaxf(mx1, s_cur[0][e + 1]), s_cur[1][e + 1]);
      }
      float mx = fmaxf(mx0, mx1);
      mx = max_across_halves(mx);
      const float m_cand = mx * sc;

      // the accumulators follow the row maximum lazily: rescale only when some row's
      // maximum has grown by more than the threshold (exact: the final division uses
      // the same reference value for numerator and denominator)
      if (__builtin_amdgcn_ballot_w64(m_cand > m_run + kRescaleThreshold) != 0) {
        const float m_new = fmaxf(m_run, m_cand);
        const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);  // exp2(-inf) = 0 at the first tile
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
      }
      const float m_use = (m_run == -INFINITY) ? 0.f : m_run;

      bf16x8 pb[4];
      float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
      for (int aa = 0; aa < 2; ++aa)
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s_cur[aa][e], sc, -m_use));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s_cur[aa][e + 1], sc, -m_use));
          ps0 += p0;
          ps1 += p1;
          pb[aa * 2 + (e >> 3)][e & 7] = (bf16_t)p0;
          pb[aa * 2 + (e >> 3)][(e & 7) + 1] = (bf16_t)p1;
        }
      l_run += ps0 + ps1;

      compute_pv(2 * TILEB + st_cur, pb);

      wait_lds_dma();
      __syncthreads();
    }

    // ---- normalise and write ---------------------------------------------------------
    const float l_tot = sum_across_halves(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (my_row < seg_hi) {
      uint16_t* orow = op + ((int64_t)my_row * Hq + head) * D + 4 * hf;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (bf16_t)(o[dt][4 * vq + e] * inv);
          *reinterpret_cast<u32x2*>(orow + 32 * dt + 8 * vq) = __builtin_bit_cast(u32x2, w);
        }
    }
  }
}

// Compacts the keep flags of a sync block into the list of kept 64-row KV tiles,
// participant after participant, plus the number of kept tiles before each
// participant.  One thread per participant (the lists are short).
__global__ __launch_bounds__(kMaxP) void build_kept_tiles_kernel(PrefillArgs a, int2* kept_tiles,
                                                                 int32_t* kept_cum) {
  __shared__ int cnt[kMaxP + 1];
  const int n = threadIdx.x;
  const int N = a.seg.n;
  int my = 0;
  if (n < N) {
    const int lo = a.seg.seg_off[n], hi = a.seg.seg_off[n + 1];
    const uint8_t* keep = a.keep_chunks + a.seg.chunk_cum[n];
    const int nc = a.seg.chunk_cum[n + 1] - a.seg.chunk_cum[n];
    for (int c = 0; c < nc; ++c) {
      if (!keep[c]) continue;
      const int clen = min(a.chunk_tokens, hi - (lo + c * a.chunk_tokens));
      my += (clen + kKvTile - 1) / kKvTile;
    }
  }
  cnt[n] = my;
  __syncthreads();
  if (n == 0) {
    int run = 0;
    for (int i = 0; i < N; ++i) {
      const int c = cnt[i];
      cnt[i] = run;
      kept_cum[i] = run;
      run += c;
    }
    cnt[N] = run;
    kept_cum[N] = run;
  }
  __syncthreads();
  if (n < N) {
    const int lo = a.seg.seg_off[n], hi = a.seg.seg_off[n + 1];
    const uint8_t* keep = a.keep_chunks + a.seg.chunk_cum[n];
    const int nc = a.seg.chunk_cum[n + 1] - a.seg.chunk_cum[n];
    int w = cnt[n];
    for (int c = 0; c < nc; ++c) {
      if (!keep[c]) continue;
      const int start = lo + c * a.chunk_tokens;
      const int clen = min(a.chunk_tokens, hi - start);
      for (int t = 0; t < clen; t += kKvTile) kept_tiles[w++] = make_int2(start + t, min(kKvTile, clen - t));
    }
  }
}

}  // namespace

hipError_t launch_prefill_mfma(const PrefillArgs& a, int n_blocks, hipStream_t s) {
  if (a.n_q_tiles == 0 || n_blocks == 0) return hipSuccess;
  const int G = a.Hq / a.Hkv;
  // causal: query tiles are paired; a local block pairs inside each segment, which
  // needs at least as many workgroups as the sequence-wide pairing of a sync block
  const int wg_tiles = a.causal ? a.seg.pair_cum[a.seg.n] : a.n_q_tiles;
  dim3 grid((unsigned)(wg_tiles * a.Hkv * (G / a.heads_per_wg)), (unsigned)n_blocks, 1);
  if (a.D == 128)
    hipLaunchKernelGGL(prefill_mfma_kernel<128>, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(prefill_mfma_kernel<64>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_build_kept_tiles(const PrefillArgs& a, int2* kept_tiles, int32_t* kept_cum,
                                   hipStream_t s) {
  hipLaunchKernelGGL(build_kept_tiles_kernel, dim3(1), dim3(kMaxP), 0, s, a, kept_tiles, kept_cum);
  return hipGetLastError();
}

}  // namespace fedattn
