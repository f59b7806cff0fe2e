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
#include <algorithm>
#include <climits>
#include <type_traits>

#include "common.h"
#include "mfma_tile.h"

namespace fedattn {

namespace {

// NG = 1: 4 wavefronts per workgroup (two workgroups share a CU when the grid is large
// enough, and one's matrix work overlaps the other's softmax: inside a wavefront the softmax
// sits between the two products that depend on it, and spreading it under the MFMAs of the
// neighbouring tiles instead measured slower).  NG = 2, for grids that would
// leave one workgroup per CU: 8 wavefronts = two groups of 4 on the same query rows;
// group g takes the KV tiles j with j mod 2 == g through its own LDS stages and the two
// partial results are merged at the end (split-KV inside the workgroup).
// FOLD: the softmax scale (and the change to base 2) is folded into the Q operand and the
// reference value of the online softmax into the starting value of the score accumulation, so
// that a score comes out of the MFMAs ready for the exponential: one vector instruction less per
// score, a quarter of the softmax's (3-4 % of the kernel's time on the large workloads).  Folding
// the scale rounds q * scale to bf16 once more; the host asks for it only when the scale does not
// exceed 1/sqrt(D), where that rounding stays well below the rounding of the weights themselves.
template <int D, int NG, bool FOLD>
__global__ __launch_bounds__(256 * NG, 2) void prefill_mfma_kernel(PrefillArgs a) {
  using TL = KvTile<D, 1>;
  constexpr int KSTEPS = TL::KSTEPS, DT = TL::DT, TILEB = TL::TILEB;
  // Per group: K and V tiles double-buffered; the group's i-th tile lives in stage i&1.
  // Layout per group: K stage 0, K stage 1, V stage 0, V stage 1 (TILEB bytes each).
  extern __shared__ __attribute__((aligned(1024))) unsigned char kv_lds[];
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave_all = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave_all >> 2;   // wavefront group (KV tile parity)
  const int wave = wave_all & 3;   // wavefront inside the group
  const int l32 = lane & 31;
  const int hf = lane >> 5;
  const lds_cptr lds0 = (lds_cptr)(lds_void_ptr)kv_lds + grp * 4 * TILEB;
  const uint32_t lds_base = lds_addr_of(kv_lds) + grp * 4 * TILEB;

  const int Hq = a.Hq, Hkv = a.Hkv;
  const int G = Hq / Hkv;
  const int HS = a.heads_per_wg;
  const int HG = G / HS;
  const int BM = a.q_tile_rows;
  const int N = a.seg.n;
  const int T = a.n_q_tiles;

  // The segment tables sit in the kernel-argument buffer.  Walking them entry by entry costs
  // one scalar-cache miss after another while nothing else is in flight, so every lane
  // fetches the entries of segment `lane` (and `lane + 64`) of all tables in one go and the
  // searches below run on ballots.  Entry 0 of every table is 0.
  struct Tab {
    int lo, hi;  // table[lane + 1], table[lane + 65]; INT_MAX past the last segment
  };
  auto load_tab = [&](const int32_t* t) __attribute__((always_inline)) {
    // the tables have kMaxP + 1 entries whatever N is: fetch first (nothing to wait for), select after
    const int lo = t[lane + 1], hi = t[lane + 65];
    Tab r;
    r.lo = lane < N ? lo : INT_MAX;
    r.hi = lane + 64 < N ? hi : INT_MAX;
    return r;
  };
  // table[idx] for a wave-uniform idx in [0, N]
  auto tab_at = [&](const Tab& t, int idx) __attribute__((always_inline)) {
    if (idx == 0) return 0;
    return idx <= 64 ? __builtin_amdgcn_readlane(t.lo, idx - 1) : __builtin_amdgcn_readlane(t.hi, idx - 65);
  };
  // number of segments s with x >= table[s + 1], i.e. the segment a cumulative index falls in
  auto tab_find = [&](const Tab& t, int x) __attribute__((always_inline)) {
    int n = __builtin_popcountll(__builtin_amdgcn_ballot_w64(x >= t.lo));
    if (N > 64) n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(x >= t.hi));
    return n;
  };
  const Tab seg_tab = load_tab(a.seg.seg_off);
  const Tab tile_tab = load_tab(a.seg.tile_cum);
  const Tab pair_tab = load_tab(a.seg.pair_cum);
  const int order_lo = a.seg_order[lane], order_hi = a.seg_order[lane + 64];

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
  if (a.n_ordered > 0) {
    // small causal launch: one query tile per workgroup, in the order the host laid out
    if (p >= a.n_ordered) return;
    tile_a = a.tile_order[p];
    // the light half waits about a microsecond: its loads then queue behind those of the heavy
    // half, whose workgroups set the length of the launch (the light ones have time to spare)
    if (p >= (a.n_ordered + 1) / 2) __builtin_amdgcn_s_sleep(32);
  } else if (!causal) {
    if (p >= T) return;
    tile_a = T - 1 - p;
  } else if (a.one_tile_heavy_first) {
    // A launch of several rounds of workgroups: equal-sized pairs would all finish together and
    // leave the last round partly empty.  One tile per workgroup instead, dispatched heaviest
    // first, so that the short walks at the end of the list fill the gaps.  Sync block: work
    // grows with the position in the sequence.  Local block: the participants in order of
    // decreasing length, each one's tiles from its last to its first.
    if (p >= T) return;
    if (is_sync) {
      tile_a = T - 1 - p;
    } else {
      const int s = tab_find(pair_tab, p);   // position in the length order
      const int pi = p - tab_at(pair_tab, s);
      const int n = s < 64 ? __builtin_amdgcn_readlane(order_lo, s) : __builtin_amdgcn_readlane(order_hi, s - 64);
      tile_a = tab_at(tile_tab, n + 1) - 1 - pi;
    }
  } else if (is_sync) {
    if (p >= (T + 1) / 2) return;
    tile_a = T - 1 - p;
    if (p < T - 1 - p) tile_b = p;
  } else {
    if (p >= tab_at(pair_tab, N)) return;
    const int n = tab_find(pair_tab, p);
    const int pi = p - tab_at(pair_tab, n);
    const int t0 = tab_at(tile_tab, n), tn = tab_at(tile_tab, n + 1) - t0;
    tile_a = t0 + tn - 1 - pi;
    if (pi < tn - 1 - pi) tile_b = t0 + pi;
  }

  const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + (int64_t)block * a.q_block_stride;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(a.k) + (int64_t)block * a.kv_block_stride + g * D;
  const uint16_t* vp = reinterpret_cast<const uint16_t*>(a.v) + (int64_t)block * a.kv_block_stride + g * D;
  const uint16_t* kp_list = reinterpret_cast<const uint16_t*>(a.k_list) + g * D;  // kept-tile list (one block)
  const uint16_t* vp_list = reinterpret_cast<const uint16_t*>(a.v_list) + g * D;
  uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + (int64_t)block * a.q_block_stride;
  const float sc = a.scale * kLog2e;
  const int row_elems = Hkv * D;  // elements between consecutive KV rows in HBM

  TL tile_io;
  tile_io.init(lane, wave, row_elems);

  // One query tile's walk through its KV tiles (all members wave-uniform): two runs of
  // the kept-tile list, then a dense range [dlo, dhi).
  struct Walk {
    int seg_hi, row0w, la_n, lb0, n_list, dlo, dhi, nt;
  };
  auto make_walk = [&](int tile, Walk& w) __attribute__((always_inline)) {
    const int n = tab_find(tile_tab, tile);
    const int seg_lo = tab_at(seg_tab, n);
    w.seg_hi = tab_at(seg_tab, n + 1);
    const int q0 = seg_lo + (tile - tab_at(tile_tab, n)) * BM;
    w.row0w = q0 + kWaveRows * (wave / HS);
    const int i_last = min(q0 + BM, w.seg_hi) - 1;
    int la_n = 0, lb0 = 0, lb_n = 0;
    if (sparse) {
      la_n = a.kept_cum[n];
      if (!causal) {
        lb0 = a.kept_cum[n + 1];
        lb_n = a.kept_cum[N] - lb0;
      }
    }
    w.la_n = la_n;
    w.lb0 = lb0;
    w.n_list = la_n + lb_n;
    w.dlo = (is_sync && !sparse) ? 0 : seg_lo;
    w.dhi = causal ? i_last + 1 : ((is_sync && !sparse) ? a.total : w.seg_hi);
    w.nt = w.n_list + (w.dhi - w.dlo + kKvTile - 1) / kKvTile;  // >= 1: the tile has a row
  };
  auto tile_desc = [&](const Walk& w, int it, int& kv0, int& len, bool& causal_tile)
                       __attribute__((always_inline)) {
    if (it < w.n_list) {
      const int idx = it < w.la_n ? it : w.lb0 + (it - w.la_n);
      const int2 t = a.kept_tiles[idx];
      kv0 = __builtin_amdgcn_readfirstlane(t.x);
      len = __builtin_amdgcn_readfirstlane(t.y);
      causal_tile = false;
    } else {
      kv0 = w.dlo + kKvTile * (it - w.n_list);
      len = min(kKvTile, w.dhi - kv0);
      causal_tile = causal;
    }
  };
  // K and V tile `it` of walk w into the stage at byte offset st of this group
  auto fetch_tile = [&](const Walk& w, int it, int st) __attribute__((always_inline)) {
    int kv0, len;
    bool ct;
    tile_desc(w, it, kv0, len, ct);
    const bool listed = it < w.n_list;
    tile_io.template dma<false>((listed ? kp_list : kp) + (int64_t)kv0 * row_elems, lds_base + st, len);
    tile_io.template dma<true>((listed ? vp_list : vp) + (int64_t)kv0 * row_elems, lds_base + 2 * TILEB + st, len);
  };
  const int head = g * G + hsub * HS + (wave % HS);
  // Q fragments (B operand of S^T): lane (q row = l32, half hf) holds
  // Q[row][16*step + 8*hf .. +8].
  auto load_q = [&](const Walk& w, bf16x8 (&qf)[KSTEPS]) __attribute__((always_inline)) {
    const int row_ld = min(w.row0w + l32, w.seg_hi - 1);
    const uint16_t* qrow = qp + ((int64_t)row_ld * Hq + head) * D + 8 * hf;
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st)
      qf[st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(qrow + 16 * st));
  };

  // The first walk's Q rows come through LDS instead: loaded as above, an instruction touches
  // 32 rows (32 bytes of each) and a launch of a few thousand tokens spends its first
  // microsecond in the address path.  Here the wavefront moves its 32 x D tile with whole-row
  // direct-to-LDS loads (4 rows of 2 D bytes per instruction) into the half of a K or V stage
  // that the first tile does not use, in the K tile's swizzled layout, and reads the fragments
  // back like K fragments.  Nobody else touches that half before the barrier below.
  constexpr int QINST = kWaveRows * TL::ROWB / 1024;  // load instructions per wavefront
  const int q_lds = (wave >> 1) * 2 * TILEB + TILEB + (wave & 1) * (TILEB / 2);  // byte offset in the group's stages
  auto fetch_q_lds = [&](const Walk& w) __attribute__((always_inline)) {
    const int rbase = min(w.row0w, w.seg_hi - 1);
    const uint16_t* qbase = qp + ((int64_t)rbase * Hq + head) * D;
#pragma unroll
    for (int i = 0; i < QINST; ++i) {
      const int sidx = i * 64 + lane;
      const int row = sidx / TL::CPR, cp = sidx % TL::CPR;
      const int row_ld = min(w.row0w + row, w.seg_hi - 1) - rbase;  // >= 0
      const uint32_t off = (uint32_t)(row_ld * (Hq * D) + ((cp ^ (row & (TL::CPR - 1))) * 8)) * 2u;
      lds_dma_16(qbase, off, lds_base + q_lds + i * 1024);
    }
  };
  auto read_q_lds = [&](bf16x8 (&qf)[KSTEPS]) __attribute__((always_inline)) {
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st)
      qf[st] = __builtin_bit_cast(
          bf16x8, *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(lds0 + (q_lds + tile_io.k_off[st])));
  };

  // The workgroup's walks run as one pipeline: the stage parity carries on from the
  // first walk into the second, whose first tile and Q fragments are fetched while
  // the first walk finishes.
  Walk cur, nxt;
  make_walk(tile_a, cur);
  bf16x8 qf[KSTEPS];
  fetch_q_lds(cur);
  if (grp < cur.nt) fetch_tile(cur, grp, 0);
  nxt = cur;
  const bool two = tile_b >= 0;
  unsigned warm = 0;
  if (two) {
    make_walk(tile_b, nxt);
    // pull the second walk's Q rows into L2 now (one dword per 128-byte line)
    const int row_ld = min(nxt.row0w + l32, nxt.seg_hi - 1);
    warm = *reinterpret_cast<const unsigned*>(qp + ((int64_t)row_ld * Hq + head) * D + (hf * 64) % D);
  }
  // Small problems (all of a KV head's K and V fit in L2 with room to spare): the launch starts
  // with every workgroup asking HBM for its Q rows and first tile at once, and the later tiles
  // of the long walks would each be one more cold miss behind that burst.  Instead the K and V
  // rows of the workgroup's own query rows are requested now, one dword per 128-byte line; all
  // workgroups together cover every row, and the walks then find their tiles in L2.
  unsigned warm_k = 0;
  if (a.warm_kv && grp == 0) {
    constexpr int LPR = TL::ROWB / 128;  // 128-byte lines per K/V row
    const int sub = wave % HS;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i % HS != sub || (i >= 2 && !two)) continue;   // wave-uniform
      const Walk& w = i >= 2 ? nxt : cur;
      const int row = min(w.row0w + lane / LPR, w.seg_hi - 1);
      const uint16_t* base = (i & 1) ? vp : kp;
      warm_k += *reinterpret_cast<const unsigned*>(base + (int64_t)row * row_elems + (lane % LPR) * 64);
    }
  }
  int git = 0;  // iterations this workgroup has run: stage of an iteration = git & 1

  for (int part = 0;; ++part) {
    const bool more = part == 0 && two;
    const int my_row = cur.row0w + l32;
    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
    float m_run = -INFINITY;  // row maximum the accumulators refer to, log2 domain
    float l_run = 0.f;        // this lane's share of the row sum
    f32x16 neg_ref;           // FOLD: minus that reference (0 while there is none) in every element; else zeros
#pragma unroll
    for (int e = 0; e < 16; ++e) neg_ref[e] = 0.f;

    const int n_it = (cur.nt + NG - 1) / NG;  // iterations of the workgroup (uniform: they carry barriers)
    wait_vmcnt<0>();
    if (part == 0) {
      asm volatile("" ::"v"(warm), "v"(warm_k));
      read_q_lds(qf);  // this wavefront's own loads: landed with the wait above; the barrier waits for the reads
    }
    if constexpr (FOLD) {
#pragma unroll
      for (int st = 0; st < KSTEPS; ++st)
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[st][e] = (bf16_t)((float)qf[st][e] * sc);
    }
    __syncthreads();

    // ---- main loop: the group's i-th tile is computed from one stage while its next tile
    // (in the last iteration: the first tile of the next walk) streams into the other ---------
    for (int it = 0; it < n_it; ++it, ++git) {
      const int j = it * NG + grp;
      const int st_cur = (git & 1) * TILEB;
      const int st_nxt = TILEB - st_cur;
      if (it + 1 < n_it) {
        if (j + NG < cur.nt) fetch_tile(cur, j + NG, st_nxt);
      } else if (more && grp < nxt.nt) {
        fetch_tile(nxt, grp, st_nxt);  // last iteration of the first walk: start on the second walk
      }

      if (j < cur.nt) {
        int kv0, len;
        bool causal_tile;
        tile_desc(cur, j, kv0, len, causal_tile);
        f32x16 s_cur[2];
        tile_io.scores(lds0, st_cur, qf, neg_ref, s_cur);

        if (len < kKvTile || (causal_tile && kv0 + kKvTile - 1 > cur.row0w)) {
          // valid kv rows of this tile for this lane's query: [0, lim)
          int lim = len;
          if (causal_tile) lim = min(lim, my_row - kv0 + 1);
          mask_scores(s_cur, lim, hf);
        }

        bf16x8 pb[4];
        if constexpr (FOLD) softmax_step_rel<DT>(s_cur, m_run, l_run, o, neg_ref, pb);
        else softmax_step<DT>(s_cur, sc, m_run, l_run, o, pb);

        tile_io.pv(lds0, 2 * TILEB + st_cur, pb, o);
      }

      wait_vmcnt<0>();
      __syncthreads();
    }

    // This walk's Q fragments are dead: fetch the next walk's behind the epilogue.  With two
    // groups the hand-over barrier comes first (group 1 has nothing else to do after it;
    // group 0 loads once it has taken group 1's partial results over).
    if (NG == 1 && more) load_q(nxt, qf);

    if constexpr (NG == 2) {
      // ---- merge the two groups: group 1 hands (m, l, O) to group 0 through LDS.  The K and
      // V stages of the last iteration are free in both groups (the other stages may be
      // receiving the next walk's first tiles): wave w gets one of these four buffers.
      __shared__ float xml[4 * 128];
      const int st_free = ((git - 1) & 1) * TILEB;
      f32x4* xo = reinterpret_cast<f32x4*>(kv_lds + (wave >> 1) * 4 * TILEB + (wave & 1) * 2 * TILEB + st_free) + lane;
      float* xm = xml + wave * 128 + lane;
      if (grp == 1) {
        xm[0] = m_run;
        xm[64] = l_run;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq)
            xo[(4 * dt + vq) * 64] = f32x4{o[dt][4 * vq], o[dt][4 * vq + 1], o[dt][4 * vq + 2], o[dt][4 * vq + 3]};
      }
      // LDS-only hand-over: wait for the LDS writes, not for the loads in flight for the next walk
      __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
      __builtin_amdgcn_s_barrier();
      if (grp == 1 && more) load_q(nxt, qf);
      if (grp == 0) {
        const float m1 = xm[0], l1 = xm[64];
        const float mm = fmaxf(m_run, m1);
        const float mu = (mm == -INFINITY) ? 0.f : mm;
        const float f0 = __builtin_amdgcn_exp2f(m_run - mu), f1 = __builtin_amdgcn_exp2f(m1 - mu);
        l_run = l_run * f0 + l1 * f1;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int vq = 0; vq < 4; ++vq) {
            const f32x4 x = xo[(4 * dt + vq) * 64];
#pragma unroll
            for (int e = 0; e < 4; ++e) o[dt][4 * vq + e] = o[dt][4 * vq + e] * f0 + x[e] * f1;
          }
        if (more) load_q(nxt, qf);
      }
    }

    // ---- normalise and write: the wave's 32 x D tile goes through a free LDS stage so
    // that every store instruction writes whole rows (a lane owns a row in registers, which
    // written directly would scatter 16-byte pieces over 32 rows per instruction) ----------
    const float l_tot = sum_across_halves(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (grp == 0) {
      constexpr int ROWO = 2 * D, CPR = D / 8, RPI = 64 / CPR;  // row bytes, 16-byte chunks per row, rows per store
      const int st_free = ((git - 1) & 1) * TILEB;
      unsigned char* stage = NG == 2 ? kv_lds + (wave >> 1) * 4 * TILEB + (wave & 1) * 2 * TILEB + st_free
                                     : kv_lds + (wave >> 1) * 2 * TILEB + st_free + (wave & 1) * (TILEB / 2);
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          bf16x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) w[e] = (bf16_t)(o[dt][4 * vq + e] * inv);
          const int c = 4 * dt + vq;
          *reinterpret_cast<u32x2*>(stage + l32 * ROWO + ((c ^ (l32 & (CPR - 1))) << 4) + 8 * hf) =
              __builtin_bit_cast(u32x2, w);
        }
      const int c = lane % CPR;
#pragma unroll
      for (int kk = 0; kk < kWaveRows / RPI; ++kk) {
        const int r = kk * RPI + lane / CPR;
        const u32x4 w = *reinterpret_cast<const u32x4*>(stage + r * ROWO + ((c ^ (r & (CPR - 1))) << 4));
        if (cur.row0w + r < cur.seg_hi)
          // streaming store: the rows are not read again in this launch, and written through
          // now they are not left for the write-back at the end of the kernel
          __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(op + ((int64_t)(cur.row0w + r) * Hq + head) * D + 8 * c));
      }
    }
    if (!more) break;
    cur = nxt;
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

// ---- keep-lists finer than a tile: the kept rows of every participant are packed ------------
// A sync block under sparse KV exchange sees, of a remote participant, only the rows the
// keep-list flags.  When a flag covers whole 64-row tiles the attention kernel visits the kept
// tiles where they are; for finer lists (down to single tokens) three small kernels first
// gather each participant's kept rows into the front of its own segment of a packed K, V copy,
// so that the attention kernel still walks dense tiles.  Among remote rows only membership
// matters (a remote participant lies entirely before or entirely after the query in the
// global order), so packing loses nothing.

// Workgroup m scans participant m's flags: src_index[lo + p] = global row of its p-th kept
// row (-1 past the last), kept_rows[m] = their number.
__global__ __launch_bounds__(256) void scan_kept_rows_kernel(PrefillArgs a, int32_t* kept_rows, int32_t* src_index) {
  __shared__ int wave_cnt[4];
  const int m = blockIdx.x;
  const int lo = a.seg.seg_off[m], hi = a.seg.seg_off[m + 1];
  const uint8_t* keep = a.keep_chunks + a.seg.chunk_cum[m];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int carry = 0;
  for (int base = lo; base < hi; base += 256) {
    const int t = base + tid;
    const bool flag = t < hi && keep[(t - lo) / a.chunk_tokens] != 0;
    const unsigned long long bal = __builtin_amdgcn_ballot_w64(flag);
    const int before = __builtin_popcountll(bal & ((1ull << lane) - 1ull));
    __syncthreads();  // wave_cnt of the previous round has been read
    if (lane == 0) wave_cnt[wave] = __builtin_popcountll(bal);
    __syncthreads();
    int pos = carry + before;
    for (int w = 0; w < wave; ++w) pos += wave_cnt[w];
    if (flag) src_index[lo + pos] = t;
    carry += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
  }
  for (int p = lo + carry + tid; p < hi; p += 256) src_index[p] = -1;
  if (tid == 0) kept_rows[m] = carry;
}

// The packed rows of participant m occupy [seg_off[m], seg_off[m] + kept_rows[m]): the list
// of their 64-row tiles (the last one ragged) and the tile count before each participant.
__global__ __launch_bounds__(kMaxP) void build_packed_tiles_kernel(PrefillArgs a, const int32_t* kept_rows,
                                                                   int2* kept_tiles, int32_t* kept_cum) {
  __shared__ int cnt[kMaxP + 1];
  const int n = threadIdx.x;
  const int N = a.seg.n;
  const int kc = n < N ? kept_rows[n] : 0;
  cnt[n] = (kc + kKvTile - 1) / kKvTile;
  __syncthreads();
  if (n == 0) {
    int run = 0;
    for (int i = 0; i < N; ++i) {
      const int c = cnt[i];
      cnt[i] = run;
      kept_cum[i] = run;
      run += c;
    }
    kept_cum[N] = run;
  }
  __syncthreads();
  if (n < N) {
    const int lo = a.seg.seg_off[n];
    int w = cnt[n];
    for (int t = 0; t < kc; t += kKvTile) kept_tiles[w++] = make_int2(lo + t, min(kKvTile, kc - t));
  }
}

// Packed row p of K and V = row src_index[p] of the block's K and V (16 bytes per thread).
__global__ __launch_bounds__(256) void gather_kept_rows_kernel(PrefillArgs a, const int32_t* src_index,
                                                               uint4* k_packed, uint4* v_packed) {
  const int row_vecs = a.Hkv * a.D / 8;  // 16-byte pieces per bf16 row
  const int rows_per_wg = max(1, 256 / row_vecs);
  const uint4* src = reinterpret_cast<const uint4*>(blockIdx.y == 0 ? a.k : a.v);
  uint4* dst = blockIdx.y == 0 ? k_packed : v_packed;
  for (int i = threadIdx.x; i < rows_per_wg * row_vecs; i += 256) {
    const int p = blockIdx.x * rows_per_wg + i / row_vecs;
    if (p >= a.total) break;
    const int from = src_index[p];
    if (from >= 0) dst[(int64_t)p * row_vecs + i % row_vecs] = src[(int64_t)from * row_vecs + i % row_vecs];
  }
}

}  // namespace

hipError_t launch_pack_kept_rows(const PrefillArgs& a, int32_t* kept_rows, int32_t* src_index, void* k_packed,
                                 void* v_packed, int2* kept_tiles, int32_t* kept_cum, hipStream_t s) {
  hipLaunchKernelGGL(scan_kept_rows_kernel, dim3((unsigned)a.seg.n), dim3(256), 0, s, a, kept_rows, src_index);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(build_packed_tiles_kernel, dim3(1), dim3(kMaxP), 0, s, a, kept_rows, kept_tiles, kept_cum);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int row_vecs = a.Hkv * a.D / 8;
  const int rows_per_wg = row_vecs >= 256 ? 1 : 256 / row_vecs;
  hipLaunchKernelGGL(gather_kept_rows_kernel, dim3((unsigned)((a.total + rows_per_wg - 1) / rows_per_wg), 2), dim3(256),
                     0, s, a, src_index, reinterpret_cast<uint4*>(k_packed), reinterpret_cast<uint4*>(v_packed));
  return hipGetLastError();
}

template <int D, int NG, bool FOLD>
hipError_t launch_prefill_mfma_t(const PrefillArgs& a, dim3 grid, hipStream_t s) {
  constexpr int smem = NG * 4 * KvTile<D, 1>::TILEB;
  static std::atomic<uint64_t> attr_done{0};
  hipError_t e0 = set_max_dynamic_lds_once(attr_done, reinterpret_cast<const void*>(&prefill_mfma_kernel<D, NG, FOLD>), smem);
  if (e0 != hipSuccess) return e0;
  hipLaunchKernelGGL((prefill_mfma_kernel<D, NG, FOLD>), grid, dim3(256 * NG), smem, s, a);
  return hipGetLastError();
}

hipError_t launch_prefill_mfma(const PrefillArgs& a_in, int n_blocks, hipStream_t s) {
  if (a_in.n_q_tiles == 0 || n_blocks == 0) return hipSuccess;
  PrefillArgs a = a_in;
  a.n_ordered = 0;
  // one block whose K and V of a KV head are at most 2 MB: the workgroups pull them into L2 up front
  a.warm_kv = (n_blocks == 1 && a.keep_chunks == nullptr && (int64_t)a.total * a.D * 4 <= (2 << 20)) ? 1 : 0;
  const int G = a.Hq / a.Hkv;
  const int per_tile = a.Hkv * (G / a.heads_per_wg);  // workgroups per query tile (or pair)
  // causal: query tiles are paired; a local block pairs inside each segment, which
  // needs at least as many workgroups as the sequence-wide pairing of a sync block
  int wg_tiles = a.causal ? a.seg.pair_cum[a.seg.n] : a.n_q_tiles;
  dim3 grid((unsigned)(wg_tiles * per_tile), (unsigned)n_blocks, 1);
  // Fewer than two 4-wave workgroups per CU: 8-wave workgroups that split the KV tiles of a
  // query tile between two groups keep two wavefronts on every SIMD, at the price of a merge
  // through LDS per query tile and a heavier start.  That pays from about 16 KV tiles per
  // workgroup on (measured at 2048 tokens: 1.06 vs 1.35 us per tile, 14.0 vs 9.6 us fixed).
  bool wide = (int64_t)grid.x * grid.y < 2 * (int64_t)a.n_cus;
  if (wide && n_blocks == 1) {
    const bool is_sync = a.sync_override >= 0 ? a.sync_override != 0 : sync_block_rule(a.sync_interval, a.block_idx0);
    const int N = a.seg.n;
    int64_t kv_tiles = 0;  // KV tiles walked by all workgroups of one (KV head, head subgroup)
    for (int n = 0; n < N; ++n) {
      const int64_t len = a.seg.seg_off[n + 1] - a.seg.seg_off[n];
      const int64_t q_tiles = a.seg.tile_cum[n + 1] - a.seg.tile_cum[n];
      const int64_t span = is_sync ? (a.causal ? a.seg.seg_off[n] + len : (int64_t)a.total) : len;  // keys a late row sees
      const int64_t first = is_sync && a.causal ? a.seg.seg_off[n] : 0;
      // causal: a query tile sees the keys up to its own rows, on average half of its segment's span
      const int64_t mean_keys = a.causal ? first + (span - first + 1) / 2 : span;
      kv_tiles += q_tiles * ((mean_keys + kKvTile - 1) / kKvTile + (a.causal ? 1 : 0));
    }
    wide = kv_tiles >= 16 * (int64_t)wg_tiles;
    // Not enough tiles per workgroup for the split, and every query tile can have a workgroup of
    // its own with all of them resident at once (two per CU): drop the pairing.  Two unrelated
    // 4-wave workgroups on a CU overlap each other's matrix and vector phases, which one
    // workgroup walking a pair cannot do with itself.  Order: heavy half first, heaviest first;
    // then the light half, lightest first, so that the workgroups that come to share a CU
    // (index p and p + half, dispatched in order) carry about the same load together.
    if (!wide && a.causal && a.n_q_tiles <= kMaxOrderedTiles && (int64_t)a.n_q_tiles * per_tile <= 2 * (int64_t)a.n_cus) {
      struct Item { int tile, work; };
      Item items[kMaxOrderedTiles];
      int cnt = 0;
      for (int n = 0; n < N; ++n) {
        const int lo = a.seg.seg_off[n], hi = a.seg.seg_off[n + 1];
        for (int t = a.seg.tile_cum[n]; t < a.seg.tile_cum[n + 1]; ++t) {
          const int last = min(lo + (t - a.seg.tile_cum[n] + 1) * a.q_tile_rows, hi);  // one past the tile's last row
          items[cnt++] = Item{t, (last - (is_sync ? 0 : lo) + kKvTile - 1) / kKvTile};
        }
      }
      std::stable_sort(items, items + cnt, [](const Item& x, const Item& y) { return x.work > y.work; });
      const int half = (cnt + 1) / 2;
      for (int i = 0; i < half; ++i) a.tile_order[i] = (uint16_t)items[i].tile;
      for (int i = half; i < cnt; ++i) a.tile_order[i] = (uint16_t)items[cnt - 1 - (i - half)].tile;
      a.n_ordered = cnt;
      wg_tiles = cnt;
      grid.x = (unsigned)(wg_tiles * per_tile);
    }
  }
  // More than one round of 4-wave workgroups (two per CU): one query tile per workgroup, heaviest first.
  if (!wide && n_blocks == 1 && a.causal && a.n_ordered == 0 && (int64_t)grid.x > 2 * (int64_t)a.n_cus) {
    const bool is_sync = a.sync_override >= 0 ? a.sync_override != 0 : sync_block_rule(a.sync_interval, a.block_idx0);
    a.one_tile_heavy_first = 1;
    if (!is_sync) {
      const int N = a.seg.n;
      int order[kMaxP];
      for (int n = 0; n < N; ++n) order[n] = n;
      std::stable_sort(order, order + N, [&](int x, int y) {
        return a.seg.tile_cum[x + 1] - a.seg.tile_cum[x] > a.seg.tile_cum[y + 1] - a.seg.tile_cum[y];
      });
      int run = 0;
      for (int i = 0; i < N; ++i) {
        a.seg_order[i] = (uint8_t)order[i];
        a.seg.pair_cum[i] = run;
        run += a.seg.tile_cum[order[i] + 1] - a.seg.tile_cum[order[i]];
      }
      a.seg.pair_cum[N] = run;
    }
    grid.x = (unsigned)(a.n_q_tiles * per_tile);
  }
  // scale folded into Q only up to the usual 1/sqrt(D): its rounding error grows with the scale
  const bool fold = (double)a.scale * (double)a.scale * a.D <= 1.0 + 1e-6;
  if (a.D == 128) {
    if (fold) return wide ? launch_prefill_mfma_t<128, 2, true>(a, grid, s) : launch_prefill_mfma_t<128, 1, true>(a, grid, s);
    return wide ? launch_prefill_mfma_t<128, 2, false>(a, grid, s) : launch_prefill_mfma_t<128, 1, false>(a, grid, s);
  }
  if (fold) return wide ? launch_prefill_mfma_t<64, 2, true>(a, grid, s) : launch_prefill_mfma_t<64, 1, true>(a, grid, s);
  return wide ? launch_prefill_mfma_t<64, 2, false>(a, grid, s) : launch_prefill_mfma_t<64, 1, false>(a, grid, s);
}

hipError_t launch_build_kept_tiles(const PrefillArgs& a, int2* kept_tiles, int32_t* kept_cum,
                                   hipStream_t s) {
  hipLaunchKernelGGL(build_kept_tiles_kernel, dim3(1), dim3(kMaxP), 0, s, a, kept_tiles, kept_cum);
  return hipGetLastError();
}

}  // namespace fedattn
