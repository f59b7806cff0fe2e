// Building blocks shared by the bf16 MFMA attention kernels (prefill and decode) on
// gfx950: direct HBM -> LDS tile loads, the swizzled LDS tile layout with its
// conflict-free operand reads, the two transposed products on
// v_mfma_f32_32x32x16_bf16, and one online-softmax step in registers.
//
// Tile = 64 KV rows x D.  Products run transposed: S^T[kv][q] = K Q^T and
// O^T[d][q] += V^T P^T, so a query row lives in lane (q mod 32) and its partner
// lane + 32: lane (l32, hf) holds, in register e of s[aa], the score of tile row
// 32 aa + 8 (e/4) + 4 hf + (e%4), and P^T is consumed as the B operand of the
// second product straight from those registers.
#pragma once

#include "common.h"

namespace fedattn {

typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_void_ptr;
typedef const __attribute__((address_space(3))) unsigned char* lds_cptr;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kRescaleThreshold = 8.f;  // log2 units a row maximum may lag behind before O is rescaled

// scheduling hints: instruction classes of __builtin_amdgcn_sched_group_barrier
#define FEDATTN_SGB_MFMA 0x008
#define FEDATTN_SGB_DS_READ 0x100



// One direct-to-LDS load: every lane fetches 16 bytes from base + off (bytes) and the
// wavefront's 1 KB lands at LDS byte address lds_addr (+16 per lane).  base and
// lds_addr must be wave-uniform.  The instruction is written out so that the compiler
// does not serialise it against unrelated LDS reads; completion is awaited explicitly
// (vmcnt) before the barrier that publishes the tile.
// STREAM: nontemporal hint, for rows that are read once (they then pass the caches without
// displacing anything).
template <bool STREAM = false>
__device__ inline void lds_dma_16(const void* base, uint32_t off, uint32_t lds_addr) {
  if constexpr (STREAM)
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2 nt"
        :
        : "s"(lds_addr), "v"(off), "s"(base)
        : "memory", "m0");
  else
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2"
        :
        : "s"(lds_addr), "v"(off), "s"(base)
        : "memory", "m0");
}

__device__ inline uint32_t lds_addr_of(const void* p) { return (uint32_t)(uintptr_t)(lds_void_ptr)p; }

// Waits until at most `n` of this wavefront's loads are outstanding (vmcnt only).
template <int N>
__device__ inline void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
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

// VSWZ selects the chunk swizzle of V tiles: the transposing reads of the 32x32x16
// product touch 4 rows x 4 chunks per 32 lanes (VSWZ = 1: f = 4 (row mod 4)), those of the
// 16x16x16 product 8 rows x 2 chunks (VSWZ = 0: f = 2 (row mod 8)).
// NW = wavefronts that load a tile together (4, or 8 for 8-wave workgroups sharing one tile).
template <int D, int VSWZ, int NW = 4>
struct KvTile {
  static constexpr int KSTEPS = D / 16;         // MFMA k-steps of S^T = K Q^T
  static constexpr int DT = D / 32;             // 32-row tiles of O^T along head_dim
  static constexpr int CPR = D / 8;             // 16-byte chunks per K/V row
  static constexpr int ROWB = D * 2;            // LDS bytes per K/V row (unpadded; chunks XOR-swizzled)
  static constexpr int TILEB = kKvTile * ROWB;  // one K or V stage
  static constexpr int NINST = TILEB / 1024;    // direct-to-LDS load instructions per tile (1 KB each)
  static constexpr int IPW = NINST / NW;        // per wavefront
  static_assert(NINST % NW == 0, "tile loads must divide evenly among the wavefronts");

  // HBM -> LDS: one load instruction moves 64 x 16 bytes to 1 KB of consecutive LDS
  // (lane l lands at +16 l).  LDS slot (row, cp) receives chunk cp ^ f(row) of the row:
  // f = row mod CPR for K (conflict-free 16-byte reads down 16 rows), v_swizzle(row) for V
  // (conflict-free 8-byte transposing reads).
  static __device__ __attribute__((always_inline)) int v_swizzle(int row) {
    if (VSWZ == 0) return (2 * (row & 7)) & (CPR - 1);
    return CPR >= 16 ? 4 * (row & 3) : 4 * ((row >> 1) & 1);
  }
  uint32_t dma_koff[IPW];  // byte offset from the tile's first row of what this lane fetches in its
  uint32_t dma_voff[IPW];  // wave's i-th instruction (full tiles; ragged tiles work theirs out on the spot)
  int lane;
  // LDS -> MFMA A operand of S^T: lane (kv row 32 aa + l32, half hf) reads chunk
  // 2 st + hf of its row; k_off[st] is its swizzled byte offset (aa goes in the
  // instruction's immediate offset).
  int k_off[KSTEPS];
  // LDS -> MFMA A operand of O^T (V^T): transposing 8-byte reads.  In each group of 16
  // lanes, lane i = 4 e + c supplies the address of V[rows + e][d0 + 4 c ..] and
  // receives V[rows + 0..3][d0 + i]; d0 = 32 dt + 16 (group & 1), rows = base + 4 hf.
  int v_off[DT];
  int wave;
  int row_elems;           // elements between consecutive KV rows in HBM

  // tile row and element offset of the chunk inside the row that this lane fetches in its wave's i-th instruction
  __device__ __attribute__((always_inline)) void dma_slot(int i, bool is_v, int& row, int& col) const {
    const int sidx = (wave * IPW + i) * 64 + lane;
    const int cp = sidx % CPR;
    row = sidx / CPR;
    col = (cp ^ (is_v ? v_swizzle(row) : (row & (CPR - 1)))) * 8;
  }

  __device__ __attribute__((always_inline)) void init(int lane_, int wave_, int row_elems_) {
    const int lane = lane_;
    this->lane = lane_;
    wave = wave_;
    row_elems = row_elems_;
    const int l32 = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      int row, kcol, vcol;
      dma_slot(i, false, row, kcol);
      dma_slot(i, true, row, vcol);
      dma_koff[i] = (uint32_t)(row * row_elems + kcol) * 2u;
      dma_voff[i] = (uint32_t)(row * row_elems + vcol) * 2u;
    }
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) k_off[st] = l32 * ROWB + (((2 * st + hf) ^ (l32 & (CPR - 1))) * 16);
    const int i16 = lane & 15, e = i16 >> 2, c = i16 & 3, dsel = (lane >> 4) & 1;
    const int vrow = 4 * hf + e;
    const int fv = v_swizzle(vrow);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
      v_off[dt] = vrow * ROWB + (((4 * dt + 2 * dsel + (c >> 1)) ^ fv) * 16) + (c & 1) * 8;
  }

  // This wavefront's share of one tile: `tile_base` points at the tile's first row
  // (wave-uniform), `lds_stage` is the LDS byte address of the stage.  Rows past the
  // tile's valid length re-read its last valid row (they are masked out of the scores).
  template <bool IS_V, bool STREAM = false>
  __device__ __attribute__((always_inline)) void dma(const uint16_t* tile_base, uint32_t lds_stage, int len) const {
    if (len == kKvTile) {
#pragma unroll
      for (int i = 0; i < IPW; ++i)
        lds_dma_16<STREAM>(tile_base, IS_V ? dma_voff[i] : dma_koff[i], lds_stage + (wave * IPW + i) * 1024);
    } else {
#pragma unroll
      for (int i = 0; i < IPW; ++i) {
        int row, col;
        dma_slot(i, IS_V, row, col);
        const uint32_t o2 = (uint32_t)(min(row, len - 1) * row_elems + col) * 2u;
        lds_dma_16<STREAM>(tile_base, o2, lds_stage + (wave * IPW + i) * 1024);
      }
    }
  }

  // S^T[kv][q] = K Q^T from the K stage at LDS byte offset kb.  LDS reads run 2 k-steps
  // ahead of the MFMAs that consume them (1 to 4 measure the same; 2 leaves the registers for `init`).
  // `init` is what the accumulation starts from: zeros, or minus the reference value of the
  // softmax in every element (the scores then come out relative to it at no cost).
  __device__ __attribute__((always_inline)) void scores(lds_cptr lds0, int kb, const bf16x8 (&qf)[KSTEPS],
                                                        const f32x16& init, f32x16 (&s)[2]) const {
    s[0] = init;
    s[1] = init;
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
    constexpr int kLook = KSTEPS > 2 ? 2 : KSTEPS - 1;
    __builtin_amdgcn_sched_group_barrier(FEDATTN_SGB_DS_READ, 2 * kLook, 0);
#pragma unroll
    for (int st = 0; st < KSTEPS - kLook; ++st) {
      __builtin_amdgcn_sched_group_barrier(FEDATTN_SGB_MFMA, 2, 0);
      __builtin_amdgcn_sched_group_barrier(FEDATTN_SGB_DS_READ, 2, 0);
    }
#pragma unroll
    for (int st = 0; st < kLook; ++st) {
      __builtin_amdgcn_sched_group_barrier(FEDATTN_SGB_MFMA, 2, 0);
    }
  }

  // O^T[d][q] += V^T P^T from the V stage at LDS byte offset vb; k-step kk covers tile
  // rows 16 kk + {4hf..4hf+3, 8+4hf..8+4hf+3}, the order in which P^T sits in the
  // lane's registers.  k-step major, so that the first MFMAs need only the first
  // quarter of P.
  __device__ __attribute__((always_inline)) void pv(lds_cptr lds0, int vb, const bf16x8 (&pb)[4],
                                                    f32x16 (&o)[DT]) const {
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
      for (int dt = 0; dt < DT; ++dt) o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kk][dt], pb[kk], o[dt], 0, 0, 0);
    constexpr int kLook = 4;    // MFMAs of lookahead
    constexpr int NM = 4 * DT;  // MFMAs in this product
    __builtin_amdgcn_sched_group_barrier(FEDATTN_SGB_DS_READ, 2 * kLook, 0);
#pragma unroll
    for (int i = 0; i < NM - kLook; ++i) {
      __builtin_amdgcn_sched_group_barrier(FEDATTN_SGB_MFMA, 1, 0);
      __builtin_amdgcn_sched_group_barrier(FEDATTN_SGB_DS_READ, 2, 0);
    }
    __builtin_amdgcn_sched_group_barrier(FEDATTN_SGB_MFMA, kLook, 0);
  }
};

// Masks the tile rows a lane's query may not see: rows [lim, 64) of the tile.
__device__ __attribute__((always_inline)) inline void mask_scores(f32x16 (&s)[2], int lim, int hf) {
  const int limh = lim - 4 * hf;
#pragma unroll
  for (int aa = 0; aa < 2; ++aa)
#pragma unroll
    for (int e = 0; e < 16; ++e)
      if (32 * aa + 8 * (e >> 2) + (e & 3) >= limh) s[aa][e] = -INFINITY;
}

// Online softmax in the log2 domain on the scores of one tile, in two parts so that
// independent matrix work can be issued between them.
// Part 1: row maxima; updates the running maximum m_run lazily (the accumulators are
// rescaled only when some row's maximum has grown by more than the threshold; exact,
// because numerator and denominator of the final division refer to the same value).
// Returns the reference value the exponentials of this tile use.
template <int DT>
__device__ __attribute__((always_inline)) inline float softmax_max(const f32x16 (&s)[2], float sc, float& m_run,
                                                                   float& l_run, f32x16 (&o)[DT]) {
  float mx0 = fmaxf(s[0][0], s[1][0]);
  float mx1 = fmaxf(s[0][1], s[1][1]);
#pragma unroll
  for (int e = 2; e < 16; e += 2) {
    mx0 = fmaxf(fmaxf(mx0, s[0][e]), s[1][e]);
    mx1 = fmaxf(fmaxf(mx1, s[0][e + 1]), s[1][e + 1]);
  }
  const float m_cand = max_across_halves(fmaxf(mx0, mx1)) * sc;
  if (__builtin_amdgcn_ballot_w64(m_cand > m_run + kRescaleThreshold) != 0) {
    const float m_new = fmaxf(m_run, m_cand);
    const float m_ref = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_ref);  // exp2(-inf) = 0 at the first tile
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
  }
  return (m_run == -INFINITY) ? 0.f : m_run;
}

// Part 2: exponentials; adds this lane's share of the row sum to l_run and leaves P^T
// in bf16 in pb.  The row sum is taken over the bf16 weights, the ones the second product
// uses (numerator and denominator of the softmax then carry the same rounding), two at a
// time with v_dot2c_f32_bf16 against (1, 1): half the additions of a sum over fp32 weights.
__device__ __attribute__((always_inline)) inline void softmax_exp(const f32x16 (&s)[2], float sc, float m_use,
                                                                   float& l_run, bf16x8 (&pb)[4]) {
  const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
  float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
  for (int aa = 0; aa < 2; ++aa)
#pragma unroll
    for (int e = 0; e < 16; e += 4) {
      const float p0 = __builtin_amdgcn_exp2f(fmaf(s[aa][e], sc, -m_use));
      const float p1 = __builtin_amdgcn_exp2f(fmaf(s[aa][e + 1], sc, -m_use));
      const float p2 = __builtin_amdgcn_exp2f(fmaf(s[aa][e + 2], sc, -m_use));
      const float p3 = __builtin_amdgcn_exp2f(fmaf(s[aa][e + 3], sc, -m_use));
      const bf16x2 q0 = {(bf16_t)p0, (bf16_t)p1};
      const bf16x2 q1 = {(bf16_t)p2, (bf16_t)p3};
      ps0 = __builtin_amdgcn_fdot2_f32_bf16(q0, ones, ps0, false);
      ps1 = __builtin_amdgcn_fdot2_f32_bf16(q1, ones, ps1, false);
      pb[aa * 2 + (e >> 3)][e & 7] = q0[0];
      pb[aa * 2 + (e >> 3)][(e & 7) + 1] = q0[1];
      pb[aa * 2 + (e >> 3)][(e & 7) + 2] = q1[0];
      pb[aa * 2 + (e >> 3)][(e & 7) + 3] = q1[1];
    }
  l_run += ps0 + ps1;
}

// The same step on scores that already are in the log2 domain and relative to the reference
// value (the Q operand carries the scale, the score accumulation starts from -reference in
// `neg_ref`): no multiply-subtract per score, and no row maxima either in the common case.
// m_run is the reference in absolute terms (-inf before the first tile), neg_ref holds
// -(m_run, or 0 while m_run is -inf) in every element.
// The reference has to move only when a weight would exceed 2^threshold.  A lane's sum of
// weights bounds each of them, and the sum is computed anyway: the exponentials are taken
// first, against the reference as it stands, and only when some lane's sum of this tile
// exceeds 2^threshold (or is not a number) are the row maxima computed, the reference moved
// there, accumulators and row sums rescaled, the scores shifted, neg_ref refilled and the
// exponentials taken again.  A first tile (no reference yet) starts with the maxima.  With a reference that lags the
// running maximum by at most the threshold every weight stays <= 2^threshold, as before.
template <int DT>
__device__ __attribute__((always_inline)) inline void softmax_step_rel(f32x16 (&s)[2], float& m_run, float& l_run,
                                                                        f32x16 (&o)[DT], f32x16& neg_ref,
                                                                        bf16x8 (&pb)[4]) {
  const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
  const float limit = __builtin_amdgcn_exp2f(kRescaleThreshold);
  float ps0, ps1;
  bool moved = false;
  bool move = __builtin_amdgcn_ballot_w64(m_run == -INFINITY) != 0;  // a first tile: straight to the maxima
  while (true) {
    if (move) {
      float mx0 = fmaxf(s[0][0], s[1][0]);
      float mx1 = fmaxf(s[0][1], s[1][1]);
#pragma unroll
      for (int e = 2; e < 16; e += 2) {
        mx0 = fmaxf(fmaxf(mx0, s[0][e]), s[1][e]);
        mx1 = fmaxf(fmaxf(mx1, s[0][e + 1]), s[1][e + 1]);
      }
      const float r = max_across_halves(fmaxf(mx0, mx1));  // row maximum relative to the reference
      const float ref_old = -neg_ref[0];
      const float m_new = fmaxf(m_run, r + ref_old);
      const float ref_new = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run - ref_new);  // exp2(-inf) = 0 at the first tile
      const float shift = ref_new - ref_old;
      m_run = m_new;
      l_run *= alpha;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        s[0][e] -= shift;
        s[1][e] -= shift;
        neg_ref[e] = -ref_new;
      }
      moved = true;
    }
    ps0 = 0.f;
    ps1 = 0.f;
#pragma unroll
    for (int aa = 0; aa < 2; ++aa)
#pragma unroll
      for (int e = 0; e < 16; e += 4) {
        const bf16x2 q0 = {(bf16_t)__builtin_amdgcn_exp2f(s[aa][e]), (bf16_t)__builtin_amdgcn_exp2f(s[aa][e + 1])};
        const bf16x2 q1 = {(bf16_t)__builtin_amdgcn_exp2f(s[aa][e + 2]), (bf16_t)__builtin_amdgcn_exp2f(s[aa][e + 3])};
        ps0 = __builtin_amdgcn_fdot2_f32_bf16(q0, ones, ps0, false);
        ps1 = __builtin_amdgcn_fdot2_f32_bf16(q1, ones, ps1, false);
        pb[aa * 2 + (e >> 3)][e & 7] = q0[0];
        pb[aa * 2 + (e >> 3)][(e & 7) + 1] = q0[1];
        pb[aa * 2 + (e >> 3)][(e & 7) + 2] = q1[0];
        pb[aa * 2 + (e >> 3)][(e & 7) + 3] = q1[1];
      }
    if (moved) break;
    move = __builtin_amdgcn_ballot_w64(!(ps0 + ps1 <= limit)) != 0;
    if (!move) break;
  }
  l_run += ps0 + ps1;
}

// Both parts back to back.
template <int DT>
__device__ __attribute__((always_inline)) inline void softmax_step(const f32x16 (&s)[2], float sc, float& m_run,
                                                                    float& l_run, f32x16 (&o)[DT], bf16x8 (&pb)[4]) {
  const float m_use = softmax_max<DT>(s, sc, m_run, l_run, o);
  softmax_exp(s, sc, m_use, l_run, pb);
}

}  // namespace fedattn
