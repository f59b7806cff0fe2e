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

template <int D>
__global__ __launch_bounds__(256, 2) void prefill_mfma_kernel(PrefillArgs a) {
  constexpr int KSTEPS = D / 16;        // MFMA k-steps of S^T = K Q^T
  constexpr int DT = D / 32;            // 32-row tiles of O^T along head_dim
  constexpr int CPR = D / 8;            // 16-byte chunks per K/V row
  constexpr int KC = (kKvTile * CPR) / 256;  // K chunks per thread
  constexpr int RSK = D * 2 + 16;       // LDS bytes per K row (padded against bank conflicts)
  constexpr int RSV = kKvTile * 2 + 16; // LDS bytes per V^T row
  __shared__ __attribute__((aligned(16))) unsigned char k_lds[kKvTile * RSK];
  __shared__ __attribute__((aligned(16))) unsigned char v_lds[D * RSV];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l32 = lane & 31;
  const int hf = lane >> 5;

  const int Hq = a.Hq, Hkv = a.Hkv;
  const int G = Hq / Hkv;
  const int HS = a.heads_per_wg;
  const int HG = G / HS;
  const int BM = a.q_tile_rows;

  // workgroup -> (kv head, head subgroup, query tile); kv head fastest so that the
  // workgroups of one KV head land on one XCD (8 XCDs, round-robin dispatch) and
  // its K/V stay in that XCD's L2; heaviest (latest) query tiles first.
  const int id = blockIdx.x;
  const int g = id % Hkv;
  const int rest = id / Hkv;
  const int hsub = rest % HG;
  const int tile = a.n_q_tiles - 1 - rest / HG;
  const int block = blockIdx.y;

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
  const bool wave_active = row0w < seg_hi;

  const bool is_sync = a.sync_override >= 0 ? (a.sync_override != 0)
                                            : sync_block_rule(a.sync_interval, a.block_idx0 + block);
  const bool causal = a.causal != 0;
  const bool sparse = is_sync && a.keep_chunks != nullptr;

  const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q) + (int64_t)block * a.q_block_stride;
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(a.k) + (int64_t)block * a.kv_block_stride;
  const uint16_t* vp = reinterpret_cast<const uint16_t*>(a.v) + (int64_t)block * a.kv_block_stride;
  uint16_t* op = reinterpret_cast<uint16_t*>(a.out) + (int64_t)block * a.q_block_stride;

  // KV tile schedule of this workgroup: two runs of the kept-tile list, then a
  // dense range.
  int la_n = 0, lb0 = 0, lb_n = 0;
  if (sparse) {
    la_n = a.kept_cum[n];
    if (!causal) {
      lb0 = a.kept_cum[n + 1];
      lb_n = a.kept_cum[a.seg.n] - lb0;
    }
  }
  const int n_list = la_n + lb_n;
  const int dlo = (is_sync && !sparse) ? 0 : seg_lo;
  const int dhi = causal ? i_last + 1 : ((is_sync && !sparse) ? a.total : seg_hi);
  const int n_dense = (dhi - dlo + kKvTile - 1) / kKvTile;
  const int nt = n_list + n_dense;

  // Q fragments (B operand of S^T): lane (q row = l32, half hf) holds
  // Q[row][16*step + 8*hf .. +8].
  bf16x8 qf[KSTEPS];
  {
    const uint16_t* qrow = qp + ((int64_t)row_ld * Hq + head) * D + 8 * hf;
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st)
      qf[st] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qrow + 16 * st));
  }

  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
  float m_run = -INFINITY;  // running row maximum, log2 domain (score * scale * log2 e)
  float l_run = 0.f;        // this lane's share of the running row sum
  const float sc = a.scale * kLog2e;

  uint4 kreg[KC];
  uint4 vreg[4];
  const int v_rg = tid & 15;  // group of 4 KV rows this thread transposes
  const int v_dc = tid >> 4;  // its 8-wide head_dim chunk
  const bool v_active = v_dc < CPR;

  auto tile_desc = [&](int it, int& kv0, int& len, bool& causal_tile) {
    if (it < n_list) {
      const int idx = it < la_n ? it : lb0 + (it - la_n);
      const int2 t = a.kept_tiles[idx];
      kv0 = t.x;
      len = t.y;
      causal_tile = false;
    } else {
      kv0 = dlo + kKvTile * (it - n_list);
      len = min(kKvTile, dhi - kv0);
      causal_tile = causal;
    }
  };

  auto load_tile = [&](int kv0, int len) {
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      const int ci = tid + 256 * c;
      const int r = min(ci / CPR, len - 1);
      const int dc = ci % CPR;
      kreg[c] = *reinterpret_cast<const uint4*>(kp + ((int64_t)(kv0 + r) * Hkv + g) * D + dc * 8);
    }
    if (v_active) {
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = min(4 * v_rg + r, len - 1);
        vreg[r] = *reinterpret_cast<const uint4*>(vp + ((int64_t)(kv0 + row) * Hkv + g) * D + v_dc * 8);
      }
    }
  };

  auto store_tile = [&]() {
#pragma unroll
    for (int c = 0; c < KC; ++c) {
      const int ci = tid + 256 * c;
      *reinterpret_cast<uint4*>(k_lds + (ci / CPR) * RSK + (ci % CPR) * 16) = kreg[c];
    }
    if (v_active) {
      // V^T[d][kv]: within each run of 16 KV rows the four 4-row groups are stored
      // in the order 0,2,1,3 so that one 16-byte read yields the 8 rows a lane
      // needs for one MFMA k-step (rows 4hf..4hf+3 and 8+4hf..8+4hf+3).
      const int gi = v_rg & 3;
      const int pos = (v_rg >> 2) * 32 + (((gi & 1) << 1) | (gi >> 1)) * 8;
      const uint32_t w0[4] = {vreg[0].x, vreg[0].y, vreg[0].z, vreg[0].w};
      const uint32_t w1[4] = {vreg[1].x, vreg[1].y, vreg[1].z, vreg[1].w};
      const uint32_t w2[4] = {vreg[2].x, vreg[2].y, vreg[2].z, vreg[2].w};
      const uint32_t w3[4] = {vreg[3].x, vreg[3].y, vreg[3].z, vreg[3].w};
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int d = 8 * v_dc + 2 * p;
        uint2 ev, od;
        ev.x = pack_lo(w0[p], w1[p]);
        ev.y = pack_lo(w2[p], w3[p]);
        od.x = pack_hi(w0[p], w1[p]);
        od.y = pack_hi(w2[p], w3[p]);
        *reinterpret_cast<uint2*>(v_lds + d * RSV + pos) = ev;
        *reinterpret_cast<uint2*>(v_lds + (d + 1) * RSV + pos) = od;
      }
    }
  };

  if (nt > 0) {
    int kv0, len;
    bool ct;
    tile_desc(0, kv0, len, ct);
    load_tile(kv0, len);
  }

  for (int it = 0; it < nt; ++it) {
    int kv0, len;
    bool causal_tile;
    tile_desc(it, kv0, len, causal_tile);

    __syncthreads();  // all waves are done reading the previous tile
    store_tile();
    __syncthreads();
    if (it + 1 < nt) {
      int nkv0, nlen;
      bool nct;
      tile_desc(it + 1, nkv0, nlen, nct);
      load_tile(nkv0, nlen);  // in flight while this tile is computed
    }

    // waves whose rows all lie before this tile (causal) or past the segment end
    // have nothing to compute here
    if (!wave_active || (causal_tile && kv0 > row0w + kWaveRows - 1)) continue;

    // ---- S^T[kv][q] = K Q^T -------------------------------------------------
    f32x16 s[2];
#pragma unroll
    for (int e = 0; e < 16; ++e) { s[0][e] = 0.f; s[1][e] = 0.f; }
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) {
#pragma unroll
      for (int aa = 0; aa < 2; ++aa) {
        const bf16x8 kf = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const uint4*>(k_lds + (32 * aa + l32) * RSK + (16 * st + 8 * hf) * 2));
        s[aa] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], s[aa], 0, 0, 0);
      }
    }
    // register e of s[aa] holds kv row 32*aa + 8*(e/4) + 4*hf + (e%4), query row l32

    if (len < kKvTile || (causal_tile && kv0 + kKvTile - 1 > row0w)) {
#pragma unroll
      for (int aa = 0; aa < 2; ++aa)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int jl = 32 * aa + 8 * (e >> 2) + 4 * hf + (e & 3);
          const bool ok = jl < len && (!causal_tile || kv0 + jl <= my_row);
          if (!ok) s[aa][e] = -INFINITY;
        }
    }

    // ---- online softmax (log2 domain) ----------------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int aa = 0; aa < 2; ++aa)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[aa][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx * sc);
    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
    m_run = m_new;

    float psum = 0.f;
    bf16x8 pb[4];
#pragma unroll
    for (int aa = 0; aa < 2; ++aa)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(fmaf(s[aa][e], sc, -m_use));
        psum += p;
        pb[aa * 2 + (e >> 3)][e & 7] = (bf16_t)p;
      }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;

    // ---- O^T[d][q] += V^T P^T --------------------------------------------------
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const bf16x8 vf = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const uint4*>(v_lds + (32 * dt + l32) * RSV + kk * 32 + hf * 16));
        o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[kk], o[dt], 0, 0, 0);
      }
    }
  }

  // ---- normalise and write -------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
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
        *reinterpret_cast<uint2*>(orow + 32 * dt + 8 * vq) = __builtin_bit_cast(uint2, w);
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
  dim3 grid((unsigned)(a.n_q_tiles * a.Hkv * (G / a.heads_per_wg)), (unsigned)n_blocks, 1);
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
