// Decode attention (Section IV-C): one new query per participant over the block's
// KV cache; bandwidth-bound, so the cache is streamed exactly once.
//
// Split-KV: a workgroup takes one chunk of one participant's cache segment for
// one KV head and ALL query rows that may see it - the G query heads of that
// participant in a local block, the N*G rows of all participants in a sync block
// (the aggregated cache is read once for everybody).  The chunk streams through a
// 4-stage LDS ring of 64-row K/V tiles filled by direct HBM -> LDS loads, three
// tiles in flight per workgroup, one workgroup per CU.  The query rows form one or
// two 32-row MFMA tiles; the wavefronts that share a query tile take the KV tiles
// round-robin, each with its own online softmax, and are merged at the end.  A
// second small kernel merges the chunks:
//   o = sum_c O_c 2^(m_c - m) / sum_c l_c 2^(m_c - m).
#include "common.h"
#include "mfma_tile.h"

namespace fedattn {

namespace {

constexpr int kDecodeStages = 4;

template <int D>
constexpr int decode_smem_bytes() { return kDecodeStages * 2 * KvTile<D>::TILEB; }

template <int D, int NQS>
__global__ __launch_bounds__(256, 1) void decode_stream_kernel(DecodeArgs a) {
  using TL = KvTile<D>;
  constexpr int KSTEPS = TL::KSTEPS, DT = TL::DT, TILEB = TL::TILEB, IPW = TL::IPW;
  constexpr int KP = 4 / NQS;        // wavefronts sharing one query tile, KV tiles round-robin
  constexpr int QCOLS = 32 * NQS;    // query columns per workgroup
  constexpr int OPAD = D + 4;        // floats per row of the merge buffer
  static_assert(QCOLS * OPAD * 4 <= kDecodeStages * 2 * TILEB, "merge buffer must fit in the tile ring");
  // stage s: K tile at s*2*TILEB, V tile at s*2*TILEB + TILEB; after the stream the
  // ring is reused as the merge buffer
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  __shared__ float m_s[4][32];
  __shared__ float l_s[4][32];
  const lds_cptr lds0 = (lds_cptr)(lds_void_ptr)smem;
  const uint32_t lds_base = lds_addr_of(smem);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;
  const int hf = lane >> 5;
  const int qs = wave % NQS;   // query tile of this wavefront
  const int kp = wave / NQS;   // its turn among the KV tiles

  const int Hq = a.Hq, Hkv = a.Hkv;
  const int G = Hq / Hkv;
  const int g = blockIdx.x % Hkv;
  const int gc = blockIdx.x / Hkv;  // chunk index over all segments
  const int cb = blockIdx.y * QCOLS;

  int m = 0;
  while (gc >= a.chunk_cum[m + 1]) ++m;
  const int c = gc - a.chunk_cum[m];
  const int own_len = a.seg_lens[m];
  const int rem_len = a.has_remote ? a.remote_lens[m] : own_len;
  const bool sync = a.is_sync != 0;
  const int rows_end = sync ? max(own_len, rem_len) : own_len;
  const int min_limit = sync ? min(own_len, rem_len) : own_len;
  const int r_lo = c * a.chunk_rows;
  const int r_hi = min(r_lo + a.chunk_rows, rows_end);
  const int nt = (r_hi - r_lo + kKvTile - 1) / kKvTile;
  const int row_elems = Hkv * D;

  const uint16_t* kbase = reinterpret_cast<const uint16_t*>(a.k_cache) + ((int64_t)(a.seg_off[m] + r_lo) * Hkv + g) * D;
  const uint16_t* vbase = reinterpret_cast<const uint16_t*>(a.v_cache) + ((int64_t)(a.seg_off[m] + r_lo) * Hkv + g) * D;

  TL tile_io;
  tile_io.init(lane, wave, row_elems);

  // this lane's query column -> (participant, head); columns past the end are zero
  // rows: local block, column = head inside the KV group; sync block, column =
  // participant * G + head inside the group.  The loads are written out (like the tile
  // loads) so that the compiler's own wait for them does not drain the tile ring; they
  // are the oldest loads of the wavefront, so the first tile wait covers them.
  const int col = cb + 32 * qs + l32;
  const bool col_ok = col < a.cols;
  const int col_part = sync ? col / G : m;
  const int col_head = g * G + (sync ? col % G : col);
  const int limit = col_ok ? (col_part == m ? own_len : rem_len) : 0;  // visible rows of this segment
  u32x4 qw[KSTEPS];
  {
    const uint16_t* qrow = reinterpret_cast<const uint16_t*>(a.q) +
                           ((int64_t)(col_ok ? col_part : 0) * Hq + (col_ok ? col_head : 0)) * D + 8 * hf;
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st)
      asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(qw[st]) : "v"(qrow + 16 * st) : "memory");
  }

  auto issue = [&](int t) __attribute__((always_inline)) {
    const int len = min(kKvTile, r_hi - r_lo - kKvTile * t);
    const uint32_t stage = lds_base + (t % kDecodeStages) * 2 * TILEB;
    tile_io.template dma<false>(kbase + (int64_t)t * kKvTile * row_elems, stage, len);
    tile_io.template dma<true>(vbase + (int64_t)t * kKvTile * row_elems, stage + TILEB, len);
  };
#pragma unroll
  for (int t = 0; t < kDecodeStages - 1; ++t)
    if (t < nt) issue(t);

  f32x16 o[DT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[dt][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = a.scale * kLog2e;

  for (int t = 0; t < nt; ++t) {
    // this wavefront's part of tile t has landed once at most the loads of the tiles
    // issued after it are outstanding
    const int after = min(nt, t + kDecodeStages - 1) - (t + 1);
    if (after >= 2)
      wait_vmcnt<2 * 2 * IPW>();
    else if (after == 1)
      wait_vmcnt<2 * IPW>();
    else
      wait_vmcnt<0>();
    __syncthreads();  // tile t is complete in LDS, and everyone is done with tile t-1
#pragma unroll
    for (int st = 0; st < KSTEPS; ++st) asm volatile("" : "+v"(qw[st]));  // the query loads have landed by now
    if (t + kDecodeStages - 1 < nt) issue(t + kDecodeStages - 1);  // into the stage tile t-1 used

    if (t % KP == kp) {
      const int kb = (t % kDecodeStages) * 2 * TILEB;
      bf16x8 qf[KSTEPS];
#pragma unroll
      for (int st = 0; st < KSTEPS; ++st) {
        const u32x4 zero = {0u, 0u, 0u, 0u};
        qf[st] = __builtin_bit_cast(bf16x8, col_ok ? qw[st] : zero);
      }
      f32x16 s[2];
      tile_io.scores(lds0, kb, qf, s);
      const int row0 = r_lo + kKvTile * t;
      if (row0 + kKvTile > min_limit) mask_scores(s, limit - row0, hf);
      bf16x8 pb[4];
      softmax_step<DT>(s, sc, m_run, l_run, o, pb);
      tile_io.pv(lds0, kb + TILEB, pb, o);
    }
  }

  // ---- merge the wavefronts that share a query tile ------------------------------------
  const float l_full = sum_across_halves(l_run);
  if (hf == 0) m_s[wave][l32] = m_run;
  __syncthreads();  // also: every wavefront is done with the tile ring
  float mm = -INFINITY;
#pragma unroll
  for (int k2 = 0; k2 < KP; ++k2) mm = fmaxf(mm, m_s[k2 * NQS + qs][l32]);
  const float mu = (mm == -INFINITY) ? 0.f : mm;
  const float f = __builtin_amdgcn_exp2f(m_run - mu);
  if (hf == 0) l_s[wave][l32] = l_full * f;
  float* o_s = reinterpret_cast<float*>(smem);
#pragma unroll
  for (int k2 = 0; k2 < KP; ++k2) {
    if (kp == k2) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          float* dst = o_s + (32 * qs + l32) * OPAD + 32 * dt + 8 * vq + 4 * hf;
          f32x4 val = {o[dt][4 * vq] * f, o[dt][4 * vq + 1] * f, o[dt][4 * vq + 2] * f, o[dt][4 * vq + 3] * f};
          if (k2 > 0) val += *reinterpret_cast<const f32x4*>(dst);
          *reinterpret_cast<f32x4*>(dst) = val;
        }
    }
    __syncthreads();
  }

  const int n_cols = min(QCOLS, a.cols - cb);
  const int64_t prow0 = ((int64_t)g * a.n_chunks + gc) * a.cols + cb;
  for (int idx = tid; idx < n_cols * (D / 4); idx += 256) {
    const int cl = idx / (D / 4), d4 = idx % (D / 4);
    *reinterpret_cast<f32x4*>(a.part_o + (prow0 + cl) * D + 4 * d4) =
        *reinterpret_cast<const f32x4*>(o_s + cl * OPAD + 4 * d4);
  }
  if (tid < n_cols) {
    const int q2 = tid >> 5, c32 = tid & 31;
    float m2 = -INFINITY, l2 = 0.f;
#pragma unroll
    for (int k2 = 0; k2 < KP; ++k2) {
      m2 = fmaxf(m2, m_s[k2 * NQS + q2][c32]);
      l2 += l_s[k2 * NQS + q2][c32];
    }
    a.part_ml[(prow0 + tid) * 2] = m2;
    a.part_ml[(prow0 + tid) * 2 + 1] = l2;
  }
}

// Merges the chunk partials of one (participant, query head) and writes the output row.
template <typename T>
__global__ __launch_bounds__(256) void decode_combine_kernel(DecodeArgs a) {
  __shared__ float w_s[256];
  __shared__ float red_s[8];
  const int n = blockIdx.x / a.Hq;
  const int h = blockIdx.x % a.Hq;
  const int G = a.Hq / a.Hkv;
  const int g = h / G, hh = h % G;
  const int c0 = a.is_sync ? 0 : a.chunk_cum[n];
  const int c1 = a.is_sync ? a.n_chunks : a.chunk_cum[n + 1];
  const int col = a.is_sync ? n * G + hh : hh;
  const int64_t base = (int64_t)g * a.n_chunks;
  const int tid = threadIdx.x;
  const int D = a.D;

  // row maximum over the chunks
  float mm = -INFINITY;
  for (int cc = c0 + tid; cc < c1; cc += blockDim.x) mm = fmaxf(mm, a.part_ml[((base + cc) * a.cols + col) * 2]);
  mm = wave_max(mm);
  if ((tid & 63) == 0) red_s[tid >> 6] = mm;
  __syncthreads();
  mm = -INFINITY;
  for (int w = 0; w < (int)(blockDim.x >> 6); ++w) mm = fmaxf(mm, red_s[w]);
  const float mu = (mm == -INFINITY) ? 0.f : mm;

  float acc = 0.f, den = 0.f;
  for (int cb = c0; cb < c1; cb += 256) {
    const int nb = min(256, c1 - cb);
    __syncthreads();
    for (int i = tid; i < nb; i += blockDim.x)
      w_s[i] = __builtin_amdgcn_exp2f(a.part_ml[((base + cb + i) * a.cols + col) * 2] - mu);
    __syncthreads();
    if (tid < D) {
      int i = 0;
      for (; i + 4 <= nb; i += 4) {
        const float* p0 = a.part_o + ((base + cb + i) * a.cols + col) * D + tid;
        const int64_t st = (int64_t)a.cols * D;
        const float x0 = p0[0], x1 = p0[st], x2 = p0[2 * st], x3 = p0[3 * st];
        acc = fmaf(x0, w_s[i], acc);
        acc = fmaf(x1, w_s[i + 1], acc);
        acc = fmaf(x2, w_s[i + 2], acc);
        acc = fmaf(x3, w_s[i + 3], acc);
      }
      for (; i < nb; ++i) acc = fmaf(a.part_o[((base + cb + i) * a.cols + col) * D + tid], w_s[i], acc);
    }
    for (int i = 0; i < nb; ++i) den = fmaf(a.part_ml[((base + cb + i) * a.cols + col) * 2 + 1], w_s[i], den);
  }
  if (tid < D) {
    const float val = den > 0.f ? acc / den : 0.f;
    T* out = reinterpret_cast<T*>(a.out) + ((int64_t)n * a.Hq + h) * D + tid;
    if constexpr (sizeof(T) == 2)
      *out = f32_to_bf16_bits(val);
    else
      *out = val;
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

template <int D>
hipError_t launch_stream(const DecodeArgs& a, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_stream_kernel<D, 1>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, decode_smem_bytes<D>());
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_stream_kernel<D, 2>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, decode_smem_bytes<D>());
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int qcols = a.cols <= 32 ? 32 : 64;
  dim3 grid((unsigned)(a.n_chunks * a.Hkv), (unsigned)((a.cols + qcols - 1) / qcols), 1);
  if (qcols == 32)
    hipLaunchKernelGGL((decode_stream_kernel<D, 1>), grid, dim3(256), decode_smem_bytes<D>(), s, a);
  else
    hipLaunchKernelGGL((decode_stream_kernel<D, 2>), grid, dim3(256), decode_smem_bytes<D>(), s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const DecodeArgs& a, int dtype, hipStream_t s) {
  if (a.N == 0) return hipSuccess;
  const bool mfma = dtype == FEDATTN_BF16 && (a.D == 64 || a.D == 128);
  if (!mfma) {
    dim3 grid((unsigned)(a.N * a.Hq));
    if (dtype == FEDATTN_F32)
      hipLaunchKernelGGL(decode_rows_kernel<float>, grid, dim3(64), 0, s, a);
    else
      hipLaunchKernelGGL(decode_rows_kernel<uint16_t>, grid, dim3(64), 0, s, a);
    return hipGetLastError();
  }
  if (a.n_chunks > 0) {
    hipError_t e = a.D == 128 ? launch_stream<128>(a, s) : launch_stream<64>(a, s);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(decode_combine_kernel<uint16_t>, dim3((unsigned)(a.N * a.Hq)), dim3(a.D <= 64 ? 64 : 128), 0,
                     s, a);
  return hipGetLastError();
}

}  // namespace fedattn
