// Decode attention (Section IV-C): one new query per participant over the block's
// KV cache; bandwidth-bound, so the cache is streamed exactly once.
//
// Split-KV: a workgroup takes one chunk of one participant's cache segment for
// one KV head and ALL query rows that may see it - the G query heads of that
// participant in a local block, the N*G rows of all participants in a sync block
// (the aggregated cache is read once for everybody).  Each of the 4 wavefronts
// streams its own 32-row sub-tiles straight from HBM into MFMA operand registers
// (K) or through a private LDS transpose (V), keeps an online softmax per query
// column, and the wavefronts are merged at the end.  A second small kernel merges
// the chunks: o = sum_c O_c 2^(m_c - m) / sum_c l_c 2^(m_c - m).
//
// Products run transposed on the 16x16x32 bf16 MFMA: S^T[kv][q] = K Q^T and
// O^T[d][q] += V^T P^T, so a query column lives in 4 lanes (lane%16) and P^T feeds
// the second product from registers.
#include "common.h"

namespace fedattn {

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int kSubRows = 32;  // cache rows per wavefront step

__device__ inline uint32_t pack_lo(uint32_t a, uint32_t b) { return (a & 0xFFFFu) | (b << 16); }
__device__ inline uint32_t pack_hi(uint32_t a, uint32_t b) { return (a >> 16) | (b & 0xFFFF0000u); }

template <int D, int NQT>
__global__ __launch_bounds__(256, (NQT <= 2 ? 2 : 1)) void decode_split_kernel(DecodeArgs a) {
  constexpr int KS = D / 32;          // MFMA k-steps of S^T
  constexpr int DT = D / 16;          // 16-row tiles of O^T along head_dim
  constexpr int VP = D / 64;          // V load passes (a wave covers 64 head_dim columns per pass)
  constexpr int QCOLS = 16 * NQT;     // query columns per workgroup
  constexpr int RSQ = D * 2 + 16;     // LDS bytes per Q row
  constexpr int RSV = kSubRows * 2 + 16;  // LDS bytes per V^T row (one wave's 32 cache rows)
  constexpr int OPAD = D + 4;         // floats per row of the merge buffer
  constexpr int VT_BYTES = 4 * D * RSV;
  constexpr int OS_BYTES = QCOLS * OPAD * 4;
  constexpr int SCR_BYTES = VT_BYTES > OS_BYTES ? VT_BYTES : OS_BYTES;
  __shared__ __attribute__((aligned(16))) unsigned char q_lds[QCOLS * RSQ];
  __shared__ __attribute__((aligned(16))) unsigned char scr[SCR_BYTES];  // V^T per wave, later the merge buffer
  __shared__ float m_s[4][QCOLS];
  __shared__ float l_s[4][QCOLS];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int l16 = lane & 15;
  const int kg = lane >> 4;

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

  const uint16_t* qp = reinterpret_cast<const uint16_t*>(a.q);
  const uint16_t* kp = reinterpret_cast<const uint16_t*>(a.k_cache) + ((int64_t)a.seg_off[m] * Hkv + g) * D;
  const uint16_t* vp = reinterpret_cast<const uint16_t*>(a.v_cache) + ((int64_t)a.seg_off[m] * Hkv + g) * D;
  const int64_t row_stride = (int64_t)Hkv * D;

  // query column -> (participant, head); columns past the end read zeros
  auto col_participant = [&](int col) { return sync ? col / G : m; };
  auto col_head = [&](int col) { return g * G + (sync ? col % G : col); };

  // stage Q into LDS
  for (int idx = tid; idx < QCOLS * (D / 8); idx += 256) {
    const int cl = idx / (D / 8), ch = idx % (D / 8);
    const int col = cb + cl;
    uint4 w = make_uint4(0, 0, 0, 0);
    if (col < a.cols)
      w = *reinterpret_cast<const uint4*>(qp + ((int64_t)col_participant(col) * Hq + col_head(col)) * D + ch * 8);
    *reinterpret_cast<uint4*>(q_lds + cl * RSQ + ch * 16) = w;
  }
  __syncthreads();

  // rows of this segment visible to the query column in lane l16 of column tile qt
  int limit[NQT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int col = cb + 16 * qt + l16;
    limit[qt] = col >= a.cols ? 0 : (col_participant(col) == m ? own_len : rem_len);
  }

  f32x4 o[DT][NQT];
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) o[dt][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run[NQT], l_run[NQT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) { m_run[qt] = -INFINITY; l_run[qt] = 0.f; }
  const float sc = a.scale * kLog2e;

  unsigned char* vt = scr + wave * (D * RSV);
  const int v_rg = lane & 7;   // group of 4 cache rows this lane transposes
  const int v_dc = lane >> 3;  // 8-wide head_dim chunk (plus 8 per pass)
  const int v_pos = (((v_rg & 3) << 1) | (v_rg >> 2)) * 8;  // groups kg and 4+kg end up adjacent

  uint4 kreg[2][KS];
  uint4 vreg[VP][4];
  auto load_sub = [&](int r0) {
#pragma unroll
    for (int aa = 0; aa < 2; ++aa) {
      const int row = min(r0 + 16 * aa + l16, r_hi - 1);
#pragma unroll
      for (int st = 0; st < KS; ++st)
        kreg[aa][st] = *reinterpret_cast<const uint4*>(kp + row * row_stride + 32 * st + 8 * kg);
    }
#pragma unroll
    for (int ps = 0; ps < VP; ++ps)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = min(r0 + 4 * v_rg + r, r_hi - 1);
        vreg[ps][r] = *reinterpret_cast<const uint4*>(vp + row * row_stride + 8 * (v_dc + 8 * ps));
      }
  };

  int r0 = r_lo + kSubRows * wave;
  if (r0 < r_hi) load_sub(r0);

  for (; r0 < r_hi; r0 += 4 * kSubRows) {
    // take this sub-tile out of the prefetch registers
    bf16x8 kf[2][KS];
#pragma unroll
    for (int aa = 0; aa < 2; ++aa)
#pragma unroll
      for (int st = 0; st < KS; ++st) kf[aa][st] = __builtin_bit_cast(bf16x8, kreg[aa][st]);
#pragma unroll
    for (int ps = 0; ps < VP; ++ps) {
      const uint32_t w0[4] = {vreg[ps][0].x, vreg[ps][0].y, vreg[ps][0].z, vreg[ps][0].w};
      const uint32_t w1[4] = {vreg[ps][1].x, vreg[ps][1].y, vreg[ps][1].z, vreg[ps][1].w};
      const uint32_t w2[4] = {vreg[ps][2].x, vreg[ps][2].y, vreg[ps][2].z, vreg[ps][2].w};
      const uint32_t w3[4] = {vreg[ps][3].x, vreg[ps][3].y, vreg[ps][3].z, vreg[ps][3].w};
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int d = 8 * (v_dc + 8 * ps) + 2 * p;
        uint2 ev, od;
        ev.x = pack_lo(w0[p], w1[p]);
        ev.y = pack_lo(w2[p], w3[p]);
        od.x = pack_hi(w0[p], w1[p]);
        od.y = pack_hi(w2[p], w3[p]);
        *reinterpret_cast<uint2*>(vt + d * RSV + v_pos) = ev;
        *reinterpret_cast<uint2*>(vt + (d + 1) * RSV + v_pos) = od;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const int r_next = r0 + 4 * kSubRows;
    if (r_next < r_hi) load_sub(r_next);  // in flight during the MFMAs below

    // ---- S^T[kv][q] = K Q^T ---------------------------------------------------
    f32x4 s[2][NQT];
#pragma unroll
    for (int aa = 0; aa < 2; ++aa)
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt) s[aa][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
      for (int st = 0; st < KS; ++st) {
        const bf16x8 qf = __builtin_bit_cast(
            bf16x8, *reinterpret_cast<const uint4*>(q_lds + (16 * qt + l16) * RSQ + (32 * st + 8 * kg) * 2));
        s[0][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[0][st], qf, s[0][qt], 0, 0, 0);
        s[1][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[1][st], qf, s[1][qt], 0, 0, 0);
      }
    // element e of s[aa][qt]: cache row r0 + 16*aa + 4*kg + e, query column 16*qt + l16

    if (r0 + kSubRows > min_limit) {
#pragma unroll
      for (int aa = 0; aa < 2; ++aa)
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (r0 + 16 * aa + 4 * kg + e >= limit[qt]) s[aa][qt][e] = -INFINITY;
    }

    // ---- online softmax per query column ----------------------------------------
    bf16x8 pb[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      float mx = -INFINITY;
#pragma unroll
      for (int aa = 0; aa < 2; ++aa)
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = fmaxf(mx, s[aa][qt][e]);
      mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run[qt], mx * sc);
      const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
      const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_use);
      m_run[qt] = m_new;
      float psum = 0.f;
#pragma unroll
      for (int aa = 0; aa < 2; ++aa)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[aa][qt][e], sc, -m_use));
          psum += p;
          pb[qt][4 * aa + e] = (bf16_t)p;
        }
      l_run[qt] = l_run[qt] * alpha + psum;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) o[dt][qt] *= alpha;
    }

    // ---- O^T[d][q] += V^T P^T -------------------------------------------------------
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const bf16x8 vf = __builtin_bit_cast(
          bf16x8, *reinterpret_cast<const uint4*>(vt + (16 * dt + l16) * RSV + kg * 16));
#pragma unroll
      for (int qt = 0; qt < NQT; ++qt)
        o[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pb[qt], o[dt][qt], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  // ---- merge the 4 wavefronts -------------------------------------------------------
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    l_run[qt] += __shfl_xor(l_run[qt], 16, 64);
    l_run[qt] += __shfl_xor(l_run[qt], 32, 64);
    if (kg == 0) m_s[wave][16 * qt + l16] = m_run[qt];
  }
  __syncthreads();  // also: every wave is done with its V^T region
  float f[NQT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int cl = 16 * qt + l16;
    const float mm = fmaxf(fmaxf(m_s[0][cl], m_s[1][cl]), fmaxf(m_s[2][cl], m_s[3][cl]));
    const float mu = (mm == -INFINITY) ? 0.f : mm;
    f[qt] = __builtin_amdgcn_exp2f(m_run[qt] - mu);
    if (kg == 0) l_s[wave][cl] = l_run[qt] * f[qt];
  }
  float* o_s = reinterpret_cast<float*>(scr);
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
          float* dst = o_s + (16 * qt + l16) * OPAD + 16 * dt + 4 * kg;
          f32x4 val = o[dt][qt] * f[qt];
          if (w > 0) val += *reinterpret_cast<const f32x4*>(dst);
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
    const float mm = fmaxf(fmaxf(m_s[0][tid], m_s[1][tid]), fmaxf(m_s[2][tid], m_s[3][tid]));
    const float ll = l_s[0][tid] + l_s[1][tid] + l_s[2][tid] + l_s[3][tid];
    a.part_ml[(prow0 + tid) * 2] = mm;
    a.part_ml[(prow0 + tid) * 2 + 1] = ll;
  }
}

// Merges the chunk partials of one (participant, query head) and writes the output row.
template <typename T>
__global__ void decode_combine_kernel(DecodeArgs a) {
  const int n = blockIdx.x / a.Hq;
  const int h = blockIdx.x % a.Hq;
  const int G = a.Hq / a.Hkv;
  const int g = h / G, hh = h % G;
  const int c0 = a.is_sync ? 0 : a.chunk_cum[n];
  const int c1 = a.is_sync ? a.n_chunks : a.chunk_cum[n + 1];
  const int col = a.is_sync ? n * G + hh : hh;
  const int64_t base = (int64_t)g * a.n_chunks;

  float mm = -INFINITY;
  for (int cc = c0; cc < c1; ++cc) mm = fmaxf(mm, a.part_ml[((base + cc) * a.cols + col) * 2]);
  const float mu = (mm == -INFINITY) ? 0.f : mm;
  for (int d = threadIdx.x; d < a.D; d += blockDim.x) {
    float num = 0.f, den = 0.f;
    for (int cc = c0; cc < c1; ++cc) {
      const int64_t prow = (base + cc) * a.cols + col;
      const float fc = __builtin_amdgcn_exp2f(a.part_ml[prow * 2] - mu);
      den = fmaf(a.part_ml[prow * 2 + 1], fc, den);
      num = fmaf(a.part_o[prow * a.D + d], fc, num);
    }
    const float val = den > 0.f ? num / den : 0.f;
    T* out = reinterpret_cast<T*>(a.out) + ((int64_t)n * a.Hq + h) * a.D + d;
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
hipError_t launch_split(const DecodeArgs& a, hipStream_t s) {
  const int qcols = a.cols <= 16 ? 16 : (a.cols <= 32 ? 32 : 64);
  dim3 grid((unsigned)(a.n_chunks * a.Hkv), (unsigned)((a.cols + qcols - 1) / qcols), 1);
  if (qcols == 16)
    hipLaunchKernelGGL((decode_split_kernel<D, 1>), grid, dim3(256), 0, s, a);
  else if (qcols == 32)
    hipLaunchKernelGGL((decode_split_kernel<D, 2>), grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((decode_split_kernel<D, 4>), grid, dim3(256), 0, s, a);
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
    hipError_t e = a.D == 128 ? launch_split<128>(a, s) : launch_split<64>(a, s);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(decode_combine_kernel<uint16_t>, dim3((unsigned)(a.N * a.Hq)),
                     dim3((unsigned)a.D), 0, s, a);
  return hipGetLastError();
}

}  // namespace fedattn
