// General prefill attention kernel (plain ALU, fp32 arithmetic): one wavefront per
// (query row, query head).  Covers every shape the boundary accepts (any head_dim
// that is a multiple of 8 up to 256, fp32 or bf16 storage, token-granular
// keep-lists, bidirectional attention); the MFMA kernel takes over for the bf16
// shapes that matter for throughput.
//
// Visibility of key j for query i (Section III-B causal mask; Phase I / Phase II;
// adaptive KV aggregation): own segment always, remote segments only in a sync
// block and only in chunks flagged as exchanged, and j <= i when causal.
#include "common.h"

namespace fedattn {

namespace {

constexpr int kKeysPerStep = 256;

template <typename T>
struct RowLoad;

template <>
struct RowLoad<float> {
  // dot of an LDS-resident fp32 vector with a global fp32 row
  static __device__ inline float dot(const float* qs, const float* row, int D) {
    float acc = 0.f;
    for (int d = 0; d < D; d += 4) {
      const float4 kv = *reinterpret_cast<const float4*>(row + d);
      acc = fmaf(qs[d + 0], kv.x, acc);
      acc = fmaf(qs[d + 1], kv.y, acc);
      acc = fmaf(qs[d + 2], kv.z, acc);
      acc = fmaf(qs[d + 3], kv.w, acc);
    }
    return acc;
  }
  static __device__ inline float at(const float* p) { return *p; }
  static __device__ inline void store(float* p, float x) { *p = x; }
};

template <>
struct RowLoad<uint16_t> {
  static __device__ inline float dot(const float* qs, const uint16_t* row, int D) {
    float acc = 0.f;
    for (int d = 0; d < D; d += 8) {
      const uint4 w = *reinterpret_cast<const uint4*>(row + d);
      const uint32_t u[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        acc = fmaf(qs[d + 2 * e], __uint_as_float(u[e] << 16), acc);
        acc = fmaf(qs[d + 2 * e + 1], __uint_as_float(u[e] & 0xFFFF0000u), acc);
      }
    }
    return acc;
  }
  static __device__ inline float at(const uint16_t* p) { return bf16_bits_to_f32(*p); }
  static __device__ inline void store(uint16_t* p, float x) { *p = f32_to_bf16_bits(x); }
};

template <typename T>
__global__ __launch_bounds__(256) void prefill_rows_kernel(PrefillArgs a) {
  __shared__ float q_s[4][256];
  __shared__ float p_s[4][kKeysPerStep];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int64_t pair = (int64_t)blockIdx.x * 4 + wave;
  const int64_t n_pairs = (int64_t)a.total * a.Hq;
  if (pair >= n_pairs) return;  // only wave-level synchronisation below

  const int block = blockIdx.y;
  const int i = (int)(pair / a.Hq);
  const int h = (int)(pair % a.Hq);
  const int g = h / (a.Hq / a.Hkv);
  const int D = a.D;
  const bool is_sync = a.sync_override >= 0 ? (a.sync_override != 0)
                                            : sync_block_rule(a.sync_interval, a.block_idx0 + block);

  const T* q = reinterpret_cast<const T*>(a.q) + (int64_t)block * a.q_block_stride;
  const T* k = reinterpret_cast<const T*>(a.k) + (int64_t)block * a.kv_block_stride;
  const T* v = reinterpret_cast<const T*>(a.v) + (int64_t)block * a.kv_block_stride;
  T* out = reinterpret_cast<T*>(a.out) + (int64_t)block * a.q_block_stride;

  int n = 0;
  while (n + 1 < a.seg.n && i >= a.seg.seg_off[n + 1]) ++n;

  float* qs = q_s[wave];
  float* ps = p_s[wave];
  for (int d = lane; d < D; d += 64) qs[d] = RowLoad<T>::at(q + ((int64_t)i * a.Hq + h) * D + d);
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();

  float m_run = -INFINITY, l_run = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};

  for (int m = 0; m < a.seg.n; ++m) {
    int lo = a.seg.seg_off[m], hi = a.seg.seg_off[m + 1];
    if (m != n && !is_sync) continue;
    if (a.causal && hi > i + 1) hi = i + 1;
    if (lo >= hi) continue;
    const bool filter = (m != n) && a.keep_chunks != nullptr;
    const int seg_lo = a.seg.seg_off[m];
    const uint8_t* keep = filter ? a.keep_chunks + a.seg.chunk_cum[m] : nullptr;

    for (int base = lo; base < hi; base += kKeysPerStep) {
      float s[4];
      float tmax = -INFINITY;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int j = base + lane + 64 * t;
        bool vis = j < hi;
        if (vis && filter) vis = keep[(j - seg_lo) / a.chunk_tokens] != 0;
        s[t] = vis ? a.scale * RowLoad<T>::dot(qs, k + ((int64_t)j * a.Hkv + g) * D, D) : -INFINITY;
        tmax = fmaxf(tmax, s[t]);
      }
      tmax = wave_max(tmax);
      if (tmax == -INFINITY) continue;  // wave-uniform
      const float m_new = fmaxf(m_run, tmax);
      const float alpha = expf(m_run - m_new);  // exp(-inf) = 0 on the first visible step
      float psum = 0.f;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float p = expf(s[t] - m_new);  // masked keys: exp(-inf) = 0
        ps[lane + 64 * t] = p;
        psum += p;
      }
      l_run = l_run * alpha + wave_sum(psum);
      m_run = m_new;
#pragma unroll
      for (int dd = 0; dd < 4; ++dd) acc[dd] *= alpha;
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
      const int cnt = min(kKeysPerStep, hi - base);
      for (int jj = 0; jj < cnt; ++jj) {
        const float p = ps[jj];
        if (p == 0.f) continue;  // wave-uniform (same address for all lanes)
        const T* vrow = v + ((int64_t)(base + jj) * a.Hkv + g) * D;
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) {
          const int d = lane + 64 * dd;
          if (d < D) acc[dd] = fmaf(p, RowLoad<T>::at(vrow + d), acc[dd]);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }

  const float inv = l_run > 0.f ? 1.f / l_run : 0.f;
#pragma unroll
  for (int dd = 0; dd < 4; ++dd) {
    const int d = lane + 64 * dd;
    if (d < D) RowLoad<T>::store(out + ((int64_t)i * a.Hq + h) * D + d, acc[dd] * inv);
  }
}

}  // namespace

hipError_t launch_prefill_generic(const PrefillArgs& a, int n_blocks, int dtype, hipStream_t s) {
  const int64_t n_pairs = (int64_t)a.total * a.Hq;
  if (n_pairs == 0 || n_blocks == 0) return hipSuccess;
  dim3 grid((unsigned)((n_pairs + 3) / 4), (unsigned)n_blocks, 1);
  if (dtype == FEDATTN_F32)
    hipLaunchKernelGGL(prefill_rows_kernel<float>, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(prefill_rows_kernel<uint16_t>, grid, dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace fedattn
