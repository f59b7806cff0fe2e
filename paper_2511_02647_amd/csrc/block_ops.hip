// The element-wise pieces of the decoder block around the attention operator in the
// end-to-end configuration: RMSNorm, rotary position embedding (with the split of the
// fused QKV projection into the attention's q, k, v tensors), SwiGLU, the residual add, and
// the residual add fused into the RMSNorm that follows it.  The block structure is the paper's (Section III-B: attention and a feed-forward
// network, each with a residual connection and a normalisation; Section IV-B local
// forward); the Llama-style variants are those of the configuration.  All four are
// bandwidth-bound passes: 16-byte accesses with the nontemporal hint (every element is touched
// once; without the hint RMSNorm ran at 4.9 TB/s instead of 6.5), fp32 arithmetic, bf16 at the
// interfaces, fp32 residual stream.  The matrix products stay plain GEMMs outside this library.
#include "common.h"

namespace fedattn {

namespace {

typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ inline f32x2 bf16_pair(uint32_t w) {
  return f32x2{__uint_as_float(w << 16), __uint_as_float(w & 0xffff0000u)};
}
__device__ inline uint32_t pack_bf16(float a, float b) {
  const bf16x2 p = {(bf16_t)a, (bf16_t)b};
  return __builtin_bit_cast(uint32_t, p);
}

// out[r] = bf16(x[r] / sqrt(mean(x[r]^2) + eps)); one wavefront per row, 4 rows per workgroup.
// ADD: the residual update of the previous half of the block is applied on the way,
// x[r] += y[r] (y bf16), and the updated row is written back: one pass over the fp32 stream
// where the separate residual-add and RMSNorm kernels take two (12 instead of 16 bytes per
// element; same arithmetic in the same order, so the results are those of the two kernels).
template <bool ADD>
__global__ __launch_bounds__(256) void rmsnorm_kernel(float* __restrict__ x, const uint16_t* __restrict__ y,
                                                      uint16_t* __restrict__ out, int64_t rows, int d_model, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  f32x4* xr = reinterpret_cast<f32x4*>(x + r * d_model);
  const u32x2_t* yr = reinterpret_cast<const u32x2_t*>(y + (ADD ? r * d_model : 0));
  const int n4 = d_model / 4;
  u32x2_t* orow = reinterpret_cast<u32x2_t*>(out + r * d_model);
  float ss = 0.f;
  // rows of up to 4096 elements stay in registers between the two passes (16 vectors per lane)
  constexpr int kHeld = 16;
  if (n4 <= kHeld * 64) {
    f32x4 held[kHeld];
    u32x2_t upd[ADD ? kHeld : 1];
#pragma unroll
    for (int j = 0; j < kHeld; ++j) {
      const int i = lane + 64 * j;
      held[j] = i < n4 ? __builtin_nontemporal_load(xr + i) : f32x4{0.f, 0.f, 0.f, 0.f};
      if constexpr (ADD) upd[j] = i < n4 ? __builtin_nontemporal_load(yr + i) : u32x2_t{0u, 0u};
    }
#pragma unroll
    for (int j = 0; j < kHeld; ++j) {
      f32x4 v = held[j];
      if constexpr (ADD) {
        const f32x2 y0 = bf16_pair(upd[j][0]), y1 = bf16_pair(upd[j][1]);
        v[0] += y0[0];
        v[1] += y0[1];
        v[2] += y1[0];
        v[3] += y1[1];
        held[j] = v;
        const int i = lane + 64 * j;
        if (i < n4) __builtin_nontemporal_store(v, xr + i);
      }
      ss += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
    }
    ss = wave_sum(ss);
    const float inv = 1.0f / sqrtf(ss / (float)d_model + eps);
#pragma unroll
    for (int j = 0; j < kHeld; ++j) {
      const int i = lane + 64 * j;
      const f32x4 v = held[j];
      if (i < n4) __builtin_nontemporal_store(u32x2_t{pack_bf16(v[0] * inv, v[1] * inv), pack_bf16(v[2] * inv, v[3] * inv)}, orow + i);
    }
    return;
  }
  for (int i = lane; i < n4; i += 64) {
    f32x4 v = xr[i];
    if constexpr (ADD) {
      const u32x2_t u = yr[i];
      const f32x2 y0 = bf16_pair(u[0]), y1 = bf16_pair(u[1]);
      v[0] += y0[0];
      v[1] += y0[1];
      v[2] += y1[0];
      v[3] += y1[1];
      xr[i] = v;   // read back below by the same lane
    }
    ss += (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
  }
  ss = wave_sum(ss);
  const float inv = 1.0f / sqrtf(ss / (float)d_model + eps);
  for (int i = lane; i < n4; i += 64) {
    const f32x4 v = xr[i];
    orow[i] = u32x2_t{pack_bf16(v[0] * inv, v[1] * inv), pack_bf16(v[2] * inv, v[3] * inv)};
  }
}

// Splits qkv [T, (Hq + 2 Hkv) D] into q [T,Hq,D], k [T,Hkv,D], v [T,Hkv,D] and rotates q and
// k: element i < D/2 pairs with i + D/2, angle = pos * theta^(-2 i / D) (rotate-half form).
// One thread per (token, 4 consecutive i): it computes its 4 angles once (in fp64 up to the
// reduction to [0, 2 pi), positions reach 10^5..10^6) and walks all heads.
__global__ __launch_bounds__(256) void rope_split_kernel(const uint16_t* __restrict__ qkv, const int32_t* __restrict__ pos,
                                                         uint16_t* __restrict__ q, uint16_t* __restrict__ k,
                                                         uint16_t* __restrict__ v, int64_t tokens, int Hq, int Hkv,
                                                         int D, float theta) {
  const int groups = D / 8;  // threads per token: 4 pairs each
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t t = idx / groups;
  if (t >= tokens) return;
  const int i0 = (int)(idx % groups) * 4;
  const double p = pos ? (double)pos[t] : (double)t;
  float c[4], s[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const double inv_freq = exp2(-2.0 * (double)(i0 + e) / (double)D * log2((double)theta));
    double ang = p * inv_freq;
    ang -= floor(ang * 0.15915494309189535) * 6.283185307179586;  // mod 2 pi
    sincosf((float)ang, &s[e], &c[e]);
  }
  const int half = D / 2;
  const int64_t in_row = (int64_t)(Hq + 2 * Hkv) * D;
  const uint16_t* src = qkv + t * in_row;
  for (int h = 0; h < Hq + Hkv; ++h) {
    const uint16_t* sp = src + h * D + i0;
    uint16_t* dp = h < Hq ? q + (t * Hq + h) * D + i0 : k + (t * Hkv + (h - Hq)) * D + i0;
    const u32x2_t lo = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(sp));
    const u32x2_t hi = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(sp + half));
    const f32x2 a0 = bf16_pair(lo[0]), a1 = bf16_pair(lo[1]), b0 = bf16_pair(hi[0]), b1 = bf16_pair(hi[1]);
    const float a[4] = {a0[0], a0[1], a1[0], a1[1]}, b[4] = {b0[0], b0[1], b1[0], b1[1]};
    float ra[4], rb[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      ra[e] = a[e] * c[e] - b[e] * s[e];
      rb[e] = b[e] * c[e] + a[e] * s[e];
    }
    __builtin_nontemporal_store(u32x2_t{pack_bf16(ra[0], ra[1]), pack_bf16(ra[2], ra[3])}, reinterpret_cast<u32x2_t*>(dp));
    __builtin_nontemporal_store(u32x2_t{pack_bf16(rb[0], rb[1]), pack_bf16(rb[2], rb[3])}, reinterpret_cast<u32x2_t*>(dp + half));
  }
  for (int h = 0; h < Hkv; ++h) {
    const uint16_t* sp = src + (Hq + Hkv + h) * D + i0;
    uint16_t* dp = v + (t * Hkv + h) * D + i0;
    __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(sp)), reinterpret_cast<u32x2_t*>(dp));
    __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(sp + half)),
                                reinterpret_cast<u32x2_t*>(dp + half));
  }
}

// out[r][f] = bf16(silu(gate) * up), gate = gate_up[r][f], up = gate_up[r][F + f]; 8 elements per thread.
__global__ __launch_bounds__(256) void swiglu_kernel(const uint16_t* __restrict__ gate_up, uint16_t* __restrict__ out,
                                                     int64_t rows, int F) {
  const int per_row = F / 8;
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t r = idx / per_row;
  if (r >= rows) return;
  const int f = (int)(idx % per_row) * 8;
  const u32x4_t g = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(gate_up + r * 2 * F + f));
  const u32x4_t u = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(gate_up + r * 2 * F + F + f));
  u32x4_t o;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const f32x2 gv = bf16_pair(g[e]), uv = bf16_pair(u[e]);
    const float a = gv[0] / (1.0f + __expf(-gv[0])) * uv[0];
    const float b = gv[1] / (1.0f + __expf(-gv[1])) * uv[1];
    o[e] = pack_bf16(a, b);
  }
  __builtin_nontemporal_store(o, reinterpret_cast<u32x4_t*>(out + r * F + f));
}

// x[i] += y[i] (fp32 residual stream, bf16 update); 4 elements per thread.
__global__ __launch_bounds__(256) void residual_add_kernel(float* __restrict__ x, const uint16_t* __restrict__ y, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  f32x4 xv = __builtin_nontemporal_load(reinterpret_cast<f32x4*>(x) + i);
  const u32x2_t yv = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(y) + i);
  const f32x2 y0 = bf16_pair(yv[0]), y1 = bf16_pair(yv[1]);
  xv[0] += y0[0];
  xv[1] += y0[1];
  xv[2] += y1[0];
  xv[3] += y1[1];
  __builtin_nontemporal_store(xv, reinterpret_cast<f32x4*>(x) + i);
}

}  // namespace

hipError_t launch_rmsnorm(const float* x, void* out, int64_t rows, int d_model, float eps, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(rmsnorm_kernel<false>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, const_cast<float*>(x),
                     static_cast<const uint16_t*>(nullptr), reinterpret_cast<uint16_t*>(out), rows, d_model, eps);
  return hipGetLastError();
}

hipError_t launch_residual_add_rmsnorm(float* x, const void* y, void* out, int64_t rows, int d_model, float eps,
                                       hipStream_t s) {
  if (rows == 0) return hipSuccess;
  hipLaunchKernelGGL(rmsnorm_kernel<true>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, x,
                     reinterpret_cast<const uint16_t*>(y), reinterpret_cast<uint16_t*>(out), rows, d_model, eps);
  return hipGetLastError();
}

hipError_t launch_rope_split(const void* qkv, const int32_t* pos, void* q, void* k, void* v, int64_t tokens, int Hq,
                             int Hkv, int D, float theta, hipStream_t s) {
  if (tokens == 0) return hipSuccess;
  const int64_t threads = tokens * (D / 8);
  hipLaunchKernelGGL(rope_split_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<const uint16_t*>(qkv), pos, reinterpret_cast<uint16_t*>(q),
                     reinterpret_cast<uint16_t*>(k), reinterpret_cast<uint16_t*>(v), tokens, Hq, Hkv, D, theta);
  return hipGetLastError();
}

hipError_t launch_swiglu(const void* gate_up, void* out, int64_t rows, int F, hipStream_t s) {
  if (rows == 0) return hipSuccess;
  const int64_t threads = rows * (F / 8);
  hipLaunchKernelGGL(swiglu_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                     reinterpret_cast<const uint16_t*>(gate_up), reinterpret_cast<uint16_t*>(out), rows, F);
  return hipGetLastError();
}

hipError_t launch_residual_add(float* x, const void* y, int64_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const int64_t n4 = n / 4;
  hipLaunchKernelGGL(residual_add_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, x,
                     reinterpret_cast<const uint16_t*>(y), n4);
  return hipGetLastError();
}

}  // namespace fedattn
