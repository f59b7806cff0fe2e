// Measurement aids, not part of the method: two kernels that give the benchmark the rates this
// GPU reaches on the bare resources the attention kernels are bound by, measured on the same
// box in the same run as the kernels themselves.
//   stream probe: reads a buffer through LDS rings with the direct HBM -> LDS loads of the
//     decode kernel and does nothing else.  Contiguous: every workgroup reads one contiguous
//     share.  Cache layout: the access pattern of the decode kernel on a [rows, Hkv, D] bf16
//     cache with Hkv = 8, D = 128: workgroup (chunk, head) reads 256-byte pieces at a 2 KB stride
//     from a K and from a V array, 64 rows per tile.
//   MFMA probe: a loop of v_mfma_f32_32x32x16_bf16 on register operands, two wavefronts per SIMD.
#include "common.h"
#include "mfma_tile.h"

namespace fedattn {

namespace {

constexpr int kProbeTile = 32768;   // bytes per ring stage (a 64-row K tile and its V tile at D = 128)
constexpr int kProbeStages = 3;

// pattern 0: workgroup b reads bytes [b * per_wg, (b + 1) * per_wg) in 32 KB tiles.
// pattern 1: workgroup b = chunk * 8 + head reads `rows` rows of 256 bytes at stride 2048 bytes from K (at src) and
//            from V (at src + v_offset), 64 rows of each per tile.
__global__ __launch_bounds__(256, 1) void stream_probe_kernel(const unsigned char* src, int64_t per_wg, int rows,
                                                              int64_t v_offset, int pattern, float* sink) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds_base = lds_addr_of(smem);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int IPW = kProbeTile / 1024 / 4;   // load instructions per wavefront and tile
  const int nt = pattern == 0 ? (int)(per_wg / kProbeTile) : rows / 64;
  const unsigned char* base = pattern == 0 ? src + (int64_t)blockIdx.x * per_wg
                                           : src + ((int64_t)(blockIdx.x / 8) * rows) * 2048 + (blockIdx.x % 8) * 256;
  auto issue = [&](int t) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int inst = wave * IPW + i;   // 0..31
      const uint32_t lds = lds_base + (t % kProbeStages) * kProbeTile + inst * 1024;
      if (pattern == 0) {
        lds_dma_16<true>(base + (int64_t)t * kProbeTile, (uint32_t)(inst * 1024 + lane * 16), lds);
      } else {
        const int unit = (inst & 15) * 64 + lane;   // 16-byte unit of a 64 x 256 byte tile
        const unsigned char* b = base + (inst < 16 ? 0 : v_offset) + (int64_t)t * 64 * 2048;
        lds_dma_16<true>(b, (uint32_t)((unit / 16) * 2048 + (unit % 16) * 16), lds);
      }
    }
  };
#pragma unroll
  for (int t = 0; t < kProbeStages - 1; ++t)
    if (t < nt) issue(t);
  float acc = 0.f;
  for (int t = 0; t < nt; ++t) {
    if (min(nt, t + kProbeStages - 1) - (t + 1) >= 1)
      wait_vmcnt<IPW>();
    else
      wait_vmcnt<0>();
    __syncthreads();
    if (t + kProbeStages - 1 < nt) issue(t + kProbeStages - 1);
    acc += *reinterpret_cast<const float*>(smem + (t % kProbeStages) * kProbeTile + tid * 16);
  }
  if (acc == 123.456f) sink[blockIdx.x] = acc;   // keeps the reads alive
}

__global__ __launch_bounds__(512, 1) void mfma_probe_kernel(float* sink, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (bf16_t)(0.001f * (float)(threadIdx.x + e));
    b[e] = (bf16_t)(1.0f + 0.01f * (float)e);
  }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int it = 0; it < iters; ++it)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i & 3], 0, 0, 0);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[i][e];
  if (s == 123.456f) sink[blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_stream_probe(const void* src, int64_t bytes, int n_wgs, int pattern, float* sink, hipStream_t s) {
  static std::atomic<uint64_t> attr_done{0};
  hipError_t e = set_max_dynamic_lds_once(attr_done, reinterpret_cast<const void*>(&stream_probe_kernel),
                                          kProbeStages * kProbeTile);
  if (e != hipSuccess) return e;
  int64_t per_wg = 0, v_offset = 0;
  int rows = 0;
  if (pattern == 0) {
    per_wg = bytes / n_wgs / kProbeTile * kProbeTile;
  } else {
    rows = (int)(bytes / 2 / 256 / n_wgs / 64 * 64);       // rows per workgroup: K and V halves, 256 bytes per row and head
    v_offset = (int64_t)(n_wgs / 8) * rows * 2048;         // the V array follows the K array
  }
  hipLaunchKernelGGL(stream_probe_kernel, dim3((unsigned)n_wgs), dim3(256), kProbeStages * kProbeTile, s,
                     reinterpret_cast<const unsigned char*>(src), per_wg, rows, v_offset, pattern, sink);
  return hipGetLastError();
}

hipError_t launch_mfma_probe(float* sink, int n_wgs, int iters, hipStream_t s) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)n_wgs), dim3(512), 0, s, sink, iters);
  return hipGetLastError();
}

}  // namespace fedattn
