// KV aggregation of a sync block (Phase II): [K V] = sum_n Pi_n [k_n v_n].  Pi_n's
// columns are the basis vectors of participant n's global positions, so the sum is
// a scatter of every local row to its global row - with contiguous segments, a
// copy of each participant's matrices to offset seg_off[n].  Pure HBM traffic:
// 16-byte loads and stores, one grid row per (participant, tensor).
#include "common.h"

namespace fedattn {

namespace {

__global__ __launch_bounds__(256) void aggregate_kv_kernel(AggregateArgs a) {
  const int n = blockIdx.y >> 1;
  const bool is_v = blockIdx.y & 1;
  const int lo = a.seg_off[n], hi = a.seg_off[n + 1];
  const int64_t units = (int64_t)(hi - lo) * (a.row_bytes / 16);
  const uint4* src = reinterpret_cast<const uint4*>(is_v ? a.v_local[n] : a.k_local[n]);
  uint4* dst = reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(is_v ? a.v_global : a.k_global) +
                                        (int64_t)lo * a.row_bytes);
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  // four loads in flight per thread before the first store: the copy is a chain of memory
  // round trips otherwise (a launch moves a few MB, i.e. a handful of units per thread)
  for (int64_t u = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; u < units; u += 4 * stride) {
    // loads past the end re-read the last unit (no branch between the loads); their stores are skipped
    const int64_t u1 = u + stride, u2 = u + 2 * stride, u3 = u + 3 * stride, last = units - 1;
    const uint4 r0 = src[u];
    const uint4 r1 = src[u1 < units ? u1 : last];
    const uint4 r2 = src[u2 < units ? u2 : last];
    const uint4 r3 = src[u3 < units ? u3 : last];
    dst[u] = r0;
    if (u1 < units) dst[u1] = r1;
    if (u2 < units) dst[u2] = r2;
    if (u3 < units) dst[u3] = r3;
  }
}

}  // namespace

hipError_t launch_aggregate(const AggregateArgs& a, hipStream_t s) {
  const int total = a.seg_off[a.n];
  if (total == 0) return hipSuccess;
  int max_len = 0;
  for (int n = 0; n < a.n; ++n) max_len = max(max_len, a.seg_off[n + 1] - a.seg_off[n]);
  const int64_t max_units = (int64_t)max_len * (a.row_bytes / 16);
  // enough workgroups per (participant, tensor) to cover the chip a few times over
  int64_t gx = (max_units + 256 * 4 - 1) / (256 * 4);
  const int64_t cap = (2048 + 2 * a.n - 1) / (2 * a.n);
  if (gx > cap) gx = cap;
  if (gx < 1) gx = 1;
  hipLaunchKernelGGL(aggregate_kv_kernel, dim3((unsigned)gx, (unsigned)(2 * a.n)), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace fedattn
