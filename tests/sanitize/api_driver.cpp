// Driver for the AddressSanitizer / UndefinedBehaviorSanitizer build of the library's host side:
// every entry point is called with arguments that must be rejected (or accepted as an empty
// problem) by validation, before any kernel would be enqueued.  No GPU is needed; the pointers
// that stand for device memory are never dereferenced on the host.  Exit status 0 = every call
// returned the expected status and the sanitizers saw nothing.
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "fedattn.h"

static int failures = 0;
#define EXPECT(call, want)                                                                         \
  do {                                                                                             \
    const int got_ = (int)(call);                                                                  \
    if (got_ != (int)(want)) {                                                                     \
      std::fprintf(stderr, "line %d: %s returned %d (%s), expected %d\n", __LINE__, #call, got_,   \
                   fedattn_last_error(), (int)(want));                                             \
      ++failures;                                                                                  \
    }                                                                                              \
  } while (0)

int main() {
  fedattn_params ok = {3, 8, 2, 128, 2, 1, FEDATTN_BF16, 0.f};
  void* dev = reinterpret_cast<void*>(0x7000000000ull);     // stands for device memory; never read here
  void* odd = reinterpret_cast<void*>(0x7000000008ull);     // misaligned
  std::vector<int32_t> seg = {0, 64, 64, 200};
  std::vector<int32_t> lens = {64, 0, 100};

  EXPECT(fedattn_is_sync_block(2, 1), 1);
  EXPECT(fedattn_is_sync_block(2, 2), 0);
  EXPECT(fedattn_is_sync_block(-1, 5), 0);

  // parameter checks, one broken field at a time
  for (int field = 0; field < 7; ++field) {
    fedattn_params p = ok;
    switch (field) {
      case 0: p.n_participants = 0; break;
      case 1: p.n_participants = FEDATTN_MAX_PARTICIPANTS + 1; break;
      case 2: p.n_kv_heads = 3; break;
      case 3: p.head_dim = 100; break;
      case 4: p.dtype = 7; break;
      case 5: p.softmax_scale = -1.f; break;
      case 6: p.causal = 2; break;
    }
    EXPECT(fedattn_prefill(&p, 0, dev, dev, dev, dev, seg.data(), nullptr, 0, -1, nullptr, 0, nullptr), FEDATTN_EINVAL);
    EXPECT(fedattn_decode(&p, 0, dev, dev, dev, dev, seg.data(), lens.data(), nullptr, -1, dev, 1 << 20, nullptr), FEDATTN_EINVAL);
    EXPECT(fedattn_workspace_bytes(&p, FEDATTN_OP_DECODE, 200, 0), 0);
  }
  EXPECT(fedattn_prefill(nullptr, 0, dev, dev, dev, dev, seg.data(), nullptr, 0, -1, nullptr, 0, nullptr), FEDATTN_EINVAL);

  // prefill: offsets, pointers, alignment, overrides, workspace
  std::vector<int32_t> bad_seg = {0, 80, 64, 200};
  EXPECT(fedattn_prefill(&ok, 0, dev, dev, dev, dev, bad_seg.data(), nullptr, 0, -1, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill(&ok, 0, dev, dev, dev, dev, nullptr, nullptr, 0, -1, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill(&ok, 0, nullptr, dev, dev, dev, seg.data(), nullptr, 0, -1, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill(&ok, 0, odd, dev, dev, dev, seg.data(), nullptr, 0, -1, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill(&ok, -1, dev, dev, dev, dev, seg.data(), nullptr, 0, -1, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill(&ok, 0, dev, dev, dev, dev, seg.data(), nullptr, 0, 2, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill(&ok, 1, dev, dev, dev, dev, seg.data(), static_cast<const uint8_t*>(dev), 0, -1, nullptr, 0, nullptr),
         FEDATTN_EINVAL);      // keep-list without a chunk size
  EXPECT(fedattn_prefill(&ok, 1, dev, dev, dev, dev, seg.data(), static_cast<const uint8_t*>(dev), 64, -1, nullptr, 0, nullptr),
         FEDATTN_EWORKSPACE);  // keep-list in a sync block without a workspace
  std::vector<int32_t> empty_seg = {0, 0, 0, 0};
  EXPECT(fedattn_prefill(&ok, 0, nullptr, nullptr, nullptr, nullptr, empty_seg.data(), nullptr, 0, -1, nullptr, 0, nullptr), FEDATTN_OK);
  EXPECT(fedattn_prefill_blocks(&ok, 0, 4, dev, dev, dev, dev, 12, 16, seg.data(), nullptr), FEDATTN_EINVAL);   // stride not a multiple of 8
  EXPECT(fedattn_prefill_blocks(&ok, 0, 70000, dev, dev, dev, dev, 16, 16, seg.data(), nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill_blocks(&ok, 0, 0, dev, dev, dev, dev, 16, 16, seg.data(), nullptr), FEDATTN_OK);

  // Phase II from local matrices: NULL tables, NULL / misaligned entries, matrices apart without a workspace
  const void* kl[3] = {dev, nullptr, static_cast<char*>(dev) + 64 * 2 * 128 * 2};
  const void* apart[3] = {dev, nullptr, static_cast<char*>(dev) + (1 << 20)};
  const void* with_null[3] = {dev, nullptr, nullptr};
  const void* with_odd[3] = {odd, nullptr, dev};
  EXPECT(fedattn_prefill_sync_local_kv(&ok, dev, nullptr, kl, dev, seg.data(), nullptr, 0, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill_sync_local_kv(&ok, dev, with_null, kl, dev, seg.data(), nullptr, 0, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill_sync_local_kv(&ok, dev, with_odd, kl, dev, seg.data(), nullptr, 0, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill_sync_local_kv(&ok, dev, apart, apart, dev, seg.data(), nullptr, 0, nullptr, 0, nullptr), FEDATTN_EWORKSPACE);
  EXPECT(fedattn_prefill_sync_local_kv(&ok, nullptr, kl, kl, dev, seg.data(), nullptr, 0, nullptr, 0, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_prefill_sync_local_kv(&ok, dev, kl, kl, dev, empty_seg.data(), nullptr, 0, nullptr, 0, nullptr), FEDATTN_OK);
  if (fedattn_workspace_bytes(&ok, FEDATTN_OP_PREFILL_SYNC_LOCAL_KV, 200, 0) < 2u * 200 * 2 * 128 * 2) ++failures;

  // decode: lengths against capacities, workspace, strides, fused block count, the built-in scratch limit
  std::vector<int32_t> cap = {0, 100, 200, 300};
  std::vector<int32_t> too_long = {101, 0, 5};
  EXPECT(fedattn_decode(&ok, 0, dev, dev, dev, dev, cap.data(), too_long.data(), nullptr, -1, dev, 1 << 24, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_decode(&ok, 0, dev, dev, dev, dev, cap.data(), lens.data(), too_long.data(), -1, dev, 1 << 24, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_decode(&ok, 0, dev, dev, dev, dev, cap.data(), nullptr, nullptr, -1, dev, 1 << 24, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_decode(&ok, 0, dev, dev, dev, dev, cap.data(), lens.data(), nullptr, -1, nullptr, 0, nullptr), FEDATTN_EWORKSPACE);
  EXPECT(fedattn_decode(&ok, 0, dev, dev, dev, dev, cap.data(), lens.data(), nullptr, -1, dev, 64, nullptr), FEDATTN_EWORKSPACE);
  EXPECT(fedattn_decode(&ok, 0, dev, dev, dev, dev, cap.data(), lens.data(), nullptr, -1, odd, 1 << 24, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_decode_blocks(&ok, 0, 2, dev, dev, dev, dev, 12, 16, cap.data(), lens.data(), nullptr, -1, dev, 1 << 24, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_decode_blocks(&ok, 0, 0, dev, dev, dev, dev, 16, 16, cap.data(), lens.data(), nullptr, -1, nullptr, 0, nullptr), FEDATTN_OK);
  EXPECT(fedattn_decode_blocks_fused(&ok, 0, 70000, dev, dev, dev, dev, 16, 16, cap.data(), lens.data(), nullptr, -1, dev, 1 << 24, nullptr),
         FEDATTN_EINVAL);
  fedattn_params wide = {128, 64, 8, 128, 1, 1, FEDATTN_BF16, 0.f};
  std::vector<int32_t> cap128(129), len128(128, 64);
  for (int n = 0; n <= 128; ++n) cap128[n] = 64 * n;
  EXPECT(fedattn_decode_static(&wide, 0, dev, dev, dev, dev, cap128.data(), len128.data(), nullptr, -1, nullptr), FEDATTN_EWORKSPACE);
  EXPECT(fedattn_decode_static(&ok, 0, dev, dev, dev, dev, cap.data(), too_long.data(), nullptr, -1, nullptr), FEDATTN_EINVAL);

  // aggregation and the element-wise block kernels
  EXPECT(fedattn_aggregate_kv(&ok, nullptr, kl, seg.data(), dev, dev, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_aggregate_kv(&ok, with_null, kl, seg.data(), dev, dev, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_aggregate_kv(&ok, kl, kl, seg.data(), odd, dev, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_aggregate_kv(&ok, kl, kl, empty_seg.data(), nullptr, nullptr, nullptr), FEDATTN_OK);
  EXPECT(fedattn_rmsnorm(static_cast<float*>(dev), dev, 4, 6, 1e-6f, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_rmsnorm(static_cast<float*>(dev), dev, 0, 8, 1e-6f, nullptr), FEDATTN_OK);
  EXPECT(fedattn_residual_add_rmsnorm(static_cast<float*>(dev), nullptr, dev, 4, 8, 1e-6f, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_residual_add_rmsnorm(static_cast<float*>(dev), dev, dev, 4, 8, -1.f, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_rope_split_qkv(dev, nullptr, dev, dev, dev, 4, 2, 1, 12, 10000.f, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_rope_split_qkv(dev, nullptr, dev, dev, dev, 4, 2, 1, 16, 0.5f, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_swiglu(dev, dev, 4, 12, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_residual_add(static_cast<float*>(dev), dev, 6, nullptr), FEDATTN_EINVAL);
  EXPECT(fedattn_residual_add(static_cast<float*>(dev), dev, 0, nullptr), FEDATTN_OK);

  if (std::strlen(fedattn_version()) == 0) ++failures;
  if (failures) {
    std::fprintf(stderr, "api driver: %d check(s) failed\n", failures);
    return 1;
  }
  std::printf("api driver: clean\n");
  return 0;
}
