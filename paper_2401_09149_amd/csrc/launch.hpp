// Host-side launchers, one per kernel file, called by the C-ABI entry points.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "attn_common.hpp"

namespace ie {

// Records the HIP error text for ie_attn_last_hip_error() and returns IE_ERR_HIP.
int hip_fail(hipError_t e);

int launch_fwd(AttnParams p, int D, hipStream_t st);
int launch_fwd_wide(AttnParams p, hipStream_t st);  // head dimension 128
// phases: bit 0 delta, bit 1 dq, bit 2 dk/dv
int launch_bwd(AttnParams p, int D, int phases, hipStream_t st);

constexpr int kMaxDevices = 64;   // per-device host state is kept for device ordinals below this

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Compute units of the current device (cached per device); 0 and *err set if the runtime refuses.
inline int cu_count(hipError_t* err) {
  static std::atomic<int> cus_of[kMaxDevices];
  int dev = 0;
  if ((*err = hipGetDevice(&dev)) != hipSuccess) return 0;
  int cus = dev < kMaxDevices ? cus_of[dev].load(std::memory_order_relaxed) : 0;
  if (cus == 0) {
    if ((*err = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return 0;
    if (dev < kMaxDevices) cus_of[dev].store(cus, std::memory_order_relaxed);
  }
  return cus;
}

// Number of `ts`-token tiles per head the grid must cover (upper bound when packed:
// every document adds at most one partial tile).
inline int64_t tiles_per_head(int64_t S, int64_t ts, const int32_t* cu, int32_t num_docs) {
  return cu ? S / ts + num_docs : ceil_div(S, ts);
}

// Head dimension 128 has two forward kernels and two workgroup sizes of the recomputing dQ kernel: 256-row items
// (one persistent workgroup per CU, the faster steady state) and 128-row items (two workgroups per CU).  With few
// 256-row items per CU a launch is as long as its heaviest item, and a 256-row item costs about 15 us around its
// key loop, as much as four of its key tiles; measured on dense causal shapes from 4K x 24 heads to 16K x 16 heads,
// the 128-row forward wins up to 4K tokens at any head count and at 8K below 2 items per CU, the 128-row dQ only at
// 8K and above below 2 items per CU.  `items_256`: 256-row items of the launch; `S`: tokens per batch entry.
inline bool few_items(int64_t items_256) {
  hipError_t e;
  const int cus = cu_count(&e);
  return cus > 0 && items_256 < 2 * (int64_t)cus;
}
// (`tile_rows_setting`: 0 = choose as above, 128 or 256 = the caller's choice, see ie_attn_set_tile_rows)
inline std::atomic<int> tile_rows_setting{0};
inline bool fwd_prefers_128_rows(int64_t items_256, int64_t S, bool packed) {
  const int forced = tile_rows_setting.load(std::memory_order_relaxed);
  if (forced) return forced == 128;
  return !packed && (S <= 4096 || (S <= 8192 && few_items(items_256)));
}
inline bool dq_prefers_128_rows(int64_t items_256, int64_t S, bool packed) {
  const int forced = tile_rows_setting.load(std::memory_order_relaxed);
  if (forced) return forced == 128;
  return !packed && S >= 8192 && few_items(items_256);
}

constexpr int kErrShape = -2;  // IE_ERR_SHAPE
constexpr int kErrBusy = -7;   // IE_ERR_BUSY

template <typename K>
inline int set_smem(K kernel, int bytes) {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  return e == hipSuccess ? 0 : hip_fail(e);
}

}  // namespace ie
