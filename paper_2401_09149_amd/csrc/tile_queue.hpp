// Work queue of a persistent launch: the grid is one workgroup per CU (times the kernel's
// occupancy) and every workgroup takes (head, tile) items until none are left, instead of one
// workgroup per item.  Two things are gained over leaving the distribution to the hardware
// dispatcher.  (1) With one resident workgroup per CU, the dispatcher can only start the next
// workgroup after the previous one has gone; measured on the forward kernel that gap (dispatch
// plus prologue) is 14 us per workgroup, 3 % of the kernel.  (2) The dispatcher deals workgroups
// to the 8 XCDs round-robin, an equal share each, but under load the XCDs do not run at one
// clock (6 % apart in the same kernel), so the slowest XCD finishes late while the others idle.
// Here every XCD has its own list (the items of "its" heads, in the order decode_tile defines, so
// that the workgroups of an XCD still stream the same head's K/V through its L2 together), and a
// workgroup whose list is empty takes from the next XCD's list.
//
// The counters of a launch (kQueueBytes, `AttnParams::q_counters`) are memory that belongs to
// that launch alone: the backward kernels take them from the caller's workspace, the forward from
// a pool of slots whose use the host tracks with events (attn_fwd_wide.hip).  They have to be zeros when the main
// kernel starts: the backward's are cleared by the call's first kernel (or, when a call runs single kernels, by a
// one-wave kernel in front of each), the forward's slots start out as zeros and are left so by every launch
// (queue_leave).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

#include "attn_common.hpp"
#include "launch.hpp"

namespace ie {

constexpr int kQueueBytes = 64;   // 8 list counters, one counter of workgroups that have left (queue_leave), padding

static __global__ void tile_queue_reset_kernel(unsigned int* counters) {
  if (threadIdx.x < kQueueBytes / 4) counters[threadIdx.x] = 0u;
}

// The XCD this wave runs on (0..7).
__device__ __forceinline__ uint32_t xcc_id() {
  uint32_t x;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(x));
  return x & 7u;
}

// The next item of this launch for the calling workgroup, or -1 when all lists are empty.  All
// threads of the workgroup call it; it contains two barriers, so on return everyone has left the
// previous item (its LDS is free) and sees the same result.  `skip` (per workgroup, starts at 0)
// remembers how many lists were already found empty.
// `s_work` points at the workgroup's queue state in LDS, which queue_init() has set up.
struct QueueState { unsigned int* counters; int work; };
__device__ __forceinline__ void queue_init(const AttnParams& p, QueueState* s) {
  // (the counters' address is parked in LDS: held in scalar registers through an item's main loop it would
  // cost the one-wave-per-SIMD kernels registers they do not have)
  if (threadIdx.x == 0) s->counters = p.q_counters;
}
__device__ __forceinline__ int next_work(const AttnParams& p, QueueState* s_work, uint32_t xcc, int& skip) {
  __syncthreads();
  if (threadIdx.x == 0) {
    int w = -1;
    unsigned int* next = s_work->counters;
    if (p.q_per_xcd > 0) {
      for (; skip < 8; ++skip) {
        const uint32_t x = (xcc + (uint32_t)skip) & 7u;
        const unsigned int s = atomicAdd(next + x, 1u);
        if (s < (unsigned int)p.q_per_xcd) { w = (int)(s * 8u + x); break; }
      }
    } else {
      const unsigned int s = atomicAdd(next, 1u);
      if (s < (unsigned int)p.q_total) w = (int)s;
    }
    s_work->work = w;
  }
  __syncthreads();
  return (int)uniform((uint32_t)s_work->work);
}

// For launches whose counters are NOT cleared in front of them (the forward's slots, which start out as zeros): every
// workgroup calls this once, after its last next_work(); the last one to do so, which knows that nobody will touch the
// counters again, clears them for the slot's next launch.
__device__ __forceinline__ void queue_leave(QueueState* s_work) {
  if (threadIdx.x == 0) {
    unsigned int* c = s_work->counters;
    if (atomicAdd(c + 8, 1u) == gridDim.x - 1) {
#pragma unroll
      for (int i = 0; i < 9; ++i) __hip_atomic_store(c + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Per kernel and device: the dynamic LDS limit is raised once, and the number of workgroups of `kernel`
// that fit on one CU together (registers, LDS; at least 1) is asked once.
struct KernelSetup { std::atomic<int> per_cu[kMaxDevices]; };
template <typename K>
static inline int kernel_setup(KernelSetup& ks, K kernel, int smem_bytes, int* per_cu, int threads = kThreads) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e);
  int n = dev < kMaxDevices ? ks.per_cu[dev].load(std::memory_order_acquire) : 0;
  if (n == 0) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes);
    if (e != hipSuccess) return hip_fail(e);
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void*>(kernel), threads, (size_t)smem_bytes) != hipSuccess || n < 1) n = 1;
    if (dev < kMaxDevices) ks.per_cu[dev].store(n, std::memory_order_release);
  }
  *per_cu = n;
  return 0;
}

// Host side: fills the queue fields of `p` for `total` items (= tiles per head x B x heads) with the
// launch's own `counters` (device memory, kQueueBytes) and clears them on `st` (unless they are clear already).  Returns the grid size for
// `per_cu` resident workgroups per CU.
struct QueueLaunch { int grid; hipError_t err; };
static inline QueueLaunch tile_queue_prepare(AttnParams& p, unsigned int* counters, int64_t total, int heads, int per_cu, hipStream_t st,
                                             bool already_clear = false) {
  QueueLaunch r{0, hipSuccess};
  const int cus = cu_count(&r.err);
  if (r.err != hipSuccess) return r;
  const int64_t nH = p.B * heads;
  p.q_counters = counters;
  p.q_total = (int32_t)total;
  p.q_per_xcd = (nH % 8 == 0) ? (int32_t)(total / 8) : 0;
  p.q_heavy = p.tiles - p.tiles * 3 / 8;   // (at 4K-16K the split makes no measurable difference; at 32K 0 % and 30 % are 1-4 % slower)
  const int64_t want = (int64_t)cus * per_cu;
  r.grid = (int)(total < want ? total : want);
  // (`already_clear`: a kernel in front of this launch on the same stream has cleared the counters)
  if (!already_clear) {
    tile_queue_reset_kernel<<<1, 64, 0, st>>>(counters);
    r.err = hipGetLastError();
  }
  return r;
}

}  // namespace ie
