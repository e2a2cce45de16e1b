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
// The counters live in a file-scope device array (one copy per translation unit that includes
// this header, and per device); a launch uses one slot of it, cleared by a one-wave kernel on
// the same stream in front of the main kernel.  Slots rotate per launch, so launches that overlap
// on different streams do not share a slot unless kQueueSlots of them are in flight at once.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>

#include "attn_common.hpp"
#include "launch.hpp"

namespace ie {

constexpr int kQueueSlots = 256;
struct TileQueue { unsigned int next[8]; };
static __device__ TileQueue g_tile_queue[kQueueSlots];

static __global__ void tile_queue_reset_kernel(int slot) {
  if (threadIdx.x < 8) g_tile_queue[slot].next[threadIdx.x] = 0u;
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
__device__ __forceinline__ int next_work(const AttnParams& p, int* s_work, uint32_t xcc, int& skip) {
  __syncthreads();
  if (threadIdx.x == 0) {
    int w = -1;
    unsigned int* next = g_tile_queue[p.q_slot].next;
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
    *s_work = w;
  }
  __syncthreads();
  return (int)uniform((uint32_t)*s_work);
}

// Workgroups of `kernel` that fit on one CU together (registers, LDS); at least 1.
template <typename K>
static inline int resident_per_cu(K kernel, int smem_bytes) {
  int n = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, reinterpret_cast<const void*>(kernel), kThreads, (size_t)smem_bytes) != hipSuccess) n = 1;
  return n < 1 ? 1 : n;
}

// Host side: fills the queue fields of `p` for `total` items (= tiles per head x B x heads) and
// clears the slot on `st`.  Returns the grid size for `per_cu` resident workgroups per CU.
// (static: every translation unit that includes this header has its own counter array and reset kernel,
// and must call its own copy of this function; a shared inline copy would clear one unit's array for all.)
struct QueueLaunch { int grid; hipError_t err; };
static inline QueueLaunch tile_queue_prepare(AttnParams& p, int64_t total, int heads, int per_cu, hipStream_t st) {
  static std::atomic<unsigned int> next_slot{0};
  QueueLaunch r{0, hipSuccess};
  const int cus = cu_count(&r.err);
  if (r.err != hipSuccess) return r;
  const int64_t nH = p.B * heads;
  p.q_slot = (int32_t)(next_slot.fetch_add(1u, std::memory_order_relaxed) % kQueueSlots);
  p.q_total = (int32_t)total;
  p.q_per_xcd = (nH % 8 == 0) ? (int32_t)(total / 8) : 0;
  const int64_t want = (int64_t)cus * per_cu;
  r.grid = (int)(total < want ? total : want);
  tile_queue_reset_kernel<<<1, 64, 0, st>>>(p.q_slot);
  r.err = hipGetLastError();
  return r;
}

}  // namespace ie
