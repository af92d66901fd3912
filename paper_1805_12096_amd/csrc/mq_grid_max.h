// Grid-wide agreement on a maximum inside one launch, for kernels whose workgroups are all resident.
//
// Per-tensor abs-max quantization (arxiv 1805.12096, Section 4.2, with the multiplier taken from the
// tensor) needs max|x| over the whole tensor before the first element can be converted.  When the data
// of every workgroup fits its registers, one launch can do both: each workgroup publishes the maximum
// of its share, waits until all shares are known, and converts from registers.
//
// Protocol.  `barrier` points to kBarrierWords words that are zero when the kernel starts.  Workgroup b
// stores the bit pattern of its (non-negative, non-NaN) maximum, plus one, in word b (of every copy of the slot array); bit patterns of
// such floats order like unsigned integers.  Then it reads all words until none is zero: the read that
// ends the wait also delivers every maximum.  Only device-scope stores and loads touch these words: no
// counter, no read-modify-write on a shared address, no cache write-back or invalidation.  The wait
// is bounded in wall-clock time.  A workgroup that gives up first raises the sticky word behind the
// slots, then reads once more; if values are still missing it goes on with a meaningless result.
// Whoever publishes the tensor's multiplier looks at the sticky word after its last store, which is
// later than any complete read, and must publish NaN instead if it is raised, so that nothing computed
// from this launch can pass for a result.
//
// Requirements on the caller: gridDim.x <= kBarrierSlots, all workgroups resident at the same time (the
// launcher checks with the occupancy query), one launch at a time per barrier area.
#pragma once

#include <hip/hip_runtime.h>

#include "mq_internal.h"

namespace mq {

constexpr unsigned kBarrierSlots = 256;
// Every workgroup's value is stored in kBarrierCopies copies of the slot array and a workgroup polls only copy
// blockIdx.x % kBarrierCopies: loads of one cache line from the whole chip are served one after the other
// (about 12 ns each), so 256 pollers on one copy would take 3 us per round, 32 take 0.4 us.
constexpr unsigned kBarrierCopies = 8;
static_assert(kBarrierSlots % 64 == 0 && kBarrierCopies * kBarrierSlots + 2 <= kBarrierWords, "barrier layout");
// Word behind the sticky one: counts the workgroups that are done with the area (see grid_max_retire).
constexpr unsigned kBarrierDoneWord = kBarrierCopies * kBarrierSlots + 1;

// Maximum of an unsigned value over the 64 lanes, the same in every lane: inside rows of 16 lanes by
// data-parallel-primitive moves (swap neighbours, swap pairs, mirror the half rows, mirror the rows),
// across the four rows through scalar registers.
__device__ __forceinline__ unsigned wave_max_u32(unsigned x) {
  x = max(x, (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true));    // quad_perm [1,0,3,2]
  x = max(x, (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, true));    // quad_perm [2,3,0,1]
  x = max(x, (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, true));   // row_half_mirror
  x = max(x, (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x140, 0xF, 0xF, true));   // row_mirror
  const unsigned a = __builtin_amdgcn_readlane((int)x, 0), b = __builtin_amdgcn_readlane((int)x, 16);
  const unsigned c = __builtin_amdgcn_readlane((int)x, 32), d = __builtin_amdgcn_readlane((int)x, 48);
  return max(max(a, b), max(c, d));
}

// One thread of the workgroup publishes the workgroup's maximum m (m >= 0, not NaN).
__device__ __forceinline__ void grid_max_publish(unsigned* barrier, float m) {
#pragma unroll
  for (unsigned c = 0; c < kBarrierCopies; ++c)
    __hip_atomic_store(barrier + c * kBarrierSlots + blockIdx.x, __float_as_uint(m) + 1u, __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

// Called by all 64 lanes of ONE wave of the workgroup after grid_max_publish: waits for every workgroup's
// value (at most `ticks` ticks of the 100 MHz wall clock) and returns the maximum over the grid in
// every lane.
__device__ __forceinline__ float grid_max_collect(unsigned* barrier, unsigned long long ticks) {
  const int lane = threadIdx.x % 64;
  const unsigned total = gridDim.x;
  const unsigned* mine = barrier + (blockIdx.x % kBarrierCopies) * kBarrierSlots;
  const unsigned long long t0 = wall_clock64();       // the same value in every lane
  unsigned best;
  bool gave_up = false;
  for (;;) {
    best = 1u;
    bool all = true;
#pragma unroll
    for (unsigned k = 0; k < kBarrierSlots / 64; ++k) {
      const unsigned i = lane + 64 * k;
      const unsigned v = i < total ? __hip_atomic_load(mine + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 1u;
      all = all && v != 0u;
      best = max(best, v);
    }
    if (__all(all)) break;
    if (gave_up) break;                                // that was the one read after giving up
    if (wall_clock64() - t0 >= ticks) {
      if (lane == 0) (void)atomicOr(barrier + kBarrierCopies * kBarrierSlots, 1u);
      gave_up = true;
      __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0): the atomic is done before the next read is issued
      continue;
    }
    __builtin_amdgcn_s_sleep(2);
  }
  return __uint_as_float(wave_max_u32(best) - 1u);
}

// For kernels that leave the area as they found it, all zero, so that the next launch needs no clearing launch
// before it.  One thread of every workgroup calls this once, after its workgroup's collect (and, for the workgroup
// that publishes the multiplier, after its look at the sticky word); the value returned to the LAST caller of the
// grid is gridDim.x - 1: by then no workgroup will read or write the area again, and that workgroup zeroes all
// kBarrierWords words.  This is the one read-modify-write on a shared word in the protocol; it is not on the
// path of anybody's wait.
__device__ __forceinline__ unsigned grid_max_retire(unsigned* barrier) {
  return atomicAdd(barrier + kBarrierDoneWord, 1u);
}

// True if some workgroup of this launch gave up waiting (to be read after the caller's own collect).
__device__ __forceinline__ bool grid_max_failed(unsigned* barrier) {
  return __hip_atomic_load(barrier + kBarrierCopies * kBarrierSlots, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u;
}

}  // namespace mq
