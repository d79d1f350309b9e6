// Chip-wide phase alignment for persistent kernels.
//
// On MI355X a kernel that streams r_g rows in and r_g rows out at the same time reaches about 5.4-5.8 TB/s,
// while the same rows read alone stream at 7.1 TB/s and written alone at 5.8 TB/s: HBM loses time whenever
// reads and writes to many address streams are interleaved.  A persistent grid that makes the whole chip read
// for some tens of microseconds (results parked in registers), then write, then read again, gets most of that
// back.  The alignment below only shapes timing; no data passes between blocks, so it needs no memory ordering,
// and every wait is bounded: a block that has waited `spin_limit` polls simply goes on (the result is the same,
// only slower) and tells the others not to wait either, so the grid drains even if its blocks are not all resident at once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define SOLON_SYNC_GROUPS 8       // arrival counters (blocks are spread over them by blockIdx & 7)
#define SOLON_SYNC_STRIDE 32      // words between counters: 128 bytes, one cache line each
#define SOLON_SYNC_GLOBAL (SOLON_SYNC_GROUPS * SOLON_SYNC_STRIDE)
#define SOLON_SYNC_EXIT (SOLON_SYNC_GLOBAL + SOLON_SYNC_STRIDE)
// polls (a microsecond or two each) before a block gives up at an alignment point: healthy waits are the skew between the blocks of
// one phase, some ten polls; a launch that shares the chip with another stream's kernels should go adrift early (measured with two
// rounds on two streams: 400 polls cost C3 25 % against one stream, 60 polls 8 %; one stream alone is the same at 60 ... 400)
#define SOLON_SPIN_LIMIT 100
#define SOLON_SYNC_ADRIFT_BIT 0x80000000u  // in the grid-wide counter: set once a block has waited in vain, nobody waits any more in this launch

// The nbar-th alignment point of this launch (nbar = 1, 2, ...; every block calls it the same number of times).
// Two levels keep the single hot address short of traffic: a block bumps the counter of its group, every
// arrival that completes a round of its group bumps the grid-wide counter, and one thread per block polls that with sleeps in between.
// A block that has polled `spin_limit` times in vain sets the launch adrift: the grid is evidently not resident as a whole
// (another kernel - a second stream's, say - holds part of the chip), so waiting at every further point would cost the full
// bound each time; from then on no block of this launch waits at all and the kernel runs like an unaligned one.
__device__ __forceinline__ void solon_phase_align(uint32_t* sync, uint32_t nbar, int spin_limit) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t x = blockIdx.x & (SOLON_SYNC_GROUPS - 1);
    const uint32_t mates = (gridDim.x + SOLON_SYNC_GROUPS - 1 - x) / SOLON_SYNC_GROUPS;
    const uint32_t old = __hip_atomic_fetch_add(sync + SOLON_SYNC_STRIDE * x, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if ((old + 1u) % mates == 0u) __hip_atomic_fetch_add(sync + SOLON_SYNC_GLOBAL, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const uint32_t ngroups = gridDim.x < SOLON_SYNC_GROUPS ? gridDim.x : SOLON_SYNC_GROUPS;
    // the adrift mark is the top bit of the grid-wide counter, so a poll stays one load
    int n = 0;
    uint32_t seen = __hip_atomic_load(sync + SOLON_SYNC_GLOBAL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    while ((seen & SOLON_SYNC_ADRIFT_BIT) == 0u && seen < nbar * ngroups) {
      if (++n > spin_limit) {
        __hip_atomic_fetch_or(sync + SOLON_SYNC_GLOBAL, SOLON_SYNC_ADRIFT_BIT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(16);
      seen = __hip_atomic_load(sync + SOLON_SYNC_GLOBAL, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();
}

// Store pacing inside a write phase.  HBM takes writes fastest when the addresses in flight chip-wide stay inside a
// few megabytes: a flat fill whose 4 KB pieces are shuffled inside 1 MB windows runs as fast as an ordered one, shuffled
// inside 64 MB windows it loses 20 %.  In a write phase every wave has a list of store steps (row after row) and step
// k of all waves together covers one contiguous window, but waves that get their stores accepted early run ahead into
// later windows.  Holding step k of every wave back until k * (window bytes / absorbable rate) after the phase began
// keeps the chip inside one or two windows; waves that HBM delays simply lag (the caller also lets a wave wait for
// its previous store before the next).  `pace8` is that interval in eighths of a tick of the constant-rate clock,
// t0 the clock when the wave entered the phase.  The wait is bounded by the clock and by a poll count.
__device__ __forceinline__ void solon_pace(unsigned long long t0, uint32_t step, uint32_t pace8) {
  const unsigned long long due = t0 + (((unsigned long long)step * pace8) >> 3);
  int n = 0;
  while ((unsigned long long)wall_clock64() < due && n < 256) {
    __builtin_amdgcn_s_sleep(1);
    ++n;
  }
}

// Called once by every block after its last alignment point: the last block to leave zeroes the counters, so
// the next launch (ordered after this one on its stream) starts from zero without a separate clearing step.
__device__ __forceinline__ void solon_phase_exit(uint32_t* sync) {
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t old = __hip_atomic_fetch_add(sync + SOLON_SYNC_EXIT, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1u == gridDim.x) {
      for (int x = 0; x < SOLON_SYNC_GROUPS; ++x)
        __hip_atomic_store(sync + SOLON_SYNC_STRIDE * x, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(sync + SOLON_SYNC_GLOBAL, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(sync + SOLON_SYNC_EXIT, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}
