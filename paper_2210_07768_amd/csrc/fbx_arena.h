// In-kernel dynamic allocation, callable from any kernel (Section 5, Algorithm 1 and "Reset GPU
// memory pool"): every thread of a workgroup brings a size; a prefix sum over the workgroup gives
// each thread the sizes before it; ONE thread adds the workgroup's total (rounded up to 128 bytes,
// so that every workgroup starts on a 128-byte line) to the pool's idle-memory head with one
// atomic add; a thread's region starts at the old head plus the sizes of the threads before it.
// (The printed listing subtracts the first thread's prefix, which is right only for equal sizes;
// the prose and Figure 5 lay the threads' regions end to end, which is what is computed.)
// Workgroups land in arrival order: offsets are unique, not ordered, across workgroups.
// Releasing is one store of the pool's base to the head.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fbx {

__device__ __forceinline__ uint64_t arena_round128(uint64_t x) { return (x + 127ull) & ~127ull; }

// Inclusive prefix sum of v over the 64 lanes of a wavefront.  Inside a row of 16 lanes the steps
// of 1, 2, 4 and 8 lanes are single data-parallel-primitive moves (row_shr: zero for a lane
// without a source); the totals of the rows before a lane's own then come through three more.
template <int D>
__device__ __forceinline__ uint32_t arena_row_shr(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x110 + D, 0xf, 0xf, false);
}
__device__ __forceinline__ uint32_t wave_prefix_u32(uint32_t v) {
  const uint32_t lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  v += arena_row_shr<1>(v);
  v += arena_row_shr<2>(v);
  v += arena_row_shr<4>(v);
  v += arena_row_shr<8>(v);
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15), r1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31),
                 r2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
  return v + (lane >= 16u ? r0 : 0u) + (lane >= 32u ? r1 : 0u) + (lane >= 48u ? r2 : 0u);
}
__device__ __forceinline__ uint64_t wave_prefix_u64(uint64_t v) {  // (sizes too large for 32-bit sums: plain shuffles)
  const uint32_t lane = __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
  for (uint32_t d = 1; d < 64u; d <<= 1) {
    const uint64_t t = __shfl_up(v, d, 64);
    if (lane >= d) v += t;
  }
  return v;
}

// Algorithm 1 for one workgroup.  Every thread of the workgroup calls it, the same number of
// times (it holds workgroup barriers), with the bytes it needs (0 is fine); the result is the
// byte offset of the thread's region from the pool's base.  s_part: LDS, blockDim.x / 64 + 2
// 64-bit words that the workgroup uses for nothing else across the call.  Two barriers, one
// atomic; nothing is checked against the pool's size (the caller compares offset + size with it).
__device__ __forceinline__ uint64_t arena_alloc_wg(uint64_t* head, uint64_t size, uint64_t* s_part) {
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6, n_waves = (blockDim.x + 63u) >> 6;
  uint64_t incl;
  if (__ballot(size >> 26) == 0ull) incl = wave_prefix_u32((uint32_t)size);  // (64 sizes below 2^26 sum below 2^32)
  else incl = wave_prefix_u64(size);
  if (lane == 63u || threadIdx.x + 1u == blockDim.x) s_part[wave] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint64_t total = 0;
    for (uint32_t w = 0; w < n_waves; ++w) {
      const uint64_t t = s_part[w];
      s_part[w] = total;  // the sizes of the wavefronts before w
      total += t;
    }
    total = arena_round128(total);
    s_part[n_waves] = total ? atomicAdd(reinterpret_cast<unsigned long long*>(head), (unsigned long long)total)
                            : *reinterpret_cast<volatile uint64_t*>(head);
  }
  __syncthreads();
  const uint64_t out = s_part[n_waves] + s_part[wave] + incl - size;
  __syncthreads();  // (s_part may be written again by the next call)
  return out;
}

}  // namespace fbx
