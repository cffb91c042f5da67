// Single-launch variant of the whole path for small token counts, where three dependent launches
// cost more than the data movement:
//   phase 1  state reduction of this workgroup's tiles          (reduce16_phase / reduce32_phase)
//   barrier  all workgroups of the head have written their partial
//   phase 2  this workgroup sums its 64-element slices of the head's partials in split order
//   barrier  the head's state is complete
//   phase 3  apply + normalize on this workgroup's tiles         (apply16_dma_phase / apply32_phase)
// grid = (splits, B*H), block = 256; the host launches it only when every workgroup of the grid is
// resident at once.  The arithmetic and its order are those of the separate kernels, so both paths
// give bit-identical results for the same number of splits.
//
// Barrier: one 64-bit word per head and barrier in the caller's workspace, holding (ticket << 32) |
// arrivals.  `ticket` is unique per call, so a word left by an earlier call (or any other content)
// reads as "zero arrivals": the workspace needs no initialisation and nothing is reset afterwards.
// Waiting is bounded: a workgroup that does not see all arrivals within `spin_limit` polls raises
// the error word and returns, so every wave reaches the end of the kernel whatever happens.
#pragma once
#include "lf_apply16_dma.hpp"
#include "lf_fp32.hpp"

namespace lf {

struct HeadSync {
  unsigned long long reduced;    // barrier after phase 1
  unsigned long long combined;   // barrier after phase 2
};

// Returns false (for every thread of the workgroup) when the wait timed out.
LF_DEV bool head_barrier(unsigned long long* word, unsigned ticket, unsigned expect, unsigned spin_limit,
                         unsigned* err, int* lds_flag) {
  __threadfence();   // this thread's global writes are visible device-wide before the arrival
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned long long tag = (unsigned long long)ticket << 32;
    unsigned long long old = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {   // at most `expect` failures: each one means another workgroup arrived
      const unsigned long long nw = ((unsigned)(old >> 32) == ticket) ? old + 1 : (tag | 1ull);
      if (__hip_atomic_compare_exchange_strong(word, &old, nw, __ATOMIC_ACQ_REL, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT))
        break;
    }
    const unsigned long long want = tag | expect;
    unsigned polls = 0;
    int ok = 1;
    while (__hip_atomic_load(word, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) != want) {
      __builtin_amdgcn_s_sleep(2);
      if (++polls > spin_limit) {
        ok = 0;
        __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
    }
    *lds_flag = ok;
  }
  __syncthreads();
  __threadfence();   // other workgroups' writes are visible to every thread from here on
  return *lds_flag != 0;
}

// phase 2: workgroup `split` sums the 64-element slices split, split + nsplit, ... of the head
LF_DEV void combine_my_slices(const float* head_partials, int nsplit, int NE, int split, float* head_state,
                              float* part) {
  for (int sl = split; sl * kCombineElems < NE; sl += nsplit) {
    combine_slice(head_partials, nsplit, NE, sl * kCombineElems, head_state, part);
    __syncthreads();
  }
}

template <typename T, int D>
constexpr int fused16_lds_bytes() {
  int a = reduce16_lds_bytes<T, D>(), b = apply16_dma_lds_bytes<T, D>();
  return a > b ? a : b;
}

template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
fused16(const u32x4* __restrict__ K, const u32x4* __restrict__ V, const u32x4* __restrict__ Q,
        u32x4* __restrict__ O, float* partials, float* state, HeadSync* sync, unsigned* err, unsigned ticket,
        unsigned spin_limit, float eps, long long N, int blk_reduce, int blk_apply) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int flag;
  constexpr int NE = D * D + D;
  const int split = blockIdx.x, nsplit = gridDim.x;
  const long long bh = blockIdx.y;
  float* head_part = partials + bh * nsplit * (long long)NE;
  float* head_state = state + bh * NE;
  reduce16_phase<T, D, FM>(K, V, head_part + (long long)split * NE, N, blk_reduce, split, nsplit, bh, smem);
  if (!head_barrier(&sync[bh].reduced, ticket, nsplit, spin_limit, err, &flag)) return;
  combine_my_slices(head_part, nsplit, NE, split, head_state, reinterpret_cast<float*>(smem));
  if (!head_barrier(&sync[bh].combined, ticket, nsplit, spin_limit, err, &flag)) return;
  apply16_dma_phase<T, D, FM, NORM>(Q, O, head_state, eps, N, blk_apply, split, nsplit, bh, smem);
}

template <int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
fused32(const f32x4* __restrict__ K, const f32x4* __restrict__ V, const f32x4* __restrict__ Q,
        float* __restrict__ O, float* partials, float* state, HeadSync* sync, unsigned* err, unsigned ticket,
        unsigned spin_limit, float eps, long long N, int blk_reduce, int blk_apply) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int flag;
  constexpr int NE = D * D + D;
  const int split = blockIdx.x, nsplit = gridDim.x;
  const long long bh = blockIdx.y;
  float* head_part = partials + bh * nsplit * (long long)NE;
  float* head_state = state + bh * NE;
  reduce32_phase<D, FM>(K, V, head_part + (long long)split * NE, N, blk_reduce, split, nsplit, bh, smem);
  if (!head_barrier(&sync[bh].reduced, ticket, nsplit, spin_limit, err, &flag)) return;
  combine_my_slices(head_part, nsplit, NE, split, head_state, reinterpret_cast<float*>(smem));
  if (!head_barrier(&sync[bh].combined, ticket, nsplit, spin_limit, err, &flag)) return;
  apply32_phase<D, FM, NORM>(Q, O, head_state, eps, N, blk_apply, split, nsplit, bh);
}

}  // namespace lf
