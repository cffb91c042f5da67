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
// Barrier: every workgroup owns one 32-bit flag per barrier in the caller's workspace and publishes
// its arrival by storing the call's `ticket` there; wave 0 of each workgroup then polls the flags of
// all workgroups of its head (one lane per flag).  There is no read-modify-write and no shared
// counter, so arrivals never contend, and because the ticket is unique per call a flag left by an
// earlier call (or any other content) reads as "not arrived": the workspace needs no initialisation
// and nothing is reset afterwards.  Waiting is bounded: a workgroup that does not see all arrivals
// within `spin_limit` polls raises the error word and returns, so every wave reaches the end of the
// kernel whatever happens.
#pragma once
#include "lf_apply16_dma.hpp"
#include "lf_fp32.hpp"

namespace lf {

// Returns false (for every thread of the workgroup) when the wait timed out.
// `flags`: the nsplit flags of this head and barrier.
LF_DEV bool head_barrier(unsigned* flags, int split, int nsplit, unsigned ticket, unsigned spin_limit,
                         unsigned* err, int* lds_flag) {
  // The partial states / states exchanged through this barrier are written with st_agent and read
  // with ld_agent, so no cache write-back or invalidation is needed here (a device-scope fence writes
  // back and invalidates the whole L2 of the XCD, measured at several microseconds per wave): it is
  // enough that every thread's stores have completed before the workgroup's arrival is published.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0): this wave's stores have been acknowledged
  __syncthreads();
  if (threadIdx.x < 64) {
    if (threadIdx.x == 0) __hip_atomic_store(flags + split, ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int ok = 1;
    unsigned polls = 0;
    for (int base = 0; base < nsplit && ok; base += 64) {
      const int i = base + (int)threadIdx.x;
      for (;;) {
        const bool arrived =
            i >= nsplit || __hip_atomic_load(flags + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == ticket;
        if (__all(arrived)) break;
        __builtin_amdgcn_s_sleep(8);
        if (++polls > spin_limit) {
          ok = 0;
          break;
        }
      }
    }
    if (threadIdx.x == 0) {
      if (!ok) __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *lds_flag = ok;
    }
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
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
        u32x4* __restrict__ O, float* partials, float* state, unsigned* flags, unsigned* err, unsigned ticket,
        unsigned spin_limit, float eps, long long N, int blk_reduce, int blk_apply) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int flag;
  constexpr int NE = D * D + D;
  const int split = blockIdx.x, nsplit = gridDim.x;
  const long long bh = blockIdx.y;
  float* head_part = partials + bh * nsplit * (long long)NE;
  float* head_state = state + bh * NE;
  reduce16_phase<T, D, FM>(K, V, head_part + (long long)split * NE, N, blk_reduce, split, nsplit, bh, smem);
  if (!head_barrier(flags + (2 * bh) * nsplit, split, nsplit, ticket, spin_limit, err, &flag)) return;
  combine_my_slices(head_part, nsplit, NE, split, head_state, reinterpret_cast<float*>(smem));
  if (!head_barrier(flags + (2 * bh + 1) * nsplit, split, nsplit, ticket, spin_limit, err, &flag)) return;
  apply16_dma_phase<T, D, FM, NORM>(Q, O, head_state, eps, N, blk_apply, split, nsplit, bh, smem);
}

template <int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
fused32(const f32x4* __restrict__ K, const f32x4* __restrict__ V, const f32x4* __restrict__ Q,
        float* __restrict__ O, float* partials, float* state, unsigned* flags, unsigned* err, unsigned ticket,
        unsigned spin_limit, float eps, long long N, int blk_reduce, int blk_apply) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int flag;
  constexpr int NE = D * D + D;
  const int split = blockIdx.x, nsplit = gridDim.x;
  const long long bh = blockIdx.y;
  float* head_part = partials + bh * nsplit * (long long)NE;
  float* head_state = state + bh * NE;
  reduce32_phase<D, FM>(K, V, head_part + (long long)split * NE, N, blk_reduce, split, nsplit, bh, smem);
  if (!head_barrier(flags + (2 * bh) * nsplit, split, nsplit, ticket, spin_limit, err, &flag)) return;
  combine_my_slices(head_part, nsplit, NE, split, head_state, reinterpret_cast<float*>(smem));
  if (!head_barrier(flags + (2 * bh + 1) * nsplit, split, nsplit, ticket, spin_limit, err, &flag)) return;
  apply32_phase<D, FM, NORM>(Q, O, head_state, eps, N, blk_apply, split, nsplit, bh);
}

}  // namespace lf
