// Single-launch variant of the whole path, for token counts where three dependent launches (and the
// drain and refill of the chip between them) cost a visible share of the time:
//   phase 1  state reduction of this workgroup's tiles          (reduce16_phase / reduce32_phase)
//   barrier  all workgroups of the head have written their partial
//            (fp16 / bf16: the first two Q tiles of every wave are requested here, see ApplyDma)
//   phase 2  this workgroup sums the elements of the head's state that it owns, over all partials
//   barrier  the head's state is complete
//   phase 3  apply + normalize on this workgroup's tiles         (ApplyDma / apply32_phase)
// grid = (splits, B*H), block = 256; the host launches it only when every workgroup of the grid is
// resident at once.  All sums run in a fixed order, so results are run-to-run bit-identical.
//
// Barrier: every workgroup owns one 64-bit flag per barrier in the caller's workspace and publishes
// its arrival by storing the call's `ticket` there; wave 0 of each workgroup then polls the flags of
// all workgroups of its head (one lane per flag).  There is no read-modify-write and no shared
// counter, so arrivals never contend.  The ticket is {t, ~t} with t unique per call and counted from a
// random per-process base, so a flag left by an earlier call reads as "not arrived", and so does any
// other content the workspace may hold (it would have to agree in all 64 bits): the workspace needs no
// initialisation and nothing is reset afterwards.  Waiting is bounded: a workgroup that does not see
// all arrivals within `spin_limit` polls records the ticket as failed and returns, so every wave
// reaches the end of the kernel whatever happens.  `rec`: two 64-bit words behind the flags,
// {ticket of the last call that ran on this workspace, ticket of the last call that gave up}.
#pragma once
#include "lf_apply16_dma.hpp"
#include "lf_fp32.hpp"

namespace lf {

// Returns false (for every thread of the workgroup) when the wait timed out.
// `flags`: the nsplit flags of this head and barrier.
LF_DEV bool head_barrier(unsigned long long* flags, int split, int nsplit, unsigned long long ticket,
                         unsigned spin_limit, unsigned long long* rec, int* lds_flag) {
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
      if (!ok) __hip_atomic_store(rec + 1, ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *lds_flag = ok;
    }
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  return *lds_flag != 0;
}

// Phase 2.  Workgroup `split` owns the state elements [split * per, (split + 1) * per), per =
// ceil(NE / nsplit).  Its 256 threads are laid out as (element, split group): thread t sums element
// t % width over the splits of group t / width in split order, with all loads of the workgroup in
// flight at once; the groups are then added in group order.  `scratch`: 256 floats of LDS.
LF_DEV void combine_owned(const float* head_partials, int nsplit, int NE, int split, float* head_state,
                          float* scratch) {
  const int per = (NE + nsplit - 1) / nsplit;
  const int lo = split * per;
  int hi = lo + per;
  if (hi > NE) hi = NE;
  for (int c0 = lo; c0 < hi; c0 += kThreads) {   // one pass unless the workgroup owns more than 256 elements
    int width = hi - c0;
    if (width > kThreads) width = kThreads;
    const int groups = kThreads / width;
    const int g = (int)threadIdx.x / width, el = (int)threadIdx.x % width;
    const int spg = (nsplit + groups - 1) / groups;
    float s = 0.0f;
    if (g < groups) {
      int p = g * spg, p1 = p + spg;
      if (p1 > nsplit) p1 = nsplit;
      const float* src = head_partials + c0 + el;
      for (; p + 8 <= p1; p += 8) {
        float a[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) a[i] = ld_agent(src + (long long)(p + i) * NE);
#pragma unroll
        for (int i = 0; i < 8; ++i) s += a[i];
      }
      for (; p < p1; ++p) s += ld_agent(src + (long long)p * NE);
    }
    scratch[threadIdx.x] = s;
    __syncthreads();
    if (g == 0) {
      float t = scratch[el];
      for (int gg = 1; gg < groups; ++gg) t += scratch[gg * width + el];
      st_agent(head_state + c0 + el, t);
    }
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
fused16(const u32x4* __restrict__ K, const u32x4* __restrict__ V, Layout lkv, const u32x4* __restrict__ Q,
        Layout lq, u32x4* __restrict__ O, Layout lo, float* partials, float* state, unsigned long long* flags, unsigned long long* rec,
        unsigned long long ticket,
        unsigned spin_limit, float eps, long long N, int blk_reduce, int blk_apply) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int flag;
  constexpr int NE = D * D + D;
  const int split = blockIdx.x, nsplit = gridDim.x;
  const long long bh = blockIdx.y;
  float* head_part = partials + bh * nsplit * (long long)NE;
  float* head_state = state + bh * NE;
  const long long okv = lkv.slice(bh);
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
    __hip_atomic_store(rec, ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  reduce16_phase<T, D, FM>(K + okv, V + okv, lkv.row, head_part + (long long)split * NE, N, blk_reduce, split, nsplit,
                           smem);
  if (!head_barrier(flags + (2 * bh) * nsplit, split, nsplit, ticket, spin_limit, rec, &flag)) return;
  ApplyDma<T, D, FM, NORM> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, blk_apply, split, nsplit, smem);
  ap.prefetch();   // Q does not depend on the state: its first tiles travel during phase 2 and the barrier
  combine_owned(head_part, nsplit, NE, split, head_state,
                reinterpret_cast<float*>(smem + ApplyDmaCfg<D>::kStageOffset));
  if (!head_barrier(flags + (2 * bh + 1) * nsplit, split, nsplit, ticket, spin_limit, rec, &flag)) {
    wait_vmcnt<0>();   // no copy into this workgroup's LDS may still be in flight when it ends
    return;
  }
  ap.template run<true>(head_state, eps);
}

template <int D> constexpr int fused32_lds_bytes() {
  return reduce32_lds_bytes<D>() > apply32_lds_bytes<D>() ? reduce32_lds_bytes<D>() : apply32_lds_bytes<D>();
}

template <int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
fused32(const f32x4* __restrict__ K, const f32x4* __restrict__ V, Layout lkv, const f32x4* __restrict__ Q,
        Layout lq, f32x4* __restrict__ O, Layout lo, float* partials, float* state, unsigned long long* flags, unsigned long long* rec,
        unsigned long long ticket,
        unsigned spin_limit, float eps, long long N, int blk_reduce, int blk_apply) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int flag;
  constexpr int NE = D * D + D;
  const int split = blockIdx.x, nsplit = gridDim.x;
  const long long bh = blockIdx.y;
  float* head_part = partials + bh * nsplit * (long long)NE;
  float* head_state = state + bh * NE;
  const long long okv = lkv.slice(bh);
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0)
    __hip_atomic_store(rec, ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  reduce32_phase<D, FM>(K + okv, V + okv, lkv.row, lkv.row, head_part + (long long)split * NE, N, blk_reduce, split, nsplit, smem);
  if (!head_barrier(flags + (2 * bh) * nsplit, split, nsplit, ticket, spin_limit, rec, &flag)) return;
  combine_owned(head_part, nsplit, NE, split, head_state, reinterpret_cast<float*>(smem));
  if (!head_barrier(flags + (2 * bh + 1) * nsplit, split, nsplit, ticket, spin_limit, rec, &flag)) return;
  Apply32Dma<D, FM, NORM> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, blk_apply, split, nsplit, smem);
  ap.prefetch();   // the combine's scratch in LDS is dead after the barrier
  ap.template load_state<true>(head_state);
  ap.stream(eps);
}

}  // namespace lf
