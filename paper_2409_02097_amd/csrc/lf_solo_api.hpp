// Host-side interface between linfusion.hip (boundary, planning) and linfusion_solo.hip (the replicated-state
// single-launch kernels of lf_solo.hpp, a translation unit of their own so that the two compile side by side).
#pragma once
#include <hip/hip_runtime.h>

#include "lf_common.hpp"

namespace lfs {

struct SoloArgs {
  const void *q, *k, *v;
  void* out;
  long long BH, N;
  int d, dtype, fm;           // d <= 64; dtype: LINFUSION_DTYPE_*
  float eps;
  bool unnorm;
  lf::Layout lq, lkv, lo;
  int G;                      // workgroups per head
  hipStream_t st;
};

// waves per workgroup of the launch for this width and type
int solo_waves(int d, int dtype);
// enqueues the one kernel; LINFUSION_OK or a LINFUSION_ERR_* code
int run_solo(const SoloArgs& a);

}  // namespace lfs
