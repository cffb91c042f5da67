// Host-side interface to the fp32 kernels of linfusion.hip for the library's other translation units: the state
// reduction (+ combine) and the apply step by themselves (the fp32 backward pass is composed of them).
#pragma once
#include <hip/hip_runtime.h>

#include "lf_common.hpp"

namespace lf32 {

// launch shape from the forward plan of the same problem size
struct Plan32 {
  int splits, blk_reduce, apply_wgs, blk_apply;
};
// LINFUSION_OK, or the forward plan's error code; `partial_bytes`: what the partial states take
int launch_plan32(int B, int H, long long N, int d, Plan32* p, size_t* partial_bytes);

// state[bh] = {S = sum_t phi(k_t)^T v_t, z = sum_t phi(k_t)}, fp32 [d*d + d]
struct Reduce32Args {
  const void *k, *v;
  int B, H;
  long long N;
  int d, fm;
  lf::Layout lk, lv;          // the two tensors may be laid out differently
  float *partials, *state;    // [B*H][splits][d*d + d] and [B*H][d*d + d]
  Plan32 plan;
  hipStream_t st;
};
// out_t = phi(q_t) S / (phi(q_t) z + eps)   (unnorm: phi(q_t) S)   from a given state
struct Apply32Args {
  const void* q;
  void* out;
  int B, H;
  long long N;
  int d, fm;
  float eps;
  bool unnorm;
  lf::Layout lq, lo;
  const float* state;
  Plan32 plan;
  hipStream_t st;
};
int run_reduce32(const Reduce32Args& a);
int run_apply32(const Apply32Args& a);

}  // namespace lf32
