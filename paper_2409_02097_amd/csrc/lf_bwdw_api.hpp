// Host-side interface between linfusion_bwd.hip (the backward entry points) and linfusion_bwdw.hip (the backward
// pass composed of the forward's kernels: fp16 at head widths above 80, fp32 at every width it has).
#pragma once
#include <hip/hip_runtime.h>

#include "lf_common.hpp"

namespace lfbw {

struct BwdWideArgs {
  const float* saved_state;   // the forward state of the same q, k, v, or null: recompute it from k, v
  const void *q, *k, *v, *g;
  void *dq, *dk, *dv;
  int B, H;
  long long N;
  int d, dtype, fm;
  float eps;
  bool unnorm;
  unsigned char* ws;          // bwd_wide_workspace_bytes, 256-byte aligned pieces inside
  hipStream_t st;
  lf::Layout lq, lkv, lg, ldq, ldkv;   // q; k and v; dout; dq; dk and dv
};

// fp16 at the wide kernels' widths; fp32 at 8 .. 64 in steps of 8
bool bwd_wide_supported(int d, int dtype);
// 0 for unsupported shapes
size_t bwd_wide_workspace_bytes(int B, int H, long long N, int d, int dtype);
// enqueues the whole pass; LINFUSION_OK or a LINFUSION_ERR_* code
int run_bwd_wide(const BwdWideArgs& a);

}  // namespace lfbw
