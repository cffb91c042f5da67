// Host-side interface between the two translation units of the library: linfusion.hip (boundary, planning,
// head widths up to 64) and linfusion_wide.hip (the kernels for head widths above 64).
#pragma once
#include <hip/hip_runtime.h>

#include "lf_common.hpp"

namespace lfw {

// launch shape of the wide kernels for one problem size (from the forward plan)
struct WidePlan {
  int splits, blk_reduce, apply_wgs, blk_apply;
  int apply_waves;            // waves per apply workgroup: 4 or 8 (apply16_wide)
  bool wave_apply;            // apply16_wave (a wave per tile, the whole state in its registers) instead
};

// state reduction + combine:  state[bh] = {S = sum_t phi(k_t)^T v_t, z = sum_t phi(k_t)}, fp32 [d*d + d]
struct WideReduceArgs {
  const void *k, *v;
  int B, H;
  long long N;
  int d, dtype, fm;           // dtype: LINFUSION_DTYPE_F16 or _BF16
  lf::Layout lk, lv;          // the two tensors may be laid out differently
  float *partials, *state;    // [B*H][splits][d*d + d] and [B*H][d*d + d], fp32
  WidePlan plan;
  hipStream_t st;
};

// pack + apply:  out_t = phi(q_t) S / (phi(q_t) z + eps)   (unnorm: phi(q_t) S)   from a given fp32 state
struct WideApplyArgs {
  const void* q;
  void* out;
  int B, H;
  long long N;
  int d, dtype, fm;
  float eps;
  bool unnorm;
  lf::Layout lq, lo;
  const float* state;         // [B*H][d*d + d]
  unsigned char* packed;      // wide_packed_bytes(d, dtype) per head: scratch for the state as apply operands
  WidePlan plan;
  hipStream_t st;
};

struct WideArgs {
  const void *q, *k, *v;
  void* out;                  // null: stop after the combine (state only)
  int B, H;
  long long N;
  int d, dtype, fm;           // dtype: LINFUSION_DTYPE_F16 or _BF16
  float eps;
  bool unnorm;
  lf::Layout lq, lkv, lo;
  float *partials, *state;    // [B*H][splits][d*d + d] and [B*H][d*d + d], fp32
  unsigned char* packed;      // wide_packed_bytes(d, dtype) per head: the state as apply operands
  WidePlan plan;
  hipStream_t st;
  hipEvent_t* ev;             // null, or four events: before reduce, after it, after combine, after apply
};

// head widths the wide kernels are built for
bool wide_supported(int d);
// whether apply16_wave is built for this width and dtype (its state operands must fit one wave's registers)
bool wave_apply_supported(int d, int dtype);
// bytes per head of the operand-ready state between the pack and apply kernels (0 if unsupported)
size_t wide_packed_bytes(int d, int dtype);
// enqueues state reduction, combine and (if out) pack and apply; returns LINFUSION_OK or a LINFUSION_ERR_* code
int run_wide(const WideArgs& a);
// the forward plan's launch shape for a wide width (linfusion.hip), and the bytes its partial states take;
// LINFUSION_ERR_UNSUPPORTED for other widths
int wide_launch_plan(int B, int H, long long N, int d, int dtype, WidePlan* wp, size_t* partial_bytes);
// the two halves by themselves (the backward pass for these widths is composed of them)
int run_wide_reduce(const WideReduceArgs& a);
int run_wide_apply(const WideApplyArgs& a);

}  // namespace lfw
