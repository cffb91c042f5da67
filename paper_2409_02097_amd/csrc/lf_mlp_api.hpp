// Host-side interface between linfusion_mlp.hip (boundary and planning of the MLP-fed mixer, kernels for whole
// token rows in one workgroup) and linfusion_mlph.hip (the routes that start with a statistics pass).
#pragma once
#include <hip/hip_runtime.h>

#include <stddef.h>

namespace lfm {

struct HeadsArgs {
  const void *a_q, *t_q, *a_k, *t_k, *v;
  void* out;
  const float *gamma_q, *beta_q, *gamma_k, *beta_k;
  int B, H;
  long long N;
  int d, dtype, fm;                                  // dtype: LINFUSION_DTYPE_F16 or _BF16
  float eps, ln_eps, slope;
  bool unnorm;
  long long in_batch, in_row, out_batch, out_row;   // strides in 16-byte units
  float *partials, *state;                           // [B*H][splits][d*d + d] and [B*H][d*d + d], fp32
  unsigned char* packed;                             // the heads' operand-ready states
  void* stats;                                       // [2][B][n_pad] pairs of floats
  long long n_pad;                                   // N rounded up to whole 32-token tiles
  int stats_wgs, splits, blk_reduce, apply_wgs, blk_apply;
  bool grouped;                                      // row-piece kernels on groups of four heads (heads_grouped)
  hipStream_t st;
  hipEvent_t* ev;             // null, or four events: before the first kernel, after the reduction, after
                              // combine + packing, after apply
};

// head widths the per-head kernels are built for; those of them that run on the wide kernels (the packed state
// then has lfw::wide_packed_bytes per head and a tile block need not be whole rounds of four waves)
bool heads_supported(int d);
bool heads_wide(int d);
// shapes the row-piece kernels on groups of four neighbouring heads take: head rows that are no whole 128-byte
// lines (the per-head kernels would read and write partial lines) in rows of whole groups
bool heads_grouped(int H, int d);
// enqueues statistics, state reduction, combine, pack and apply; returns LINFUSION_OK or a LINFUSION_ERR_* code
int run_heads(const HeadsArgs& a);

}  // namespace lfm
