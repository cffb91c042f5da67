// Sixth translation unit of the library: the MLP-fed mixer for the shapes whose token rows do not fit one
// workgroup.  A statistics pass (mlp_rowstats16), then per shape: row-piece kernels on groups of four heads
// (lf_mlp16.hpp), per-head kernels (lf_mlph16.hpp), or the wide kernels for widths above 64 (lf_mlpw16.hpp).
#include "../../include/linfusion.h"

#include <stdint.h>

#include "lf_host_api.hpp"
#include "lf_mlp_api.hpp"
#include "lf_mlp16.hpp"
#include "lf_mlph16.hpp"
#include "lf_mlpw16.hpp"

namespace {

using lfh::allow_lds;
using lfm::HeadsArgs;

template <typename T, int D, int FM, bool NORM>
int run_heads_t(const HeadsArgs& a) {
  using namespace lf;
  constexpr int NE = D * D + D;
  constexpr int lds_r = reduce16_mlph_lds_bytes<T, D>();
  constexpr int lds_p = apply16_dma_lds_bytes<T, D>();
  constexpr int lds_a = apply16_mlph_lds_bytes<T, D>();
  static_assert(lds_r <= 160 * 1024 && lds_a <= 160 * 1024, "workgroup LDS limit of the device");
  static_assert(Pack16<T, D>::kFrags == NSplit<T>::value * ((D / 2 + 2 + 15) / 16) * ((D / 8 + 1) / 2),
                "the planner's workspace size formula must match the packed layout");
  if (!allow_lds(state_reduce16_mlph<T, D, FM>, lds_r) || !allow_lds(pack_state16<T, D, NORM>, lds_p) ||
      !allow_lds(apply16_mlph<T, D, FM, NORM>, lds_a))
    return LINFUSION_ERR_HIP;
  hipStream_t st = a.st;
  const int row = (int)a.in_row, row_o = (int)a.out_row;
  const unsigned heads = (unsigned)(a.B * a.H);
  f32x2* stats_q = reinterpret_cast<f32x2*>(a.stats);
  f32x2* stats_k = stats_q + (long long)a.B * a.n_pad;
  if (a.ev) (void)hipEventRecord(a.ev[0], st);
  mlp_rowstats16<T><<<dim3(a.stats_wgs, 2u * a.B), dim3(kThreads), 0, st>>>(
      (const u32x4*)a.t_q, (const u32x4*)a.t_k, a.in_batch, row, a.H * D / 8, a.ln_eps, a.N, a.n_pad, stats_q);
  state_reduce16_mlph<T, D, FM><<<dim3(a.splits, heads), dim3(kThreads), lds_r, st>>>(
      (const u32x4*)a.a_k, (const u32x4*)a.t_k, (const u32x4*)a.v, a.in_batch, row, a.H, stats_k, a.n_pad, a.gamma_k,
      a.beta_k, a.slope, a.partials, a.N, a.blk_reduce);
  if (a.ev) (void)hipEventRecord(a.ev[1], st);
  combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, heads), dim3(kCombineThreads), 0, st>>>(
      a.partials, a.splits, NE, a.state);
  pack_state16<T, D, NORM><<<dim3(heads), dim3(kThreads), lds_p, st>>>(a.state, a.packed);
  if (a.ev) (void)hipEventRecord(a.ev[2], st);
  apply16_mlph<T, D, FM, NORM><<<dim3(a.apply_wgs, heads), dim3(kThreads), lds_a, st>>>(
      (const u32x4*)a.a_q, (const u32x4*)a.t_q, a.in_batch, row, (u32x4*)a.out, a.out_batch, row_o, a.H, stats_q, a.n_pad,
      a.gamma_q, a.beta_q, a.slope, a.packed, a.eps, a.N, a.blk_apply);
  if (a.ev) (void)hipEventRecord(a.ev[3], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

// head widths above 64: the wide kernels, eight waves per apply workgroup
template <typename T, int D, int FM, bool NORM>
int run_wide_t(const HeadsArgs& a) {
  using namespace lf;
  constexpr int NE = D * D + D, WA = 8;
  constexpr int lds_r = reduce16_wide_mlp_lds_bytes<T, D>();
  constexpr int lds_a = ApplyWide<T, D, FM, NORM, WA, true>::kLdsBytes;
  static_assert(lds_r <= 160 * 1024 && lds_a <= 160 * 1024, "workgroup LDS limit of the device");
  if (!allow_lds(state_reduce16_wide_mlp<T, D, FM>, lds_r) || !allow_lds(apply16_wide_mlp<T, D, FM, NORM, WA>, lds_a))
    return LINFUSION_ERR_HIP;
  hipStream_t st = a.st;
  const int row = (int)a.in_row, row_o = (int)a.out_row;
  const unsigned heads = (unsigned)(a.B * a.H);
  f32x2* stats_q = reinterpret_cast<f32x2*>(a.stats);
  f32x2* stats_k = stats_q + (long long)a.B * a.n_pad;
  if (a.ev) (void)hipEventRecord(a.ev[0], st);
  mlp_rowstats16<T><<<dim3(a.stats_wgs, 2u * a.B), dim3(kThreads), 0, st>>>(
      (const u32x4*)a.t_q, (const u32x4*)a.t_k, a.in_batch, row, a.H * D / 8, a.ln_eps, a.N, a.n_pad, stats_q);
  state_reduce16_wide_mlp<T, D, FM><<<dim3(a.splits, heads), dim3(kThreads), lds_r, st>>>(
      (const u32x4*)a.a_k, (const u32x4*)a.t_k, (const u32x4*)a.v, a.in_batch, row, a.H, stats_k, a.n_pad, a.gamma_k,
      a.beta_k, a.slope, a.partials, a.N, a.blk_reduce);
  if (a.ev) (void)hipEventRecord(a.ev[1], st);
  combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, heads), dim3(kCombineThreads), 0, st>>>(
      a.partials, a.splits, NE, a.state);
  // A wave per 16-token tile with the head's whole state in its registers (apply16_wave_mlp), one long-lived
  // workgroup per CU.  (LINFUSION_MLPW_WAVE_APPLY = 2 under tuning: the workgroup-shared kernel instead)
  {
    if (lfh::env_int("LINFUSION_MLPW_WAVE_APPLY", 1) == 1) {
      constexpr int lds_w = ApplyWaveMlpShape<D>::kLdsBytes;
      if (!allow_lds(apply16_wave_mlp<T, D, FM, NORM>, lds_w)) return LINFUSION_ERR_HIP;
      pack_state_wave<D><<<dim3(ApplyWaveShape<D>::kKS, heads), dim3(kThreads), 0, st>>>(a.state, a.packed, NORM ? 1 : 0);
      if (a.ev) (void)hipEventRecord(a.ev[2], st);
      const long long tiles = (a.N + ApplyWaveMlpShape<D>::kTok - 1) / ApplyWaveMlpShape<D>::kTok;
      const long long most = (tiles + kWavesPerWG - 1) / kWavesPerWG;   // every wave gets a tile
      long long wgs = lfh::env_int("LINFUSION_MLPW_WAVE_WGS", lfh::num_cu()) / (long long)heads;
      wgs = wgs > most ? most : (wgs < 1 ? 1 : wgs);
      apply16_wave_mlp<T, D, FM, NORM><<<dim3((unsigned)wgs, heads), dim3(kThreads), lds_w, st>>>(
          (const u32x4*)a.a_q, (const u32x4*)a.t_q, a.in_batch, row, (u32x4*)a.out, a.out_batch, row_o, a.H, stats_q,
          a.n_pad, a.gamma_q, a.beta_q, a.slope, a.packed, a.eps, a.N, kWavesPerWG);
      if (a.ev) (void)hipEventRecord(a.ev[3], st);
      return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
    }
  }
  pack_state_wide<T, D, WA><<<dim3(ApplyWideShape<D, WA>::kKS, heads), dim3(64 * WA), 0, st>>>(a.state, a.packed,
                                                                                             NORM ? 1 : 0);
  if (a.ev) (void)hipEventRecord(a.ev[2], st);
  apply16_wide_mlp<T, D, FM, NORM, WA><<<dim3(a.apply_wgs, heads), dim3(64 * WA), lds_a, st>>>(
      (const u32x4*)a.a_q, (const u32x4*)a.t_q, a.in_batch, row, (u32x4*)a.out, a.out_batch, row_o, a.H, stats_q, a.n_pad,
      a.gamma_q, a.beta_q, a.slope, a.packed, a.eps, a.N, a.blk_apply);
  if (a.ev) (void)hipEventRecord(a.ev[3], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T, int D>
int run_wide_fm(const HeadsArgs& a) {
  switch (a.fm) {
    case 0: return a.unnorm ? run_wide_t<T, D, 0, false>(a) : run_wide_t<T, D, 0, true>(a);
    case 1: return a.unnorm ? run_wide_t<T, D, 1, false>(a) : run_wide_t<T, D, 1, true>(a);
    default: return a.unnorm ? run_wide_t<T, D, 2, false>(a) : run_wide_t<T, D, 2, true>(a);
  }
}

// groups of four neighbouring heads (row-piece kernels): for head rows that are no whole 128-byte lines
template <typename T, int D, int FM, bool NORM>
int run_groups_t(const HeadsArgs& a) {
  using namespace lf;
  constexpr int NE = D * D + D, W = 4;
  constexpr int lds_r = ReduceMlpCfg<T, D, W>::kLdsBytes;
  constexpr int lds_p = apply16_dma_lds_bytes<T, D>();
  constexpr int lds_a = apply16_mlpg_lds_bytes<T, D>(W);
  static_assert(lds_r <= 160 * 1024 && lds_a <= 160 * 1024, "workgroup LDS limit of the device");
  static_assert(Pack16<T, D>::kFrags == NSplit<T>::value * ((D / 2 + 2 + 15) / 16) * ((D / 8 + 1) / 2),
                "the planner's workspace size formula must match the packed layout");
  if (!allow_lds(state_reduce16_mlp<T, D, FM, W, true>, lds_r) || !allow_lds(pack_state16<T, D, NORM>, lds_p) ||
      !allow_lds(apply16_mlpg<T, D, FM, NORM, W>, lds_a))
    return LINFUSION_ERR_HIP;
  hipStream_t st = a.st;
  const int row = (int)a.in_row, row_o = (int)a.out_row, gpb = a.H / W;
  const unsigned heads = (unsigned)(a.B * a.H), groups = (unsigned)(a.B * gpb);
  f32x2* stats_q = reinterpret_cast<f32x2*>(a.stats);
  f32x2* stats_k = stats_q + (long long)a.B * a.n_pad;
  if (a.ev) (void)hipEventRecord(a.ev[0], st);
  mlp_rowstats16<T><<<dim3(a.stats_wgs, 2u * a.B), dim3(kThreads), 0, st>>>(
      (const u32x4*)a.t_q, (const u32x4*)a.t_k, a.in_batch, row, a.H * D / 8, a.ln_eps, a.N, a.n_pad, stats_q);
  state_reduce16_mlp<T, D, FM, W, true><<<dim3(a.splits, groups), dim3(64 * W), lds_r, st>>>(
      (const u32x4*)a.a_k, (const u32x4*)a.t_k, (const u32x4*)a.v, a.in_batch, row, a.gamma_k, a.beta_k, a.ln_eps, a.slope,
      a.partials, a.N, a.blk_reduce, gpb, stats_k, a.n_pad);
  if (a.ev) (void)hipEventRecord(a.ev[1], st);
  combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, heads), dim3(kCombineThreads), 0, st>>>(
      a.partials, a.splits, NE, a.state);
  pack_state16<T, D, NORM><<<dim3(heads), dim3(kThreads), lds_p, st>>>(a.state, a.packed);
  if (a.ev) (void)hipEventRecord(a.ev[2], st);
  apply16_mlpg<T, D, FM, NORM, W><<<dim3(a.apply_wgs, groups), dim3(64 * W), lds_a, st>>>(
      (const u32x4*)a.a_q, (const u32x4*)a.t_q, a.in_batch, row, (u32x4*)a.out, a.out_batch, row_o, gpb, stats_q, a.n_pad,
      a.gamma_q, a.beta_q, a.slope, a.packed, a.eps, a.N, a.blk_apply);
  if (a.ev) (void)hipEventRecord(a.ev[3], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T, int D>
int run_groups_fm(const HeadsArgs& a) {
  switch (a.fm) {
    case 0: return a.unnorm ? run_groups_t<T, D, 0, false>(a) : run_groups_t<T, D, 0, true>(a);
    case 1: return a.unnorm ? run_groups_t<T, D, 1, false>(a) : run_groups_t<T, D, 1, true>(a);
    default: return a.unnorm ? run_groups_t<T, D, 2, false>(a) : run_groups_t<T, D, 2, true>(a);
  }
}

template <typename T, int D>
int run_heads_fm(const HeadsArgs& a) {
  switch (a.fm) {
    case 0: return a.unnorm ? run_heads_t<T, D, 0, false>(a) : run_heads_t<T, D, 0, true>(a);
    case 1: return a.unnorm ? run_heads_t<T, D, 1, false>(a) : run_heads_t<T, D, 1, true>(a);
    default: return a.unnorm ? run_heads_t<T, D, 2, false>(a) : run_heads_t<T, D, 2, true>(a);
  }
}

}  // namespace

namespace lfm {

bool heads_supported(int d) { return d >= 8 && d % 8 == 0 && (d <= 64 || d == 80 || heads_wide(d)); }
bool heads_wide(int d) { return d == 96 || d == 128 || d == 160; }
bool heads_grouped(int H, int d) { return H % 4 == 0 && d >= 8 && d % 8 == 0 && (d <= 56 || d == 80); }

int run_heads(const HeadsArgs& a) {
  const bool f16 = a.dtype == LINFUSION_DTYPE_F16;
  if (a.grouped) {
    switch (a.d) {
#define X(DD) case DD: return f16 ? run_groups_fm<lf::F16, DD>(a) : run_groups_fm<lf::BF16, DD>(a);
      X(8) X(16) X(24) X(32) X(40) X(48) X(56) X(80)
#undef X
    }
    return LINFUSION_ERR_UNSUPPORTED;
  }
  switch (a.d) {
#define X(DD) case DD: return f16 ? run_heads_fm<lf::F16, DD>(a) : run_heads_fm<lf::BF16, DD>(a);
    X(8) X(16) X(24) X(32) X(40) X(48) X(56) X(64) X(80)
#undef X
#define X(DD) case DD: return f16 ? run_wide_fm<lf::F16, DD>(a) : run_wide_fm<lf::BF16, DD>(a);
    X(96) X(128) X(160)
#undef X
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

}  // namespace lfm
