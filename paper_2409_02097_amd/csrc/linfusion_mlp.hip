// Fourth translation unit of the library: the mixer fed from the two-branch MLPs f', g' (lf_mlp16.hpp).
#include "../../include/linfusion.h"

#include <stdint.h>

#include <cmath>

#include "lf_host_api.hpp"
#include "lf_mlp16.hpp"
#include "lf_mlp_api.hpp"
#include "lf_wide_api.hpp"

namespace {


struct MlpPlan {
  int route;                      // 0: whole token rows in one workgroup; 1: per-head kernels + statistics pass;
                                  // 2: statistics pass + row-piece kernels on groups of four heads
  long long n_pad;                // route 1: tokens rounded up to whole tiles
  int stats_wgs;
  size_t ws_stats;
  int W;                          // heads = waves per workgroup
  int splits, blk_reduce;         // state reduction: workgroups per batch, tiles per block
  int apply_wgs, blk_apply;
  size_t ne, ws_partials, ws_state, ws_pack, ws_total;
};

// Which shapes the kernels for whole token rows take: the workgroup must cover a row (H = W in {4, 8}) and both
// rings of the apply kernel must fit the 160 KiB of LDS (eight heads: d <= 48; four heads: d <= 80).  Every other
// shape with a per-head kernel width goes the per-head way.
bool rows_supported(int H, int d) {
  if (d < 8 || d % 8 != 0) return false;
  if (H == 8) return d <= 48;
  if (H == 4) return d <= 64 || d == 80;
  return false;
}

size_t pack_bytes(int d, int dtype) {
  const size_t ns = dtype == LINFUSION_DTYPE_BF16 ? 2 : 1;
  const size_t frags = ns * (size_t)((d / 2 + 2 + 15) / 16) * (size_t)((d / 8 + 1) / 2);   // Pack16<T, D>::kFrags
  return 256 + frags * 1024;
}

int make_mlp_plan(int B, int H, long long N, int d, int dtype, MlpPlan* p) {
  if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return LINFUSION_ERR_INVALID;
  if (B > 65535) return LINFUSION_ERR_INVALID;   // grid.y limit
  if (dtype != LINFUSION_DTYPE_F16 && dtype != LINFUSION_DTYPE_BF16) return LINFUSION_ERR_UNSUPPORTED;
  if (d < 8 || d % 8 != 0 || !lfm::heads_supported(d)) return LINFUSION_ERR_UNSUPPORTED;
  if (N > (1LL << 40) / ((long long)H * d)) return LINFUSION_ERR_INVALID;
  const long long n_tiles = (N + lf::kTile - 1) / lf::kTile;
  p->ne = (size_t)d * d + d;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  // LINFUSION_MLP_ROUTE=1 sends every shape the per-head way, =2 every shape with whole groups of four heads
  // through the group kernels (test aids)
  const int forced = lfh::env_int("LINFUSION_MLP_ROUTE", 0);
  const bool groupable = lfm::heads_grouped(H, d);
  p->route = forced == 1 ? 1 : ((forced == 2 && groupable) ? 2 : (rows_supported(H, d) ? 0 : (groupable ? 2 : 1)));
  if (p->route == 2) {
    // as the whole-row plan below with B * (H / 4) units of four heads; the apply kernel's rings leave room for
    // one workgroup per CU from d = 40 on
    if ((long long)B * H > 65535 || 2LL * B > 65535) return LINFUSION_ERR_INVALID;   // grid.y limits
    p->W = 4;
    p->n_pad = n_tiles * lf::kTile;
    const long long units = (long long)B * (H / 4);
    auto per_group = [&](int want_total, int blk_dflt, int* blk) {
      long long s = want_total / units;
      if (s > n_tiles) s = n_tiles;
      if (s < 1) s = 1;
      long long t = (n_tiles + s - 1) / s;
      *blk = (int)(blk_dflt < t ? blk_dflt : t);
      return (int)((n_tiles + t - 1) / t);
    };
    const int slot = (lf::kTile * d * 2 + 1023) / 1024 * 1024;
    const int lds_apply = 2 * 3 * slot * 4 + 3 * 1024;
    const int resident = 160 * 1024 / lds_apply > 0 ? 160 * 1024 / lds_apply : 1;
    p->splits = per_group(lfh::env_int("LINFUSION_MLPG_REDUCE_WGS", 2 * lfh::num_cu()), lfh::env_int("LINFUSION_MLPG_REDUCE_BLK", 2),
                          &p->blk_reduce);
    p->apply_wgs = per_group(lfh::env_int("LINFUSION_MLPG_APPLY_WGS", resident * lfh::num_cu()),
                             lfh::env_int("LINFUSION_MLPG_APPLY_BLK", 2), &p->blk_apply);
    long long sw = (N + 15) / 16, cap = lfh::env_int("LINFUSION_MLPH_STATS_WGS", 8 * lfh::num_cu()) / (2 * B);
    if (cap < 1) cap = 1;
    p->stats_wgs = (int)(sw < cap ? sw : cap);
    p->ws_partials = up((size_t)B * H * p->splits * p->ne * sizeof(float));
    p->ws_state = up((size_t)B * H * p->ne * sizeof(float));
    p->ws_pack = up((size_t)B * H * pack_bytes(d, dtype));
    p->ws_stats = up((size_t)2 * B * p->n_pad * 2 * sizeof(float));
    p->ws_total = p->ws_partials + p->ws_state + p->ws_pack + p->ws_stats;
    return LINFUSION_OK;
  }
  if (p->route == 1) {
    if ((long long)B * H > 65535 || 2LL * B > 65535) return LINFUSION_ERR_INVALID;   // grid.y limits
    p->W = 0;
    p->n_pad = n_tiles * lf::kTile;
    const long long units = (long long)B * H;
    const bool wide = lfm::heads_wide(d);   // there every wave of a workgroup visits every tile of its blocks
    auto per_head = [&](int want_total, int blk_dflt, int* blk) {
      long long s = want_total / units;
      const long long most = wide ? n_tiles : (n_tiles + 3) / 4;  // four waves, a tile each at least
      if (s > most) s = most;
      if (s < 1) s = 1;
      long long t = (n_tiles + s - 1) / s;
      t = blk_dflt < t ? blk_dflt : t;
      if (!wide) t = (t + 3) / 4 * 4;                             // a block is whole rounds of the four waves
      *blk = (int)t;
      const long long g = (n_tiles + t - 1) / t;                  // blocks are dealt round-robin to the workgroups
      return (int)(g < s ? g : s);
    };
    // apply: one resident round (two rings of three slots and the statistics deposits per wave decide how many
    // workgroups a CU holds); measured at 1 M tokens, 10 heads of 64: 0.725 ms with 256 workgroups, 0.77 with 2048
    const int slot = (lf::kTile * d * 2 + 1023) / 1024 * 1024;
    const int lds_apply = (2 * 3 * slot + 3 * 1024) * lf::kWavesPerWG;
    const int resident = (!wide && 160 * 1024 / lds_apply > 0) ? 160 * 1024 / lds_apply : 1;
    p->splits = per_head(lfh::env_int("LINFUSION_MLPH_REDUCE_WGS", 2 * lfh::num_cu()),
                         lfh::env_int("LINFUSION_MLPH_REDUCE_BLK", wide ? 4 : 8), &p->blk_reduce);
    p->apply_wgs = per_head(lfh::env_int("LINFUSION_MLPH_APPLY_WGS", resident * lfh::num_cu()),
                            lfh::env_int("LINFUSION_MLPH_APPLY_BLK", wide ? 1 : 8), &p->blk_apply);
    long long sw = (N + 15) / 16, cap = lfh::env_int("LINFUSION_MLPH_STATS_WGS", 8 * lfh::num_cu()) / (2 * B);
    if (cap < 1) cap = 1;
    p->stats_wgs = (int)(sw < cap ? sw : cap);
    p->ws_partials = up((size_t)units * p->splits * p->ne * sizeof(float));
    p->ws_state = up((size_t)units * p->ne * sizeof(float));
    p->ws_pack = up((size_t)units * (wide ? lfw::wide_packed_bytes(d, dtype) : pack_bytes(d, dtype)));
    p->ws_stats = up((size_t)2 * B * p->n_pad * 2 * sizeof(float));
    p->ws_total = p->ws_partials + p->ws_state + p->ws_pack + p->ws_stats;
    return LINFUSION_OK;
  }
  p->W = H;
  p->n_pad = 0;
  p->stats_wgs = 0;
  p->ws_stats = 0;
  auto per_batch = [&](int want_total, int blk_dflt, int* blk) {
    long long s = want_total / B;
    if (s > n_tiles) s = n_tiles;
    if (s < 1) s = 1;
    long long t = (n_tiles + s - 1) / s;
    *blk = (int)(blk_dflt < t ? blk_dflt : t);
    return (int)((n_tiles + t - 1) / t);
  };
  // (defaults in 256-thread units, as for the row-piece kernels: a workgroup of eight waves counts twice)
  const int unit = H / lf::kWavesPerWG;
  // fp16 up to d = 40 (bf16 up to 32) on eight heads: the reduction fits two workgroups per CU
  // (ReduceMlpCfg::kWavesPerSimd)
  const int rounds = (H == 8 && (d <= 32 || (dtype == LINFUSION_DTYPE_F16 && d <= 40))) ? 2 : 1;
  p->splits = per_batch(lfh::env_int("LINFUSION_MLP_REDUCE_WGS", 2 * lfh::num_cu() * rounds) / unit,
                        lfh::env_int("LINFUSION_MLP_REDUCE_BLK", 2), &p->blk_reduce);
  p->apply_wgs = per_batch(lfh::env_int("LINFUSION_MLP_APPLY_WGS", 2 * lfh::num_cu()) / unit,
                           lfh::env_int("LINFUSION_MLP_APPLY_BLK", H == 8 ? 1 : 2), &p->blk_apply);
  p->ws_partials = up((size_t)B * H * p->splits * p->ne * sizeof(float));
  p->ws_state = up((size_t)B * H * p->ne * sizeof(float));
  p->ws_pack = up((size_t)B * H * pack_bytes(d, dtype));
  p->ws_total = p->ws_partials + p->ws_state + p->ws_pack;
  return LINFUSION_OK;
}

using lfh::allow_lds;

struct MlpArgs {
  const void *a_q, *t_q, *a_k, *t_k, *v;
  void* out;
  const float *gamma_q, *beta_q, *gamma_k, *beta_k;
  int B;
  long long N;
  int fm;
  float eps, ln_eps, slope;
  bool unnorm;
  const MlpPlan* p;
  unsigned char* ws;
  hipStream_t st;
  hipEvent_t* ev;
  long long in_batch, in_row, out_batch, out_row;   // strides in 16-byte units: the five inputs; out
};

template <typename T, int D, int W, int FM, bool NORM>
int run_mlp(const MlpArgs& a) {
  using namespace lf;
  const MlpPlan& p = *a.p;
  constexpr int NE = D * D + D;
  static_assert(W * D % 8 == 0, "rows are whole 16-byte chunks");
  const int row = (int)a.in_row, row_o = (int)a.out_row;   // token strides in 16-byte units (W D / 8 when dense)
  const long long batch = a.in_batch, batch_o = a.out_batch;
  float* partials = reinterpret_cast<float*>(a.ws);
  float* state = reinterpret_cast<float*>(a.ws + p.ws_partials);
  unsigned char* packed = a.ws + p.ws_partials + p.ws_state;
  hipStream_t st = a.st;
  constexpr int lds_r = ReduceMlpCfg<T, D, W>::kLdsBytes;
  constexpr int lds_p = apply16_dma_lds_bytes<T, D>();
  constexpr int lds_a = apply16_mlp_lds_bytes<T, D>(W);
  static_assert(lds_r <= 160 * 1024 && lds_a <= 160 * 1024, "workgroup LDS limit of the device");
  static_assert(Pack16<T, D>::kFrags == NSplit<T>::value * ((D / 2 + 2 + 15) / 16) * ((D / 8 + 1) / 2),
                "the workspace size formula must match the packed layout");
  if (!allow_lds(state_reduce16_mlp<T, D, FM, W>, lds_r) || !allow_lds(pack_state16<T, D, NORM>, lds_p) ||
      !allow_lds(apply16_mlp<T, D, FM, NORM, W>, lds_a))
    return LINFUSION_ERR_HIP;
  if (a.ev) (void)hipEventRecord(a.ev[0], st);
  state_reduce16_mlp<T, D, FM, W><<<dim3(p.splits, (unsigned)a.B), dim3(64 * W), lds_r, st>>>(
      (const u32x4*)a.a_k, (const u32x4*)a.t_k, (const u32x4*)a.v, batch, row, a.gamma_k, a.beta_k, a.ln_eps, a.slope,
      partials, a.N, p.blk_reduce);
  if (a.ev) (void)hipEventRecord(a.ev[1], st);
  combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, (unsigned)(a.B * W)), dim3(kCombineThreads), 0, st>>>(
      partials, p.splits, NE, state);
  pack_state16<T, D, NORM><<<dim3((unsigned)(a.B * W)), dim3(kThreads), lds_p, st>>>(state, packed);
  if (a.ev) (void)hipEventRecord(a.ev[2], st);
  apply16_mlp<T, D, FM, NORM, W><<<dim3(p.apply_wgs, (unsigned)a.B), dim3(64 * W), lds_a, st>>>(
      (const u32x4*)a.a_q, (const u32x4*)a.t_q, batch, row, (u32x4*)a.out, batch_o, row_o, a.gamma_q, a.beta_q, a.ln_eps,
      a.slope, packed, a.eps, a.N, p.blk_apply);
  if (a.ev) (void)hipEventRecord(a.ev[3], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T, int D, int W>
int run_mlp_fm(const MlpArgs& a) {
  switch (a.fm) {
    case 0: return a.unnorm ? run_mlp<T, D, W, 0, false>(a) : run_mlp<T, D, W, 0, true>(a);
    case 1: return a.unnorm ? run_mlp<T, D, W, 1, false>(a) : run_mlp<T, D, W, 1, true>(a);
    default: return a.unnorm ? run_mlp<T, D, W, 2, false>(a) : run_mlp<T, D, W, 2, true>(a);
  }
}

template <int D, int W>
int run_mlp_dtype(int dtype, const MlpArgs& a) {
  return dtype == LINFUSION_DTYPE_F16 ? run_mlp_fm<lf::F16, D, W>(a) : run_mlp_fm<lf::BF16, D, W>(a);
}

int dispatch_mlp(int H, int d, int dtype, const MlpArgs& a) {
  if (H == 8) {
    switch (d) {
#define X(DD) case DD: return run_mlp_dtype<DD, 8>(dtype, a);
      X(8) X(16) X(24) X(32) X(40) X(48)
#undef X
    }
  } else if (H == 4) {
    switch (d) {
#define X(DD) case DD: return run_mlp_dtype<DD, 4>(dtype, a);
      X(8) X(16) X(24) X(32) X(40) X(48) X(56) X(64) X(80)
#undef X
    }
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

using lfh::overlaps;

}  // namespace

extern "C" {

size_t linfusion_attn_mlp_workspace_bytes(int B, int H, long long N, int d, int dtype) {
  MlpPlan p;
  if (make_mlp_plan(B, H, N, d, dtype, &p) != LINFUSION_OK) return 0;
  return p.ws_total;
}

// `sin`, `sout`: element strides {batch, token} of the five inputs (shared) and of out; null = dense [B, N, H*d]
static int mlp_impl(const void* a_q, const void* t_q, const void* a_k, const void* t_k, const void* v, void* out,
                    const float* gamma_q, const float* beta_q, const float* gamma_k, const float* beta_k, int B, int H,
                    long long N, int d, int dtype, int feature_map, float eps, float ln_eps, float slope, unsigned flags,
                    const long long* sin, const long long* sout, void* workspace, size_t workspace_bytes, void* stream,
                    void* events[4]) {
  if (!a_q || !t_q || !a_k || !t_k || !v || !out || !gamma_q || !beta_q || !gamma_k || !beta_k)
    return LINFUSION_ERR_INVALID;
  if (!(eps >= 0.0f) || std::isinf(eps)) return LINFUSION_ERR_INVALID;
  if (!(ln_eps > 0.0f) || std::isinf(ln_eps)) return LINFUSION_ERR_INVALID;
  if (!(slope >= 0.0f && slope <= 1.0f)) return LINFUSION_ERR_INVALID;
  if (flags & ~LINFUSION_FLAG_UNNORMALIZED) return LINFUSION_ERR_INVALID;
  MlpPlan p;
  int rc = make_mlp_plan(B, H, N, d, dtype, &p);
  if (rc != LINFUSION_OK) return rc;
  if (feature_map < 0 || feature_map > 2) return LINFUSION_ERR_UNSUPPORTED;
  const void* ins[5] = {a_q, t_q, a_k, t_k, v};
  for (const void* x : ins)
    if ((uintptr_t)x & 15) return LINFUSION_ERR_MISALIGNED;
  if ((uintptr_t)out & 15) return LINFUSION_ERR_MISALIGNED;
  const float* vecs[4] = {gamma_q, beta_q, gamma_k, beta_k};
  for (const float* x : vecs)
    if ((uintptr_t)x & 3) return LINFUSION_ERR_MISALIGNED;
  const long long C = (long long)H * d;
  const long long dense[2] = {N * C, C};
  const long long* si = sin ? sin : dense;
  const long long* so = sout ? sout : dense;
  for (const long long* st2 : {si, so}) {
    if (st2[0] < 0 || st2[1] < 0) return LINFUSION_ERR_INVALID;
    if (st2[0] % 8 || st2[1] % 8) return LINFUSION_ERR_MISALIGNED;          // 16-byte aligned rows
    if (st2[1] / 8 >= (1LL << 24)) return LINFUSION_ERR_INVALID;            // 32 rows * stride stays in int
    if ((long double)(B - 1) * st2[0] + (long double)(N - 1) * st2[1] + C >= (long double)(1LL << 45))
      return LINFUSION_ERR_INVALID;
  }
  if (si[1] < C && N > 1) return LINFUSION_ERR_INVALID;                     // a token row must hold all heads
  if (so[1] < C && N > 1) return LINFUSION_ERR_OVERLAP;                     // written rows must be disjoint
  if (B > 1 && so[0] < (N - 1) * so[1] + C) return LINFUSION_ERR_OVERLAP;
  const size_t tbytes = (size_t)((B - 1) * si[0] + (N - 1) * si[1] + C) * 2;
  const size_t obytes = (size_t)((B - 1) * so[0] + (N - 1) * so[1] + C) * 2;
  const size_t vbytes = (size_t)C * sizeof(float);
  for (const void* x : ins)
    if (overlaps(out, obytes, x, tbytes)) return LINFUSION_ERR_OVERLAP;
  for (const float* x : vecs)
    if (overlaps(out, obytes, x, vbytes)) return LINFUSION_ERR_OVERLAP;
  if (!workspace) return LINFUSION_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 15) return LINFUSION_ERR_MISALIGNED;
  if (workspace_bytes < p.ws_total) return LINFUSION_ERR_WORKSPACE;
  for (const void* x : ins)
    if (overlaps(workspace, p.ws_total, x, tbytes)) return LINFUSION_ERR_OVERLAP;
  for (const float* x : vecs)
    if (overlaps(workspace, p.ws_total, x, vbytes)) return LINFUSION_ERR_OVERLAP;
  if (overlaps(workspace, p.ws_total, out, obytes)) return LINFUSION_ERR_OVERLAP;
  rc = lfh::check_device();
  if (rc != LINFUSION_OK) return rc;
  if (p.route != 0) {
    unsigned char* ws = (unsigned char*)workspace;
    lfm::HeadsArgs h{a_q, t_q, a_k, t_k, v, out, gamma_q, beta_q, gamma_k, beta_k, B, H, N, d, dtype, feature_map, eps,
                     ln_eps, slope, (flags & LINFUSION_FLAG_UNNORMALIZED) != 0, si[0] / 8, si[1] / 8, so[0] / 8,
                     so[1] / 8, reinterpret_cast<float*>(ws), reinterpret_cast<float*>(ws + p.ws_partials),
                     ws + p.ws_partials + p.ws_state, ws + p.ws_partials + p.ws_state + p.ws_pack, p.n_pad,
                     p.stats_wgs, p.splits, p.blk_reduce, p.apply_wgs, p.blk_apply, p.route == 2, (hipStream_t)stream,
                     reinterpret_cast<hipEvent_t*>(events)};
    return lfm::run_heads(h);
  }
  MlpArgs a{a_q, t_q, a_k, t_k, v, out, gamma_q, beta_q, gamma_k, beta_k, B, N, feature_map, eps, ln_eps, slope,
            (flags & LINFUSION_FLAG_UNNORMALIZED) != 0, &p, (unsigned char*)workspace, (hipStream_t)stream,
            reinterpret_cast<hipEvent_t*>(events), si[0] / 8, si[1] / 8, so[0] / 8, so[1] / 8};
  return dispatch_mlp(H, d, dtype, a);
}

int linfusion_attn_fwd_mlp(const void* a_q, const void* t_q, const void* a_k, const void* t_k, const void* v, void* out,
                           const float* gamma_q, const float* beta_q, const float* gamma_k, const float* beta_k, int B,
                           int H, long long N, int d, int dtype, int feature_map, float eps, float ln_eps, float slope,
                           unsigned flags, void* workspace, size_t workspace_bytes, void* stream, void* events[4]) {
  return mlp_impl(a_q, t_q, a_k, t_k, v, out, gamma_q, beta_q, gamma_k, beta_k, B, H, N, d, dtype, feature_map, eps,
                  ln_eps, slope, flags, nullptr, nullptr, workspace, workspace_bytes, stream, events);
}

int linfusion_attn_fwd_mlp_strided(const void* a_q, const void* t_q, const void* a_k, const void* t_k, const void* v,
                                   void* out, const float* gamma_q, const float* beta_q, const float* gamma_k,
                                   const float* beta_k, int B, int H, long long N, int d, int dtype, int feature_map,
                                   float eps, float ln_eps, float slope, unsigned flags, const long long in_strides[2],
                                   const long long out_strides[2], void* workspace, size_t workspace_bytes,
                                   void* stream, void* events[4]) {
  return mlp_impl(a_q, t_q, a_k, t_k, v, out, gamma_q, beta_q, gamma_k, beta_k, B, H, N, d, dtype, feature_map, eps,
                  ln_eps, slope, flags, in_strides, out_strides, workspace, workspace_bytes, stream, events);
}

}  // extern "C"
