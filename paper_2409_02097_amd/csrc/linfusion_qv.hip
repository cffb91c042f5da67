// Fifth translation unit of the library: feature width of q, k different from the value width (lf_qv16.hpp).
#include "../../include/linfusion.h"

#include <stdint.h>

#include <cmath>

#include "lf_host_api.hpp"
#include "lf_qv16.hpp"

namespace {


struct QvPlan {
  int splits, blk_reduce, apply_wgs, blk_apply;
  size_t ne, ws_partials, ws_state, ws_total;
};

// the pairs (d_qk, d_v) that have kernels
bool qv_supported(int dk, int dv) {
  if (dk == dv) return false;
  const bool dv_ok = dv == 40 || dv == 64;
  const bool dk_ok = dk == 16 || dk == 32 || dk == 40 || dk == 64 || dk == 80;
  return dv_ok && dk_ok;
}

int make_qv_plan(int B, int H, long long N, int dk, int dv, int dtype, QvPlan* p) {
  if (B <= 0 || H <= 0 || N <= 0 || dk <= 0 || dv <= 0) return LINFUSION_ERR_INVALID;
  if ((long long)B * H > 65535) return LINFUSION_ERR_INVALID;   // grid.y limit
  if (dtype != LINFUSION_DTYPE_F16 && dtype != LINFUSION_DTYPE_BF16) return LINFUSION_ERR_UNSUPPORTED;
  if (!qv_supported(dk, dv)) return LINFUSION_ERR_UNSUPPORTED;
  if (N > (1LL << 40) / (dk > dv ? dk : dv)) return LINFUSION_ERR_INVALID;
  const long long BH = (long long)B * H;
  const long long n_tiles = (N + lf::kTile - 1) / lf::kTile;
  const long long max_s = (n_tiles + lf::kWavesPerWG - 1) / lf::kWavesPerWG;
  auto per_head = [&](int want_total, int blk_dflt, int* blk) {
    long long s = want_total / BH;
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    long long t = (n_tiles + s - 1) / s;
    long long b = blk_dflt < t ? blk_dflt : t;
    *blk = (int)((b + lf::kWavesPerWG - 1) / lf::kWavesPerWG * lf::kWavesPerWG);
    return (int)((n_tiles + t - 1) / t);
  };
  const bool mid = (double)BH * (double)N * (2.0 * dk + 2.0 * dv) * 2.0 <
                   (double)lfh::env_int("LINFUSION_APPLY_ONE_ROUND_MB", 768) * 1048576.0;
  p->splits = per_head(lfh::env_int("LINFUSION_REDUCE_WGS", 2 * lfh::num_cu()), lfh::env_int("LINFUSION_REDUCE_BLK", 16),
                       &p->blk_reduce);
  p->apply_wgs = per_head(lfh::env_int("LINFUSION_APPLY_WGS", (mid ? 2 : 8) * lfh::num_cu()),
                          lfh::env_int("LINFUSION_APPLY_BLK", 8), &p->blk_apply);
  p->ne = (size_t)dk * dv + dk;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  p->ws_partials = up((size_t)BH * p->splits * p->ne * sizeof(float));
  p->ws_state = up((size_t)BH * p->ne * sizeof(float));
  p->ws_total = p->ws_partials + p->ws_state;
  return LINFUSION_OK;
}

using lfh::allow_lds;

struct QvArgs {
  const void *q, *k, *v;
  void* out;
  long long BH, N;
  int fm;
  float eps;
  bool unnorm;
  const QvPlan* p;
  unsigned char* ws;
  hipStream_t st;
  hipEvent_t* ev;
};

template <typename T, int DK, int DV, int FM, bool NORM>
int run_qv(const QvArgs& a) {
  using namespace lf;
  const QvPlan& p = *a.p;
  constexpr int NE = DK * DV + DK;
  float* partials = reinterpret_cast<float*>(a.ws);
  float* state = reinterpret_cast<float*>(a.ws + p.ws_partials);
  hipStream_t st = a.st;
  constexpr int lds_r = reduce16_qv_lds_bytes<T, DK, DV>();
  constexpr int lds_a = apply16_dma_lds_bytes<T, DK, DV>();
  static_assert(lds_r <= 160 * 1024 && lds_a <= 160 * 1024, "workgroup LDS limit of the device");
  if (!allow_lds(state_reduce16_qv<T, DK, DV, FM>, lds_r) || !allow_lds(apply16_qv<T, DK, DV, FM, NORM>, lds_a))
    return LINFUSION_ERR_HIP;
  if (a.ev) (void)hipEventRecord(a.ev[0], st);
  state_reduce16_qv<T, DK, DV, FM><<<dim3(p.splits, (unsigned)a.BH), dim3(kThreads), lds_r, st>>>(
      (const u32x4*)a.k, (const u32x4*)a.v, partials, a.N, p.blk_reduce);
  if (a.ev) (void)hipEventRecord(a.ev[1], st);
  combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, (unsigned)a.BH), dim3(kCombineThreads), 0, st>>>(
      partials, p.splits, NE, state);
  if (a.ev) (void)hipEventRecord(a.ev[2], st);
  apply16_qv<T, DK, DV, FM, NORM><<<dim3(p.apply_wgs, (unsigned)a.BH), dim3(kThreads), lds_a, st>>>(
      (const u32x4*)a.q, (u32x4*)a.out, state, a.eps, a.N, p.blk_apply);
  if (a.ev) (void)hipEventRecord(a.ev[3], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T, int DK, int DV>
int run_qv_fm(const QvArgs& a) {
  switch (a.fm) {
    case 0: return a.unnorm ? run_qv<T, DK, DV, 0, false>(a) : run_qv<T, DK, DV, 0, true>(a);
    case 1: return a.unnorm ? run_qv<T, DK, DV, 1, false>(a) : run_qv<T, DK, DV, 1, true>(a);
    default: return a.unnorm ? run_qv<T, DK, DV, 2, false>(a) : run_qv<T, DK, DV, 2, true>(a);
  }
}

#define LFQ_FOR_PAIRS(X) X(16, 40) X(32, 40) X(64, 40) X(80, 40) X(16, 64) X(32, 64) X(40, 64) X(80, 64)

int dispatch_qv(int dk, int dv, int dtype, const QvArgs& a) {
#define X(DK, DV)                                                                                          \
  if (dk == DK && dv == DV)                                                                                \
    return dtype == LINFUSION_DTYPE_F16 ? run_qv_fm<lf::F16, DK, DV>(a) : run_qv_fm<lf::BF16, DK, DV>(a);
  LFQ_FOR_PAIRS(X)
#undef X
  return LINFUSION_ERR_UNSUPPORTED;
}

using lfh::overlaps;

}  // namespace

extern "C" {

size_t linfusion_attn_qv_workspace_bytes(int B, int H, long long N, int d_qk, int d_v, int dtype) {
  QvPlan p;
  if (make_qv_plan(B, H, N, d_qk, d_v, dtype, &p) != LINFUSION_OK) return 0;
  return p.ws_total;
}

int linfusion_attn_fwd_qv(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d_qk,
                          int d_v, int dtype, int feature_map, float eps, unsigned flags, void* workspace,
                          size_t workspace_bytes, void* stream, void* events[4]) {
  if (!q || !k || !v || !out) return LINFUSION_ERR_INVALID;
  if (!(eps >= 0.0f) || std::isinf(eps)) return LINFUSION_ERR_INVALID;
  if (flags & ~LINFUSION_FLAG_UNNORMALIZED) return LINFUSION_ERR_INVALID;
  QvPlan p;
  int rc = make_qv_plan(B, H, N, d_qk, d_v, dtype, &p);
  if (rc != LINFUSION_OK) return rc;
  if (feature_map < 0 || feature_map > 2) return LINFUSION_ERR_UNSUPPORTED;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)out) & 15) return LINFUSION_ERR_MISALIGNED;
  const size_t qbytes = (size_t)B * H * (size_t)N * d_qk * 2, vbytes = (size_t)B * H * (size_t)N * d_v * 2;
  if (overlaps(out, vbytes, q, qbytes) || overlaps(out, vbytes, k, qbytes) || overlaps(out, vbytes, v, vbytes))
    return LINFUSION_ERR_OVERLAP;
  if (!workspace) return LINFUSION_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 15) return LINFUSION_ERR_MISALIGNED;
  if (workspace_bytes < p.ws_total) return LINFUSION_ERR_WORKSPACE;
  if (overlaps(workspace, p.ws_total, q, qbytes) || overlaps(workspace, p.ws_total, k, qbytes) ||
      overlaps(workspace, p.ws_total, v, vbytes) || overlaps(workspace, p.ws_total, out, vbytes))
    return LINFUSION_ERR_OVERLAP;
  rc = lfh::check_device();
  if (rc != LINFUSION_OK) return rc;
  QvArgs a{q, k, v, out, (long long)B * H, N, feature_map, eps, (flags & LINFUSION_FLAG_UNNORMALIZED) != 0,
           &p, (unsigned char*)workspace, (hipStream_t)stream, reinterpret_cast<hipEvent_t*>(events)};
  return dispatch_qv(d_qk, d_v, dtype, a);
}

}  // extern "C"
