// Third translation unit of the library: the backward pass (lf_backward16.hpp) and its entry points.
#include "../../include/linfusion.h"

#include <stdint.h>

#include <cmath>

#include "lf_backward16.hpp"
#include "lf_backward16_rows.hpp"
#include "lf_bwdw_api.hpp"
#include "lf_host_api.hpp"

namespace {


struct BwdPlan {
  int splits, blk_reduce, apply_wgs, blk_apply;
  int apply1_wgs, blk_apply1;   // launch shape of the gradient kernels of which one workgroup fills a CU
  int gsplits, gblk_reduce;   // the state-gradient reduction's own launch shape
  int most;                   // partial states per head the workspace has room for
  bool wide;                  // widths above 80: the composed pass of linfusion_bwdw.hip (its own workspace layout)
  size_t ne, ws_partials, ws_state, ws_scal, ws_pack, ws_total;
  bool kv_packed;             // dK / dV from operands packed once per head, many short-lived workgroups
  int kvp_wgs, kvp_blk;
};

// bytes per head of bwd_pack_kv16's output (PackKV16<T, D>::kHeadBytes, kept in step by a static_assert at the launch)
size_t kv_pack_head_bytes(int d, int dtype) {
  const int ns = dtype == LINFUSION_DTYPE_BF16 ? 2 : 1;
  const int mtb = (d / 2 + 15) / 16, ks = (d / 8 + 1) / 2;
  return 1024 + (size_t)2 * ns * mtb * ks * 64 * 16;
}

bool bwd_supported_d(int d) { return (d >= 8 && d <= 64 && d % 8 == 0) || d == 80; }

int make_bwd_plan(int B, int H, long long N, int d, int dtype, BwdPlan* p) {
  if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return LINFUSION_ERR_INVALID;
  if ((long long)B * H > 65535) return LINFUSION_ERR_INVALID;
  p->wide = lfbw::bwd_wide_supported(d, dtype);   // the composed pass: fp16 above 80, fp32
  if (dtype != LINFUSION_DTYPE_F16 && dtype != LINFUSION_DTYPE_BF16 && !p->wide) return LINFUSION_ERR_UNSUPPORTED;
  if (!bwd_supported_d(d) && !p->wide) return LINFUSION_ERR_UNSUPPORTED;
  if (N > (1LL << 40) / d) return LINFUSION_ERR_INVALID;
  if (p->wide) {
    p->ne = (size_t)d * d + d;
    p->ws_total = lfbw::bwd_wide_workspace_bytes(B, H, N, d, dtype);
    return p->ws_total ? LINFUSION_OK : LINFUSION_ERR_UNSUPPORTED;
  }
  const long long BH = (long long)B * H;
  const long long n_tiles = (N + lf::kTile - 1) / lf::kTile;
  const long long max_s = (n_tiles + lf::kWavesPerWG - 1) / lf::kWavesPerWG;
  auto per_head = [&](int want_total, int blk_dflt, int* blk) {
    long long s = want_total / BH;   // rounded down: one workgroup too many costs a whole extra round
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    long long t = (n_tiles + s - 1) / s;
    long long b = blk_dflt < t ? blk_dflt : t;
    *blk = (int)((b + lf::kWavesPerWG - 1) / lf::kWavesPerWG * lf::kWavesPerWG);
    return (int)((n_tiles + t - 1) / t);
  };
  // Launch sizes measured on MI355X: up to a few hundred MB of tensor traffic two workgroups per CU (one resident
  // round) are best for the gradient kernels too; at GB sizes four (dQ, dK/dV) and eight (state gradient) per CU.
  const bool mid = 4.0 * (double)BH * (double)N * d * 2.0 < (double)lfh::env_int("LINFUSION_APPLY_ONE_ROUND_MB", 768) * 1048576.0;
  p->splits = per_head(lfh::env_int("LINFUSION_REDUCE_WGS", 2 * lfh::num_cu()), lfh::env_int("LINFUSION_REDUCE_BLK", 16),
                       &p->blk_reduce);
  p->gsplits = per_head(lfh::env_int("LINFUSION_BWD_REDUCE_WGS", (mid ? 2 : 8) * lfh::num_cu()),
                        lfh::env_int("LINFUSION_BWD_REDUCE_BLK", 16), &p->gblk_reduce);
  p->apply_wgs = per_head(lfh::env_int("LINFUSION_BWD_APPLY_WGS", (mid ? 2 : 4) * lfh::num_cu()),
                          lfh::env_int("LINFUSION_BWD_APPLY_BLK", 8), &p->blk_apply);
  p->apply1_wgs = per_head(lfh::env_int("LINFUSION_BWD_APPLY1_WGS", lfh::num_cu()),
                           lfh::env_int("LINFUSION_BWD_APPLY1_BLK", 8), &p->blk_apply1);
  p->ne = (size_t)d * d + d;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  int most = p->splits > p->gsplits ? p->splits : p->gsplits;
  if (p->apply_wgs > most) most = p->apply_wgs;   // the merged dQ + state-gradient kernel writes one partial each
  if (p->apply1_wgs > most) most = p->apply1_wgs;
  p->most = most;
  p->ws_partials = up((size_t)BH * most * p->ne * sizeof(float));
  p->ws_state = up((size_t)BH * p->ne * sizeof(float));
  p->ws_scal = up((size_t)BH * (size_t)N * 2 * sizeof(float));
  p->ws_pack = up((size_t)BH * kv_pack_head_bytes(d, dtype));
  p->ws_total = p->ws_partials + 2 * p->ws_state + p->ws_scal + p->ws_pack;
  // Large fp16 problems: dK / dV as many short-lived workgroups of a few tiles each (the hardware deals them out in
  // order, so the chip reads and writes one narrow moving window of memory), which needs a start-up of a few loads:
  // the head's operands are packed once.  Measured at 1.3 GB per tensor, long-lived / 32 tiles per short-lived
  // workgroup: fp16 d = 40 1.92 / 1.88 ms per backward call; d = 64 2.02 / 2.03, d = 80 1.11 / 1.12, bf16 d = 40
  // 2.58 / 2.56 (operands two to four times as large): taken for fp16 up to d = 48.
  const int pk = lfh::env_int("LINFUSION_BWD_KV_PACKED", 1);   // 1: by size and type, 2: never, 3: always
  p->kv_packed = pk == 3 || (pk == 1 && !mid && dtype == LINFUSION_DTYPE_F16 && d <= 48);
  p->kvp_blk = (lfh::env_int("LINFUSION_BWD_KVP_BLK", 32) + lf::kWavesPerWG - 1) / lf::kWavesPerWG * lf::kWavesPerWG;
  if (p->kvp_blk < lf::kWavesPerWG) p->kvp_blk = lf::kWavesPerWG;
  const long long kw = (n_tiles + p->kvp_blk - 1) / p->kvp_blk;
  p->kvp_wgs = (int)(kw < 1048576 ? kw : 1048576);   // blocks beyond that are taken cyclically
  return LINFUSION_OK;
}

using lfh::allow_lds;

struct BwdArgs {
  const float* saved_state;   // the forward state of the same q, k, v, or null: recompute it from k, v
  const void *q, *k, *v, *g;
  void *dq, *dk, *dv;
  int B, H;
  long long N;
  float eps;
  bool unnorm;
  const BwdPlan* p;
  unsigned char* ws;
  hipStream_t st;
  lf::Layout lq, lkv, lg, ldq, ldkv;   // q; k and v; dout; dq; dk and dv
};

// The row-piece kernels run one workgroup of W waves per group and tile, with a longer prologue than the per-head
// kernels: measured token-major, fp16 8 x 40, per-head / row-piece: 5 MB per tensor 43 / 50 us, 21 MB 106 / 102 us,
// 84 MB 408 / 322 us, 1.3 GB 7.0 / 2.6 ms.  They are picked from 24 MB up.
inline bool rows_pay(const BwdArgs& a, int d) {
  return (double)a.B * a.H * (double)a.N * d * 2.0 >= (double)lfh::env_int("LINFUSION_BWD_ROWS_MIN_MB", 24) * 1048576.0;
}

// dK, dV: the row-piece kernel on groups of W heads where the heads of a token are neighbours in memory (k, v and
// dk, dv alike), a head's row is no whole 128-byte line and the heads make whole groups; else the per-head kernel.
template <typename T, int D, int FM, int W>
int launch_kv_rows(const BwdArgs& a, const float* stateD) {
  using namespace lf;
  constexpr int lds = BwdRowsCfg<D, W>::lds_bytes();
  static_assert(lds <= 160 * 1024, "workgroup LDS limit of the device");
  if (!allow_lds(bwd_kv16_rows<T, D, FM, W>, lds)) return LINFUSION_ERR_HIP;
  const int gpb = a.H / W;
  const long long groups = (long long)a.B * gpb;
  const long long n_tiles = (a.N + kTile - 1) / kTile;
  const int resident = 160 * 1024 / lds > 0 ? 160 * 1024 / lds : 1;
  long long wgs = lfh::env_int("LINFUSION_BWD_ROWS_WGS", resident * lfh::num_cu()) / groups;
  if (wgs > n_tiles) wgs = n_tiles;
  if (wgs < 1) wgs = 1;
  long long blk = lfh::env_int("LINFUSION_BWD_ROWS_BLK", 1);
  const long long share = (n_tiles + wgs - 1) / wgs;
  if (blk > share) blk = share;
  bwd_kv16_rows<T, D, FM, W><<<dim3((unsigned)wgs, (unsigned)groups), dim3(64 * W), lds, a.st>>>(
      (const u32x4*)a.k, (const u32x4*)a.v, a.lkv, (u32x4*)a.dk, (u32x4*)a.dv, a.ldkv, gpb, stateD, a.N, (int)blk);
  return LINFUSION_OK;
}

// dQ and the state gradient in one pass (fp16, d <= 48) on groups of heads: as launch_kv_rows; *wgs_used = partial
// states per head written for combine_state
template <typename T, int D, int FM, bool NORM, int W>
int launch_qs_rows(const BwdArgs& a, const float* stateS, float* partials, int* wgs_used) {
  using namespace lf;
  constexpr int lds = BwdRowsCfg<D, W>::lds_bytes() + 64 * W;
  static_assert(lds <= 160 * 1024, "workgroup LDS limit of the device");
  if (!allow_lds(bwd_qs16_rows<T, D, FM, NORM, W>, lds)) return LINFUSION_ERR_HIP;
  const int gpb = a.H / W;
  const long long groups = (long long)a.B * gpb;
  const long long n_tiles = (a.N + kTile - 1) / kTile;
  const int resident = 160 * 1024 / lds > 0 ? 160 * 1024 / lds : 1;
  long long wgs = lfh::env_int("LINFUSION_BWD_ROWS_WGS", resident * lfh::num_cu()) / groups;
  if (wgs > a.p->most) wgs = a.p->most;   // room for the partial states
  if (wgs > n_tiles) wgs = n_tiles;
  if (wgs < 1) wgs = 1;
  long long blk = lfh::env_int("LINFUSION_BWD_ROWS_BLK", 1);
  const long long share = (n_tiles + wgs - 1) / wgs;
  if (blk > share) blk = share;
  bwd_qs16_rows<T, D, FM, NORM, W><<<dim3((unsigned)wgs, (unsigned)groups), dim3(64 * W), lds, a.st>>>(
      (const u32x4*)a.q, a.lq, (const u32x4*)a.g, a.lg, (u32x4*)a.dq, a.ldq, gpb, stateS, partials, a.eps, a.N,
      (int)blk);
  *wgs_used = (int)wgs;
  return LINFUSION_OK;
}

// dQ and the per-token scalars (the separate-kernel path: bf16, d > 48) on groups of heads
template <typename T, int D, int FM, bool NORM, int W>
int launch_q_rows(const BwdArgs& a, const float* stateS, lf::f32x2* scal) {
  using namespace lf;
  constexpr int lds = BwdRowsCfg<D, W>::lds_bytes();
  static_assert(lds <= 160 * 1024, "workgroup LDS limit of the device");
  if (!allow_lds(bwd_q16_rows<T, D, FM, NORM, W>, lds)) return LINFUSION_ERR_HIP;
  const int gpb = a.H / W;
  const long long groups = (long long)a.B * gpb;
  const long long n_tiles = (a.N + kTile - 1) / kTile;
  const int resident = 160 * 1024 / lds > 0 ? 160 * 1024 / lds : 1;
  long long wgs = lfh::env_int("LINFUSION_BWD_ROWS_WGS", resident * lfh::num_cu()) / groups;
  if (wgs > n_tiles) wgs = n_tiles;
  if (wgs < 1) wgs = 1;
  long long blk = lfh::env_int("LINFUSION_BWD_ROWS_BLK", 1);
  const long long share = (n_tiles + wgs - 1) / wgs;
  if (blk > share) blk = share;
  bwd_q16_rows<T, D, FM, NORM, W><<<dim3((unsigned)wgs, (unsigned)groups), dim3(64 * W), lds, a.st>>>(
      (const u32x4*)a.q, a.lq, (const u32x4*)a.g, a.lg, (u32x4*)a.dq, a.ldq, gpb, stateS, scal, a.eps, a.N, (int)blk);
  return LINFUSION_OK;
}

// whether q_rows below takes the dQ launch (bf16 has no row-piece form of the merged kernel and keeps the separate
// row-piece kernels wherever they would be picked)
template <int D>
bool q_rows_wanted(const BwdArgs& a) {
  constexpr int CPR = D / 8;
  if constexpr ((D * 2) % 128 == 0) {
    return false;
  } else {
    if (a.lq.head != CPR || a.lg.head != CPR || a.ldq.head != CPR) return false;
    const int mode = lfh::env_int("LINFUSION_BWD_ROWS", 1);
    if (mode == 2 || (mode != 3 && !rows_pay(a, D))) return false;
    if constexpr (D <= 48) {
      if (a.H % 8 == 0) return true;
    }
    if constexpr (D <= 56 || D == 80) {
      if (a.H % 4 == 0) return true;
    }
    return false;
  }
}

template <typename T, int D, int FM, bool NORM>
bool q_rows(const BwdArgs& a, const float* stateS, lf::f32x2* scal, int* rc) {
  constexpr int CPR = D / 8;
  if constexpr ((D * 2) % 128 == 0) {
    return false;
  } else {
    if (a.lq.head != CPR || a.lg.head != CPR || a.ldq.head != CPR) return false;
    const int mode = lfh::env_int("LINFUSION_BWD_ROWS", 1);   // 1: by size, 2: never, 3: always (a test aid)
    if (mode == 2 || (mode != 3 && !rows_pay(a, D))) return false;
    if constexpr (D <= 48) {
      if (a.H % 8 == 0) { *rc = launch_q_rows<T, D, FM, NORM, 8>(a, stateS, scal); return true; }
    }
    if constexpr (D <= 56 || D == 80) {
      if (a.H % 4 == 0) { *rc = launch_q_rows<T, D, FM, NORM, 4>(a, stateS, scal); return true; }
    }
    return false;
  }
}

template <typename T, int D, int FM, bool NORM>
bool qs_rows(const BwdArgs& a, const float* stateS, float* partials, int* wgs_used, int* rc) {
  constexpr int CPR = D / 8;
  if constexpr ((D * 2) % 128 == 0 || lf::NSplit<T>::value != 1 || D > 48) {
    return false;
  } else {
    if (a.lq.head != CPR || a.lg.head != CPR || a.ldq.head != CPR) return false;
    const int mode = lfh::env_int("LINFUSION_BWD_ROWS", 1);   // 1: by size, 2: never, 3: always (a test aid)
    if (mode == 2 || (mode != 3 && !rows_pay(a, D))) return false;
    if (a.H % 8 == 0) { *rc = launch_qs_rows<T, D, FM, NORM, 8>(a, stateS, partials, wgs_used); return true; }
    if (a.H % 4 == 0) { *rc = launch_qs_rows<T, D, FM, NORM, 4>(a, stateS, partials, wgs_used); return true; }
    return false;
  }
}

// the forward state of token-major k, v by the row-piece reduction (as the forward pass does); *nparts = partial
// states per head written for combine_state
template <typename T, int D, int FM, int W>
int launch_state_rows(const BwdArgs& a, float* partials, int* nparts) {
  using namespace lf;
  constexpr int lds = ReduceRowsCfg<T, D, W>::kLdsBytes;
  if (!allow_lds(state_reduce16_rows<T, D, FM, W>, lds)) return LINFUSION_ERR_HIP;
  const int gpb = a.H / W;
  const long long groups = (long long)a.B * gpb;
  const long long n_tiles = (a.N + kTile - 1) / kTile;
  long long s = lfh::env_int("LINFUSION_GROUP_REDUCE_WGS", 2 * lfh::num_cu()) / (W / kWavesPerWG) / groups;
  if (s > a.p->most) s = a.p->most;   // room for the partial states
  if (s > n_tiles) s = n_tiles;
  if (s < 1) s = 1;
  long long blk = lfh::env_int("LINFUSION_GROUP_REDUCE_BLK", 2);
  const long long share = (n_tiles + s - 1) / s;
  if (blk > share) blk = share;
  state_reduce16_rows<T, D, FM, W><<<dim3((unsigned)s, (unsigned)groups), dim3(64 * W), lds, a.st>>>(
      (const u32x4*)a.k, (const u32x4*)a.v, a.lkv, gpb, partials, a.N, (int)blk);
  *nparts = (int)s;
  return LINFUSION_OK;
}

template <typename T, int D, int FM>
bool state_rows(const BwdArgs& a, float* partials, int* nparts, int* rc) {
  constexpr int CPR = D / 8;
  if constexpr ((D * 2) % 128 == 0) return false;
  if (a.lkv.head != CPR) return false;
  const int mode = lfh::env_int("LINFUSION_BWD_ROWS", 1);   // 1: by size, 2: never, 3: always (a test aid)
  if (mode == 2 || (mode != 3 && !rows_pay(a, D))) return false;
  if constexpr (D <= 64) {
    if (a.H % 8 == 0) { *rc = launch_state_rows<T, D, FM, 8>(a, partials, nparts); return true; }
  }
  if (a.H % 4 == 0) { *rc = launch_state_rows<T, D, FM, 4>(a, partials, nparts); return true; }
  return false;
}

template <int D> constexpr bool kRowsW8 = D <= 48;                       // three slots of eight regions fit the LDS
template <int D> constexpr bool kRowsW4 = D <= 56 || D == 80;

// returns true (and sets *rc) when the row-piece kernel took the launch
template <typename T, int D, int FM>
bool kv_rows(const BwdArgs& a, const float* stateD, int* rc) {
  constexpr int CPR = D / 8;
  if constexpr ((D * 2) % 128 == 0) return false;
  if (a.lkv.head != CPR || a.ldkv.head != CPR) return false;
  const int mode = lfh::env_int("LINFUSION_BWD_ROWS", 1);   // 1: by size, 2: never, 3: always (a test aid)
  if (mode == 2 || (mode != 3 && !rows_pay(a, D))) return false;
  if constexpr (kRowsW8<D>) {
    if (a.H % 8 == 0) { *rc = launch_kv_rows<T, D, FM, 8>(a, stateD); return true; }
  }
  if constexpr (kRowsW4<D>) {
    if (a.H % 4 == 0) { *rc = launch_kv_rows<T, D, FM, 4>(a, stateD); return true; }
  }
  return false;
}

// dK, dV by the per-head kernel: long-lived workgroups that stage the state gradient themselves, or (large fp16
// problems) operands packed once per head and many short-lived workgroups
template <typename T, int D, int FM>
int launch_kv(const BwdArgs& a, const float* stateD) {
  using namespace lf;
  const BwdPlan& p = *a.p;
  const long long BH = (long long)a.B * a.H;
  constexpr int lds_a = BwdCfg<D>::lds_bytes();
  const u32x4* K = (const u32x4*)a.k;
  const u32x4* V = (const u32x4*)a.v;
  if (p.kv_packed) {
    using PK = PackKV16<T, D>;
    unsigned char* packed = a.ws + p.ws_partials + 2 * p.ws_state + p.ws_scal;
    if ((size_t)PK::kHeadBytes != kv_pack_head_bytes(D, NSplit<T>::value == 2 ? LINFUSION_DTYPE_BF16 : LINFUSION_DTYPE_F16))
      return LINFUSION_ERR_WORKSPACE;
    constexpr int lds_ring = BwdCfg<D>::kRing * kWavesPerWG * BwdCfg<D>::kSlotBytes;
    if (!allow_lds(bwd_pack_kv16<T, D>, lds_a) || !allow_lds(bwd_kv16_packed<T, D, FM>, lds_ring)) return LINFUSION_ERR_HIP;
    bwd_pack_kv16<T, D><<<dim3((unsigned)BH), dim3(kThreads), lds_a, a.st>>>(stateD, packed);
    bwd_kv16_packed<T, D, FM><<<dim3((unsigned)p.kvp_wgs, (unsigned)BH), dim3(kThreads), lds_ring, a.st>>>(
        K, V, a.lkv, (u32x4*)a.dk, (u32x4*)a.dv, a.ldkv, packed, a.N, p.kvp_blk);
    return LINFUSION_OK;
  }
  if (!allow_lds(bwd_kv16<T, D, FM>, lds_a)) return LINFUSION_ERR_HIP;
  bwd_kv16<T, D, FM><<<dim3(p.apply_wgs, (unsigned)BH), dim3(kThreads), lds_a, a.st>>>(
      K, V, a.lkv, (u32x4*)a.dk, (u32x4*)a.dv, a.ldkv, stateD, a.N, p.blk_apply);
  return LINFUSION_OK;
}

template <typename T, int D, int FM, bool NORM>
int run_bwd(const BwdArgs& a) {
  using namespace lf;
  const BwdPlan& p = *a.p;
  constexpr int NE = D * D + D;
  const long long BH = (long long)a.B * a.H;
  float* partials = reinterpret_cast<float*>(a.ws);
  float* stateS = reinterpret_cast<float*>(a.ws + p.ws_partials);
  float* stateD = reinterpret_cast<float*>(a.ws + p.ws_partials + p.ws_state);
  f32x2* scal = reinterpret_cast<f32x2*>(a.ws + p.ws_partials + 2 * p.ws_state);
  const u32x4* Q = (const u32x4*)a.q;
  const u32x4* K = (const u32x4*)a.k;
  const u32x4* V = (const u32x4*)a.v;
  const u32x4* G = (const u32x4*)a.g;
  const dim3 blk(kThreads);
  hipStream_t st = a.st;
  const HeadSubset all{0, a.H};
  const dim3 gr(p.splits, (unsigned)BH), ga(p.apply_wgs, (unsigned)BH);
  const dim3 gc((NE + kCombineElems - 1) / kCombineElems, (unsigned)BH);

  constexpr int lds_r = reduce16_lds_bytes<T, D>();
  constexpr int lds_a = BwdCfg<D>::lds_bytes();
  constexpr int lds_s = bwd_state_lds_bytes<T, D>();
  if (!allow_lds(state_reduce16<T, D, FM>, lds_r) || !allow_lds(bwd_q16<T, D, FM, NORM>, lds_a) ||
      !allow_lds(bwd_state16<T, D, FM, NORM>, lds_s) || !allow_lds(bwd_kv16<T, D, FM>, lds_a))
    return LINFUSION_ERR_HIP;

  if (a.saved_state) {
    stateS = const_cast<float*>(a.saved_state);   // only read below
  } else {
    int nparts = p.splits, rcs = LINFUSION_OK;
    if (!state_rows<T, D, FM>(a, partials, &nparts, &rcs))
      state_reduce16<T, D, FM><<<gr, blk, lds_r, st>>>(K, V, a.lkv, all, partials, a.N, p.blk_reduce);
    if (rcs != LINFUSION_OK) return rcs;
    combine_state<0><<<gc, dim3(kCombineThreads), 0, st>>>(partials, nparts, NE, stateS);
  }
  // dQ and the state gradient in one pass over Q and dout.  Its row-piece form exists for fp16 up to d = 48; where
  // the layout asks for row-piece kernels and that form is missing, the separate row-piece kernels are kept.
  constexpr bool kMerged = !(NSplit<T>::value == 2 && D == 80);   // bf16 at d = 80: measured slower than the separate kernels
  constexpr bool kQsRows = NSplit<T>::value == 1 && D <= 48;
  if constexpr (kMerged) {
    bool merged = lfh::env_int("LINFUSION_BWD_MERGED", 1) == 1;
    if (!kQsRows && q_rows_wanted<D>(a)) merged = false;
    if (merged) {
      constexpr int lds_qs = qs_lds_bytes<T, D>();
      static_assert(lds_qs <= 160 * 1024, "workgroup LDS limit of the device");
      if (!allow_lds(bwd_qs16<T, D, FM, NORM>, lds_qs)) return LINFUSION_ERR_HIP;
      const bool two = qs_two_per_cu<T, D>();
      const int qs_wgs = two ? p.apply_wgs : p.apply1_wgs, qs_blk = two ? p.blk_apply : p.blk_apply1;
      if (qs_wgs > p.most) return LINFUSION_ERR_WORKSPACE;   // one partial state per workgroup must fit
      int nparts = qs_wgs, rcq = LINFUSION_OK;
      if (!qs_rows<T, D, FM, NORM>(a, stateS, partials, &nparts, &rcq))
        bwd_qs16<T, D, FM, NORM><<<dim3(qs_wgs, (unsigned)BH), blk, lds_qs, st>>>(
            Q, a.lq, G, a.lg, (u32x4*)a.dq, a.ldq, stateS, partials, a.eps, a.N, qs_blk);
      if (rcq != LINFUSION_OK) return rcq;
      combine_state<0><<<gc, dim3(kCombineThreads), 0, st>>>(partials, nparts, NE, stateD);
      int rck = LINFUSION_OK;
      if (!kv_rows<T, D, FM>(a, stateD, &rck)) rck = launch_kv<T, D, FM>(a, stateD);
      if (rck != LINFUSION_OK) return rck;
      return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
    }
  }
  int rcq = LINFUSION_OK;
  if (!q_rows<T, D, FM, NORM>(a, stateS, scal, &rcq))
    bwd_q16<T, D, FM, NORM><<<ga, blk, lds_a, st>>>(Q, a.lq, G, a.lg, (u32x4*)a.dq, a.ldq, stateS, scal, a.eps, a.N,
                                                    p.blk_apply);
  if (rcq != LINFUSION_OK) return rcq;
  bwd_state16<T, D, FM, NORM><<<dim3(p.gsplits, (unsigned)BH), blk, lds_s, st>>>(Q, a.lq, G, a.lg, scal, stateS,
                                                                                  partials, a.N, p.gblk_reduce);
  combine_state<0><<<gc, dim3(kCombineThreads), 0, st>>>(partials, p.gsplits, NE, stateD);
  int rck = LINFUSION_OK;
  if (!kv_rows<T, D, FM>(a, stateD, &rck)) rck = launch_kv<T, D, FM>(a, stateD);
  if (rck != LINFUSION_OK) return rck;
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T, int D>
int run_bwd_fm(int fm, const BwdArgs& a) {
  switch (fm) {
    case 0: return a.unnorm ? run_bwd<T, D, 0, false>(a) : run_bwd<T, D, 0, true>(a);
    case 1: return a.unnorm ? run_bwd<T, D, 1, false>(a) : run_bwd<T, D, 1, true>(a);
    default: return a.unnorm ? run_bwd<T, D, 2, false>(a) : run_bwd<T, D, 2, true>(a);
  }
}

#define LFB_FOR_D(X) X(8) X(16) X(24) X(32) X(40) X(48) X(56) X(64) X(80)

int dispatch_bwd(int d, int dtype, int fm, const BwdArgs& a) {
  switch (d) {
#define X(DD) \
  case DD: return dtype == LINFUSION_DTYPE_F16 ? run_bwd_fm<lf::F16, DD>(fm, a) : run_bwd_fm<lf::BF16, DD>(fm, a);
    LFB_FOR_D(X)
#undef X
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

using lfh::overlaps;

}  // namespace

extern "C" {

size_t linfusion_attn_bwd_workspace_bytes(int B, int H, long long N, int d, int dtype) {
  BwdPlan p;
  if (make_bwd_plan(B, H, N, d, dtype, &p) != LINFUSION_OK) return 0;
  return p.ws_total;
}

// strides: q; k and v; dout; dq; dk and dv -- element strides {batch, head, token}, null = contiguous [B, H, N, d]
static int bwd_impl(const void* q, const void* k, const void* v, const void* dout, const float* state, void* dq,
                    void* dk, void* dv, int B, int H, long long N, int d, int dtype, int feature_map, float eps,
                    unsigned flags, const long long* const strides[5], void* workspace, size_t workspace_bytes,
                    void* stream) {
  if (!q || !k || !v || !dout || !dq || !dk || !dv) return LINFUSION_ERR_INVALID;
  if (!(eps >= 0.0f) || std::isinf(eps)) return LINFUSION_ERR_INVALID;
  if (flags & ~LINFUSION_FLAG_UNNORMALIZED) return LINFUSION_ERR_INVALID;
  BwdPlan p;
  int rc = make_bwd_plan(B, H, N, d, dtype, &p);
  if (rc != LINFUSION_OK) return rc;
  if (feature_map < 0 || feature_map > 2) return LINFUSION_ERR_UNSUPPORTED;
  const void* ins[4] = {q, k, v, dout};
  void* outs[3] = {dq, dk, dv};
  for (const void* x : ins)
    if ((uintptr_t)x & 15) return LINFUSION_ERR_MISALIGNED;
  for (void* x : outs)
    if ((uintptr_t)x & 15) return LINFUSION_ERR_MISALIGNED;
  const size_t esz = dtype == LINFUSION_DTYPE_F32 ? 4 : 2;
  const long long dense[3] = {(long long)H * N * d, N * d, (long long)d};
  const long long* st5[5];
  for (int i = 0; i < 5; ++i) st5[i] = (strides && strides[i]) ? strides[i] : dense;
  for (int i = 0; i < 5; ++i)
    if ((rc = lfh::check_strides(st5[i], B, H, N, d, esz, i >= 3)) != LINFUSION_OK) return rc;
  // spans of q, k, v, dout and of dq, dk, dv
  const size_t in_span[4] = {lfh::span_bytes(st5[0], B, H, N, d, esz), lfh::span_bytes(st5[1], B, H, N, d, esz),
                             lfh::span_bytes(st5[1], B, H, N, d, esz), lfh::span_bytes(st5[2], B, H, N, d, esz)};
  const size_t out_span[3] = {lfh::span_bytes(st5[3], B, H, N, d, esz), lfh::span_bytes(st5[4], B, H, N, d, esz),
                              lfh::span_bytes(st5[4], B, H, N, d, esz)};
  for (int i = 0; i < 3; ++i) {
    for (int j = 0; j < 4; ++j)
      if (overlaps(outs[i], out_span[i], ins[j], in_span[j])) return LINFUSION_ERR_OVERLAP;
    for (int j = i + 1; j < 3; ++j)
      if (overlaps(outs[i], out_span[i], outs[j], out_span[j])) return LINFUSION_ERR_OVERLAP;
  }
  if (!workspace) return LINFUSION_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 15) return LINFUSION_ERR_MISALIGNED;
  if (workspace_bytes < p.ws_total) return LINFUSION_ERR_WORKSPACE;
  if (state) {
    const size_t sbytes = (size_t)B * H * p.ne * sizeof(float);
    if ((uintptr_t)state & 15) return LINFUSION_ERR_MISALIGNED;
    if (overlaps(workspace, p.ws_total, state, sbytes)) return LINFUSION_ERR_OVERLAP;
    for (int i = 0; i < 3; ++i)
      if (overlaps(outs[i], out_span[i], state, sbytes)) return LINFUSION_ERR_OVERLAP;
  }
  for (int j = 0; j < 4; ++j)
    if (overlaps(workspace, p.ws_total, ins[j], in_span[j])) return LINFUSION_ERR_OVERLAP;
  for (int i = 0; i < 3; ++i)
    if (overlaps(workspace, p.ws_total, outs[i], out_span[i])) return LINFUSION_ERR_OVERLAP;
  rc = lfh::check_device();
  if (rc != LINFUSION_OK) return rc;
  const int per = 16 / (int)esz;   // elements per 16-byte unit
  auto lay = [&](const long long* s) { return lf::Layout{s[0] / per, s[1] / per, (int)(s[2] / per), H}; };   // 16-byte units
  if (p.wide) {
    const lfbw::BwdWideArgs w{state, q, k, v, dout, dq, dk, dv, B, H, N, d, dtype, feature_map, eps,
                              (flags & LINFUSION_FLAG_UNNORMALIZED) != 0, (unsigned char*)workspace,
                              (hipStream_t)stream, lay(st5[0]), lay(st5[1]), lay(st5[2]), lay(st5[3]), lay(st5[4])};
    return lfbw::run_bwd_wide(w);
  }
  BwdArgs a{state, q, k, v, dout, dq, dk, dv, B, H, N, eps, (flags & LINFUSION_FLAG_UNNORMALIZED) != 0,
            &p, (unsigned char*)workspace, (hipStream_t)stream,
            lay(st5[0]), lay(st5[1]), lay(st5[2]), lay(st5[3]), lay(st5[4])};
  return dispatch_bwd(d, dtype, feature_map, a);
}

int linfusion_attn_bwd(const void* q, const void* k, const void* v, const void* dout, const float* state, void* dq,
                       void* dk, void* dv, int B, int H, long long N, int d, int dtype, int feature_map, float eps,
                       unsigned flags, void* workspace, size_t workspace_bytes, void* stream) {
  return bwd_impl(q, k, v, dout, state, dq, dk, dv, B, H, N, d, dtype, feature_map, eps, flags, nullptr, workspace,
                  workspace_bytes, stream);
}

int linfusion_attn_bwd_strided(const void* q, const void* k, const void* v, const void* dout, const float* state,
                               void* dq, void* dk, void* dv, int B, int H, long long N, int d, int dtype,
                               int feature_map, float eps, unsigned flags, const long long q_strides[3],
                               const long long kv_strides[3], const long long dout_strides[3],
                               const long long dq_strides[3], const long long dkv_strides[3], void* workspace,
                               size_t workspace_bytes, void* stream) {
  const long long* const strides[5] = {q_strides, kv_strides, dout_strides, dq_strides, dkv_strides};
  return bwd_impl(q, k, v, dout, state, dq, dk, dv, B, H, N, d, dtype, feature_map, eps, flags, strides, workspace,
                  workspace_bytes, stream);
}

}  // extern "C"
