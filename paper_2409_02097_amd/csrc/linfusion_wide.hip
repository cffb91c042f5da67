// Second translation unit of the library: launches of the kernels for head widths above 64
// (lf_wide16.hpp).  Kept apart from linfusion.hip so that the two compile side by side.
#include "../../include/linfusion.h"

#include "lf_wave16.hpp"
#include "lf_host_api.hpp"
#include "lf_wide_api.hpp"

namespace lfw {

namespace {

using lfh::allow_lds;

// apply16_wave holds the (d + 2) x d fp16 operands of a head in one wave's registers, for both storage types
// (query rows are scaled into fp16's range as they are read): built for every wide width.
template <typename T, int D> constexpr bool wave_ok() { return true; }

template <typename T, int D>
int reduce(const WideReduceArgs& a, hipEvent_t* ev) {
  using namespace lf;
  constexpr int NE = D * D + D;
  const long long BH = (long long)a.B * a.H;
  const dim3 blk(kThreads);
  const u32x4* K = (const u32x4*)a.k;
  const u32x4* V = (const u32x4*)a.v;
  const HeadSubset all{0, a.H};
  hipStream_t st = a.st;
  constexpr int lds1 = reduce16_wide_lds_bytes<T, D>();
  const dim3 g1(a.plan.splits, (unsigned)BH);
  // one workgroup per head: its partial is the state (same layout), and there is nothing to combine
  const bool direct = a.plan.splits == 1;
  float* part = direct ? a.state : a.partials;
  if (ev) (void)hipEventRecord(ev[0], st);
#define LFW_REDUCE(FM)                                                                       \
  {                                                                                          \
    if (!allow_lds(state_reduce16_wide<T, D, FM>, lds1)) return LINFUSION_ERR_HIP;           \
    state_reduce16_wide<T, D, FM><<<g1, blk, lds1, st>>>(K, a.lk, V, a.lv, all, part, a.N, a.plan.blk_reduce); \
  }
  switch (a.fm) {
    case 0: LFW_REDUCE(0) break;
    case 1: LFW_REDUCE(1) break;
    default: LFW_REDUCE(2) break;
  }
#undef LFW_REDUCE
  if (ev) (void)hipEventRecord(ev[1], st);
  if (!direct)
    combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, (unsigned)BH), dim3(kCombineThreads), 0, st>>>(
        a.partials, a.plan.splits, NE, a.state);
  if (ev) (void)hipEventRecord(ev[2], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T, int D>
int apply(const WideApplyArgs& a) {
  using namespace lf;
  const long long BH = (long long)a.B * a.H;
  const dim3 blk(kThreads);
  const u32x4* Q = (const u32x4*)a.q;
  u32x4* O = (u32x4*)a.out;
  const HeadSubset all{0, a.H};
  hipStream_t st = a.st;
  const dim3 g2(a.plan.apply_wgs, (unsigned)BH);
#define LFW_APPLY_W(FM, NORM, WW)                                                                            \
  {                                                                                                          \
    constexpr int lds2 = apply16_wide_lds_bytes<T, D, WW>();                                                 \
    if (!allow_lds(apply16_wide<T, D, FM, NORM, WW>, lds2)) return LINFUSION_ERR_HIP;                        \
    pack_state_wide<T, D, WW><<<dim3(ApplyWideShape<D, WW>::kKS, (unsigned)BH), dim3(64 * WW), 0, st>>>(     \
        a.state, a.packed, NORM ? 1 : 0);                                                                    \
    apply16_wide<T, D, FM, NORM, WW><<<g2, dim3(64 * WW), lds2, st>>>(Q, a.lq, O, a.lo, all, a.packed, a.eps, \
                                                                      a.N, a.plan.blk_apply);                \
  }
#define LFW_APPLY_WAVE(FM, NORM)                                                                             \
  if constexpr (wave_ok<T, D>()) {                                                                          \
    constexpr int lds2 = apply16_wave_lds_bytes<D>();                                                        \
    if (!allow_lds(apply16_wave<T, D, FM, NORM>, lds2)) return LINFUSION_ERR_HIP;                            \
    pack_state_wave<D><<<dim3(ApplyWaveShape<D>::kKS, (unsigned)BH), blk, 0, st>>>(a.state, a.packed,        \
                                                                                  NORM ? 1 : 0);             \
    apply16_wave<T, D, FM, NORM><<<g2, blk, lds2, st>>>(Q, a.lq, O, a.lo, all, a.packed, a.eps, a.N,         \
                                                        a.plan.blk_apply);                                   \
  } else {                                                                                                   \
    return LINFUSION_ERR_UNSUPPORTED;                                                                        \
  }
#define LFW_APPLY(FM, NORM)                                        \
  if (a.plan.wave_apply) { LFW_APPLY_WAVE(FM, NORM) }              \
  else if (a.plan.apply_waves == 8) LFW_APPLY_W(FM, NORM, 8) else LFW_APPLY_W(FM, NORM, 4)
  switch (a.fm) {
    case 0: if (a.unnorm) { LFW_APPLY(0, false) } else { LFW_APPLY(0, true) } break;
    case 1: if (a.unnorm) { LFW_APPLY(1, false) } else { LFW_APPLY(1, true) } break;
    default: if (a.unnorm) { LFW_APPLY(2, false) } else { LFW_APPLY(2, true) } break;
  }
#undef LFW_APPLY
#undef LFW_APPLY_WAVE
#undef LFW_APPLY_W
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T, int D>
int run(const WideArgs& a) {
  const WideReduceArgs r{a.k, a.v, a.B, a.H, a.N, a.d, a.dtype, a.fm, a.lkv, a.lkv, a.partials, a.state, a.plan, a.st};
  int rc = reduce<T, D>(r, a.ev);
  if (rc != LINFUSION_OK) return rc;
  if (a.out) {
    const WideApplyArgs p{a.q, a.out, a.B, a.H, a.N, a.d, a.dtype, a.fm, a.eps, a.unnorm, a.lq, a.lo, a.state,
                          a.packed, a.plan, a.st};
    rc = apply<T, D>(p);
  }
  if (a.ev) (void)hipEventRecord(a.ev[3], a.st);
  return rc;
}

}  // namespace

#define LFW_FOR_D(X) X(96) X(128) X(160)

// room for the operands of any of the apply kernels
template <typename T, int D>
constexpr size_t pack_bytes() {
  size_t b = lf::PackWide<T, D, 4>::kHeadBytes > lf::PackWide<T, D, 8>::kHeadBytes ? lf::PackWide<T, D, 4>::kHeadBytes
                                                                                   : lf::PackWide<T, D, 8>::kHeadBytes;
  if (wave_ok<T, D>() && (size_t)lf::PackWave<D>::kHeadBytes > b) b = lf::PackWave<D>::kHeadBytes;
  return b;
}

bool wide_supported(int d) {
  switch (d) {
#define X(DD) case DD:
    LFW_FOR_D(X)
#undef X
    return true;
  }
  return false;
}

bool wave_apply_supported(int d, int dtype) {
  switch (d) {
#define X(DD) \
  case DD: return dtype == LINFUSION_DTYPE_F16 ? wave_ok<lf::F16, DD>() : wave_ok<lf::BF16, DD>();
    LFW_FOR_D(X)
#undef X
  }
  return false;
}

size_t wide_packed_bytes(int d, int dtype) {
  switch (d) {
#define X(DD) \
  case DD: return dtype == LINFUSION_DTYPE_F16 ? pack_bytes<lf::F16, DD>() : pack_bytes<lf::BF16, DD>();
    LFW_FOR_D(X)
#undef X
  }
  return 0;
}

int run_wide_reduce(const WideReduceArgs& a) {
  switch (a.d) {
#define X(DD) \
  case DD: return a.dtype == LINFUSION_DTYPE_F16 ? reduce<lf::F16, DD>(a, nullptr) : reduce<lf::BF16, DD>(a, nullptr);
    LFW_FOR_D(X)
#undef X
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

int run_wide_apply(const WideApplyArgs& a) {
  switch (a.d) {
#define X(DD) \
  case DD: return a.dtype == LINFUSION_DTYPE_F16 ? apply<lf::F16, DD>(a) : apply<lf::BF16, DD>(a);
    LFW_FOR_D(X)
#undef X
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

int run_wide(const WideArgs& a) {
  switch (a.d) {
#define X(DD) \
  case DD: return a.dtype == LINFUSION_DTYPE_F16 ? run<lf::F16, DD>(a) : run<lf::BF16, DD>(a);
    LFW_FOR_D(X)
#undef X
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

}  // namespace lfw
