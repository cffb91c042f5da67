// Launches of the replicated-state single-launch kernels (lf_solo.hpp); see lf_solo_api.hpp.
#include "../../include/linfusion.h"

#include "lf_host_api.hpp"
#include "lf_solo.hpp"
#include "lf_solo_api.hpp"

namespace {

using lfh::allow_lds;

#define LF_SWITCH_FM_NORM(CALL)                 \
  switch (a.fm) {                               \
    case 0: if (a.unnorm) { CALL(0, false) } else { CALL(0, true) } break;  \
    case 1: if (a.unnorm) { CALL(1, false) } else { CALL(1, true) } break;  \
    default: if (a.unnorm) { CALL(2, false) } else { CALL(2, true) } break; \
  }

template <typename T, int D>
int solo16_launch(const lfs::SoloArgs& a) {
  using namespace lf;
  constexpr int W = Solo16Cfg<T, D>::kWaves;
  constexpr int lds = Solo16Cfg<T, D>::kLdsBytes;
  const dim3 g((unsigned)(a.G * a.BH));
#define LF_SOLO(FM, NORM)                                                                           \
  if (!allow_lds(solo16<T, D, FM, NORM>, lds)) return LINFUSION_ERR_HIP;                            \
  solo16<T, D, FM, NORM><<<g, dim3(64 * W), lds, a.st>>>((const u32x4*)a.k, (const u32x4*)a.v, a.lkv, (const u32x4*)a.q, \
                                                        a.lq, (u32x4*)a.out, a.lo, a.eps, a.N, a.G, W);
  LF_SWITCH_FM_NORM(LF_SOLO)
#undef LF_SOLO
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <int D>
int solo32_launch(const lfs::SoloArgs& a) {
  using namespace lf;
  constexpr int W = Solo32Cfg<D>::kWaves;
  constexpr int lds = Solo32Cfg<D>::kLdsBytes;
  const dim3 g((unsigned)(a.G * a.BH));
#define LF_SOLO(FM, NORM)                                                                           \
  if (!allow_lds(solo32<D, FM, NORM>, lds)) return LINFUSION_ERR_HIP;                               \
  solo32<D, FM, NORM><<<g, dim3(64 * W), lds, a.st>>>((const f32x4*)a.k, (const f32x4*)a.v, a.lkv, (const f32x4*)a.q,    \
                                                     a.lq, (f32x4*)a.out, a.lo, a.eps, a.N, a.G, W);
  LF_SWITCH_FM_NORM(LF_SOLO)
#undef LF_SOLO
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

}  // namespace

namespace lfs {

int solo_waves(int d, int dtype) {
  if (dtype == LINFUSION_DTYPE_F32) return lf::solo32_waves(d);
  return lf::solo16_waves(d, dtype == LINFUSION_DTYPE_BF16 ? 2 : 1);
}

int run_solo(const SoloArgs& a) {
#define LF_FOR_D(X) X(8) X(16) X(24) X(32) X(40) X(48) X(56) X(64)
  switch (a.dtype) {
    case LINFUSION_DTYPE_F16:
      switch (a.d) {
#define X(DD) case DD: return solo16_launch<lf::F16, DD>(a);
        LF_FOR_D(X)
#undef X
      }
      break;
    case LINFUSION_DTYPE_BF16:
      switch (a.d) {
#define X(DD) case DD: return solo16_launch<lf::BF16, DD>(a);
        LF_FOR_D(X)
#undef X
      }
      break;
    default:
      switch (a.d) {
#define X(DD) case DD: return solo32_launch<DD>(a);
        LF_FOR_D(X)
#undef X
      }
      break;
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

}  // namespace lfs
