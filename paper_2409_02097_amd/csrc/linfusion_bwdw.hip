// Translation unit of the library: the composed backward pass (lf_backward_wide.hpp) -- fp16 at head widths above
// 80 on the forward's wide state reduction and apply kernels, fp32 on the fp32 ones -- and its small kernels.
#include "../../include/linfusion.h"

#include "lf_backward_wide.hpp"
#include "lf_bwdw_api.hpp"
#include "lf_f32_api.hpp"
#include "lf_host_api.hpp"
#include "lf_wide_api.hpp"

namespace lfbw {

namespace {

size_t up(size_t x) { return (x + 255) & ~(size_t)255; }

struct Regions {
  lfw::WidePlan wplan;        // fp16: the wide kernels' launch shape
  lf32::Plan32 fplan;         // fp32: the fp32 kernels'
  int zsplits;
  size_t ne;
  size_t partials, state, tstate, dstate, tdstate, packed, aux, dzpart, scal, u, gp, tk, total;   // byte offsets
};

int make_regions(int B, int H, long long N, int d, int dtype, Regions* r) {
  size_t pbytes = 0;
  const bool f32 = dtype == LINFUSION_DTYPE_F32;
  int rc = f32 ? lf32::launch_plan32(B, H, N, d, &r->fplan, &pbytes) : lfw::wide_launch_plan(B, H, N, d, dtype, &r->wplan, &pbytes);
  if (rc != LINFUSION_OK) return rc;
  const size_t BH = (size_t)B * H;
  r->ne = (size_t)d * d + d;
  long long zs = (N + 31) / 32;   // dz partials: at least 32 tokens each
  r->zsplits = (int)(zs < 1 ? 1 : (zs > 64 ? 64 : zs));
  const size_t st = up(BH * r->ne * sizeof(float));
  const size_t tensor = up(BH * (size_t)N * d * (f32 ? 4 : 2));
  size_t o = 0;
  r->partials = o; o += up(pbytes);
  r->state = o; o += st;
  r->tstate = o; o += st;
  r->dstate = o; o += st;
  r->tdstate = o; o += st;
  r->packed = o; o += f32 ? 0 : up(BH * lfw::wide_packed_bytes(d, dtype));
  r->aux = o; o += up(BH * 2 * sizeof(float));
  r->dzpart = o; o += up(BH * r->zsplits * d * sizeof(float));
  r->scal = o; o += up(BH * (size_t)N * sizeof(float));
  r->u = o; o += tensor;
  r->gp = o; o += tensor;
  r->tk = o; o += tensor;
  r->total = o;
  return LINFUSION_OK;
}

// the two primitives on either set of kernels
template <typename T>
int reduce_to_state(const BwdWideArgs& a, const Regions& r, const void* k, lf::Layout lk, const void* v, lf::Layout lv,
                    int fm, float* partials, float* state) {
  if constexpr (std::is_same<T, lf::F32>::value) {
    const lf32::Reduce32Args x{k, v, a.B, a.H, a.N, a.d, fm, lk, lv, partials, state, r.fplan, a.st};
    return lf32::run_reduce32(x);
  } else {
    const lfw::WideReduceArgs x{k, v, a.B, a.H, a.N, a.d, a.dtype, fm, lk, lv, partials, state, r.wplan, a.st};
    return lfw::run_wide_reduce(x);
  }
}
// out = phi(in) state, no normalizer
template <typename T>
int apply_state(const BwdWideArgs& a, const Regions& r, const void* in, lf::Layout li, void* out, lf::Layout lo, int fm,
                const float* state) {
  if constexpr (std::is_same<T, lf::F32>::value) {
    const lf32::Apply32Args x{in, out, a.B, a.H, a.N, a.d, fm, 0.0f, true, li, lo, state, r.fplan, a.st};
    return lf32::run_apply32(x);
  } else {
    const lfw::WideApplyArgs x{in, out, a.B, a.H, a.N, a.d, a.dtype, fm, 0.0f, true, li, lo, state, a.ws + r.packed,
                               r.wplan, a.st};
    return lfw::run_wide_apply(x);
  }
}

template <typename T, int D, int FM, bool NORM>
int run(const BwdWideArgs& a, const Regions& r) {
  using namespace lf;
  using Elem = typename RowChunk<T>::Elem;
  constexpr int CPR = D / RowChunk<T>::kPer;
  const long long BH = (long long)a.B * a.H;
  hipStream_t st = a.st;
  unsigned char* ws = a.ws;
  float* partials = reinterpret_cast<float*>(ws + r.partials);
  float* raw = reinterpret_cast<float*>(ws + r.state);      // the forward state if computed here; later dS' as reduced
  float* tstate = reinterpret_cast<float*>(ws + r.tstate);
  float* dstate = reinterpret_cast<float*>(ws + r.dstate);
  float* tdstate = reinterpret_cast<float*>(ws + r.tdstate);
  float* aux = reinterpret_cast<float*>(ws + r.aux);
  float* dzpart = reinterpret_cast<float*>(ws + r.dzpart);
  float* scal = reinterpret_cast<float*>(ws + r.scal);
  void* U = ws + r.u;
  void* GP = ws + r.gp;
  void* TK = ws + r.tk;
  // dense [B, H, N, D] temporaries, in 16-byte units
  const Layout dense{(long long)a.H * a.N * CPR, a.N * CPR, CPR, a.H};
  const dim3 blk(kBwdWideThreads);
  const dim3 per_token((unsigned)((a.N + 3) / 4), (unsigned)BH);
  const dim3 strips(D / kBwdStrip, (unsigned)BH);
  int rc;

  // the forward state, unless the caller kept it
  const float* state = a.saved_state;
  if (!state) {
    if ((rc = reduce_to_state<T>(a, r, a.k, a.lkv, a.v, a.lkv, FM, partials, raw)) != LINFUSION_OK) return rc;
    state = raw;
  }
  bwdw_prep_state<D, NORM><<<strips, blk, 0, st>>>(state, tstate, aux);
  // u' = S' g
  if ((rc = apply_state<T>(a, r, a.g, a.lg, U, dense, kPhiIdentity, tstate)) != LINFUSION_OK) return rc;
  bwdw_q_finish<T, D, FM, NORM><<<per_token, blk, 0, st>>>((const u32x4*)a.q, a.lq, (const u32x4*)a.g, a.lg,
                                                           (const u32x4*)U, tstate, aux, (u32x4*)a.dq, a.ldq,
                                                           (u32x4*)GP, scal, a.eps, a.N);
  // dS' = sum phi(q)^T gp;  dz' = sum phi(q) e'
  if ((rc = reduce_to_state<T>(a, r, a.q, a.lq, GP, dense, FM, partials, raw)) != LINFUSION_OK) return rc;
  bwdw_dz<T, D, FM><<<dim3(r.zsplits, (unsigned)BH), blk, 0, st>>>((const Elem*)a.q, a.lq, scal, dzpart, a.N);
  bwdw_finish_state<D><<<strips, blk, 0, st>>>(raw, dstate, tdstate, dzpart, r.zsplits, aux);
  // dv = dS^T phi(k)
  if ((rc = apply_state<T>(a, r, a.k, a.lkv, a.dv, a.ldkv, FM, dstate)) != LINFUSION_OK) return rc;
  // t = dS v;  dk = (t + dz) phi'(k)
  if ((rc = apply_state<T>(a, r, a.v, a.lkv, TK, dense, kPhiIdentity, tdstate)) != LINFUSION_OK) return rc;
  bwdw_k_finish<T, D, FM><<<per_token, blk, 0, st>>>((const u32x4*)a.k, a.lkv, (const u32x4*)TK, dstate,
                                                     (u32x4*)a.dk, a.ldkv, a.N);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T, int D>
int run_fm(const BwdWideArgs& a, const Regions& r) {
  switch (a.fm) {
    case 0: return a.unnorm ? run<T, D, 0, false>(a, r) : run<T, D, 0, true>(a, r);
    case 1: return a.unnorm ? run<T, D, 1, false>(a, r) : run<T, D, 1, true>(a, r);
    default: return a.unnorm ? run<T, D, 2, false>(a, r) : run<T, D, 2, true>(a, r);
  }
}

}  // namespace

bool bwd_wide_supported(int d, int dtype) {
  if (dtype == LINFUSION_DTYPE_F16) return lfw::wide_supported(d);
  return dtype == LINFUSION_DTYPE_F32 && d >= 8 && d <= 64 && d % 8 == 0;
}

size_t bwd_wide_workspace_bytes(int B, int H, long long N, int d, int dtype) {
  Regions r;
  if (!bwd_wide_supported(d, dtype) || make_regions(B, H, N, d, dtype, &r) != LINFUSION_OK) return 0;
  return r.total;
}

int run_bwd_wide(const BwdWideArgs& a) {
  if (!bwd_wide_supported(a.d, a.dtype)) return LINFUSION_ERR_UNSUPPORTED;
  if ((a.N + 3) / 4 > 0x7fffffffLL) return LINFUSION_ERR_INVALID;
  Regions r;
  const int rc = make_regions(a.B, a.H, a.N, a.d, a.dtype, &r);
  if (rc != LINFUSION_OK) return rc;
  if (a.dtype == LINFUSION_DTYPE_F32) {
    switch (a.d) {
#define X(DD) case DD: return run_fm<lf::F32, DD>(a, r);
      X(8) X(16) X(24) X(32) X(40) X(48) X(56) X(64)
#undef X
    }
    return LINFUSION_ERR_UNSUPPORTED;
  }
  switch (a.d) {
    case 96: return run_fm<lf::F16, 96>(a, r);
    case 128: return run_fm<lf::F16, 128>(a, r);
    case 160: return run_fm<lf::F16, 160>(a, r);
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

}  // namespace lfbw
