// Translation unit of the library: the backward pass for head widths above 80 (lf_backward_wide.hpp), composed
// of the forward's wide state reduction and apply kernels and a few small kernels of its own.
#include "../../include/linfusion.h"

#include "lf_backward_wide.hpp"
#include "lf_bwdw_api.hpp"
#include "lf_host_api.hpp"
#include "lf_wide_api.hpp"

namespace lfbw {

namespace {

size_t up(size_t x) { return (x + 255) & ~(size_t)255; }

struct Regions {
  lfw::WidePlan plan;
  int zsplits;
  size_t ne;
  size_t partials, state, tstate, dstate, tdstate, packed, aux, dzpart, scal, u, gp, tk, total;   // byte offsets
};

int make_regions(int B, int H, long long N, int d, int dtype, Regions* r) {
  size_t pbytes = 0;
  int rc = lfw::wide_launch_plan(B, H, N, d, dtype, &r->plan, &pbytes);
  if (rc != LINFUSION_OK) return rc;
  const size_t BH = (size_t)B * H;
  r->ne = (size_t)d * d + d;
  long long zs = (N + 31) / 32;   // dz partials: at least 32 tokens each
  r->zsplits = (int)(zs < 1 ? 1 : (zs > 64 ? 64 : zs));
  const size_t st = up(BH * r->ne * sizeof(float));
  const size_t tensor = up(BH * (size_t)N * d * 2);
  size_t o = 0;
  r->partials = o; o += up(pbytes);
  r->state = o; o += st;
  r->tstate = o; o += st;
  r->dstate = o; o += st;
  r->tdstate = o; o += st;
  r->packed = o; o += up(BH * lfw::wide_packed_bytes(d, dtype));
  r->aux = o; o += up(BH * 2 * sizeof(float));
  r->dzpart = o; o += up(BH * r->zsplits * d * sizeof(float));
  r->scal = o; o += up(BH * (size_t)N * sizeof(float));
  r->u = o; o += tensor;
  r->gp = o; o += tensor;
  r->tk = o; o += tensor;
  r->total = o;
  return LINFUSION_OK;
}

template <typename T, int D, int FM, bool NORM>
int run(const BwdWideArgs& a, const Regions& r) {
  using namespace lf;
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
  const Layout dense{(long long)a.H * a.N * (D / 8), a.N * (D / 8), D / 8, a.H};
  const dim3 blk(kBwdWideThreads);
  const dim3 per_token((unsigned)((a.N + 3) / 4), (unsigned)BH);
  int rc;

  // the forward state, unless the caller kept it
  const float* state = a.saved_state;
  if (!state) {
    float* own = reinterpret_cast<float*>(ws + r.state);
    const lfw::WideReduceArgs fr{a.k, a.v, a.B, a.H, a.N, D, a.dtype, FM, a.lkv, a.lkv, partials, own, r.plan, st};
    if ((rc = lfw::run_wide_reduce(fr)) != LINFUSION_OK) return rc;
    state = own;
  }
  bwdw_prep_state<D, NORM><<<dim3(D / 16, (unsigned)BH), blk, 0, st>>>(state, tstate, aux);
  // u' = S' g
  {
    const lfw::WideApplyArgs ap{a.g, U, a.B, a.H, a.N, D, a.dtype, kPhiIdentity, 0.0f, true, a.lg, dense, tstate,
                                ws + r.packed, r.plan, st};
    if ((rc = lfw::run_wide_apply(ap)) != LINFUSION_OK) return rc;
  }
  bwdw_q_finish<T, D, FM, NORM><<<per_token, blk, 0, st>>>((const u32x4*)a.q, a.lq, (const u32x4*)a.g, a.lg,
                                                           (const u32x4*)U, tstate, aux, (u32x4*)a.dq, a.ldq,
                                                           (u32x4*)GP, scal, a.eps, a.N);
  // dS' = sum phi(q)^T gp;  dz' = sum phi(q) e'
  {
    const lfw::WideReduceArgs gr{a.q, GP, a.B, a.H, a.N, D, a.dtype, FM, a.lq, dense, partials, raw, r.plan, st};
    if ((rc = lfw::run_wide_reduce(gr)) != LINFUSION_OK) return rc;
  }
  bwdw_dz<T, D, FM><<<dim3(r.zsplits, (unsigned)BH), blk, 0, st>>>((const uint16_t*)a.q, a.lq, scal, dzpart, a.N);
  bwdw_finish_state<D><<<dim3(D / 16, (unsigned)BH), blk, 0, st>>>(raw, dstate, tdstate, dzpart, r.zsplits, aux);
  // dv = dS^T phi(k)
  {
    const lfw::WideApplyArgs ap{a.k, a.dv, a.B, a.H, a.N, D, a.dtype, FM, 0.0f, true, a.lkv, a.ldkv, dstate,
                                ws + r.packed, r.plan, st};
    if ((rc = lfw::run_wide_apply(ap)) != LINFUSION_OK) return rc;
  }
  // t = dS v;  dk = (t + dz) phi'(k)
  {
    const lfw::WideApplyArgs ap{a.v, TK, a.B, a.H, a.N, D, a.dtype, kPhiIdentity, 0.0f, true, a.lkv, dense, tdstate,
                                ws + r.packed, r.plan, st};
    if ((rc = lfw::run_wide_apply(ap)) != LINFUSION_OK) return rc;
  }
  bwdw_k_finish<T, D, FM><<<per_token, blk, 0, st>>>((const u32x4*)a.k, a.lkv, (const u32x4*)TK, dstate,
                                                     (u32x4*)a.dk, a.ldkv, a.N);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <int D>
int run_fm(const BwdWideArgs& a, const Regions& r) {
  using T = lf::F16;
  switch (a.fm) {
    case 0: return a.unnorm ? run<T, D, 0, false>(a, r) : run<T, D, 0, true>(a, r);
    case 1: return a.unnorm ? run<T, D, 1, false>(a, r) : run<T, D, 1, true>(a, r);
    default: return a.unnorm ? run<T, D, 2, false>(a, r) : run<T, D, 2, true>(a, r);
  }
}

}  // namespace

bool bwd_wide_supported(int d, int dtype) { return dtype == LINFUSION_DTYPE_F16 && lfw::wide_supported(d); }

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
  switch (a.d) {
    case 96: return run_fm<96>(a, r);
    case 128: return run_fm<128>(a, r);
    case 160: return run_fm<160>(a, r);
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

}  // namespace lfbw
