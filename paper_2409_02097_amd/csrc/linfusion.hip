// Host side of the C ABI declared in include/linfusion.h: argument validation, launch plan,
// kernel dispatch.  Every arithmetic step of the method runs in the kernels of
// lf_kernels16.hpp (fp16 / bf16) and lf_kernels32.hpp (fp32).
#include "../../include/linfusion.h"

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <cmath>
#include <mutex>

#include "lf_kernels16.hpp"
#include "lf_apply16_dma.hpp"
#include "lf_kernels32.hpp"

namespace {

constexpr int kVersion = 100;  // 0.1.0
constexpr int kMaxDevices = 16;

// ---- launch plan (pure function of the shape; the library targets one chip: 256 CUs) --------
struct Plan {
  int path;             // 0 = split-N three-kernel path, 1 = fused single launch
  int splits;           // state-reduction workgroups per head
  int tiles_per_split;  // tiles per contiguous block of a reduction workgroup
  int apply_wgs;        // apply workgroups per head
  int tiles_per_wg;     // tiles per contiguous block of an apply workgroup
  long long n_tiles;
  size_t state_floats;     // d*d + d: one partial, and one head's state
  size_t ws_partials, ws_state, ws_total;
};

int env_int(const char* name, int dflt) {
  const char* s = getenv(name);
  if (!s || !*s) return dflt;
  int v = atoi(s);
  return v > 0 ? v : dflt;
}

// tiles per contiguous block of a workgroup, at most its whole share, rounded up to a multiple of
// the waves per workgroup; the environment override is a tuning aid
int block_tiles(int share, const char* env, int dflt) {
  int b = env_int(env, dflt);
  if (b > share) b = share;
  return (b + lf::kWavesPerWG - 1) / lf::kWavesPerWG * lf::kWavesPerWG;
}

bool supported_d(int d) { return d >= 8 && d <= 64 && d % 8 == 0; }

int make_plan(int B, int H, long long N, int d, int dtype, unsigned flags, Plan* p) {
  if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return LINFUSION_ERR_INVALID;
  if ((long long)B * H > 65535) return LINFUSION_ERR_INVALID;   // grid.y limit
  if (flags & ~(LINFUSION_FLAG_UNNORMALIZED | LINFUSION_FLAG_FORCE_SPLIT | LINFUSION_FLAG_FORCE_FUSED))
    return LINFUSION_ERR_INVALID;
  if ((flags & LINFUSION_FLAG_FORCE_SPLIT) && (flags & LINFUSION_FLAG_FORCE_FUSED)) return LINFUSION_ERR_INVALID;
  if (dtype < 0 || dtype > 2) return LINFUSION_ERR_UNSUPPORTED;
  if (!supported_d(d)) return LINFUSION_ERR_UNSUPPORTED;
  if (N > (1LL << 40) / d) return LINFUSION_ERR_INVALID;
  const long long BH = (long long)B * H;
  const int tile = dtype == LINFUSION_DTYPE_F32 ? lf::kTile32 : lf::kTile;
  p->n_tiles = (N + tile - 1) / tile;
  p->path = 0;
  // state reduction (read-only stream): two workgroups per CU on 256 CUs measured best -- fewer,
  // longer streams keep DRAM pages open; at least one tile per wave
  const int want1 = env_int("LINFUSION_REDUCE_WGS", 512);
  long long s = (want1 + BH - 1) / BH;
  long long max_s = (p->n_tiles + lf::kWavesPerWG - 1) / lf::kWavesPerWG;
  if (s > max_s) s = max_s;
  if (s < 1) s = 1;
  long long tps = (p->n_tiles + s - 1) / s;
  s = (p->n_tiles + tps - 1) / tps;
  p->splits = (int)s;
  p->tiles_per_split = block_tiles((int)tps, "LINFUSION_REDUCE_BLK", 16);
  // apply (read + write streams): more, smaller workgroups that sweep memory in one moving window
  const int want2 = env_int("LINFUSION_APPLY_WGS", 2048);
  long long a = (want2 + BH - 1) / BH;
  if (a > max_s) a = max_s;
  if (a < 1) a = 1;
  long long tpw = (p->n_tiles + a - 1) / a;
  a = (p->n_tiles + tpw - 1) / tpw;
  p->apply_wgs = (int)a;
  p->tiles_per_wg = block_tiles((int)tpw, "LINFUSION_APPLY_BLK", 8);
  p->state_floats = (size_t)d * d + d;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  p->ws_partials = up((size_t)BH * p->splits * p->state_floats * sizeof(float));
  p->ws_state = up((size_t)BH * p->state_floats * sizeof(float));
  p->ws_total = p->ws_partials + p->ws_state;
  return LINFUSION_OK;
}

// ---- device check (cached per device) ------------------------------------------------------------
int g_dev_ok[kMaxDevices];   // 0 = unknown, 1 = gfx950, -1 = something else
std::mutex g_mu;

int check_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) { (void)hipGetLastError(); return LINFUSION_ERR_DEVICE; }
  if (dev >= kMaxDevices) return LINFUSION_ERR_DEVICE;
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_dev_ok[dev] == 0) {
    hipDeviceProp_t pr;
    if (hipGetDeviceProperties(&pr, dev) != hipSuccess) { (void)hipGetLastError(); return LINFUSION_ERR_DEVICE; }
    g_dev_ok[dev] = strncmp(pr.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
  }
  return g_dev_ok[dev] == 1 ? LINFUSION_OK : LINFUSION_ERR_DEVICE;
}

bool overlaps(const void* a, size_t na, const void* b, size_t nb) {
  uintptr_t x = (uintptr_t)a, y = (uintptr_t)b;
  return x < y + nb && y < x + na;
}

// ---- kernel dispatch ---------------------------------------------------------------------------------
#define LF_FOR_D(X) X(8) X(16) X(24) X(32) X(40) X(48) X(56) X(64)

template <typename T, int D>
int run16(const void* q, const void* k, const void* v, void* out, long long BH, long long N, int fm, float eps,
          bool unnorm, const Plan& p, unsigned char* ws, float* state_out, hipStream_t st, hipEvent_t* ev) {
  using namespace lf;
  float* partials = reinterpret_cast<float*>(ws);
  float* state = state_out ? state_out : reinterpret_cast<float*>(ws + p.ws_partials);
  constexpr int NE = D * D + D;
  const dim3 g1(p.splits, (unsigned)BH), blk(kThreads);
  const size_t lds = reduce16_lds_bytes<T, D>();
  const u32x4* K = (const u32x4*)k;
  const u32x4* V = (const u32x4*)v;
  if (ev) (void)hipEventRecord(ev[0], st);
  switch (fm) {
    case 0: state_reduce16<T, D, 0><<<g1, blk, lds, st>>>(K, V, partials, N, p.tiles_per_split); break;
    case 1: state_reduce16<T, D, 1><<<g1, blk, lds, st>>>(K, V, partials, N, p.tiles_per_split); break;
    default: state_reduce16<T, D, 2><<<g1, blk, lds, st>>>(K, V, partials, N, p.tiles_per_split); break;
  }
  if (ev) (void)hipEventRecord(ev[1], st);
  combine_state<<<dim3((NE + kCombineElems - 1) / kCombineElems, (unsigned)BH), dim3(kCombineThreads), 0, st>>>(
      partials, p.splits, NE, state);
  if (ev) (void)hipEventRecord(ev[2], st);
  if (out) {
    const dim3 g2(p.apply_wgs, (unsigned)BH);
    const u32x4* Q = (const u32x4*)q;
    u32x4* O = (u32x4*)out;
    const bool dma = env_int("LINFUSION_APPLY_IMPL", 2) == 2;
    const size_t lds2 = dma ? apply16_dma_lds_bytes<T, D>() : apply16_lds_bytes<T, D>();
#define LF_APPLY(FM)                                                                                       \
  if (dma) {                                                                                               \
    if (unnorm) apply16_dma<T, D, FM, false><<<g2, blk, lds2, st>>>(Q, O, state, eps, N, p.tiles_per_wg);  \
    else apply16_dma<T, D, FM, true><<<g2, blk, lds2, st>>>(Q, O, state, eps, N, p.tiles_per_wg);          \
  } else if (unnorm) apply16<T, D, FM, false><<<g2, blk, lds2, st>>>(Q, O, state, eps, N, p.tiles_per_wg); \
  else apply16<T, D, FM, true><<<g2, blk, lds2, st>>>(Q, O, state, eps, N, p.tiles_per_wg);
    switch (fm) {
      case 0: LF_APPLY(0) break;
      case 1: LF_APPLY(1) break;
      default: LF_APPLY(2) break;
    }
#undef LF_APPLY
  }
  if (ev) (void)hipEventRecord(ev[3], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <typename T>
int run16_d(int d, const void* q, const void* k, const void* v, void* out, long long BH, long long N, int fm,
            float eps, bool unnorm, const Plan& p, unsigned char* ws, float* state_out, hipStream_t st,
            hipEvent_t* ev) {
  switch (d) {
#define X(DD) case DD: return run16<T, DD>(q, k, v, out, BH, N, fm, eps, unnorm, p, ws, state_out, st, ev);
    LF_FOR_D(X)
#undef X
    default: return LINFUSION_ERR_UNSUPPORTED;
  }
}

int run32_d(int d, const void* q, const void* k, const void* v, void* out, long long BH, long long N, int fm,
            float eps, bool unnorm, const Plan& p, unsigned char* ws, float* state_out, hipStream_t st,
            hipEvent_t* ev) {
  float* partials = reinterpret_cast<float*>(ws);
  float* state = state_out ? state_out : reinterpret_cast<float*>(ws + p.ws_partials);
  switch (d) {
#define X(DD)                                                                                             \
  case DD:                                                                                                \
    return lf::run32<DD>((const float*)q, (const float*)k, (const float*)v, (float*)out, BH, N, fm, eps, \
                         unnorm, p.splits, p.tiles_per_split, p.apply_wgs, p.tiles_per_wg, partials,      \
                         state, st, ev) == hipSuccess                                             \
               ? LINFUSION_OK                                                                             \
               : LINFUSION_ERR_HIP;
    LF_FOR_D(X)
#undef X
    default: return LINFUSION_ERR_UNSUPPORTED;
  }
}

int validate_common(const void* k, const void* v, int B, int H, long long N, int d, int dtype, int feature_map,
                    unsigned flags, Plan* p) {
  if (!k || !v) return LINFUSION_ERR_INVALID;
  int rc = make_plan(B, H, N, d, dtype, flags, p);
  if (rc != LINFUSION_OK) return rc;
  if (feature_map < 0 || feature_map > 2) return LINFUSION_ERR_UNSUPPORTED;
  if (((uintptr_t)k | (uintptr_t)v) & 15) return LINFUSION_ERR_MISALIGNED;
  return LINFUSION_OK;
}

// library-owned scratch for the convenience entry points
void* g_ws[kMaxDevices];
size_t g_ws_bytes[kMaxDevices];

int owned_workspace(size_t need, void** ws) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return LINFUSION_ERR_DEVICE; }
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_ws_bytes[dev] < need) {
    if (hipDeviceSynchronize() != hipSuccess) { (void)hipGetLastError(); return LINFUSION_ERR_HIP; }
    if (g_ws[dev]) (void)hipFree(g_ws[dev]);
    g_ws[dev] = nullptr;
    g_ws_bytes[dev] = 0;
    size_t cap = need + need / 4;
    if (hipMalloc(&g_ws[dev], cap) != hipSuccess) { (void)hipGetLastError(); return LINFUSION_ERR_HIP; }
    g_ws_bytes[dev] = cap;
  }
  *ws = g_ws[dev];
  return LINFUSION_OK;
}

int fwd_owned(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d, int dtype,
              int feature_map, float eps, void* stream) {
  size_t need = linfusion_attn_workspace_bytes(B, H, N, d, dtype);
  void* ws = nullptr;
  if (need == 0) {
    // let the general entry point name the error (nothing is enqueued for invalid arguments)
    return linfusion_attn_fwd_ex(q, k, v, out, B, H, N, d, dtype, feature_map, eps, 0u, nullptr, 0, stream);
  }
  int rc = check_device();
  if (rc != LINFUSION_OK) return rc;
  rc = owned_workspace(need, &ws);
  if (rc != LINFUSION_OK) return rc;
  return linfusion_attn_fwd_ex(q, k, v, out, B, H, N, d, dtype, feature_map, eps, 0u, ws, g_ws_bytes[0] ? need : need, stream);
}

}  // namespace

extern "C" {

static int fwd_impl(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d,
                    int dtype, int feature_map, float eps, unsigned flags, void* workspace,
                    size_t workspace_bytes, void* stream, hipEvent_t* ev) {
  if (!q || !out) return LINFUSION_ERR_INVALID;
  if (!(eps >= 0.0f) || std::isinf(eps)) return LINFUSION_ERR_INVALID;
  Plan p;
  int rc = validate_common(k, v, B, H, N, d, dtype, feature_map, flags, &p);
  if (rc != LINFUSION_OK) return rc;
  if (((uintptr_t)q | (uintptr_t)out) & 15) return LINFUSION_ERR_MISALIGNED;
  const size_t esz = dtype == LINFUSION_DTYPE_F32 ? 4 : 2;
  const size_t tbytes = (size_t)B * H * (size_t)N * d * esz;
  if (overlaps(out, tbytes, k, tbytes) || overlaps(out, tbytes, v, tbytes)) return LINFUSION_ERR_OVERLAP;
  if (out != q && overlaps(out, tbytes, q, tbytes)) return LINFUSION_ERR_OVERLAP;
  if (!workspace) return LINFUSION_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 15) return LINFUSION_ERR_MISALIGNED;
  if (workspace_bytes < p.ws_total) return LINFUSION_ERR_WORKSPACE;
  if (overlaps(workspace, p.ws_total, out, tbytes) || overlaps(workspace, p.ws_total, q, tbytes) ||
      overlaps(workspace, p.ws_total, k, tbytes) || overlaps(workspace, p.ws_total, v, tbytes))
    return LINFUSION_ERR_OVERLAP;
  rc = check_device();
  if (rc != LINFUSION_OK) return rc;
  const bool unnorm = (flags & LINFUSION_FLAG_UNNORMALIZED) != 0;
  hipStream_t st = (hipStream_t)stream;
  const long long BH = (long long)B * H;
  unsigned char* ws = (unsigned char*)workspace;
  switch (dtype) {
    case LINFUSION_DTYPE_F16: return run16_d<lf::F16>(d, q, k, v, out, BH, N, feature_map, eps, unnorm, p, ws, nullptr, st, ev);
    case LINFUSION_DTYPE_BF16: return run16_d<lf::BF16>(d, q, k, v, out, BH, N, feature_map, eps, unnorm, p, ws, nullptr, st, ev);
    default: return run32_d(d, q, k, v, out, BH, N, feature_map, eps, unnorm, p, ws, nullptr, st, ev);
  }
}

int linfusion_attn_fwd_ex(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d,
                          int dtype, int feature_map, float eps, unsigned flags, void* workspace,
                          size_t workspace_bytes, void* stream) {
  return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, flags, workspace, workspace_bytes, stream, nullptr);
}

int linfusion_attn_fwd_profile(const void* q, const void* k, const void* v, void* out, int B, int H, long long N,
                               int d, int dtype, int feature_map, float eps, unsigned flags, void* workspace,
                               size_t workspace_bytes, void* stream, void* events[4]) {
  if (!events || !events[0] || !events[1] || !events[2] || !events[3]) return LINFUSION_ERR_INVALID;
  hipEvent_t ev[4] = {(hipEvent_t)events[0], (hipEvent_t)events[1], (hipEvent_t)events[2], (hipEvent_t)events[3]};
  return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, flags, workspace, workspace_bytes, stream, ev);
}

size_t linfusion_attn_workspace_bytes(int B, int H, long long N, int d, int dtype) {
  Plan p;
  if (make_plan(B, H, N, d, dtype, 0u, &p) != LINFUSION_OK) return 0;
  return p.ws_total;
}

int linfusion_attn_state(const void* k, const void* v, float* state_out, int B, int H, long long N, int d, int dtype,
                         int feature_map, void* workspace, size_t workspace_bytes, void* stream) {
  if (!state_out) return LINFUSION_ERR_INVALID;
  Plan p;
  int rc = validate_common(k, v, B, H, N, d, dtype, feature_map, 0u, &p);
  if (rc != LINFUSION_OK) return rc;
  if ((uintptr_t)state_out & 15) return LINFUSION_ERR_MISALIGNED;
  if (!workspace) return LINFUSION_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 15) return LINFUSION_ERR_MISALIGNED;
  if (workspace_bytes < p.ws_total) return LINFUSION_ERR_WORKSPACE;
  rc = check_device();
  if (rc != LINFUSION_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const long long BH = (long long)B * H;
  unsigned char* ws = (unsigned char*)workspace;
  switch (dtype) {
    case LINFUSION_DTYPE_F16: return run16_d<lf::F16>(d, nullptr, k, v, nullptr, BH, N, feature_map, 0.f, false, p, ws, state_out, st, nullptr);
    case LINFUSION_DTYPE_BF16: return run16_d<lf::BF16>(d, nullptr, k, v, nullptr, BH, N, feature_map, 0.f, false, p, ws, state_out, st, nullptr);
    default: return run32_d(d, nullptr, k, v, nullptr, BH, N, feature_map, 0.f, false, p, ws, state_out, st, nullptr);
  }
}

int linfusion_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d,
                       int feature_map, float eps, void* stream) {
  return fwd_owned(q, k, v, out, B, H, N, d, LINFUSION_DTYPE_F16, feature_map, eps, stream);
}
int linfusion_attn_fwd_f16(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d,
                           int feature_map, float eps, void* stream) {
  return fwd_owned(q, k, v, out, B, H, N, d, LINFUSION_DTYPE_F16, feature_map, eps, stream);
}
int linfusion_attn_fwd_bf16(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d,
                            int feature_map, float eps, void* stream) {
  return fwd_owned(q, k, v, out, B, H, N, d, LINFUSION_DTYPE_BF16, feature_map, eps, stream);
}
int linfusion_attn_fwd_f32(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d,
                           int feature_map, float eps, void* stream) {
  return fwd_owned(q, k, v, out, B, H, N, d, LINFUSION_DTYPE_F32, feature_map, eps, stream);
}

void linfusion_release(void) {
  std::lock_guard<std::mutex> lk(g_mu);
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess) { (void)hipGetLastError(); return; }
  for (int dev = 0; dev < kMaxDevices; ++dev) {
    if (!g_ws[dev]) continue;
    if (hipSetDevice(dev) == hipSuccess) {
      (void)hipDeviceSynchronize();
      (void)hipFree(g_ws[dev]);
    }
    g_ws[dev] = nullptr;
    g_ws_bytes[dev] = 0;
  }
  (void)hipSetDevice(cur);
  (void)hipGetLastError();
}

const char* linfusion_status_string(int status) {
  switch (status) {
    case LINFUSION_OK: return "ok";
    case LINFUSION_ERR_INVALID: return "invalid argument";
    case LINFUSION_ERR_UNSUPPORTED: return "unsupported head width, dtype or feature map";
    case LINFUSION_ERR_MISALIGNED: return "pointer not 16-byte aligned";
    case LINFUSION_ERR_WORKSPACE: return "workspace missing or too small";
    case LINFUSION_ERR_HIP: return "HIP runtime or launch error";
    case LINFUSION_ERR_DEVICE: return "no gfx950 device";
    case LINFUSION_ERR_OVERLAP: return "buffers overlap";
    default: return "unknown status";
  }
}

int linfusion_version(void) { return kVersion; }

int linfusion_attn_plan(int B, int H, long long N, int d, int dtype, unsigned flags, int plan[4]) {
  if (!plan) return LINFUSION_ERR_INVALID;
  Plan p;
  int rc = make_plan(B, H, N, d, dtype, flags, &p);
  if (rc != LINFUSION_OK) return rc;
  plan[0] = p.path;
  plan[1] = p.splits;
  plan[2] = p.apply_wgs;
  plan[3] = dtype == LINFUSION_DTYPE_F32 ? lf::kTile32 : lf::kTile;
  return LINFUSION_OK;
}

}  // extern "C"
