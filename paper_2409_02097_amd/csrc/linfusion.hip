// Host side of the C ABI declared in include/linfusion.h: argument validation, launch plan,
// kernel dispatch.  Every arithmetic step of the method runs in the kernels of lf_reduce16.hpp,
// lf_apply16_dma.hpp (fp16 / bf16), lf_fp32.hpp (fp32) and lf_fused.hpp (single-launch variant).
#include "../../include/linfusion.h"

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <chrono>
#include <cmath>
#include <mutex>
#include <random>

#include "lf_fused.hpp"
#include "lf_reduce32s.hpp"
#include "lf_solo_api.hpp"
#include "lf_host_api.hpp"
#include "lf_f32_api.hpp"
#include "lf_wide_api.hpp"

namespace {

constexpr int kVersion = 600;  // 0.6.0
constexpr int kMaxDevices = 16;
constexpr int kDefaultCU = 256;   // compute units assumed while no device can be asked (one whole MI355X)

// ---- per-device facts, asked once ---------------------------------------------------------------
std::mutex g_mu;
int g_dev_ok[kMaxDevices];   // 0 = unknown, 1 = gfx950, -1 = something else
int g_dev_cu[kMaxDevices];   // compute units of the device (valid once g_dev_ok != 0)

// fills g_dev_ok / g_dev_cu for the current device; returns its index or -1
int probe_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0) { (void)hipGetLastError(); return -1; }
  if (dev >= kMaxDevices) return -1;
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_dev_ok[dev] == 0) {
    hipDeviceProp_t pr;
    if (hipGetDeviceProperties(&pr, dev) != hipSuccess) { (void)hipGetLastError(); return -1; }
    g_dev_ok[dev] = strncmp(pr.gcnArchName, "gfx950", 6) == 0 ? 1 : -1;
    g_dev_cu[dev] = pr.multiProcessorCount > 0 ? pr.multiProcessorCount : kDefaultCU;
  }
  return dev;
}

// Compute units of the current device: launch sizes and the residency test of the single-launch kernel follow
// it (a partitioned device has fewer than the whole chip's 256).  kDefaultCU when no device is visible, so the
// size queries still answer on a host without a GPU.
int num_cu() {
  const int dev = probe_device();
  return dev >= 0 ? g_dev_cu[dev] : kDefaultCU;
}

// ---- tuning switch ---------------------------------------------------------------------------------
// The LINFUSION_* environment variables (launch shapes, forced routes, the barrier poll limit) are development
// aids.  They are looked at only while tuning is on -- LINFUSION_TUNE=1 in the environment when the library is
// first used, or linfusion_set_tuning(1) -- so the default path reads no environment at all and the launch
// plan is a function of the shape and the device alone.
std::atomic<int> g_tuning{-1};   // -1 = not decided yet

bool tuning_on() {
  int t = g_tuning.load(std::memory_order_relaxed);
  if (t < 0) {
    const char* s = getenv("LINFUSION_TUNE");
    t = (s && *s && atoi(s) > 0) ? 1 : 0;
    g_tuning.store(t, std::memory_order_relaxed);
  }
  return t == 1;
}

// ---- launch plan (pure function of the shape and flags) ----------------------------------------
struct Plan {
  int path;             // 0 = split-N three-kernel path, 1 = fused single launch, 2 = replicated-state launch
  int solo_g;           // replicated-state launch: workgroups per head (0 = the shape cannot use it)
  int splits;           // split path: state-reduction workgroups per head
  int blk_reduce;       //   tiles per contiguous block of a reduction workgroup
  int apply_wgs;        //   apply workgroups per head
  int blk_apply;        //   tiles per contiguous block of an apply workgroup
  int fsplits;          // fused path: workgroups per head (0 = the shape cannot use it)
  int fblk_reduce, fblk_apply;
  // row-piece kernels (heads adjacent in memory): whole groups of gwaves (8 if H % 8 == 0, else 4)
  // heads, one wave per head; workgroups per group
  int gwaves, groups, gsplits, gblk_reduce, gapply_wgs, gblk_apply;
  int apply_waves;      // waves per workgroup of the packed per-head apply (1, 2 or 4)
  bool wave_apply;      // widths above 80: apply16_wave (a wave per tile) instead of apply16_wide
  bool apply_packed;    // per-head apply from operands prepared by pack_state16 (many short-lived workgroups)
  long long n_tiles;
  size_t state_floats;  // d*d + d: one partial, and one head's state
  size_t ws_partials, ws_state, ws_sync, ws_pack, ws_total;   // ws_pack: operand-ready state (row-piece apply)
};

int env_int(const char* name, int dflt) {
  if (!tuning_on()) return dflt;
  const char* s = getenv(name);
  if (!s || !*s) return dflt;
  int v = atoi(s);
  return v > 0 ? v : dflt;
}

// tiles per contiguous block of a workgroup, at most its whole share, rounded up to a multiple of
// the waves per workgroup; the environment override is a tuning aid
int block_tiles(long long share, const char* env, int dflt, int multiple = lf::kWavesPerWG) {
  long long b = env_int(env, dflt);
  if (b > share) b = share;
  if (b > (1 << 28)) b = 1 << 28;
  return (int)((b + multiple - 1) / multiple * multiple);
}

// head widths up to 64 in steps of 8 for every dtype; for the 16-bit types also 80 (same kernels) and the
// wide kernels' widths
bool is_wide(int d) { return d > 80; }
bool supported_d(int d, int dtype) {
  if (d >= 8 && d <= 64 && d % 8 == 0) return true;
  return dtype != LINFUSION_DTYPE_F32 && (d == 80 || lfw::wide_supported(d));
}

// Workgroups of the fused kernel that fit one CU at once (registers and LDS of the largest phase);
// conservative figures, re-checked against the runtime's occupancy query before each fused launch.
int fused_wgs_per_cu(int d, int dtype) {
  if (dtype == LINFUSION_DTYPE_F32) return 2;
  if (d > 64) return 1;
  if (dtype == LINFUSION_DTYPE_BF16) return d <= 40 ? 4 : (d <= 48 ? 3 : 2);
  return d <= 48 ? 4 : 2;
}

// Workgroups of the per-head apply kernel that one CU holds at once (registers and LDS).
int apply_wgs_per_cu(int d, int dtype) {
  if (dtype == LINFUSION_DTYPE_F32) return 2;
  if (d > 64) return 2;
  return fused_wgs_per_cu(d, dtype);
}

// the wide kernels' share of a plan
lfw::WidePlan wide_plan_of(const Plan& p, int dtype) {
  return lfw::WidePlan{p.splits, p.blk_reduce, p.apply_wgs, p.blk_apply,
                       env_int("LINFUSION_WIDE_APPLY_WAVES", dtype == LINFUSION_DTYPE_BF16 ? 8 : 4) == 8 ? 8 : 4,
                       p.wave_apply};
}

// `compact`: size the scratch for the three-kernel path alone (no room for the single launch's partials and
// flags, which take most of the general workspace) -- the plan of the entry point with the fixed scratch array.
int make_plan(int B, int H, long long N, int d, int dtype, unsigned flags, Plan* p, bool compact = false) {
  if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return LINFUSION_ERR_INVALID;
  if ((long long)B * H > 65535) return LINFUSION_ERR_INVALID;   // grid.y limit
  if (flags & ~(LINFUSION_FLAG_UNNORMALIZED | LINFUSION_FLAG_FORCE_SPLIT | LINFUSION_FLAG_FORCE_FUSED |
                LINFUSION_FLAG_FORCE_SOLO))
    return LINFUSION_ERR_INVALID;
  {
    const unsigned forced = flags & (LINFUSION_FLAG_FORCE_SPLIT | LINFUSION_FLAG_FORCE_FUSED | LINFUSION_FLAG_FORCE_SOLO);
    if (forced & (forced - 1)) return LINFUSION_ERR_INVALID;   // at most one path may be forced
  }
  if (dtype < 0 || dtype > 2) return LINFUSION_ERR_UNSUPPORTED;
  if (!supported_d(d, dtype)) return LINFUSION_ERR_UNSUPPORTED;
  if (N > (1LL << 40) / d) return LINFUSION_ERR_INVALID;
  const long long BH = (long long)B * H;
  const int tile = dtype == LINFUSION_DTYPE_F32 ? lf::kTile32 : lf::kTile;
  p->n_tiles = (N + tile - 1) / tile;
  if (is_wide(d)) {
    // wide kernels: every wave of a workgroup visits every tile of its blocks; three-kernel path only
    auto per_head = [&](int want_total, int blk_dflt, const char* env_blk, int* blk) {
      long long s = want_total / BH;   // rounded down: one workgroup too many costs a whole extra round
      if (s > p->n_tiles) s = p->n_tiles;
      if (s < 1) s = 1;
      const long long t = (p->n_tiles + s - 1) / s;
      *blk = block_tiles(t, env_blk, blk_dflt, 1);
      return (int)((p->n_tiles + t - 1) / t);
    };
    // reduction workgroups per CU: two; from 768 MB of tensor traffic on, what fits below d = 160 measured faster
    // (d = 128: three, 3-5 %; d = 96: three for fp16, four for bf16, 6-15 %), while smaller problems lose to the
    // longer combine
    int reduce_per_cu = 2;
    {
      const double bytes = 4.0 * (double)BH * (double)N * d * 2.0;
      if (d <= 128 && bytes >= 768.0 * 1048576.0) reduce_per_cu = (d <= 96 && dtype == LINFUSION_DTYPE_BF16) ? 4 : 3;
    }
    p->splits = per_head(env_int("LINFUSION_WIDE_REDUCE_WGS", reduce_per_cu * num_cu()), 4, "LINFUSION_WIDE_REDUCE_BLK", &p->blk_reduce);
    // a head of one or two tiles: one workgroup sums them and writes the state itself (no partials, no combine
    // launch; from four tiles on a workgroup's tiles in sequence cost more than the launch saved)
    if (p->n_tiles <= env_int("LINFUSION_WIDE_ONE_SPLIT_TILES", 2)) {
      p->splits = 1;
      p->blk_reduce = (int)p->n_tiles;
    }
    // apply: a wave per tile with the head's whole state in its registers where that fits (one workgroup
    // per CU, long-lived: its prologue loads the (d + 2) x d operands), else the workgroup-shared tiles
    p->wave_apply = lfw::wave_apply_supported(d, dtype) && env_int("LINFUSION_WIDE_WAVE_APPLY", 1) == 1;   // 2: never
    if (p->wave_apply) {
      const long long max_a = (p->n_tiles + lf::kWavesPerWG - 1) / lf::kWavesPerWG;   // every wave gets a tile
      // (d = 96 leaves room for a second workgroup per CU: at 2^18 tokens of 8 heads apply 166 -> 157 us; measured
      // slower at d = 128 and 160)
      const bool two_per_cu = d <= 96 && 4.0 * (double)BH * (double)N * d * 2.0 >= 768.0 * 1048576.0;
      long long s = env_int("LINFUSION_WIDE_APPLY_WGS", (two_per_cu ? 2 : 1) * num_cu()) / BH;
      if (s > max_a) s = max_a;
      if (s < 1) s = 1;
      const long long t = (p->n_tiles + s - 1) / s;
      p->apply_wgs = (int)((p->n_tiles + t - 1) / t);
      p->blk_apply = block_tiles(t, "LINFUSION_WIDE_APPLY_BLK", lf::kWavesPerWG);
    } else {
      p->apply_wgs = per_head(env_int("LINFUSION_WIDE_APPLY_WGS", 2 * num_cu()), 1, "LINFUSION_WIDE_APPLY_BLK", &p->blk_apply);
    }
    p->fsplits = 0;
    p->fblk_reduce = p->fblk_apply = 1;
    p->gwaves = lf::kWavesPerWG;
    p->groups = p->gsplits = p->gapply_wgs = 0;
    p->gblk_reduce = p->gblk_apply = 1;
    p->apply_packed = false;
    p->apply_waves = lf::kWavesPerWG;
    p->path = 0;
    p->solo_g = 0;
    if (flags & (LINFUSION_FLAG_FORCE_FUSED | LINFUSION_FLAG_FORCE_SOLO)) return LINFUSION_ERR_UNSUPPORTED;
    p->state_floats = (size_t)d * d + d;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    p->ws_partials = up((size_t)BH * p->splits * p->state_floats * sizeof(float));
    p->ws_state = up((size_t)BH * p->state_floats * sizeof(float));
    // in place of the single-launch flags: the state as apply operands
    p->ws_sync = up((size_t)BH * lfw::wide_packed_bytes(d, dtype));
    p->ws_pack = 0;
    p->ws_total = p->ws_partials + p->ws_state + p->ws_sync;
    return LINFUSION_OK;
  }
  const long long max_s = (p->n_tiles + lf::kWavesPerWG - 1) / lf::kWavesPerWG;   // >= one tile per wave
  auto per_head = [&](int want_total, long long* share) {
    long long s = want_total / BH;   // rounded down: one workgroup too many costs a whole extra round
    if (s > max_s) s = max_s;
    if (s < 1) s = 1;
    long long t = (p->n_tiles + s - 1) / s;
    *share = t;
    return (int)((p->n_tiles + t - 1) / t);
  };
  long long share = 0;
  // state reduction (read-only stream): two workgroups per CU measured best -- fewer, longer
  // streams keep DRAM pages open
  const size_t esz = dtype == LINFUSION_DTYPE_F32 ? 4 : 2;
  const double bytes = 4.0 * (double)BH * (double)N * d * (double)esz;
  // From 768 MB of tensor traffic on, the narrow heads whose tiles carry more vector work than bytes run faster with
  // more, shorter streams (sweeps at 2-4 M tokens of 8 heads: bf16 d = 8 / 16 / 24 / 32 / 40 -30 / -13 / -9 / -3.5 /
  // -3.5 % per call with eight workgroups per CU, fp16 d = 8 / 16 / 24 -32 / -9 / -3 %, fp32 d = 8 -14 % with four;
  // the other widths measured equal or slower that way, smaller problems equal).  Not for the entry point with the
  // fixed scratch array, whose partials are sized for two.
  int reduce_per_cu = 2;
  if (!compact && bytes >= 768.0 * 1048576.0) {
    if (dtype == LINFUSION_DTYPE_F32) reduce_per_cu = d <= 8 ? 4 : 2;
    else if (d <= 24 || (dtype == LINFUSION_DTYPE_BF16 && d <= 40)) reduce_per_cu = 8;
  }
  p->splits = per_head(env_int("LINFUSION_REDUCE_WGS", reduce_per_cu * num_cu()), &share);
  p->blk_reduce = block_tiles(share, "LINFUSION_REDUCE_BLK", 16);
  // apply (read + write streams): more, smaller workgroups that sweep memory in one moving window.
  // Up to a few hundred MB of tensor traffic one resident round measured best (a second, partly filled
  // round costs more than its finer balance gains); beyond that eight workgroups per CU.
  const bool one_round = bytes < (double)env_int("LINFUSION_APPLY_ONE_ROUND_MB", 768) * 1048576.0;
  const int apply_dflt = (one_round ? apply_wgs_per_cu(d, dtype) : 8) * num_cu();
  // Large 16-bit problems: the head's operands are packed once (pack_state16) and apply runs as many short-lived
  // workgroups of about 16 tiles each, dealt out by the hardware in order, so that the chip reads and writes one
  // narrow moving window (measured on the 2 M-token workload: 443 us against 488 us for 2048 long-lived
  // workgroups that each stage and pack the fp32 state themselves).
  const int packed_mode = env_int("LINFUSION_APPLY_PACKED", 1);   // 1 = by size, 2 = never, 3 = always
  p->apply_packed = dtype != LINFUSION_DTYPE_F32 && (packed_mode == 3 || (packed_mode == 1 && !one_round));
  p->apply_waves = lf::kWavesPerWG;
  p->wave_apply = false;
  int apply_want = apply_dflt, blk_dflt = 8;
  if (p->apply_packed) {
    const int w = env_int("LINFUSION_APPLY_WAVES", lf::kWavesPerWG);
    p->apply_waves = (w == 1 || w == 2) ? w : lf::kWavesPerWG;
    const long long by_tiles = BH * p->n_tiles / (4 * p->apply_waves);   // four tiles per wave
    // bf16 operands are twice as large (high and low halves), and at these widths the resident grid of
    // eight long-lived workgroups per CU measured 9-14 % faster than the short-lived ones (d = 32 and 48
    // measured 3-9 % slower that way, fp16 within 1 % either way)
    const bool resident = dtype == LINFUSION_DTYPE_BF16 && (d == 40 || d >= 64);
    if (!one_round && !resident && by_tiles > apply_want) apply_want = by_tiles > (1 << 24) ? (1 << 24) : (int)by_tiles;
    blk_dflt = p->apply_waves;                                           // one tile per wave and round
  }
  {
    // every wave gets at least one tile
    const long long max_a = (p->n_tiles + p->apply_waves - 1) / p->apply_waves;
    long long s = env_int("LINFUSION_APPLY_WGS", apply_want) / BH;
    if (s > max_a) s = max_a;
    if (s < 1) s = 1;
    share = (p->n_tiles + s - 1) / s;
    p->apply_wgs = (int)((p->n_tiles + share - 1) / share);
  }
  p->blk_apply = block_tiles(share, "LINFUSION_APPLY_BLK", blk_dflt, p->apply_waves);
  // fused single launch: every workgroup must be resident at once
  const long long cap = (long long)fused_wgs_per_cu(d, dtype) * num_cu();
  p->fsplits = 0;
  if (BH <= cap && !compact) {
    p->fsplits = per_head((int)(cap / BH * BH), &share);
    if ((long long)p->fsplits * BH > cap) p->fsplits = 0;
    p->fblk_reduce = block_tiles(share, "LINFUSION_REDUCE_BLK", 16);
    p->fblk_apply = block_tiles(share, "LINFUSION_APPLY_BLK", 8);
  }
  // row-piece kernels: a workgroup covers a whole group of four heads, every wave walks all of its tiles
  p->gwaves = (H % 8 == 0 && d <= 64 && env_int("LINFUSION_GROUP_WAVES", 8) == 8) ? 8 : 4;   // d = 80: registers
  p->groups = compact ? 0 : B * (H / p->gwaves);   // (compact: contiguous tensors only, whose heads are never neighbours)
  if (p->groups > 0) {
    auto per_group = [&](int want_total, long long* sh) {
      long long s = want_total / p->groups;
      if (s > p->n_tiles) s = p->n_tiles;
      if (s < 1) s = 1;
      long long t = (p->n_tiles + s - 1) / s;
      *sh = t;
      return (int)((p->n_tiles + t - 1) / t);
    };
    // (the defaults are in 256-thread units: a workgroup of eight waves counts twice)
    const int unit = p->gwaves / lf::kWavesPerWG;
    // (the widths and sizes that take more reduction workgroups per CU above do here as well: four, eight at d = 8;
    // token-major bf16 8 x 40 at 2 M tokens 0.999 -> 0.971 ms, d = 24 0.616 -> 0.556, fp16 d = 8 0.577 -> 0.407)
    const int greduce_per_cu = reduce_per_cu == 8 ? (d <= 8 ? 8 : 4) : 2;
    p->gsplits = per_group(env_int("LINFUSION_GROUP_REDUCE_WGS", greduce_per_cu * num_cu()) / unit, &share);
    p->gblk_reduce = block_tiles(share, "LINFUSION_GROUP_REDUCE_BLK", 2, 1);
    // up to a few hundred MB one workgroup of eight waves (two of four) per CU; large problems as many short-lived
    // workgroups of about `kGroupTilesPerWG` tiles each (the hardware deals them out in order: one narrow moving
    // window of memory, as for the per-head apply; 2 M tokens of 8 x 40: 472 -> 445 us); tiles dealt out one at
    // a time
    constexpr long long kGroupTilesPerWG = 8;
    long long gwant = 2 * num_cu();
    if (!one_round && p->groups * p->n_tiles / kGroupTilesPerWG * unit > gwant)
      gwant = p->groups * p->n_tiles / kGroupTilesPerWG * unit;
    if (gwant > (1 << 24)) gwant = 1 << 24;
    p->gapply_wgs = per_group(env_int("LINFUSION_GROUP_APPLY_WGS", (int)gwant) / unit, &share);
    p->gblk_apply = block_tiles(share, "LINFUSION_GROUP_APPLY_BLK", p->gwaves == 8 ? 1 : 2, 1);
  } else {
    p->gsplits = p->gapply_wgs = 0;
    p->gblk_reduce = p->gblk_apply = lf::kWavesPerWG;
  }
  // Measured on MI355X: with the apply launch sized to one resident round the three short kernels match
  // or beat the single launch (two in-kernel barriers) nearly everywhere; the single launch still wins
  // by 4-7 % for 16-bit heads of 56 and 64 channels between ~128 MB and ~1 GB of tensor traffic (no
  // drain and refill of the chip between phases), so only there it is chosen unasked.
  const double fused_min = (double)env_int("LINFUSION_FUSED_MIN_MB", 128) * 1048576.0;
  const double fused_max = (double)env_int("LINFUSION_FUSED_MAX_MB", 1024) * 1048576.0;
  const bool fused_pays = dtype != LINFUSION_DTYPE_F32 && d > 48 && d <= 64 && bytes >= fused_min && bytes <= fused_max;
  p->path = 0;
  if (p->fsplits > 0 && !(flags & (LINFUSION_FLAG_FORCE_SPLIT | LINFUSION_FLAG_FORCE_SOLO)) &&
      ((flags & LINFUSION_FLAG_FORCE_FUSED) || fused_pays))
    p->path = 1;
  // Replicated-state launch (lf_solo.hpp): one kernel, every workgroup reduces its head's whole state itself.
  // Workgroups per head: one workgroup per CU, but no more than there are blocks of apply tiles.
  p->solo_g = 0;
  if (d <= 64 && !compact && BH <= 32768) {
    const int waves = lfs::solo_waves(d, dtype);
    long long g = num_cu() / BH;
    const long long blocks = (p->n_tiles + waves - 1) / waves;
    if (g > blocks) g = blocks;
    if (g < 1) g = 1;
    if (g * BH <= (1 << 20)) p->solo_g = (int)g;
    // Measured on MI355X it never beat three launches: the repeated reduction runs on ONE compute unit per workgroup
    // and is bound by that unit's vector rate (phi, conversions: about 0.6 us per 32-token tile and SIMD), so it costs
    // 36 us at 4096 tokens of 8 x 40 fp16 (three kernels: 22 us), 51 us at 1024 fp32 tokens (16 us), and only ties
    // below 256 tokens, where the host's call overhead hides everything.  It is therefore taken only when asked for
    // (LINFUSION_FLAG_FORCE_SOLO; LINFUSION_SOLO_MAX_KB under the tuning switch): a launch that needs no workspace
    // content, no barrier and no ticket, e.g. for capture into a graph of very small layers.
    const double kv_head = 2.0 * (double)N * d * (double)esz;
    const bool solo_pays = kv_head <= (double)env_int("LINFUSION_SOLO_MAX_KB", 0) * 1024.0 && BH <= num_cu() &&
                           env_int("LINFUSION_SOLO_MAX_KB", 0) > 0;
    if (p->solo_g > 0 && !(flags & (LINFUSION_FLAG_FORCE_SPLIT | LINFUSION_FLAG_FORCE_FUSED)) &&
        ((flags & LINFUSION_FLAG_FORCE_SOLO) || solo_pays))
      p->path = 2;
  }
  if ((flags & LINFUSION_FLAG_FORCE_SOLO) && p->path != 2) return LINFUSION_ERR_UNSUPPORTED;
  p->state_floats = (size_t)d * d + d;
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  int smax = p->splits > p->fsplits ? p->splits : p->fsplits;
  if (dtype != LINFUSION_DTYPE_F32 && p->gsplits > smax) smax = p->gsplits;
  p->ws_partials = up((size_t)BH * smax * p->state_floats * sizeof(float));
  p->ws_state = up((size_t)BH * p->state_floats * sizeof(float));
  // single launch: one 64-bit flag per workgroup and barrier, then two 64-bit records {last call, failed call}
  p->ws_sync = up((size_t)BH * 2 * (p->fsplits > 0 ? p->fsplits : 1) * sizeof(unsigned long long) + 16);
  p->ws_pack = 0;
  if (dtype != LINFUSION_DTYPE_F32 && (p->groups > 0 || p->apply_packed)) {
    const size_t ns = dtype == LINFUSION_DTYPE_BF16 ? 2 : 1;
    const size_t frags = ns * (size_t)((d / 2 + 2 + 15) / 16) * (size_t)((d / 8 + 1) / 2);   // Pack16<T, D>::kFrags
    p->ws_pack = up((size_t)BH * (256 + frags * 1024));
  }
  p->ws_total = p->ws_partials + p->ws_state + p->ws_sync + p->ws_pack;
  return LINFUSION_OK;
}

// ---- device check (cached per device) ------------------------------------------------------------
int check_device() {
  const int dev = probe_device();
  if (dev < 0) return LINFUSION_ERR_DEVICE;
  return g_dev_ok[dev] == 1 ? LINFUSION_OK : LINFUSION_ERR_DEVICE;
}

using lfh::overlaps;

// Barrier tickets of the single-launch kernel.  A call's ticket is a 64-bit word {t, ~t}: t counts up from a
// base drawn at random once per process, so no earlier call of this or another process used it, and a word the
// (uninitialised) workspace happens to hold equals it only if all 64 bits agree -- a stale flag, a counter, a
// bool or a float pattern never has its upper half equal to the complement of its lower half and to this t.
std::atomic<unsigned> g_ticket{0};
std::once_flag g_ticket_once;

unsigned long long next_ticket() {
  std::call_once(g_ticket_once, [] {
    std::random_device rd;
    const unsigned long long mix = ((unsigned long long)rd() << 32) ^ rd() ^
                                   (unsigned long long)std::chrono::steady_clock::now().time_since_epoch().count();
    g_ticket.store((unsigned)(mix ^ (mix >> 32)) | 1u, std::memory_order_relaxed);
  });
  unsigned t = g_ticket.fetch_add(1, std::memory_order_relaxed);
  if (t == 0) t = g_ticket.fetch_add(1, std::memory_order_relaxed);
  return ((unsigned long long)t << 32) | (unsigned long long)(~t);
}

// true when `grid` workgroups of `kernel` (256 threads, `lds` dynamic bytes) are resident at once
template <typename KernelT>
bool fits_resident(KernelT kernel, size_t lds, long long grid) {
  int per_cu = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, lf::kThreads, lds) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return (long long)per_cu * num_cu() >= grid;
}

using lfh::allow_lds;

// The single-launch kernel's barriers compare flags against a ticket that is new for every call; a captured
// launch would replay an old ticket (its flags already match), so under stream capture the three-kernel path runs.
bool capturing(hipStream_t st) {
  hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &status) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return status != hipStreamCaptureStatusNone;
}

struct Args {
  const void *q, *k, *v;
  void* out;
  long long BH, N;
  int fm;
  float eps;
  bool unnorm;
  const Plan* p;
  unsigned char* ws;
  float* state_out;
  hipStream_t st;
  hipEvent_t* ev;
  lf::Layout lq, lkv, lo;
  bool group_reduce, group_apply;   // use the one-head-per-wave kernels
};

// polls (of about a microsecond each) before a single-launch call gives up at a barrier; the
// environment override exists so that a test can force the give-up path from the host
unsigned spin_limit() {
  if (tuning_on()) {
    const char* s = getenv("LINFUSION_FUSED_SPIN_LIMIT");
    if (s && *s) return (unsigned)strtoul(s, nullptr, 10);
  }
  return 4u << 20;
}

// ---- kernel dispatch ---------------------------------------------------------------------------------
#define LF_FOR_D(X) X(8) X(16) X(24) X(32) X(40) X(48) X(56) X(64)

#define LF_SWITCH_FM_NORM(CALL)                 \
  switch (a.fm) {                               \
    case 0: if (a.unnorm) { CALL(0, false) } else { CALL(0, true) } break;  \
    case 1: if (a.unnorm) { CALL(1, false) } else { CALL(1, true) } break;  \
    default: if (a.unnorm) { CALL(2, false) } else { CALL(2, true) } break; \
  }
#define LF_SWITCH_FM(CALL)      \
  switch (a.fm) {               \
    case 0: CALL(0) break;      \
    case 1: CALL(1) break;      \
    default: CALL(2) break;     \
  }

template <typename T, int D>
int run16(const Args& a) {
  using namespace lf;
  const Plan& p = *a.p;
  float* partials = reinterpret_cast<float*>(a.ws);
  float* state = a.state_out ? a.state_out : reinterpret_cast<float*>(a.ws + p.ws_partials);
  constexpr int NE = D * D + D;
  const dim3 blk(kThreads);
  const u32x4* K = (const u32x4*)a.k;
  const u32x4* V = (const u32x4*)a.v;
  const u32x4* Q = (const u32x4*)a.q;
  u32x4* O = (u32x4*)a.out;
  hipStream_t st = a.st;
  if (p.path == 1 && a.out && !(a.group_reduce || a.group_apply) && !capturing(a.st)) {
    unsigned long long* sync = reinterpret_cast<unsigned long long*>(a.ws + p.ws_partials + p.ws_state);
    unsigned long long* err = sync + a.BH * 2 * p.fsplits;
    const dim3 g(p.fsplits, (unsigned)a.BH);
    const size_t lds = fused16_lds_bytes<T, D>();
    bool launched = false;
#define LF_FUSED(FM, NORM)                                                                               \
  if (allow_lds(fused16<T, D, FM, NORM>, (int)lds) &&                                                    \
      fits_resident(fused16<T, D, FM, NORM>, lds, (long long)p.fsplits * a.BH)) {                        \
    if (a.ev) (void)hipEventRecord(a.ev[0], st);                                                         \
    fused16<T, D, FM, NORM><<<g, blk, lds, st>>>(K, V, a.lkv, Q, a.lq, O, a.lo, partials, state, sync, err,  \
                                                 next_ticket(), spin_limit(), a.eps, a.N, p.fblk_reduce,     \
                                                 p.fblk_apply);                                              \
    launched = true;                                                                                     \
  }
    LF_SWITCH_FM_NORM(LF_FUSED)
#undef LF_FUSED
    if (launched) {
      if (a.ev) { (void)hipEventRecord(a.ev[1], st); (void)hipEventRecord(a.ev[2], st); (void)hipEventRecord(a.ev[3], st); }
      return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
    }
  }
  const size_t lds1 = reduce16_lds_bytes<T, D>();
  if (a.ev) (void)hipEventRecord(a.ev[0], st);
  const int H = a.lkv.H, B = (int)(a.BH / H);
  const int gpb = H / p.gwaves, rest = H % p.gwaves;   // whole groups of heads, heads left over
  const HeadSubset all{0, H}, tail{H - rest, rest > 0 ? rest : 1};
  if (a.group_reduce) {
    const dim3 g1(p.gsplits, (unsigned)p.groups);
#define LF_REDUCE_W(FM, WW)                                                                              \
  {                                                                                                      \
    constexpr int ldsr = ReduceRowsCfg<T, D, WW>::kLdsBytes;                                             \
    if (!allow_lds(state_reduce16_rows<T, D, FM, WW>, ldsr)) return LINFUSION_ERR_HIP;                   \
    state_reduce16_rows<T, D, FM, WW><<<g1, dim3(64 * WW), ldsr, st>>>(K, V, a.lkv, gpb, partials, a.N,  \
                                                                       p.gblk_reduce);                   \
  }
#define LF_REDUCE(FM)                                   \
  if constexpr (D <= 64) {                              \
    if (p.gwaves == 8) LF_REDUCE_W(FM, 8) else LF_REDUCE_W(FM, 4) \
  } else LF_REDUCE_W(FM, 4)
    LF_SWITCH_FM(LF_REDUCE)
#undef LF_REDUCE
#undef LF_REDUCE_W
    if (rest > 0) {   // same number of partials per head, so that one combine serves all heads
      const dim3 g1t(p.gsplits, (unsigned)(B * rest));
#define LF_REDUCE(FM)                                                                    \
  if (!allow_lds(state_reduce16<T, D, FM>, (int)lds1)) return LINFUSION_ERR_HIP;         \
  state_reduce16<T, D, FM><<<g1t, blk, lds1, st>>>(K, V, a.lkv, tail, partials, a.N, p.blk_reduce);
      LF_SWITCH_FM(LF_REDUCE)
#undef LF_REDUCE
    }
  } else {
    const dim3 g1(p.splits, (unsigned)a.BH);
#define LF_REDUCE(FM)                                                                    \
  if (!allow_lds(state_reduce16<T, D, FM>, (int)lds1)) return LINFUSION_ERR_HIP;         \
  state_reduce16<T, D, FM><<<g1, blk, lds1, st>>>(K, V, a.lkv, all, partials, a.N, p.blk_reduce);
    LF_SWITCH_FM(LF_REDUCE)
#undef LF_REDUCE
  }
  if (a.ev) (void)hipEventRecord(a.ev[1], st);
  combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, (unsigned)a.BH), dim3(kCombineThreads), 0, st>>>(
      partials, a.group_reduce ? p.gsplits : p.splits, NE, state);
  if (a.ev && !(a.out && (a.group_apply || p.apply_packed))) (void)hipEventRecord(a.ev[2], st);
  if (a.out) {
    const size_t lds2 = apply16_dma_lds_bytes<T, D>();
    if (a.group_apply) {
      const dim3 g2(p.gapply_wgs, (unsigned)p.groups);
      unsigned char* packed = a.ws + p.ws_partials + p.ws_state + p.ws_sync;
      static_assert(Pack16<T, D>::kFrags == NSplit<T>::value * ((D / 2 + 2 + 15) / 16) * ((D / 8 + 1) / 2),
                    "the workspace size formula must match the packed layout");
      if (!allow_lds(pack_state16<T, D, true>, (int)lds2) || !allow_lds(pack_state16<T, D, false>, (int)lds2))
        return LINFUSION_ERR_HIP;
      if (a.unnorm) pack_state16<T, D, false><<<dim3((unsigned)a.BH), blk, lds2, st>>>(state, packed);
      else pack_state16<T, D, true><<<dim3((unsigned)a.BH), blk, lds2, st>>>(state, packed);
      if (a.ev) (void)hipEventRecord(a.ev[2], st);   // the operand packing counts with the combine
#define LF_APPLY_W(FM, NORM, WW)                                                                          \
  {                                                                                                       \
    constexpr int ldsa = apply16_dma_lds_bytes<T, D>(WW);                                                 \
    if (!allow_lds(apply16_rows<T, D, FM, NORM, WW>, ldsa)) return LINFUSION_ERR_HIP;                     \
    apply16_rows<T, D, FM, NORM, WW><<<g2, dim3(64 * WW), ldsa, st>>>(Q, a.lq, O, a.lo, gpb, packed, a.eps, \
                                                                      a.N, p.gblk_apply);                 \
  }
#define LF_APPLY(FM, NORM)                                          \
  if constexpr (D <= 64) {                                          \
    if (p.gwaves == 8) LF_APPLY_W(FM, NORM, 8) else LF_APPLY_W(FM, NORM, 4) \
  } else LF_APPLY_W(FM, NORM, 4)
      LF_SWITCH_FM_NORM(LF_APPLY)
#undef LF_APPLY
#undef LF_APPLY_W
      if (rest > 0) {
        const dim3 g2t(p.apply_wgs, (unsigned)(B * rest));
#define LF_APPLY(FM, NORM)                                                               \
  if (!allow_lds(apply16_dma<T, D, FM, NORM>, (int)lds2)) return LINFUSION_ERR_HIP;      \
  apply16_dma<T, D, FM, NORM><<<g2t, blk, lds2, st>>>(Q, a.lq, O, a.lo, tail, state, a.eps, a.N, p.blk_apply);
        LF_SWITCH_FM_NORM(LF_APPLY)
#undef LF_APPLY
      }
    } else if (p.apply_packed) {
      const dim3 g2(p.apply_wgs, (unsigned)a.BH);
      unsigned char* packed = a.ws + p.ws_partials + p.ws_state + p.ws_sync;
      if (!allow_lds(pack_state16<T, D, true>, (int)lds2) || !allow_lds(pack_state16<T, D, false>, (int)lds2))
        return LINFUSION_ERR_HIP;
      if (a.unnorm) pack_state16<T, D, false><<<dim3((unsigned)a.BH), blk, lds2, st>>>(state, packed);
      else pack_state16<T, D, true><<<dim3((unsigned)a.BH), blk, lds2, st>>>(state, packed);
      if (a.ev) (void)hipEventRecord(a.ev[2], st);   // the operand packing counts with the combine
#define LF_APPLY_W(FM, NORM, WW)                                                                          \
  {                                                                                                       \
    constexpr size_t lds3 = (size_t)ApplyDmaCfg<D>::kRing * ApplyDmaCfg<D>::kSlotBytes * WW;              \
    if (!allow_lds(apply16_packed<T, D, FM, NORM, WW>, (int)lds3)) return LINFUSION_ERR_HIP;             \
    apply16_packed<T, D, FM, NORM, WW><<<g2, dim3(64 * WW), lds3, st>>>(Q, a.lq, O, a.lo, all, packed, a.eps, a.N, \
                                                                        p.blk_apply);                    \
  }
#define LF_APPLY(FM, NORM)                                                        \
  if (p.apply_waves == 1) LF_APPLY_W(FM, NORM, 1) else if (p.apply_waves == 2) LF_APPLY_W(FM, NORM, 2) else LF_APPLY_W(FM, NORM, 4)
      LF_SWITCH_FM_NORM(LF_APPLY)
#undef LF_APPLY
#undef LF_APPLY_W
    } else {
      const dim3 g2(p.apply_wgs, (unsigned)a.BH);
#define LF_APPLY(FM, NORM)                                                               \
  if (!allow_lds(apply16_dma<T, D, FM, NORM>, (int)lds2)) return LINFUSION_ERR_HIP;      \
  apply16_dma<T, D, FM, NORM><<<g2, blk, lds2, st>>>(Q, a.lq, O, a.lo, all, state, a.eps, a.N, p.blk_apply);
      LF_SWITCH_FM_NORM(LF_APPLY)
#undef LF_APPLY
    }
  }
  if (a.ev) (void)hipEventRecord(a.ev[3], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

// fp32 state reduction of the split path: on the 16-bit matrix cores through three bf16 terms per value
// (state_reduce32_split), or on the fp32 instruction (state_reduce32).  Measured on MI355X, B=1, H=8, whole step:
// d = 8: 249 against 942 us at 2^20 tokens, d = 16: 393 / 939, d = 24: 306 / 531 at 2^19, d = 32: 738 / 1138 at
// 2^20, d = 40: 502 / 632 at 2^19, d = 48: 344 / 355 at 2^18; d = 56: 434 / 422 and d = 64: 495 / 459 the other way
// (its six 16-bit tiles per wave leave one workgroup per CU there); below about 8192 tokens per head the fp32
// instruction's shorter prologue wins (d = 40, N = 2048: 24.8 / 20.6 us, N = 8192: 36.7 / 37.2).
template <int D, int FM>
int launch_reduce32(const lf::f32x4* K, lf::Layout lk, const lf::f32x4* V, lf::Layout lv, float* partials, long long N,
                    int splits, int blk, long long BH, hipStream_t st) {
  using namespace lf;
  const dim3 g1(splits, (unsigned)BH), b(kThreads);
  const int mode = env_int("LINFUSION_F32_SPLIT", 1);   // 1 = by shape, 2 = never, 3 = always
  if (mode == 3 || (mode == 1 && D <= 48 && N >= 8192)) {
    constexpr int lds = reduce32s_lds_bytes<D>();
    if (!lfh::allow_lds(state_reduce32_split<D, FM>, lds)) return LINFUSION_ERR_HIP;
    // the plan counts 16-token tiles; this kernel's are 32 tokens
    const int blk32 = ((blk / 2 + kWavesPerWG - 1) / kWavesPerWG) * kWavesPerWG;
    state_reduce32_split<D, FM><<<g1, b, lds, st>>>(K, lk, V, lv, partials, N, blk32 < kWavesPerWG ? kWavesPerWG : blk32);
  } else {
    constexpr size_t lds = reduce32_lds_bytes<D>() > 1024 ? reduce32_lds_bytes<D>() : 1024;
    state_reduce32<D, FM><<<g1, b, lds, st>>>(K, lk, V, lv, partials, N, blk);
  }
  return LINFUSION_OK;
}

template <int D>
int run32(const Args& a) {
  using namespace lf;
  const Plan& p = *a.p;
  float* partials = reinterpret_cast<float*>(a.ws);
  float* state = a.state_out ? a.state_out : reinterpret_cast<float*>(a.ws + p.ws_partials);
  constexpr int NE = D * D + D;
  const dim3 blk(kThreads);
  const f32x4* K = (const f32x4*)a.k;
  const f32x4* V = (const f32x4*)a.v;
  const f32x4* Q = (const f32x4*)a.q;
  f32x4* O = (f32x4*)a.out;
  hipStream_t st = a.st;
  constexpr size_t ldsf = fused32_lds_bytes<D>();
  constexpr size_t ldsa = apply32_lds_bytes<D>();
  if (p.path == 1 && a.out && !capturing(a.st)) {
    unsigned long long* sync = reinterpret_cast<unsigned long long*>(a.ws + p.ws_partials + p.ws_state);
    unsigned long long* err = sync + a.BH * 2 * p.fsplits;
    const dim3 g(p.fsplits, (unsigned)a.BH);
    bool launched = false;
#define LF_FUSED(FM, NORM)                                                                           \
  if (fits_resident(fused32<D, FM, NORM>, ldsf, (long long)p.fsplits * a.BH)) {                       \
    if (a.ev) (void)hipEventRecord(a.ev[0], st);                                                     \
    fused32<D, FM, NORM><<<g, blk, ldsf, st>>>(K, V, a.lkv, Q, a.lq, O, a.lo, partials, state, sync, err, \
                                              next_ticket(), spin_limit(), a.eps, a.N, p.fblk_reduce,   \
                                              p.fblk_apply);                                            \
    launched = true;                                                                                 \
  }
    LF_SWITCH_FM_NORM(LF_FUSED)
#undef LF_FUSED
    if (launched) {
      if (a.ev) { (void)hipEventRecord(a.ev[1], st); (void)hipEventRecord(a.ev[2], st); (void)hipEventRecord(a.ev[3], st); }
      return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
    }
  }
  if (a.ev) (void)hipEventRecord(a.ev[0], st);
#define LF_REDUCE(FM)                                                                                              \
  if (int rc = launch_reduce32<D, FM>(K, a.lkv, V, a.lkv, partials, a.N, p.splits, p.blk_reduce, a.BH, st)) return rc;
  LF_SWITCH_FM(LF_REDUCE)
#undef LF_REDUCE
  if (a.ev) (void)hipEventRecord(a.ev[1], st);
  combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, (unsigned)a.BH), dim3(kCombineThreads), 0, st>>>(
      partials, p.splits, NE, state);
  if (a.ev) (void)hipEventRecord(a.ev[2], st);
  if (a.out) {
    const dim3 g2(p.apply_wgs, (unsigned)a.BH);
#define LF_APPLY(FM, NORM) apply32<D, FM, NORM><<<g2, blk, ldsa, st>>>(Q, a.lq, O, a.lo, state, a.eps, a.N, p.blk_apply);
    LF_SWITCH_FM_NORM(LF_APPLY)
#undef LF_APPLY
  }
  if (a.ev) (void)hipEventRecord(a.ev[3], st);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

int dispatch(int d, int dtype, const Args& a) {
  if (a.p->path == 2 && a.out) {      // replicated-state single launch: no workspace, one kernel
    if (a.ev) (void)hipEventRecord(a.ev[0], a.st);
    const lfs::SoloArgs s{a.q, a.k, a.v, a.out, a.BH, a.N, d, dtype, a.fm, a.eps, a.unnorm, a.lq, a.lkv, a.lo,
                          a.p->solo_g, a.st};
    const int rc = lfs::run_solo(s);
    if (a.ev) { (void)hipEventRecord(a.ev[1], a.st); (void)hipEventRecord(a.ev[2], a.st); (void)hipEventRecord(a.ev[3], a.st); }
    return rc;
  }
  if (is_wide(d)) {
    const Plan& p = *a.p;
    lfw::WideArgs w{a.q, a.k, a.v, a.out, (int)(a.BH / a.lkv.H), a.lkv.H, a.N, d, dtype, a.fm, a.eps, a.unnorm,
                    a.lq, a.lkv, a.lo, reinterpret_cast<float*>(a.ws),
                    a.state_out ? a.state_out : reinterpret_cast<float*>(a.ws + p.ws_partials),
                    a.ws + p.ws_partials + p.ws_state, wide_plan_of(p, dtype), a.st, a.ev};
    return lfw::run_wide(w);
  }
  switch (dtype) {
    case LINFUSION_DTYPE_F16:
      switch (d) {
#define X(DD) case DD: return run16<lf::F16, DD>(a);
        LF_FOR_D(X) X(80)
#undef X
      }
      break;
    case LINFUSION_DTYPE_BF16:
      switch (d) {
#define X(DD) case DD: return run16<lf::BF16, DD>(a);
        LF_FOR_D(X) X(80)
#undef X
      }
      break;
    default:
      switch (d) {
#define X(DD) case DD: return run32<DD>(a);
        LF_FOR_D(X)
#undef X
      }
      break;
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

int validate_common(const void* k, const void* v, int B, int H, long long N, int d, int dtype, int feature_map,
                    unsigned flags, Plan* p, bool compact = false) {
  if (!k || !v) return LINFUSION_ERR_INVALID;
  int rc = make_plan(B, H, N, d, dtype, flags, p, compact);
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

// ---- tensor layouts ------------------------------------------------------------------------------
// Strides in elements between batches, heads and tokens; the d channels of a token are contiguous.
struct Strides { long long b, h, n; };

Strides contiguous_strides(int H, long long N, int d) { return Strides{(long long)H * N * d, N * d, (long long)d}; }

// bytes from the first to one past the last element the layout touches
size_t span_bytes(const Strides& s, int B, int H, long long N, int d, size_t esz) {
  return (size_t)((B - 1) * s.b + (H - 1) * s.h + (N - 1) * s.n + d) * esz;
}

// LINFUSION_OK when the kernels can address the layout: non-negative strides that keep every token row
// 16-byte aligned and within the index widths the kernels use.  `written`: additionally no two
// (batch, head, token) rows may share memory -- checked by ordering the dimensions by stride and
// requiring each stride to clear the span of the smaller ones.
int check_strides(const Strides& s, int B, int H, long long N, int d, size_t esz, bool written) {
  const long long vec = (long long)(16 / esz);
  if (s.b < 0 || s.h < 0 || s.n < 0) return LINFUSION_ERR_INVALID;
  if (s.b % vec || s.h % vec || s.n % vec) return LINFUSION_ERR_MISALIGNED;
  if (s.n / vec >= (1LL << 24)) return LINFUSION_ERR_INVALID;           // 32 rows * stride stays in int
  const long double span = (long double)(B - 1) * s.b + (long double)(H - 1) * s.h + (long double)(N - 1) * s.n + d;
  if (span * esz >= (long double)(1LL << 46)) return LINFUSION_ERR_INVALID;
  if (written) {
    struct Dim { long long extent, stride; } dims[4] = {{d, 1}, {N, s.n}, {H, s.h}, {B, s.b}};
    int n = 0;
    for (int i = 0; i < 4; ++i)
      if (dims[i].extent > 1) dims[n++] = dims[i];
    for (int i = 1; i < n; ++i)            // insertion sort by stride
      for (int j = i; j > 0 && dims[j].stride < dims[j - 1].stride; --j) { Dim t = dims[j]; dims[j] = dims[j - 1]; dims[j - 1] = t; }
    long long reach = 1;                   // elements spanned by the dimensions seen so far
    for (int i = 0; i < n; ++i) {
      if (dims[i].stride < reach) return LINFUSION_ERR_OVERLAP;
      reach = (dims[i].extent - 1) * dims[i].stride + reach;
    }
  }
  return LINFUSION_OK;
}

lf::Layout device_layout(const Strides& s, int H, size_t esz) {
  const long long vec = (long long)(16 / esz);
  return lf::Layout{s.b / vec, s.h / vec, (int)(s.n / vec), H};
}

// `sq`, `skv`, `so`: strides of q, of k and v, and of out; null = contiguous [B, H, N, d]
int fwd_impl(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d, int dtype,
             int feature_map, float eps, unsigned flags, void* workspace, size_t workspace_bytes, void* stream,
             hipEvent_t* ev, const long long* sq = nullptr, const long long* skv = nullptr,
             const long long* so = nullptr, bool compact = false) {
  if (!q || !out) return LINFUSION_ERR_INVALID;
  if (!(eps >= 0.0f) || std::isinf(eps)) return LINFUSION_ERR_INVALID;
  Plan p;
  int rc = validate_common(k, v, B, H, N, d, dtype, feature_map, flags, &p, compact);
  if (rc != LINFUSION_OK) return rc;
  if (((uintptr_t)q | (uintptr_t)out) & 15) return LINFUSION_ERR_MISALIGNED;
  const size_t esz = dtype == LINFUSION_DTYPE_F32 ? 4 : 2;
  const Strides dense = contiguous_strides(H, N, d);
  const Strides lq = sq ? Strides{sq[0], sq[1], sq[2]} : dense;
  const Strides lkv = skv ? Strides{skv[0], skv[1], skv[2]} : dense;
  const Strides lo = so ? Strides{so[0], so[1], so[2]} : dense;
  if ((rc = check_strides(lq, B, H, N, d, esz, false)) != LINFUSION_OK) return rc;
  if ((rc = check_strides(lkv, B, H, N, d, esz, false)) != LINFUSION_OK) return rc;
  if ((rc = check_strides(lo, B, H, N, d, esz, true)) != LINFUSION_OK) return rc;
  const size_t nq = span_bytes(lq, B, H, N, d, esz), nkv = span_bytes(lkv, B, H, N, d, esz);
  const size_t no = span_bytes(lo, B, H, N, d, esz);
  if (overlaps(out, no, k, nkv) || overlaps(out, no, v, nkv)) return LINFUSION_ERR_OVERLAP;
  // in place on q: every tile is read before the same wave writes it, provided both views coincide
  const bool same_view = out == q && lq.b == lo.b && lq.h == lo.h && lq.n == lo.n;
  if (!same_view && overlaps(out, no, q, nq)) return LINFUSION_ERR_OVERLAP;
  if (!workspace) return LINFUSION_ERR_WORKSPACE;
  if ((uintptr_t)workspace & 15) return LINFUSION_ERR_MISALIGNED;
  if (workspace_bytes < p.ws_total) return LINFUSION_ERR_WORKSPACE;
  if (overlaps(workspace, p.ws_total, out, no) || overlaps(workspace, p.ws_total, q, nq) ||
      overlaps(workspace, p.ws_total, k, nkv) || overlaps(workspace, p.ws_total, v, nkv))
    return LINFUSION_ERR_OVERLAP;
  rc = check_device();
  if (rc != LINFUSION_OK) return rc;
  // The row-piece kernels pay where the heads of a token are neighbours in memory and a head's row is
  // not a whole number of 128-byte lines: a group of four heads is then moved as contiguous pieces that
  // single heads would touch as scattered fragments.  (Not used by the single-launch kernel, so a
  // forced single launch keeps the one-head-per-workgroup mapping.)
  auto heads_adjacent = [&](const Strides& s) { return p.groups > 0 && s.h == d && s.n > d; };
  // Measured (token-major, d = 40): from about 40 MB of tensor traffic up the row-piece kernels match the
  // contiguous layout's speed and the per-head kernels fall behind (2x at 170 MB, 3x at 2.7 GB); below
  // about 20 MB the per-head kernels' shorter start wins.
  const double tensor_bytes = 4.0 * (double)B * H * (double)N * d * (double)esz;
  const bool big = tensor_bytes >= (double)env_int("LINFUSION_GROUP_MIN_MB", 24) * 1048576.0;
  const int group_mode = env_int("LINFUSION_HEAD_GROUPS", 1);   // 1 = by size, 2 = never, 3 = whenever possible
  const bool frag = (group_mode == 3 || (group_mode == 1 && big)) && dtype != LINFUSION_DTYPE_F32 &&
                    (d * esz) % 128 != 0 && !(flags & LINFUSION_FLAG_FORCE_FUSED);
  const bool group_reduce = frag && heads_adjacent(lkv);
  const bool group_apply = frag && heads_adjacent(lo) && heads_adjacent(lq);
  // (where the row-piece kernels are due -- large token-major tensors -- they go before the replicated-state launch,
  // whose per-head accesses would touch the rows as fragments)
  if (p.path == 2 && (group_reduce || group_apply) && !(flags & LINFUSION_FLAG_FORCE_SOLO)) p.path = 0;
  Args a{q, k, v, out, (long long)B * H, N, feature_map, eps, (flags & LINFUSION_FLAG_UNNORMALIZED) != 0,
         &p, (unsigned char*)workspace, nullptr, (hipStream_t)stream, ev,
         device_layout(lq, H, esz), device_layout(lkv, H, esz), device_layout(lo, H, esz), group_reduce, group_apply};
  return dispatch(d, dtype, a);
}

int fwd_owned(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d, int dtype,
              int feature_map, float eps, void* stream) {
  size_t need = linfusion_attn_workspace_bytes(B, H, N, d, dtype);
  if (need == 0)   // let the general entry point name the error (nothing is enqueued for invalid arguments)
    return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, 0u, nullptr, 0, stream, nullptr);
  int rc = check_device();
  if (rc != LINFUSION_OK) return rc;
  void* ws = nullptr;
  rc = owned_workspace(need, &ws);
  if (rc != LINFUSION_OK) return rc;
  // the three-kernel path, which cannot time out: the caller of these entry points has no workspace to ask about
  return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, LINFUSION_FLAG_FORCE_SPLIT, ws, need, stream, nullptr);
}

// ---- scratch that no call has to allocate ------------------------------------------------------------
// One fixed array per device, part of the library's device image (each GPU the library runs on holds its
// own copy at its own address until the process ends).  In host code the array's name is only a stand-in
// for the symbol, not a device address: the address is asked once per device with hipGetSymbolAddress and
// only that pointer is ever handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
void* g_scratch_ptr[kMaxDevices];

// device address of `scratch` on the current device (asked on first use, with that device current)
int static_scratch(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return LINFUSION_ERR_DEVICE; }
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return LINFUSION_ERR_HIP; }
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return LINFUSION_OK;
}

}  // namespace

namespace lf32 {

int launch_plan32(int B, int H, long long N, int d, Plan32* out, size_t* partial_bytes) {
  Plan p;
  const int rc = make_plan(B, H, N, d, LINFUSION_DTYPE_F32, LINFUSION_FLAG_FORCE_SPLIT, &p);
  if (rc != LINFUSION_OK) return rc;
  *out = Plan32{p.splits, p.blk_reduce, p.apply_wgs, p.blk_apply};
  *partial_bytes = p.ws_partials;
  return LINFUSION_OK;
}

namespace {
template <int D>
int reduce32(const Reduce32Args& a) {
  using namespace lf;
  constexpr int NE = D * D + D;
  const long long BH = (long long)a.B * a.H;
  const f32x4* K = (const f32x4*)a.k;
  const f32x4* V = (const f32x4*)a.v;
  int rc;
  switch (a.fm) {
    case 0: rc = launch_reduce32<D, 0>(K, a.lk, V, a.lv, a.partials, a.N, a.plan.splits, a.plan.blk_reduce, BH, a.st); break;
    case 1: rc = launch_reduce32<D, 1>(K, a.lk, V, a.lv, a.partials, a.N, a.plan.splits, a.plan.blk_reduce, BH, a.st); break;
    default: rc = launch_reduce32<D, 2>(K, a.lk, V, a.lv, a.partials, a.N, a.plan.splits, a.plan.blk_reduce, BH, a.st); break;
  }
  if (rc != LINFUSION_OK) return rc;
  combine_state<0><<<dim3((NE + kCombineElems - 1) / kCombineElems, (unsigned)BH), dim3(kCombineThreads), 0, a.st>>>(
      a.partials, a.plan.splits, NE, a.state);
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}

template <int D>
int apply32(const Apply32Args& a) {
  using namespace lf;
  constexpr size_t ldsa = apply32_lds_bytes<D>();
  const long long BH = (long long)a.B * a.H;
  const dim3 g2(a.plan.apply_wgs, (unsigned)BH), blk(kThreads);
  const f32x4* Q = (const f32x4*)a.q;
  f32x4* O = (f32x4*)a.out;
#define LF_APPLY(FM, NORM) \
  lf::apply32<D, FM, NORM><<<g2, blk, ldsa, a.st>>>(Q, a.lq, O, a.lo, a.state, a.eps, a.N, a.plan.blk_apply);
  LF_SWITCH_FM_NORM(LF_APPLY)
#undef LF_APPLY
  return hipGetLastError() == hipSuccess ? LINFUSION_OK : LINFUSION_ERR_HIP;
}
}  // namespace

int run_reduce32(const Reduce32Args& a) {
  switch (a.d) {
#define X(DD) case DD: return reduce32<DD>(a);
    LF_FOR_D(X)
#undef X
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

int run_apply32(const Apply32Args& a) {
  switch (a.d) {
#define X(DD) case DD: return apply32<DD>(a);
    LF_FOR_D(X)
#undef X
  }
  return LINFUSION_ERR_UNSUPPORTED;
}

}  // namespace lf32

namespace lfw {
int wide_launch_plan(int B, int H, long long N, int d, int dtype, WidePlan* wp, size_t* partial_bytes) {
  Plan p;
  const int rc = make_plan(B, H, N, d, dtype, 0, &p);
  if (rc != LINFUSION_OK) return rc;
  if (!is_wide(d)) return LINFUSION_ERR_UNSUPPORTED;
  *wp = wide_plan_of(p, dtype);
  *partial_bytes = p.ws_partials;
  return LINFUSION_OK;
}
}  // namespace lfw

namespace lfh {
int check_device() { return ::check_device(); }
int env_int(const char* name, int dflt) { return ::env_int(name, dflt); }
int num_cu() { return ::num_cu(); }
int check_strides(const long long s[3], int B, int H, long long N, int d, size_t esz, bool written) {
  return ::check_strides(Strides{s[0], s[1], s[2]}, B, H, N, d, esz, written);
}
size_t span_bytes(const long long s[3], int B, int H, long long N, int d, size_t esz) {
  return ::span_bytes(Strides{s[0], s[1], s[2]}, B, H, N, d, esz);
}
}  // namespace lfh

extern "C" {

int linfusion_attn_fwd_ex(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d,
                          int dtype, int feature_map, float eps, unsigned flags, void* workspace,
                          size_t workspace_bytes, void* stream) {
  return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, flags, workspace, workspace_bytes, stream, nullptr);
}

int linfusion_attn_fwd_strided(const void* q, const void* k, const void* v, void* out, int B, int H, long long N,
                               int d, int dtype, int feature_map, float eps, unsigned flags,
                               const long long q_strides[3], const long long kv_strides[3],
                               const long long out_strides[3], void* workspace, size_t workspace_bytes,
                               void* stream) {
  return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, flags, workspace, workspace_bytes, stream, nullptr,
                  q_strides, kv_strides, out_strides);
}

int linfusion_attn_fwd_profile(const void* q, const void* k, const void* v, void* out, int B, int H, long long N,
                               int d, int dtype, int feature_map, float eps, unsigned flags,
                               const long long q_strides[3], const long long kv_strides[3],
                               const long long out_strides[3], void* workspace, size_t workspace_bytes,
                               void* stream, void* events[4]) {
  if (!events || !events[0] || !events[1] || !events[2] || !events[3]) return LINFUSION_ERR_INVALID;
  hipEvent_t ev[4] = {(hipEvent_t)events[0], (hipEvent_t)events[1], (hipEvent_t)events[2], (hipEvent_t)events[3]};
  return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, flags, workspace, workspace_bytes, stream, ev,
                  q_strides, kv_strides, out_strides);
}

int linfusion_attn_last_error(const void* workspace, size_t workspace_bytes, int B, int H, long long N, int d,
                              int dtype, void* stream) {
  if (!workspace) return LINFUSION_ERR_INVALID;
  Plan p;
  int rc = make_plan(B, H, N, d, dtype, 0u, &p);
  if (rc != LINFUSION_OK) return rc;
  if (workspace_bytes < p.ws_total) return LINFUSION_ERR_WORKSPACE;
  rc = check_device();
  if (rc != LINFUSION_OK) return rc;
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) { (void)hipGetLastError(); return LINFUSION_ERR_HIP; }
  if (p.fsplits == 0) return LINFUSION_OK;   // no single-launch path for this shape: nothing can time out
  const unsigned char* ws = (const unsigned char*)workspace;
  const unsigned long long* rec = reinterpret_cast<const unsigned long long*>(ws + p.ws_partials + p.ws_state) +
                                  (size_t)B * H * 2 * p.fsplits;
  // {ticket of the last single-launch call that ran on this workspace, ticket of the last one that gave up}:
  // both written by the kernels themselves, so the answer belongs to this workspace whatever ran elsewhere.
  // A well-formed ticket has its lower half equal to the complement of its upper half; anything else is the
  // workspace's undefined initial content (no single-launch call has used it yet).
  unsigned long long pair[2] = {0, 0};
  if (hipMemcpy(pair, rec, sizeof(pair), hipMemcpyDeviceToHost) != hipSuccess) { (void)hipGetLastError(); return LINFUSION_ERR_HIP; }
  const bool formed = (unsigned)(pair[0] >> 32) == ~(unsigned)pair[0];
  return (formed && pair[1] == pair[0]) ? LINFUSION_ERR_TIMEOUT : LINFUSION_OK;
}

size_t linfusion_attn_workspace_state_offset(int B, int H, long long N, int d, int dtype) {
  Plan p;
  if (make_plan(B, H, N, d, dtype, 0u, &p) != LINFUSION_OK) return 0;
  return p.ws_partials;
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
  p.path = 0;
  const size_t esz = dtype == LINFUSION_DTYPE_F32 ? 4 : 2;
  const lf::Layout dense = device_layout(contiguous_strides(H, N, d), H, esz);
  Args a{nullptr, k, v, nullptr, (long long)B * H, N, feature_map, 0.0f, false,
         &p, (unsigned char*)workspace, state_out, (hipStream_t)stream, nullptr, dense, dense, dense, false, false};
  return dispatch(d, dtype, a);
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

size_t linfusion_attn_static_scratch_bytes(void) { return kStaticScratchBytes; }

int linfusion_init(void) {
  int rc = check_device();
  if (rc != LINFUSION_OK) return rc;
  void* p = nullptr;
  return static_scratch(&p);
}

int linfusion_attn_fwd_static(const void* q, const void* k, const void* v, void* out, int B, int H, long long N, int d,
                              int dtype, int feature_map, float eps, unsigned flags, void* stream) {
  // the three-kernel path only: its scratch needs no initial content, and nothing in it can time out
  if (flags & LINFUSION_FLAG_FORCE_FUSED) return LINFUSION_ERR_INVALID;
  const unsigned f = flags | LINFUSION_FLAG_FORCE_SPLIT;
  Plan p;
  int rc = make_plan(B, H, N, d, dtype, f, &p, true);
  if (rc != LINFUSION_OK)   // let the general entry point name the error in its own order of checks
    return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, f, nullptr, 0, stream, nullptr);
  if (p.ws_total > kStaticScratchBytes) return LINFUSION_ERR_WORKSPACE;
  rc = check_device();
  if (rc != LINFUSION_OK) return rc;
  void* ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != LINFUSION_OK) return rc;
  return fwd_impl(q, k, v, out, B, H, N, d, dtype, feature_map, eps, f, ws, kStaticScratchBytes, stream, nullptr,
                  nullptr, nullptr, nullptr, true);
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
    case LINFUSION_ERR_TIMEOUT: return "single-launch barrier wait expired";
    default: return "unknown status";
  }
}

int linfusion_version(void) { return kVersion; }

void linfusion_set_tuning(int on) { g_tuning.store(on ? 1 : 0, std::memory_order_relaxed); }

const char* linfusion_attn_apply_kernel(int B, int H, long long N, int d, int dtype, unsigned flags) {
  Plan p;
  if (make_plan(B, H, N, d, dtype, flags, &p) != LINFUSION_OK) return "";
  if (is_wide(d)) return p.wave_apply ? "apply16_wave" : "apply16_wide";
  if (p.path == 2) return dtype == LINFUSION_DTYPE_F32 ? "solo32" : "solo16";
  if (p.path == 1) return dtype == LINFUSION_DTYPE_F32 ? "fused32" : "fused16";
  if (dtype == LINFUSION_DTYPE_F32) return "apply32";
  return p.apply_packed ? "apply16_packed" : "apply16_dma";
}

int linfusion_attn_plan(int B, int H, long long N, int d, int dtype, unsigned flags, int plan[4]) {
  if (!plan) return LINFUSION_ERR_INVALID;
  Plan p;
  int rc = make_plan(B, H, N, d, dtype, flags, &p);
  if (rc != LINFUSION_OK) return rc;
  plan[0] = p.path;
  plan[1] = p.path == 2 ? p.solo_g : (p.path == 1 ? p.fsplits : p.splits);
  plan[2] = p.path == 2 ? p.solo_g : (p.path == 1 ? p.fsplits : p.apply_wgs);
  plan[3] = dtype == LINFUSION_DTYPE_F32 ? lf::kTile32 : lf::kTile;
  return LINFUSION_OK;
}

}  // extern "C"
