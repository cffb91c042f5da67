// Single launch without any exchange between workgroups, for small token counts (Prop. 2: the state g'(X)^T X is
// independent of the token a query belongs to, so whoever applies it may as well have computed it):
//   every workgroup computes the WHOLE state of its head from all N tokens of K and V -- the G workgroups of a head
//   repeat that work; K and V of a head are a few hundred KB that stay in the XCD's L2 after the first touch --
//   keeps it in its own LDS, and applies it to its share of the head's query tiles.
// One kernel, no workspace, no barrier between workgroups, no flags: the three-kernel path pays three launches and
// three fills and drains of the chip (each 3 to 19 us for the SD-sized layers), the single launch with barriers pays two
// device-wide round trips; here the price is the repeated reduction, which is small while N is.  All workgroups of
// a head sum in the same fixed order, so they hold bit-identical states and results are run-to-run identical.
// grid = (G * B*H), block = 64 * waves: workgroup u works on head u / G, part u % G.  The hardware deals
// consecutive workgroups to the eight XCDs in turn; the index is remapped so that the G workgroups of a head share
// an XCD (and its L2) whenever the grid is a multiple of eight.
#pragma once
#include "lf_apply16_dma.hpp"
#include "lf_fp32.hpp"

namespace lf {

// workgroups dealt round-robin to 8 XCDs: unit = (linear % 8) * (total / 8) + linear / 8 keeps consecutive
// units on one XCD
LF_DEV int solo_unit(int linear, int total) {
  return (total % 8 == 0) ? (linear % 8) * (total / 8) + linear / 8 : linear;
}

// Waves per workgroup: as many as the two phases' LDS allows (the state phase is bound by memory latency per
// wave): sixteen if the reduction's wave-private tiles and the apply ring fit 160 KB, else eight.  Plain integer
// arithmetic so that the host's launch plan uses the same function; `levels` = 16-bit operand levels of phi(K).
constexpr int solo16_lds_bytes(int d, int levels, int waves) {
  const int dp = (d + 15) / 16 * 16;
  const int rs = dp + ((d % 16) != 0 ? 0 : 8);
  const int reduce = (levels + 1) * kTile * rs * 2 * waves;
  const int slot = (kTile * (d / 8) + 63) / 64 * 1024;
  const int ring = 3 * slot * waves;
  const int stage = 2 * slot * waves + (d * d + d) * 4 + 256;
  const int a = ring > stage ? ring : stage;
  return reduce > a ? reduce : a;
}
constexpr int solo16_waves(int d, int levels) { return solo16_lds_bytes(d, levels, 16) <= 160 * 1024 ? 16 : 8; }
constexpr int solo32_waves(int d) { return d <= 48 ? 16 : 8; }

template <typename T, int D> struct Solo16Cfg {
  static constexpr int kWaves = solo16_waves(D, NSplit<T>::value);
  using AC = ApplyDmaCfg<D>;
  static constexpr int kStageOffset = (AC::kRing - 1) * kWaves * AC::kSlotBytes;
  static_assert(reduce_copies(kWaves, D) * (D * D + D) * 4 <= kStageOffset,
                "the cross-wave copies must lie below the area the finished state is written to");
  static constexpr int kLdsBytes = reduce16_lds_bytes<T, D>(kWaves) > apply16_dma_lds_bytes<T, D>(kWaves)
                                       ? reduce16_lds_bytes<T, D>(kWaves) : apply16_dma_lds_bytes<T, D>(kWaves);
  static_assert(kLdsBytes <= solo16_lds_bytes(D, NSplit<T>::value, kWaves), "solo16_lds_bytes must cover both phases");
  static_assert(kLdsBytes <= 160 * 1024, "workgroup LDS limit of the device");
};

template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__((64 * Solo16Cfg<T, D>::kWaves))
solo16(const u32x4* __restrict__ K, const u32x4* __restrict__ V, Layout lkv, const u32x4* __restrict__ Q, Layout lq,
       u32x4* __restrict__ O, Layout lo, float eps, long long N, int G, int blk_apply) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Cfg = Solo16Cfg<T, D>;
  constexpr int W = Cfg::kWaves;
  const int u = solo_unit((int)blockIdx.x, (int)gridDim.x);
  const long long bh = u / G;
  const int part = u % G;
  const long long okv = lkv.slice(bh);
  const long long n_tiles = (N + kTile - 1) / kTile;
  const int blk_all = (int)((n_tiles + W - 1) / W * W);      // one block: the workgroup walks every tile of the head
  float* st = reinterpret_cast<float*>(smem + Cfg::kStageOffset);
  reduce16_phase<T, D, FM, W, true>(K + okv, V + okv, lkv.row, st, N, blk_all, 0, 1, smem);
  __syncthreads();      // the state is complete where the apply prologue expects it; the tiles below it are dead
  ApplyDma<T, D, FM, NORM, 0, false, D, false, W> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, blk_apply,
                                                     part, G, smem);
  ap.prefetch();
  ap.template load_state<false, true>(nullptr, eps, true);
  ap.stream();
}

template <int D> struct Solo32Cfg {
  static constexpr int kWaves = solo32_waves(D);
  using AC = Apply32Cfg<D>;
  static constexpr int kStateOffset = (AC::kRing - 1) * kWaves * AC::kSlotBytes;   // third slot block: free until the stream starts
  static_assert(reduce_copies(kWaves, D) * (D * D + D) * 4 <= kStateOffset, "copies below the finished state");
  static constexpr int kNeed = kStateOffset + (D * D + D) * 4;
  static constexpr int kLdsBytes = kNeed > apply32_lds_bytes<D>(kWaves) ? kNeed : apply32_lds_bytes<D>(kWaves);
  static_assert(kLdsBytes <= 160 * 1024, "workgroup LDS limit of the device");
};

template <int D, int FM, bool NORM>
__global__ void __launch_bounds__((64 * Solo32Cfg<D>::kWaves))
solo32(const f32x4* __restrict__ K, const f32x4* __restrict__ V, Layout lkv, const f32x4* __restrict__ Q, Layout lq,
       f32x4* __restrict__ O, Layout lo, float eps, long long N, int G, int blk_apply) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Cfg = Solo32Cfg<D>;
  constexpr int W = Cfg::kWaves;
  const int u = solo_unit((int)blockIdx.x, (int)gridDim.x);
  const long long bh = u / G;
  const int part = u % G;
  const long long okv = lkv.slice(bh);
  const long long n_tiles = (N + kTile32 - 1) / kTile32;
  const int blk_all = (int)((n_tiles + W - 1) / W * W);
  float* st = reinterpret_cast<float*>(smem + Cfg::kStateOffset);
  reduce32_phase<D, FM, W, true>(K + okv, V + okv, lkv.row, lkv.row, st, N, blk_all, 0, 1, smem);
  __syncthreads();
  Apply32Dma<D, FM, NORM, W> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, blk_apply, part, G, smem);
  ap.prefetch();                           // slots 0 and 1: the cross-wave copies there are dead
  ap.template load_state<false>(st);       // operands into registers: plain reads of the workgroup's own LDS
  __syncthreads();                         // before the stream loop refills the third slot block
  ap.stream(eps);
}

}  // namespace lf
