// fp16 / bf16 state reduction and the dtype-independent combine of the split-N path:
//   state_reduce16  S_p = sum_{j in chunk} phi(k_j)^T v_j,  z_p = sum phi(k_j)       (Prop. 2: g'(X)^T X)
//   combine_state   S = sum_p S_p, z = sum_p z_p in a fixed order                      (Eq. 5: Z, non-causal)
// The apply + normalize kernel is in lf_apply16_dma.hpp.  Each step is a __device__ "phase" function
// so that the single-launch kernel (lf_fused.hpp) runs exactly the same code as the separate kernels.
#pragma once
#include "lf_common.hpp"

namespace lf {

constexpr int kWavesPerWG = 4;
constexpr int kThreads = 64 * kWavesPerWG;
constexpr int kTile = 32;   // tokens per tile, both in the reduction (one 16x16x32 k-step) and in apply

// ==========================================================================================
// State reduction.  grid = (splits, B*H), block = 256.  Workgroup (split, bh) owns blocks of
// tiles_per_block consecutive tiles of head bh (see TileIter); its four waves take them
// round-robin and each wave streams on its own: global -> registers (128-bit, coalesced over
// the contiguous tile) -> phi on K -> wave-private LDS tile -> transposing LDS reads give the
// token-major operands -> 16x16x32 matrix-core products accumulate S (and z through a column
// of ones) in fp32.  No workgroup barrier inside the stream loop.
// Partial written per workgroup: S as [D][D] row-major then z as [D], fp32.
// ==========================================================================================
template <int D> struct Reduce16Cfg {
  using Sh = Shape16<D>;
  // LDS row stride in 16-bit elements: padded so that the 4 rows x 32 bytes a 16-lane group
  // reads with one transposing load fall in distinct banks.
  static constexpr int kRS = Sh::kDP + (Sh::kSpareCol ? 0 : 8);
  static constexpr int kTileElems = kTile * kRS;
  static constexpr int kChunks = kTile * Sh::kChunksPerRow;   // 16-byte chunks per tile
  static constexpr int kNL = (kChunks + 63) / 64;              // loads per lane per tensor
};

// copies of the accumulators in the cross-wave sum: one per wave for the four waves of the separate kernels up to
// d = 64 (every wave stores at once: one barrier, no read-add-write round, whose 40 dependent LDS round trips per
// lane cost 1.5 us of a small launch), two beyond (the copies would take a second workgroup's LDS); workgroups of
// more waves (the replicated-state kernel) take four where they fit below the apply phase's staging area
constexpr int reduce_copies(int waves, int d) { return waves > 4 ? (d <= 48 ? 4 : 2) : (d <= 64 ? 4 : 2); }

template <typename T, int D>
constexpr int reduce16_lds_bytes(int waves = kWavesPerWG) {
  // per wave: NSplit tiles of phi(K) + one of V; reused by the cross-wave reduction (copies of the accumulators)
  int tiles = (NSplit<T>::value + 1) * Reduce16Cfg<D>::kTileElems * 2 * waves;
  int red = reduce_copies(waves, D) * (D * D + D) * 4;
  return tiles > red ? tiles : red;
}

// `dst`: where this workgroup's partial goes ([D*D + D] floats).  `smem`: reduce16_lds_bytes<T,D>(WAVES)
// bytes of LDS.  Ends with every thread having written its share of `dst` (no trailing barrier).
// `Kh`, `Vh`: first token row of this head; `rs`: row stride in 16-byte units.
// WAVES: waves of the workgroup.  TO_LDS: `dst` lies in the workgroup's own LDS (beyond the first
// reduce_copies(WAVES, D) * (D*D + D) floats of `smem`) and takes plain stores; else it is global memory that other
// workgroups read.
template <typename T, int D, int FM, int WAVES = kWavesPerWG, bool TO_LDS = false>
LF_DEV void reduce16_phase(const u32x4* __restrict__ Kh, const u32x4* __restrict__ Vh, int rs,
                           float* __restrict__ dst, long long N, int tiles_per_block, int split, int nsplit,
                           unsigned char* smem) {
  using Sh = Shape16<D>;
  using Cfg = Reduce16Cfg<D>;
  constexpr int NS = NSplit<T>::value;
  constexpr int RS = Cfg::kRS, NL = Cfg::kNL, CPR = Sh::kChunksPerRow, MT = Sh::kMT;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  uint16_t* wbase = reinterpret_cast<uint16_t*>(smem) + wave * (NS + 1) * Cfg::kTileElems;
  uint16_t* ldsP[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) ldsP[s] = wbase + s * Cfg::kTileElems;
  uint16_t* ldsV = wbase + NS * Cfg::kTileElems;

  // per-lane constants: which chunks of a tile this lane moves (token row, offset from the tile's
  // first row in memory), and where they land in LDS
  int lds_off[NL], trow[NL], goff[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    int c = u * 64 + lane;
    trow[u] = c / CPR;
    goff[u] = trow[u] * rs + c % CPR;
    lds_off[u] = trow[u] * RS + (c % CPR) * 8;
  }
  // transposing-read base: lane j of 16-lane group g reads row 8g + 4r + j/4, columns 4*(j%4)..
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);

  const long long n_tiles = (N + kTile - 1) / kTile;

  f32x4 acc[MT][MT];
  f32x4 accz[MT];
  const uint32_t one2 = (uint32_t)OneBits<T>::value * 0x10001u;
  const u32x4 ones = {one2, one2, one2, one2};

  u32x4 kr[NL], vr[NL];
  auto issue_loads = [&](long long tile) {
    // number of valid token rows in this tile (ragged last tile of the head)
    long long rem = N - tile * kTile;
    int lim = rem < kTile ? (int)rem : kTile;
    const u32x4* kp = Kh + tile * kTile * rs;
    const u32x4* vp = Vh + tile * kTile * rs;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (u * 64 + lane < Cfg::kChunks && trow[u] < lim) {
        if constexpr (TO_LDS) {      // every workgroup of the head reads these rows: keep them in the L2
          kr[u] = kp[goff[u]];
          vr[u] = vp[goff[u]];
        } else {
          kr[u] = ld_stream(kp + goff[u]);
          vr[u] = ld_stream(vp + goff[u]);
        }
      } else {
        kr[u] = u32x4{LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value};   // phi maps it to 0
        vr[u] = u32x4{0, 0, 0, 0};
      }
    }
    return lim;
  };

  // fp16 with elu+1: phi(k) = exp(k) of keys far below zero leaves fp16's normal range (bits are lost below -10,
  // everything below -17), which matters when ALL keys a wave sees are that small: nothing larger dominates its
  // sums then.  Such a stream shows in the wave's normalizer sums: z_c >= every phi(k_jc) that went into it, so if
  // all z_c stay below 2^-11 per token summed, no single phi(k) can have been above 2^-11 either... and conversely a
  // stream whose largest phi(k) is below 2^-11 always has every z_c below (tokens) * 2^-11.  Only then (never for
  // ordinary data) the wave goes through its tiles again: once to find its largest key m, and, if m is below
  // kRescanBelow, once more with phi(k) evaluated as exp(k - m) (m not below kShiftFloor, so that the rows past
  // the end of a head, which are loaded as the most negative fp16 value, still map to 0); the factor exp(m) is
  // taken out of the fp32 sums afterwards.
  constexpr bool kRescan = NS == 1 && FM == kPhiEluPlusOne;
  constexpr float kRescanBelow = -5.0f, kShiftFloor = -64.0f, kLog2e = 1.44269504088896340736f;

  // Fill of the wave's tiles (after the stream's first loads have been issued, so that it runs under their
  // latency): phi(K) pad columns zero; V pad columns zero except the ones column at index D (when a spare column
  // exists) which makes z fall out of the products.  16 bytes per lane and store; LDS operations of a wave
  // complete in order, so the ones land on the zeros.
  auto fill_tiles = [&]() {
    static_assert(((NS + 1) * Cfg::kTileElems * 2) % 16 == 0, "whole 16-byte pieces");
    u32x4* w16 = reinterpret_cast<u32x4*>(wbase);
    for (int i = lane; i < (NS + 1) * Cfg::kTileElems / 8; i += 64) w16[i] = u32x4{0, 0, 0, 0};
    if constexpr (Sh::kSpareCol) {
      if (lane < kTile) ldsV[lane * RS + D] = OneBits<T>::value;
    }
  };

  // the wave's whole stream: sums of phi(k) 2^kc (x) v into acc / accz; returns the token rows summed
  auto run_stream = [&](const float kc) {
    TileIter it(split, nsplit, wave, tiles_per_block, n_tiles, WAVES);
#pragma unroll
    for (int a = 0; a < MT; ++a) {
      accz[a] = f32x4{0, 0, 0, 0};
#pragma unroll
      for (int b = 0; b < MT; ++b) acc[a][b] = f32x4{0, 0, 0, 0};
    }
    int lim = 0;
    long long tokens = 0;
    if (it.valid()) lim = issue_loads(it.t);
    fill_tiles();
    while (it.valid()) {
      tokens += lim;
      // ---- phi(K) -> 16-bit (hi [, lo]) -> LDS ; V -> LDS --------------------------------------
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        int c = u * 64 + lane;
        if (c < Cfg::kChunks) {
          const bool ok = trow[u] < lim;
          u32x4 ph, pl;
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            if constexpr (NS == 1 && kPhiKillsLowest<FM>) {
              ph[w] = kRescan ? phi_pack2_scaled<T, FM>(kr[u][w], kc) : phi_pack2<T, FM>(kr[u][w]);
              continue;
            }
            float x0, x1;
            unpack2<T>(kr[u][w], x0, x1);
            float p0 = kRescan ? phi_scaled<FM>(x0, kc) : phi<FM>(x0);
            float p1 = kRescan ? phi_scaled<FM>(x1, kc) : phi<FM>(x1);
            if constexpr (!kPhiKillsLowest<FM>) {
              p0 = ok ? p0 : 0.0f;
              p1 = ok ? p1 : 0.0f;
            }
            if constexpr (NS == 1) {
              ph[w] = pack2<T>(p0, p1);
            } else {
              uint32_t h, l;
              pack2_split<T>(p0, p1, h, l);
              ph[w] = h;
              pl[w] = l;
            }
          }
          *reinterpret_cast<u32x4*>(ldsP[0] + lds_off[u]) = ph;
          if constexpr (NS == 2) *reinterpret_cast<u32x4*>(ldsP[1] + lds_off[u]) = pl;
          *reinterpret_cast<u32x4*>(ldsV + lds_off[u]) = vr[u];
        }
      }
      // ---- prefetch the wave's next tile while this one is multiplied -------------------------
      it.next();
      int next_lim = 0;
      if (it.valid()) next_lim = issue_loads(it.t);

      // ---- token-major operands by transposing LDS reads, then the outer products -------------
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      u32x4 bfrag[MT];
#pragma unroll
      for (int b = 0; b < MT; ++b) {
        u32x2 r0 = lds_read_tr16(ldsV + tr_base + 16 * b);
        u32x2 r1 = lds_read_tr16(ldsV + tr_base + 4 * RS + 16 * b);
        bfrag[b] = u32x4{r0[0], r0[1], r1[0], r1[1]};
      }
#pragma unroll
      for (int s = 0; s < NS; ++s) {
#pragma unroll
        for (int a = 0; a < MT; ++a) {
          u32x2 r0 = lds_read_tr16(ldsP[s] + tr_base + 16 * a);
          u32x2 r1 = lds_read_tr16(ldsP[s] + tr_base + 4 * RS + 16 * a);
          u32x4 afrag = u32x4{r0[0], r0[1], r1[0], r1[1]};
#pragma unroll
          for (int b = 0; b < MT; ++b) acc[a][b] = mfma_16x16x32<T>(afrag, bfrag[b], acc[a][b]);
          if constexpr (!Sh::kSpareCol) accz[a] = mfma_16x16x32<T>(afrag, ones, accz[a]);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      lim = next_lim;
    }
    return tokens;
  };

  const long long tokens = run_stream(0.0f);

  if constexpr (kRescan) {
    // largest normalizer sum of the wave (spare column: column D of the last block row holds z; else accz, whose
    // columns all hold it)
    float zm = 0.0f;
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (Sh::kSpareCol) zm = fmaxf(zm, j16 == D % 16 ? acc[a][D / 16][i] : 0.0f);
        else zm = fmaxf(zm, accz[a][i]);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) zm = fmaxf(zm, __shfl_xor(zm, o));
    if (zm < (float)tokens * 0x1p-11f) {      // never for ordinary data, a wave without tiles (0 < 0) or NaNs
      // the stream's largest key
      f16x2 kmax2 = __builtin_bit_cast(f16x2, LowestBits<F16>::value);
      {
        TileIter it(split, nsplit, wave, tiles_per_block, n_tiles, WAVES);
        while (it.valid()) {
          (void)issue_loads(it.t);
#pragma unroll
          for (int u = 0; u < NL; ++u) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              const uint32_t word = kr[u][w];
              kmax2 = __builtin_elementwise_max(kmax2, __builtin_bit_cast(f16x2, word));
            }
          }
          it.next();
        }
      }
      float m = fmaxf((float)kmax2[0], (float)kmax2[1]);
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
      // (not small after all -- many tokens of middling keys -- or nothing but the most negative value: keep the sums)
      if (m < kRescanBelow && m > -65504.0f) {
        const float kc = fmaxf(m, kShiftFloor) * -kLog2e;
        (void)run_stream(kc);
        const float back = __builtin_amdgcn_exp2f(-kc);      // the rescanned sums carry 2^kc
#pragma unroll
        for (int a = 0; a < MT; ++a) {
          accz[a] *= back;
#pragma unroll
          for (int b = 0; b < MT; ++b) acc[a][b] *= back;
        }
      }
    }
  }

  // ---- cross-wave sum in a fixed order: wave w adds into LDS copy w % COPIES ([D*D] S then [D] z) in round
  //      w / COPIES (round 0 stores), so copy c = w_c + w_(c+COPIES) + ...; then all threads add the copies in
  //      order and write the partial.  Four waves: (w0 + w2) + (w1 + w3), with two copies or four. ----------
  __syncthreads();
  constexpr int NE = D * D + D;
  constexpr int COPIES = reduce_copies(WAVES, D);
  static_assert(WAVES % COPIES == 0, "whole rounds");
  float* red = reinterpret_cast<float*>(smem);
  float* mine = red + (wave % COPIES) * NE;
#pragma unroll
  for (int round = 0; round < WAVES / COPIES; ++round) {
    if (wave / COPIES == round) {
#pragma unroll
      for (int a = 0; a < MT; ++a) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = a * 16 + 4 * g4 + i;
          if (row < D) {
#pragma unroll
            for (int b = 0; b < MT; ++b) {
              const int col = b * 16 + j16;
              float* p = nullptr;
              if (col < D) p = mine + row * D + col;
              else if (Sh::kSpareCol && col == D) p = mine + D * D + row;
              if (p) *p = (round == 0) ? acc[a][b][i] : *p + acc[a][b][i];
            }
            if constexpr (!Sh::kSpareCol) {
              if (j16 == 0) {
                float* p = mine + D * D + row;
                *p = (round == 0) ? accz[a][i] : *p + accz[a][i];
              }
            }
          }
        }
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < NE; i += 64 * WAVES) {
    float v;
    if constexpr (COPIES == 4 && WAVES == 4) v = (red[i] + red[2 * NE + i]) + (red[NE + i] + red[3 * NE + i]);   // (w0 + w2) + (w1 + w3)
    else if constexpr (COPIES == 4) v = ((red[i] + red[NE + i]) + red[2 * NE + i]) + red[3 * NE + i];
    else v = red[i] + red[NE + i];
    if constexpr (TO_LDS) dst[i] = v;
    else st_agent(dst + i, v);
  }
}

template <typename T, int D, int FM>
__global__ void __launch_bounds__(kThreads)
state_reduce16(const u32x4* __restrict__ K, const u32x4* __restrict__ V, Layout kv, HeadSubset hs,
               float* __restrict__ partials, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = hs.bh(blockIdx.y, kv.H);
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)(D * D + D);
  const long long off = kv.slice(bh);
  reduce16_phase<T, D, FM>(K + off, V + off, kv.row, dst, N, tiles_per_block, blockIdx.x, gridDim.x, smem);
}

// ==========================================================================================
// State reduction on groups of W (4 or 8) heads that are neighbours in memory (a token row of the group
// is one contiguous piece of W d elements, as in the token-major [B, N, H*d] layout).
// grid = (splits, B * groups_per_batch), block = 64 W: workgroup (x, y) takes heads W (y % gpb) .. + W-1
// of batch y / gpb; heads beyond the last whole group are left to state_reduce16.
// All threads fetch each tile as whole row pieces (coalesced over W d elements instead of W scattered
// d-element rows), apply phi to the K pieces and scatter the chunks into per-head LDS tiles; after a
// workgroup barrier wave w multiplies head w's tiles exactly as state_reduce16 does and keeps that
// head's accumulators, so a partial is one wave's sum over all the workgroup's tiles.  The LDS tiles
// are double-buffered where two sets fit in 64 KiB (one barrier per tile), else single (two).
// ==========================================================================================
template <typename T, int D, int W> struct ReduceRowsCfg {
  using Sh = Shape16<D>;
  using RC = Reduce16Cfg<D>;
  static constexpr int kNS = NSplit<T>::value;
  static constexpr int kThreadsW = 64 * W;
  static constexpr int kPiece = W * Sh::kChunksPerRow;      // 16-byte chunks per row piece
  static constexpr int kChunks = kTile * kPiece;                       // chunks per tile of row pieces
  static constexpr int kNL = (kChunks + kThreadsW - 1) / kThreadsW;      // loads per thread per tensor
  static constexpr int kHeadElems = (kNS + 1) * RC::kTileElems;        // phi(K) level tiles, then the V tile
  static constexpr int kBufElems = W * kHeadElems;
  static constexpr bool kDouble = 2 * kBufElems * 2 <= 65536;
  static constexpr int kLdsBytes = (kDouble ? 2 : 1) * kBufElems * 2;
};

template <typename T, int D, int FM, int W>
__global__ void __launch_bounds__(64 * W)
state_reduce16_rows(const u32x4* __restrict__ K, const u32x4* __restrict__ V, Layout kv, int groups_per_batch,
                    float* __restrict__ partials, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Sh = Shape16<D>;
  using RC = Reduce16Cfg<D>;
  using Cfg = ReduceRowsCfg<T, D, W>;
  constexpr int NT = Cfg::kThreadsW;
  constexpr int NS = Cfg::kNS, RS = RC::kRS, NL = Cfg::kNL, CPR = Sh::kChunksPerRow, MT = Sh::kMT;
  constexpr int PC = Cfg::kPiece, TE = RC::kTileElems;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long b = blockIdx.y / groups_per_batch;
  const long long h0 = (long long)(blockIdx.y % groups_per_batch) * W;
  const u32x4* Kg = K + (b * kv.batch + h0 * kv.head);
  const u32x4* Vg = V + (b * kv.batch + h0 * kv.head);
  const int rs = kv.row;
  uint16_t* lds = reinterpret_cast<uint16_t*>(smem);

  // per-thread constants: chunk p = 64 W u + tid of a tile is chunk p % PC of token row p / PC; it
  // belongs to head (p % PC) / CPR and lands in that head's LDS tiles
  int goff[NL], loff[NL], trow[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    const int p = u * NT + tid;
    const int r = p / PC, c = p % PC;
    const bool in = p < Cfg::kChunks;
    trow[u] = in ? r : kTile;              // kTile: never below the row limit
    goff[u] = r * rs + c;
    loff[u] = in ? (c / CPR) * Cfg::kHeadElems + r * RS + (c % CPR) * 8 : 0;
  }
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);

  const long long n_tiles = (N + kTile - 1) / kTile;

  f32x4 acc[MT][MT];
  f32x4 accz[MT];
  const uint32_t one2 = (uint32_t)OneBits<T>::value * 0x10001u;
  const u32x4 ones = {one2, one2, one2, one2};

  u32x4 kr[NL], vr[NL];
  auto issue_loads = [&](long long tile) {
    long long rem = N - tile * kTile;
    int lim = rem < kTile ? (int)rem : kTile;
    const u32x4* kp = Kg + tile * kTile * rs;
    const u32x4* vp = Vg + tile * kTile * rs;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (trow[u] < lim) {
        kr[u] = ld_stream(kp + goff[u]);
        vr[u] = ld_stream(vp + goff[u]);
      } else {
        kr[u] = u32x4{LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value};   // phi maps it to 0
        vr[u] = u32x4{0, 0, 0, 0};
      }
    }
    return lim;
  };

  // one-time fill: pad columns zero, ones column (index D, where a spare column exists) in the V tiles
  for (int i = tid; i < (Cfg::kDouble ? 2 : 1) * Cfg::kBufElems; i += NT) {
    const int tile_idx = i / TE, within = i % TE;
    const bool is_v = tile_idx % (NS + 1) == NS;
    lds[i] = (is_v && Sh::kSpareCol && within % RS == D) ? OneBits<T>::value : (uint16_t)0;
  }
  __syncthreads();

  // fp16 with elu+1: a head whose keys are all far below zero is summed a second time relative to its largest
  // key (see reduce16_phase).  Here the waves of a workgroup move in step, so the workgroup decides together;
  // `hshift`: per head of the group, first the largest key (as an ordered integer), then the shift 2^kc.
  constexpr bool kRescan = NS == 1 && FM == kPhiEluPlusOne;
  constexpr float kRescanBelow = -5.0f, kShiftFloor = -64.0f, kLog2e = 1.44269504088896340736f;
  __shared__ int hmax[8];
  __shared__ float hshift[8];
  int head_of[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) head_of[u] = ((u * NT + tid) % PC) / CPR;

  // the workgroup's whole stream; `shifted`: chunk u's phi(k) carries 2^hshift[its head]; returns token rows summed
  auto run_stream = [&](const bool shifted) {
    TileIter it(blockIdx.x, gridDim.x, 0, tiles_per_block, n_tiles, 1);   // every wave walks every tile
#pragma unroll
    for (int a = 0; a < MT; ++a) {
      accz[a] = f32x4{0, 0, 0, 0};
#pragma unroll
      for (int bb = 0; bb < MT; ++bb) acc[a][bb] = f32x4{0, 0, 0, 0};
    }
    float kcu[NL];
#pragma unroll
    for (int u = 0; u < NL; ++u) kcu[u] = shifted ? hshift[head_of[u]] : 0.0f;
    int lim = 0;
    long long tokens = 0;
    if (it.valid()) lim = issue_loads(it.t);
    int buf = 0;
    while (it.valid()) {
      tokens += lim;
      uint16_t* bufp = lds + buf * Cfg::kBufElems;
      // ---- phi(K) -> 16-bit (hi [, lo]) -> the owning head's tiles ; V likewise ------------------
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        if (u * NT + tid < Cfg::kChunks) {
          const bool ok = trow[u] < lim;
          u32x4 ph, pl;
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            if constexpr (NS == 1 && kPhiKillsLowest<FM>) {
              ph[w] = (kRescan && shifted) ? phi_pack2_scaled<T, FM>(kr[u][w], kcu[u]) : phi_pack2<T, FM>(kr[u][w]);
              continue;
            }
            float x0, x1;
            unpack2<T>(kr[u][w], x0, x1);
            float p0 = (kRescan && shifted) ? phi_scaled<FM>(x0, kcu[u]) : phi<FM>(x0);
            float p1 = (kRescan && shifted) ? phi_scaled<FM>(x1, kcu[u]) : phi<FM>(x1);
            if constexpr (!kPhiKillsLowest<FM>) {
              p0 = ok ? p0 : 0.0f;
              p1 = ok ? p1 : 0.0f;
            }
            if constexpr (NS == 1) {
              ph[w] = pack2<T>(p0, p1);
            } else {
              uint32_t h, l;
              pack2_split<T>(p0, p1, h, l);
              ph[w] = h;
              pl[w] = l;
            }
          }
          *reinterpret_cast<u32x4*>(bufp + loff[u]) = ph;
          if constexpr (NS == 2) *reinterpret_cast<u32x4*>(bufp + TE + loff[u]) = pl;
          *reinterpret_cast<u32x4*>(bufp + NS * TE + loff[u]) = vr[u];
        }
      }
      it.next();
      int next_lim = 0;
      if (it.valid()) next_lim = issue_loads(it.t);
      lds_barrier();   // the tile is complete in LDS

      // ---- wave w: head w's outer products ----------------------------------------------------
      const uint16_t* hp = bufp + wave * Cfg::kHeadElems;
      const uint16_t* ldsV = hp + NS * TE;
      u32x4 bfrag[MT];
#pragma unroll
      for (int bb = 0; bb < MT; ++bb) {
        u32x2 r0 = lds_read_tr16(ldsV + tr_base + 16 * bb);
        u32x2 r1 = lds_read_tr16(ldsV + tr_base + 4 * RS + 16 * bb);
        bfrag[bb] = u32x4{r0[0], r0[1], r1[0], r1[1]};
      }
#pragma unroll
      for (int s = 0; s < NS; ++s) {
#pragma unroll
        for (int a = 0; a < MT; ++a) {
          u32x2 r0 = lds_read_tr16(hp + s * TE + tr_base + 16 * a);
          u32x2 r1 = lds_read_tr16(hp + s * TE + tr_base + 4 * RS + 16 * a);
          u32x4 afrag = u32x4{r0[0], r0[1], r1[0], r1[1]};
#pragma unroll
          for (int bb = 0; bb < MT; ++bb) acc[a][bb] = mfma_16x16x32<T>(afrag, bfrag[bb], acc[a][bb]);
          if constexpr (!Sh::kSpareCol) accz[a] = mfma_16x16x32<T>(afrag, ones, accz[a]);
        }
      }
      if constexpr (Cfg::kDouble) buf ^= 1;
      else lds_barrier();   // single buffer: everyone is done reading before the next tile is written
      lim = next_lim;
    }
    return tokens;
  };

  const long long tokens = run_stream(false);

  if constexpr (kRescan) {
    float zm = 0.0f;      // largest normalizer sum of this wave's head
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if constexpr (Sh::kSpareCol) zm = fmaxf(zm, j16 == D % 16 ? acc[a][D / 16][i] : 0.0f);
        else zm = fmaxf(zm, accz[a][i]);
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) zm = fmaxf(zm, __shfl_xor(zm, o));
    const bool suspicious = zm < (float)tokens * 0x1p-11f;     // never for ordinary data
    if (__syncthreads_or(suspicious ? 1 : 0)) {
      // rare: every head's largest key (an ordered integer image of the float, so that an integer maximum does it)
      if (tid < 8) hmax[tid] = (int)0x80000000;
      __syncthreads();
      f16x2 kmax2[NL];
#pragma unroll
      for (int u = 0; u < NL; ++u) kmax2[u] = __builtin_bit_cast(f16x2, LowestBits<F16>::value);
      {
        TileIter it(blockIdx.x, gridDim.x, 0, tiles_per_block, n_tiles, 1);
        while (it.valid()) {
          (void)issue_loads(it.t);
#pragma unroll
          for (int u = 0; u < NL; ++u) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              const uint32_t word = kr[u][w];
              kmax2[u] = __builtin_elementwise_max(kmax2[u], __builtin_bit_cast(f16x2, word));
            }
          }
          it.next();
        }
      }
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        if (u * NT + tid < Cfg::kChunks) {
          const float m = fmaxf((float)kmax2[u][0], (float)kmax2[u][1]);
          const int bits = __builtin_bit_cast(int, m);
          atomicMax(&hmax[head_of[u]], bits >= 0 ? bits : bits ^ 0x7fffffff);
        }
      }
      __syncthreads();
      if (lane == 0) {      // wave w decides for head w (its own `suspicious` is wave-uniform)
        const int key = hmax[wave];
        const float m = __builtin_bit_cast(float, key >= 0 ? key : key ^ 0x7fffffff);
        const bool shift = suspicious && m < kRescanBelow && m > -65504.0f;
        hshift[wave] = shift ? fmaxf(m, kShiftFloor) * -kLog2e : 0.0f;
      }
      __syncthreads();
      (void)run_stream(true);      // (heads without a shift come out as before)
      const float back = __builtin_amdgcn_exp2f(-hshift[wave]);
#pragma unroll
      for (int a = 0; a < MT; ++a) {
        accz[a] *= back;
#pragma unroll
        for (int bb = 0; bb < MT; ++bb) acc[a][bb] *= back;
      }
    }
  }

  // ---- each wave owns a whole partial: straight from the accumulator layout (lane: rows 4 (l / 16) + i,
  //      column l % 16 of each 16 x 16 block) to memory ----------------------------------------------
  float* dst = partials + (((b * kv.H + h0 + wave) * gridDim.x) + blockIdx.x) * (long long)(D * D + D);
#pragma unroll
  for (int a = 0; a < MT; ++a) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = a * 16 + 4 * g4 + i;
      if (row < D) {
#pragma unroll
        for (int bb = 0; bb < MT; ++bb) {
          const int col = bb * 16 + j16;
          if (col < D) st_agent(dst + row * D + col, acc[a][bb][i]);
          else if (Sh::kSpareCol && col == D) st_agent(dst + D * D + row, acc[a][bb][i]);
        }
        if constexpr (!Sh::kSpareCol) {
          if (j16 == 0) st_agent(dst + D * D + row, accz[a][i]);
        }
      }
    }
  }
}

// ==========================================================================================
// Combine.  Thread (e, sg) sums element e of the head's partials over the sg-th quarter of the
// splits in split order; the four quarters are then added in order 0..3.  Fixed order =>
// run-to-run identical.  Output: the fp32 state of the head, S as [d][d] row-major then z as [d].
// One call handles the 64 elements [e0, e0 + 64) with 256 threads; `part` is 256 floats of LDS.
// ==========================================================================================
constexpr int kCombineThreads = 256;
constexpr int kCombineElems = 64;

LF_DEV void combine_slice(const float* __restrict__ head_partials, int splits, int NE, int e0,
                          float* __restrict__ head_state, float* part) {
  const int el = threadIdx.x & 63, sg = threadIdx.x >> 6;
  const int e = e0 + el;
  const int per = (splits + 3) / 4;
  int p0 = sg * per, p1 = p0 + per;
  if (p1 > splits) p1 = splits;
  float s = 0.0f;
  if (e < NE) {
    const float* src = head_partials + e;
    int p = p0;
    for (; p + 8 <= p1; p += 8) {   // eight loads in flight, added in split order
      float a[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = ld_agent(src + (long long)(p + i) * NE);
#pragma unroll
      for (int i = 0; i < 8; ++i) s += a[i];
    }
    for (; p < p1; ++p) s += ld_agent(src + (long long)p * NE);
  }
  part[sg * kCombineElems + el] = s;
  __syncthreads();
  if (sg == 0 && e < NE)
    st_agent(head_state + e,
             ((part[el] + part[kCombineElems + el]) + part[2 * kCombineElems + el]) + part[3 * kCombineElems + el]);
}

// grid = (ceil(NE / 64), B*H), block = 256, NE = d*d + d.  (A template only so that the two translation
// units of the library may both hold it.)
template <int kUnused>
__global__ void __launch_bounds__(kCombineThreads)
combine_state(const float* __restrict__ partials, int splits, int NE, float* __restrict__ state) {
  __shared__ float part[4 * kCombineElems];
  const long long bh = blockIdx.y;
  combine_slice(partials + (bh * splits) * (long long)NE, splits, NE, blockIdx.x * kCombineElems, state + bh * NE, part);
}

LF_DEV float pow2_scale_for(float mx) {
  // power of two alpha with alpha * mx in [2^13, 2^14); 1 when mx is zero or not finite
  if (!(mx > 0.0f) || !(mx < 3.0e38f)) return 1.0f;
  int e;
  (void)__builtin_frexpf(mx, &e);     // mx = m * 2^e, m in [0.5, 1)
  int k = 14 - e;
  k = k > 100 ? 100 : (k < -100 ? -100 : k);
  return __builtin_ldexpf(1.0f, k);
}

}  // namespace lf
