// fp32 state reduction on the 16-bit matrix cores (Prop. 2's g'(X)^T X state; Eq. 5's normalizer).
//
// state_reduce32 multiplies with v_mfma_f32_16x16x4_f32, whose rate (1/16 of the bf16 instruction's) makes the
// reduction matrix-core bound at large N: at d = 40 a 16-token tile costs 48 products of 32 cycles, about what the
// tile's bytes take to arrive at the full memory rate.  Here every fp32 value is split into three bf16 terms,
// x = x1 + x2 + x3 (each the bf16 rounding of what the terms before it left: 24 bits in all, nothing of an fp32
// number is lost), and S = sum phi(k)^T v is accumulated in fp32 from the six products whose weight is 2^-16 of
// the leading one or more:  a1 v1,  a1 v2,  a2 v1,  a2 v2,  a1 v3,  a3 v1   (a = phi(k); dropped: a2 v3, a3 v2,
// a3 v3, each below 2^-24 of a1 v1 -- the size of fp32's own rounding).  bf16 x bf16 products are exact in the
// fp32 accumulator, so the only roundings are those of the accumulation, as on the fp32 instruction.
// Per 32-token tile and wave: 6 MT^2 products of 16 cycles (54 at d = 40, a third of the fp32 instruction's time),
// paid for with about 11 vector instructions per element for the splitting.
//
// Structure: state_reduce16's (each wave streams 32-token tiles of its own: coalesced fp32 loads -> phi -> three
// 16-bit tiles per tensor in wave-private LDS -> transposing reads -> products; no workgroup barrier in the loop;
// z through a ones column where d leaves one free, else through a ones operand).  Same partial layout and the same
// cross-wave sum as the other reductions, so combine_state and apply32 follow unchanged.
#pragma once
#include "lf_reduce16.hpp"

namespace lf {

template <int D> struct Reduce32sCfg {
  using Sh = Shape16<D>;
  static constexpr int kRS = Reduce16Cfg<D>::kRS;          // LDS row stride in 16-bit elements
  static constexpr int kTileElems = kTile * kRS;
  static constexpr int kCPR = D / 4;                       // 16-byte chunks (four floats) per token row
  static constexpr int kNL = D / 8;                        // loads per lane and tensor: kTile * kCPR / 64, no remainder
  static constexpr int kLevels = 3;
  static_assert(D % 8 == 0, "whole loads");
};

template <int D>
constexpr int reduce32s_lds_bytes() {
  // per wave: three tiles of phi(K) and three of V; reused by the cross-wave sum (two copies of the accumulators)
  int tiles = 2 * Reduce32sCfg<D>::kLevels * Reduce32sCfg<D>::kTileElems * 2 * kWavesPerWG;
  int red = 2 * (D * D + D) * 4;
  return tiles > red ? tiles : red;
}

// x = h + m + l with each term the bf16 rounding of what was left
LF_DEV void split3_bf16(const float (&x)[4], u32x2& h, u32x2& m, u32x2& l) {
  float r[4], t0, t1;
  h = u32x2{pack2<BF16>(x[0], x[1]), pack2<BF16>(x[2], x[3])};
  unpack2<BF16>(h[0], t0, t1);
  r[0] = x[0] - t0;
  r[1] = x[1] - t1;
  unpack2<BF16>(h[1], t0, t1);
  r[2] = x[2] - t0;
  r[3] = x[3] - t1;
  m = u32x2{pack2<BF16>(r[0], r[1]), pack2<BF16>(r[2], r[3])};
  unpack2<BF16>(m[0], t0, t1);
  r[0] -= t0;
  r[1] -= t1;
  unpack2<BF16>(m[1], t0, t1);
  r[2] -= t0;
  r[3] -= t1;
  l = u32x2{pack2<BF16>(r[0], r[1]), pack2<BF16>(r[2], r[3])};
}

// grid = (splits, B*H), block = 256, dynamic LDS reduce32s_lds_bytes<D>()
template <int D, int FM>
__global__ void __launch_bounds__(kThreads)
state_reduce32_split(const f32x4* __restrict__ K, Layout kl, const f32x4* __restrict__ V, Layout vl,
                     float* __restrict__ partials, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Sh = Shape16<D>;
  using Cfg = Reduce32sCfg<D>;
  constexpr int RS = Cfg::kRS, NL = Cfg::kNL, CPR = Cfg::kCPR, MT = Sh::kMT, TE = Cfg::kTileElems, L = Cfg::kLevels;
  constexpr int NE = D * D + D;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long bh = blockIdx.y;
  const f32x4* Kh = K + kl.slice(bh);
  const f32x4* Vh = V + vl.slice(bh);
  const int rs = kl.row, rsv = vl.row;
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)NE;

  // per wave: tiles 0..2 = the three terms of phi(K), tiles 3..5 = those of V
  uint16_t* wbase = reinterpret_cast<uint16_t*>(smem) + wave * 2 * L * TE;

  int lds_off[NL], trow[NL], goffk[NL], goffv[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    const int c = u * 64 + lane;
    trow[u] = c / CPR;
    goffk[u] = trow[u] * rs + c % CPR;
    goffv[u] = trow[u] * rsv + c % CPR;
    lds_off[u] = trow[u] * RS + (c % CPR) * 4;
  }
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);

  f32x4 acc[MT][MT];
  f32x4 accz[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    accz[a] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < MT; ++b) acc[a][b] = f32x4{0, 0, 0, 0};
  }
  const uint32_t one2 = (uint32_t)OneBits<BF16>::value * 0x10001u;
  const u32x4 ones = {one2, one2, one2, one2};

  // one-time fill: pad columns zero; column D of V's leading term holds ones where a spare column exists, so that z
  // falls out of the products a1 v1, a2 v1, a3 v1
  for (int i = lane; i < 2 * L * TE; i += 64)
    wbase[i] = (Sh::kSpareCol && i >= L * TE && i < (L + 1) * TE && (i % RS) == D) ? OneBits<BF16>::value : (uint16_t)0;

  const long long n_tiles = (N + kTile - 1) / kTile;
  TileIter it(blockIdx.x, gridDim.x, wave, tiles_per_block, n_tiles);

  f32x4 kr[NL], vr[NL];
  auto issue_loads = [&](long long tile) {
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    const f32x4* kp = Kh + tile * kTile * rs;
    const f32x4* vp = Vh + tile * kTile * rsv;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (trow[u] < lim) {
        kr[u] = __builtin_nontemporal_load(kp + goffk[u]);
        vr[u] = __builtin_nontemporal_load(vp + goffv[u]);
      } else {
        kr[u] = f32x4{0, 0, 0, 0};
        vr[u] = f32x4{0, 0, 0, 0};
      }
    }
    return lim;
  };

  int lim = 0;
  if (it.valid()) lim = issue_loads(it.t);
  while (it.valid()) {
    // ---- phi(K) and V -> three bf16 terms each -> LDS -------------------------------------------------
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const bool ok = trow[u] < lim;   // else a row past the end: phi(0) = 1 must not be added
      float p[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        p[i] = ok ? phi<FM, true>(kr[u][i]) : 0.0f;
        w[i] = vr[u][i];
      }
      u32x2 h, m, l;
      split3_bf16(p, h, m, l);
      *reinterpret_cast<u32x2*>(wbase + lds_off[u]) = h;
      *reinterpret_cast<u32x2*>(wbase + TE + lds_off[u]) = m;
      *reinterpret_cast<u32x2*>(wbase + 2 * TE + lds_off[u]) = l;
      split3_bf16(w, h, m, l);
      *reinterpret_cast<u32x2*>(wbase + 3 * TE + lds_off[u]) = h;
      *reinterpret_cast<u32x2*>(wbase + 4 * TE + lds_off[u]) = m;
      *reinterpret_cast<u32x2*>(wbase + 5 * TE + lds_off[u]) = l;
    }
    it.next();
    int next_lim = 0;
    if (it.valid()) next_lim = issue_loads(it.t);

    // ---- token-major operands by transposing LDS reads, then the six products per block --------------------
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    u32x4 bfrag[L][MT];
#pragma unroll
    for (int s = 0; s < L; ++s)
#pragma unroll
      for (int b = 0; b < MT; ++b) {
        const uint16_t* base = wbase + (L + s) * TE;
        u32x2 r0 = lds_read_tr16(base + tr_base + 16 * b);
        u32x2 r1 = lds_read_tr16(base + tr_base + 4 * RS + 16 * b);
        bfrag[s][b] = u32x4{r0[0], r0[1], r1[0], r1[1]};
      }
#pragma unroll
    for (int a = 0; a < MT; ++a) {
      u32x4 afrag[L];
#pragma unroll
      for (int s = 0; s < L; ++s) {
        u32x2 r0 = lds_read_tr16(wbase + s * TE + tr_base + 16 * a);
        u32x2 r1 = lds_read_tr16(wbase + s * TE + tr_base + 4 * RS + 16 * a);
        afrag[s] = u32x4{r0[0], r0[1], r1[0], r1[1]};
      }
#pragma unroll
      for (int b = 0; b < MT; ++b) {
        // smallest terms first, so that they meet before they meet the large sum
        acc[a][b] = mfma_16x16x32<BF16>(afrag[2], bfrag[0][b], acc[a][b]);   // a3 v1
        acc[a][b] = mfma_16x16x32<BF16>(afrag[0], bfrag[2][b], acc[a][b]);   // a1 v3
        acc[a][b] = mfma_16x16x32<BF16>(afrag[1], bfrag[1][b], acc[a][b]);   // a2 v2
        acc[a][b] = mfma_16x16x32<BF16>(afrag[1], bfrag[0][b], acc[a][b]);   // a2 v1
        acc[a][b] = mfma_16x16x32<BF16>(afrag[0], bfrag[1][b], acc[a][b]);   // a1 v2
        acc[a][b] = mfma_16x16x32<BF16>(afrag[0], bfrag[0][b], acc[a][b]);   // a1 v1
      }
      if constexpr (!Sh::kSpareCol) {
#pragma unroll
        for (int s = L - 1; s >= 0; --s) accz[a] = mfma_16x16x32<BF16>(afrag[s], ones, accz[a]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    lim = next_lim;
  }

  // ---- cross-wave sum in a fixed order, (w0 + w2) + (w1 + w3), as in state_reduce16 -------------------------
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);
  float* mine = red + (wave & 1) * NE;
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if ((wave >> 1) == round) {
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
  for (int i = threadIdx.x; i < NE; i += kThreads) st_agent(dst + i, red[i] + red[NE + i]);
}

}  // namespace lf
