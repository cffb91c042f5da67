// The two-branch module (lf_mlp16.hpp) on per-head kernels with a statistics pass of its own.
#pragma once
#include "lf_apply16_dma.hpp"

namespace lf {

// ==========================================================================================================
// The same module for any head count and every head width the per-head kernels have (token rows that do not
// fit one workgroup: 10 or 20 heads of 64 channels, 8 of 80): the LayerNorm statistics get a pass of their own
// (mlp_rowstats16: reads t_q and t_k once more, writes 8 bytes per token and branch), then the per-head
// kernels form q and k per element from a, t, the token's {rstd, -mean rstd} and the head's gamma, beta.
// Eight tensor passes instead of six.
// ==========================================================================================================

// LayerNorm statistics of the token rows of t_q (blockIdx.y even) and t_k (odd).  grid = (wgs, 2 B), block = 256:
// sixteen lanes per row, each over its 16-byte chunks with its own first value as the pivot (deviations from a
// common offset are small, nothing cancels), the sixteen (count, mean, centred square sum) merged pairwise.
// `stats`: [2][B][n_pad] pairs {rstd, -mean * rstd}; `C8` = C / 8 chunks per row; `row`, `batch`: 16-byte units.
template <typename T>
__global__ void __launch_bounds__(kThreads)
mlp_rowstats16(const u32x4* __restrict__ Tq, const u32x4* __restrict__ Tk, long long batch, int row, int C8,
               float ln_eps, long long N, long long n_pad, f32x2* __restrict__ stats) {
  const int which = blockIdx.y & 1;
  const long long b = blockIdx.y >> 1;
  const u32x4* Tg = (which ? Tk : Tq) + b * batch;
  f32x2* out = stats + ((long long)which * (gridDim.y >> 1) + b) * n_pad;
  const int sub = threadIdx.x & 15;
  const long long rows_per_step = (long long)gridDim.x * (kThreads / 16);
  for (long long n = (long long)blockIdx.x * (kThreads / 16) + (threadIdx.x >> 4); n < N; n += rows_per_step) {
    const u32x4* rp = Tg + n * row;
    float cnt = 0.0f, s1 = 0.0f, s2 = 0.0f, pivot = 0.0f;
#pragma unroll 2
    for (int c = sub; c < C8; c += 16) {
      const u32x4 raw = ld_stream(rp + c);
      float x[8];
#pragma unroll
      for (int w = 0; w < 4; ++w) unpack2<T>(raw[w], x[2 * w], x[2 * w + 1]);
      if (c == sub) pivot = x[0];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float dlt = x[e] - pivot;
        s1 += dlt;
        s2 = __builtin_fmaf(dlt, dlt, s2);
      }
      cnt += 8.0f;
    }
    float mean = 0.0f, m2 = 0.0f;
    if (cnt > 0.0f) {
      const float m = s1 / cnt;
      mean = pivot + m;
      m2 = fmaxf(__builtin_fmaf(-m, s1, s2), 0.0f);
    }
#pragma unroll
    for (int o = 1; o < 16; o <<= 1) {   // the partner's triple joins in; both lanes of a pair end with the same one
      const float cnt_o = __shfl_xor(cnt, o), mean_o = __shfl_xor(mean, o), m2_o = __shfl_xor(m2, o);
      const float tot = cnt + cnt_o;
      if (tot > 0.0f) {
        const float dlt = mean_o - mean;
        const float f = cnt_o / tot;
        m2 = m2 + m2_o + dlt * dlt * cnt * f;
        mean = __builtin_fmaf(dlt, f, mean);
      }
      cnt = tot;
    }
    if (sub == 0) {
      const float rstd = __builtin_amdgcn_rsqf(m2 / cnt + ln_eps);
      out[n] = f32x2{rstd, -mean * rstd};
    }
  }
}

template <typename T, int D>
constexpr int reduce16_mlph_lds_bytes() { return reduce16_lds_bytes<T, D>() + 2 * D * 4; }

// State reduction of one head from the branch results of g' and the rows' statistics: state_reduce16 with
// k formed per element.  grid = (splits, B * H), block = 256.  `row`, `batch`: strides in 16-byte units of the
// token-major tensors; `stats`: this branch's [B][n_pad] pairs; gamma, beta: all H * D channels.
template <typename T, int D, int FM>
__global__ void __launch_bounds__(kThreads)
state_reduce16_mlph(const u32x4* __restrict__ Ak, const u32x4* __restrict__ Tk, const u32x4* __restrict__ V,
                    long long batch, int row, int H, const f32x2* __restrict__ stats, long long n_pad,
                    const float* __restrict__ gamma, const float* __restrict__ beta, float slope,
                    float* __restrict__ partials, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Sh = Shape16<D>;
  using Cfg = Reduce16Cfg<D>;
  constexpr int NS = NSplit<T>::value;
  constexpr int RS = Cfg::kRS, NL = Cfg::kNL, CPR = Sh::kChunksPerRow, MT = Sh::kMT;
  constexpr int NE = D * D + D;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long bh = blockIdx.y;
  const long long b = bh / H;
  const int h = (int)(bh % H);
  const long long off = b * batch + (long long)h * CPR;
  const u32x4* Ah = Ak + off;
  const u32x4* Th = Tk + off;
  const u32x4* Vh = V + off;
  const f32x2* sb = stats + b * n_pad;
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)NE;

  uint16_t* wbase = reinterpret_cast<uint16_t*>(smem) + wave * (NS + 1) * Cfg::kTileElems;
  uint16_t* ldsP[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) ldsP[s] = wbase + s * Cfg::kTileElems;
  uint16_t* ldsV = wbase + NS * Cfg::kTileElems;
  float* aff = reinterpret_cast<float*>(smem + reduce16_lds_bytes<T, D>());   // gamma[D] then beta[D] of this head
  for (int i = threadIdx.x; i < 2 * D; i += kThreads) aff[i] = i < D ? gamma[h * D + i] : beta[h * D + i - D];

  int lds_off[NL], trow[NL], goff[NL], ch0[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    const int c = u * 64 + lane;
    trow[u] = c / CPR;
    goff[u] = trow[u] * row + c % CPR;
    lds_off[u] = trow[u] * RS + (c % CPR) * 8;
    ch0[u] = (c % CPR) * 8;
  }
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);

  const long long n_tiles = (N + kTile - 1) / kTile;
  TileIter it(blockIdx.x, gridDim.x, wave, tiles_per_block, n_tiles);

  f32x4 acc[MT][MT];
  f32x4 accz[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    accz[a] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int bb = 0; bb < MT; ++bb) acc[a][bb] = f32x4{0, 0, 0, 0};
  }
  const uint32_t one2 = (uint32_t)OneBits<T>::value * 0x10001u;
  const u32x4 ones = {one2, one2, one2, one2};
  constexpr uint32_t LOW = LowestBits<T>::value;

  u32x4 ar[NL], tr[NL], vr[NL];
  f32x2 sr[NL];
  auto issue_loads = [&](long long tile) {
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    const long long base = tile * kTile * row;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (u * 64 + lane < Cfg::kChunks && trow[u] < lim) {
        ar[u] = ld_stream(Ah + base + goff[u]);
        tr[u] = ld_stream(Th + base + goff[u]);
        vr[u] = ld_stream(Vh + base + goff[u]);
        sr[u] = sb[tile * kTile + trow[u]];
      } else {   // a row past the end: k = lowest + LeakyReLU(beta), which phi still maps to 0
        ar[u] = u32x4{LOW, LOW, LOW, LOW};
        tr[u] = u32x4{0, 0, 0, 0};
        vr[u] = u32x4{0, 0, 0, 0};
        sr[u] = f32x2{0.0f, 0.0f};
      }
    }
    return lim;
  };

  int lim = 0;
  if (it.valid()) lim = issue_loads(it.t);
  for (int i = lane; i < Cfg::kTileElems; i += 64) {
#pragma unroll
    for (int s = 0; s < NS; ++s) ldsP[s][i] = 0;
    ldsV[i] = (Sh::kSpareCol && (i % RS) == D) ? OneBits<T>::value : (uint16_t)0;
  }
  __syncthreads();   // the head's affine is in place

  while (it.valid()) {
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (u * 64 + lane < Cfg::kChunks) {
        const bool ok = trow[u] < lim;
        const f32x4 g0 = *reinterpret_cast<const f32x4*>(aff + ch0[u]);
        const f32x4 g1 = *reinterpret_cast<const f32x4*>(aff + ch0[u] + 4);
        const f32x4 b0 = *reinterpret_cast<const f32x4*>(aff + D + ch0[u]);
        const f32x4 b1 = *reinterpret_cast<const f32x4*>(aff + D + ch0[u] + 4);
        const float gg[8] = {g0[0], g0[1], g0[2], g0[3], g1[0], g1[1], g1[2], g1[3]};
        const float bb[8] = {b0[0], b0[1], b0[2], b0[3], b1[0], b1[1], b1[2], b1[3]};
        const float rstd = sr[u][0], cn = sr[u][1];
        u32x4 ph, pl;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float x0, x1, t0, t1;
          unpack2<T>(ar[u][w], x0, x1);
          unpack2<T>(tr[u][w], t0, t1);
          const float y0 = __builtin_fmaf(gg[2 * w], __builtin_fmaf(t0, rstd, cn), bb[2 * w]);
          const float y1 = __builtin_fmaf(gg[2 * w + 1], __builtin_fmaf(t1, rstd, cn), bb[2 * w + 1]);
          x0 += fmaxf(y0, slope * y0);   // LeakyReLU for slopes up to one
          x1 += fmaxf(y1, slope * y1);
          float p0 = phi<FM>(x0), p1 = phi<FM>(x1);
          if constexpr (!kPhiKillsLowest<FM>) {
            p0 = ok ? p0 : 0.0f;
            p1 = ok ? p1 : 0.0f;
          }
          if constexpr (NS == 1) {
            ph[w] = pack2<T>(p0, p1);
          } else {
            uint32_t hh, ll;
            pack2_split<T>(p0, p1, hh, ll);
            ph[w] = hh;
            pl[w] = ll;
          }
        }
        *reinterpret_cast<u32x4*>(ldsP[0] + lds_off[u]) = ph;
        if constexpr (NS == 2) *reinterpret_cast<u32x4*>(ldsP[1] + lds_off[u]) = pl;
        *reinterpret_cast<u32x4*>(ldsV + lds_off[u]) = vr[u];
      }
    }
    it.next();
    int next_lim = 0;
    if (it.valid()) next_lim = issue_loads(it.t);

    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    u32x4 bfrag[MT];
#pragma unroll
    for (int bq = 0; bq < MT; ++bq) {
      u32x2 r0 = lds_read_tr16(ldsV + tr_base + 16 * bq);
      u32x2 r1 = lds_read_tr16(ldsV + tr_base + 4 * RS + 16 * bq);
      bfrag[bq] = u32x4{r0[0], r0[1], r1[0], r1[1]};
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
#pragma unroll
      for (int a = 0; a < MT; ++a) {
        u32x2 r0 = lds_read_tr16(ldsP[s] + tr_base + 16 * a);
        u32x2 r1 = lds_read_tr16(ldsP[s] + tr_base + 4 * RS + 16 * a);
        u32x4 afrag = u32x4{r0[0], r0[1], r1[0], r1[1]};
#pragma unroll
        for (int bq = 0; bq < MT; ++bq) acc[a][bq] = mfma_16x16x32<T>(afrag, bfrag[bq], acc[a][bq]);
        if constexpr (!Sh::kSpareCol) accz[a] = mfma_16x16x32<T>(afrag, ones, accz[a]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    lim = next_lim;
  }

  // cross-wave sum in a fixed order, (w0 + w2) + (w1 + w3), through two LDS copies of the partial
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
          const int r = a * 16 + 4 * g4 + i;
          if (r < D) {
#pragma unroll
            for (int bq = 0; bq < MT; ++bq) {
              const int col = bq * 16 + j16;
              float* p = nullptr;
              if (col < D) p = mine + r * D + col;
              else if (Sh::kSpareCol && col == D) p = mine + D * D + r;
              if (p) *p = (round == 0) ? acc[a][bq][i] : *p + acc[a][bq][i];
            }
            if constexpr (!Sh::kSpareCol) {
              if (j16 == 0) {
                float* p = mine + D * D + r;
                *p = (round == 0) ? accz[a][i] : *p + accz[a][i];
              }
            }
          }
        }
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < NE; i += kThreads) dst[i] = red[i] + red[NE + i];
}

template <typename T, int D>
constexpr int apply16_mlph_lds_bytes() {
  return 2 * ApplyDmaCfg<D>::kRing * ApplyDmaCfg<D>::kSlotBytes * kWavesPerWG + ApplyDmaCfg<D>::kRing * kWavesPerWG * 1024;
}

// Apply of one head from the branch results of f' and the rows' statistics.  grid = (wgs, B * H), block = 256;
// `packed`: the heads' operand-ready states (pack_state16); `stats`: this branch's [B][n_pad] pairs, n_pad a
// multiple of the tile so that a whole last tile can be read.
template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply16_mlph(const u32x4* __restrict__ Aq, const u32x4* __restrict__ Tq, long long batch_q, int row_q,
             u32x4* __restrict__ O, long long batch_o, int row_o, int H, const f32x2* __restrict__ stats,
             long long n_pad, const float* __restrict__ gamma, const float* __restrict__ beta, float slope,
             const unsigned char* __restrict__ packed, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.y;
  const long long b = bh / H;
  const int h = (int)(bh % H);
  const long long off_q = b * batch_q + (long long)h * (D / 8);
  ApplyDma<T, D, FM, NORM, 0, true, D, true> ap(Aq + off_q, row_q, O + b * batch_o + (long long)h * (D / 8), row_o, N,
                                               tiles_per_block, blockIdx.x, gridDim.x, smem);
  ap.set_mlp(Tq + off_q, gamma + h * D, beta + h * D, 0.0f, slope);
  ap.set_stats(stats + b * n_pad);
  ap.prefetch();
  ap.load_packed(packed + bh * Pack16<T, D>::kHeadBytes, eps);
  ap.stream();
}

}  // namespace lf
