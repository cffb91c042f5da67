// The two-branch module (lf_mlp16.hpp) for head widths above 64 (SD-v1.5's third level: 8 heads of 160): the wide
// kernels of lf_wide16.hpp with q and k formed per element from a, t, the rows' LayerNorm statistics (computed by
// mlp_rowstats16, lf_mlph16.hpp) and the head's gamma, beta.
#pragma once
#include "lf_wide16.hpp"

namespace lf {

template <typename T, int D>
constexpr int reduce16_wide_mlp_lds_bytes() { return reduce16_wide_lds_bytes<T, D>() + 2 * D * 4; }

// state_reduce16_wide on k = a + LeakyReLU(gamma (t rstd + cn) + beta).  grid = (splits, B * H), block = 256.
// `row`, `batch`: strides in 16-byte units of the token-major tensors; `stats`: this branch's [B][n_pad] pairs.
template <typename T, int D, int FM>
__global__ void __launch_bounds__(kThreads, 2)
state_reduce16_wide_mlp(const u32x4* __restrict__ Ak, const u32x4* __restrict__ Tk, const u32x4* __restrict__ V,
                        long long batch, int row, int H, const f32x2* __restrict__ stats, long long n_pad,
                        const float* __restrict__ gamma, const float* __restrict__ beta, float slope,
                        float* __restrict__ partials, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Sw = ShapeWide<D>;
  constexpr int NS = NSplit<T>::value, RS = Sw::kRS, NL = Sw::kNLR, CPR = Sw::kCPR, MT = Sw::kMT, NBW = Sw::kNBW;
  constexpr int TE = Sw::kTileElems, BUF = (NS + 1) * TE;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long bh = blockIdx.y;
  const long long b = bh / H;
  const int h = (int)(bh % H);
  const long long off = b * batch + (long long)h * CPR;
  const u32x4* Ah = Ak + off;
  const u32x4* Th = Tk + off;
  const u32x4* Vh = V + off;
  const f32x2* sb = stats + b * n_pad;
  uint16_t* lds = reinterpret_cast<uint16_t*>(smem);
  float* aff = reinterpret_cast<float*>(smem + reduce16_wide_lds_bytes<T, D>());   // gamma[D] then beta[D]

  int goff[NL], loff[NL], trow[NL], ch0[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    const int p = u * kThreads + tid;
    const int r = p / CPR, c = p % CPR;
    const bool in = p < Sw::kChunks;
    trow[u] = in ? r : kTile;              // kTile: never below the row limit
    goff[u] = r * row + c;
    loff[u] = in ? r * RS + c * 8 : 0;
    ch0[u] = c * 8;
  }
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);

  const long long n_tiles = (N + kTile - 1) / kTile;
  TileIter it(blockIdx.x, gridDim.x, 0, tiles_per_block, n_tiles, 1);

  f32x4 acc[MT][NBW];
  f32x4 accz[NBW];
#pragma unroll
  for (int i = 0; i < NBW; ++i) {
    accz[i] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int a = 0; a < MT; ++a) acc[a][i] = f32x4{0, 0, 0, 0};
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
      if (trow[u] < lim) {
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
  for (int i = tid; i < 2 * BUF; i += kThreads) lds[i] = 0;   // pad columns stay zero
  for (int i = tid; i < 2 * D; i += kThreads) aff[i] = i < D ? gamma[h * D + i] : beta[h * D + i - D];
  __syncthreads();

  int buf = 0;
  while (it.valid()) {
    uint16_t* bufp = lds + buf * BUF;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (u * kThreads + tid < Sw::kChunks) {
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
        *reinterpret_cast<u32x4*>(bufp + loff[u]) = ph;
        if constexpr (NS == 2) *reinterpret_cast<u32x4*>(bufp + TE + loff[u]) = pl;
        *reinterpret_cast<u32x4*>(bufp + NS * TE + loff[u]) = vr[u];
      }
    }
    it.next();
    int next_lim = 0;
    if (it.valid()) next_lim = issue_loads(it.t);
    lds_barrier();   // the tile is complete in this buffer; the other buffer is free to be rewritten

    const uint16_t* ldsV = bufp + NS * TE;
    u32x4 bfrag[NBW];
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
      const int bq = wave + kWavesPerWG * i;
      bfrag[i] = u32x4{0, 0, 0, 0};
      if (bq < MT) {
        u32x2 r0 = lds_read_tr16(ldsV + tr_base + 16 * bq);
        u32x2 r1 = lds_read_tr16(ldsV + tr_base + 4 * RS + 16 * bq);
        bfrag[i] = u32x4{r0[0], r0[1], r1[0], r1[1]};
      }
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
#pragma unroll
      for (int a = 0; a < MT; ++a) {
        u32x2 r0 = lds_read_tr16(bufp + s * TE + tr_base + 16 * a);
        u32x2 r1 = lds_read_tr16(bufp + s * TE + tr_base + 4 * RS + 16 * a);
        u32x4 afrag = u32x4{r0[0], r0[1], r1[0], r1[1]};
#pragma unroll
        for (int i = 0; i < NBW; ++i)
          if (wave + kWavesPerWG * i < MT) acc[a][i] = mfma_16x16x32<T>(afrag, bfrag[i], acc[a][i]);
        if (a % kWavesPerWG == wave) accz[a / kWavesPerWG] = mfma_16x16x32<T>(afrag, ones, accz[a / kWavesPerWG]);
      }
    }
    buf ^= 1;
    lim = next_lim;
  }

  // each wave writes its columns of the partial (lane: rows 4 (l / 16) + i, column l % 16 of a block)
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)(D * D + D);
#pragma unroll
  for (int a = 0; a < MT; ++a) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = a * 16 + 4 * g4 + i;
#pragma unroll
      for (int c = 0; c < NBW; ++c) {
        const int bq = wave + kWavesPerWG * c;
        if (bq < MT) dst[r * D + bq * 16 + j16] = acc[a][c][i];
      }
      if (a % kWavesPerWG == wave && j16 == 0) dst[D * D + r] = accz[a / kWavesPerWG][i];
    }
  }
}

// apply16_wide on q = a + LeakyReLU(gamma (t rstd + cn) + beta).  grid = (wgs, B * H), block = 64 W.
template <typename T, int D, int FM, bool NORM, int W>
__global__ void __launch_bounds__(64 * W)
apply16_wide_mlp(const u32x4* __restrict__ Aq, const u32x4* __restrict__ Tq, long long batch_q, int row_q,
                 u32x4* __restrict__ O, long long batch_o, int row_o, int H, const f32x2* __restrict__ stats,
                 long long n_pad, const float* __restrict__ gamma, const float* __restrict__ beta, float slope,
                 const unsigned char* __restrict__ packed, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.y;
  const long long b = bh / H;
  const int h = (int)(bh % H);
  const long long off_q = b * batch_q + (long long)h * (D / 8);
  ApplyWide<T, D, FM, NORM, W, true> ap(Aq + off_q, row_q, O + b * batch_o + (long long)h * (D / 8), row_o, N,
                                        tiles_per_block, blockIdx.x, gridDim.x, smem);
  ap.set_mlp(Tq + off_q, stats + b * n_pad, gamma + h * D, beta + h * D, slope);
  ap.prefetch();
  ap.load_packed(packed + bh * PackWide<T, D, W>::kHeadBytes, eps);
  ap.stream();
}

}  // namespace lf
