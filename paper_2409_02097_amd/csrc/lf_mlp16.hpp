// The mixer fed straight from the two-branch MLPs f', g' of Sec. 3.1 (Implementation Details) (fp16 / bf16, token-major rows):
//   q = a_q + LeakyReLU(LayerNorm_C(t_q)),   k = a_k + LeakyReLU(LayerNorm_C(t_k)),   C = H d,
// where a_* is the result of the linear branch and t_* the result of the second branch's Linear.  The sum,
// the LayerNorm over all channels of a token and the activation happen inside the state-reduction and the
// apply kernels, on tiles that are in registers / LDS anyway, so q and k never exist in memory: per token
// the kernels read a_k, t_k, v and a_q, t_q and write out -- six tensor passes where forming q and k first
// costs ten.  Both kernels are the row-piece kernels (lf_reduce16.hpp, lf_apply16_dma.hpp) with the
// workgroup covering whole token rows (H = W heads, one wave per head), which is what lets the LayerNorm
// statistics be found without a pass of their own.  For rows of several groups of four heads the same kernels
// take the statistics from an earlier pass instead (PRE; mlp_rowstats16 in lf_mlph16.hpp): state_reduce16_mlp<PRE>
// and apply16_mlpg, eight tensor passes.
#pragma once
#include "lf_apply16_dma.hpp"

namespace lf {

template <typename T, int D, int W> struct ReduceMlpCfg {
  using Base = ReduceRowsCfg<T, D, W>;
  static constexpr int kPartOffset = Base::kLdsBytes;                     // (mean, M2) of every 8-channel chunk
  static constexpr int kPartBytes = kTile * Base::kPiece * 8;
  static constexpr int kRowOffset = kPartOffset + kPartBytes;             // (rstd, -mean * rstd) of every token row
  static constexpr int kAffineOffset = kRowOffset + kTile * 8;             // gamma[C] then beta[C], fp32
  static constexpr int kLdsBytes = kAffineOffset + 2 * W * D * 4;
  static constexpr int kTPR = Base::kThreadsW / kTile;                    // threads that reduce one row
  static_assert(kTPR == 8 || kTPR == 16, "a row's partials are reduced inside one wave by shuffles");
  // fp16 up to d = 40 (bf16 up to 32) fits 128 registers, so two 8-wave workgroups share a CU and cover each other's barrier
  // waits (0.85 -> 0.67 ms at 2 M tokens); four heads of 80 fit 256 (two 4-wave workgroups; bf16 with four spilled
  // registers, still 0.72 -> 0.58 ms at 2^19 tokens); the other shapes would spill 34 to 52 registers (measured
  // with that: bf16 d = 40 0.88 -> 1.41 ms, fp16 d = 48 0.92 -> 1.15 ms) and keep one workgroup
  static constexpr int kWavesPerSimd = (W == 8 && (D <= 32 || (NSplit<T>::value == 1 && D <= 40)))
                                           ? 4
                                           : ((W == 4 && D == 80) ? 2 : W / 4);
};

// State reduction from the branch results of g'.  grid = (splits, B), block = 64 W, H = W heads.
// Per tile: chunk statistics of t (registers, two passes) -> LDS -> barrier -> row statistics by kTPR threads per
// row -> LDS -> barrier -> k = a + LeakyReLU(gamma (t - mean) rstd + beta), phi(k) and v into the heads' LDS tiles
// -> barrier -> each wave its head's matrix-core products.  `row`: token stride in 16-byte units (= W D / 8 for
// dense rows); a_k, t_k and v share it.
// PRE (rows of gpb groups of W heads, too wide for one workgroup): grid = (splits, B * gpb), workgroup (x, y) takes
// heads W (y % gpb) .. + W - 1 of batch y / gpb; the rows' {rstd, -mean rstd} come from an earlier kernel
// (`stats`: [B][n_pad] pairs), loaded with the tile by the first 32 threads, and the two statistics levels are
// skipped.  gamma, beta: all channels of a row.
template <typename T, int D, int FM, int W, bool PRE = false>
__global__ void __launch_bounds__(64 * W, (ReduceMlpCfg<T, D, W>::kWavesPerSimd))
state_reduce16_mlp(const u32x4* __restrict__ Ak, const u32x4* __restrict__ Tk, const u32x4* __restrict__ V,
                   long long batch_stride, int row, const float* __restrict__ gamma, const float* __restrict__ beta,
                   float ln_eps, float slope, float* __restrict__ partials, long long N, int tiles_per_block,
                   int gpb = 1, const f32x2* __restrict__ stats = nullptr, long long n_pad = 0) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Sh = Shape16<D>;
  using RC = Reduce16Cfg<D>;
  using Cfg = ReduceRowsCfg<T, D, W>;
  using MC = ReduceMlpCfg<T, D, W>;
  constexpr int NT = Cfg::kThreadsW;
  constexpr int NS = Cfg::kNS, RS = RC::kRS, NL = Cfg::kNL, CPR = Sh::kChunksPerRow, MT = Sh::kMT;
  constexpr int PC = Cfg::kPiece, TE = RC::kTileElems, TPR = MC::kTPR;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long b = PRE ? blockIdx.y / gpb : blockIdx.y;
  const int grp = PRE ? (int)(blockIdx.y % gpb) : 0;
  const long long goff = b * batch_stride + (long long)grp * (W * D / 8);
  const u32x4* Ag = Ak + goff;
  const u32x4* Tg = Tk + goff;
  const u32x4* Vg = V + goff;
  const f32x2* sb = stats + b * n_pad;
  gamma += grp * (W * D);
  beta += grp * (W * D);
  uint16_t* lds = reinterpret_cast<uint16_t*>(smem);
  f32x2* part = reinterpret_cast<f32x2*>(smem + MC::kPartOffset);
  f32x2* rowstat = reinterpret_cast<f32x2*>(smem + MC::kRowOffset);

  // chunk p = NT u + tid of a tile is chunk p % PC of token row p / PC (head (p % PC) / CPR)
  int loff[NL], trow[NL], coff[NL];   // (the global offset of a chunk is rebuilt from row and column: registers)
  float* affine = reinterpret_cast<float*>(smem + MC::kAffineOffset);
  for (int i = tid; i < W * D; i += NT) {
    affine[i] = gamma[i];
    affine[W * D + i] = beta[i];
  }
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    const int p = u * NT + tid;
    const int r = p / PC, c = p % PC;
    const bool in = p < Cfg::kChunks;
    trow[u] = in ? r : kTile;
    loff[u] = in ? (c / CPR) * Cfg::kHeadElems + r * RS + (c % CPR) * 8 : 0;
    coff[u] = c * 8;
  }
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);
  const int srow = tid / TPR, ssub = tid % TPR;

  const long long n_tiles = (N + kTile - 1) / kTile;
  TileIter it(blockIdx.x, gridDim.x, 0, tiles_per_block, n_tiles, 1);   // every wave walks every tile

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

  u32x4 ar[NL], tr[NL], vr[NL];
  f32x2 srow_next = f32x2{0.0f, 0.0f};   // PRE: thread r < 32 carries row r's pair of the tile on its way
  auto issue_loads = [&](long long tile) {
    long long rem = N - tile * kTile;
    int lim = rem < kTile ? (int)rem : kTile;
    const long long base = tile * kTile * row;
    if constexpr (PRE) {
      srow_next = f32x2{0.0f, 0.0f};
      if (tid < lim) srow_next = sb[tile * kTile + tid];
    }
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (trow[u] < lim) {
        const long long at = base + trow[u] * row + (coff[u] >> 3);
        ar[u] = ld_stream(Ag + at);
        tr[u] = ld_stream(Tg + at);
        vr[u] = ld_stream(Vg + at);
      } else {
        ar[u] = u32x4{LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value};   // stays hugely negative after the branch sum: phi maps it to 0
        tr[u] = u32x4{0, 0, 0, 0};
        vr[u] = u32x4{0, 0, 0, 0};
      }
    }
    return lim;
  };

  int lim = 0;
  if (it.valid()) lim = issue_loads(it.t);

  // one-time fill: pad columns zero, ones column (index D, where a spare column exists) in the V tiles
  for (int i = tid; i < (Cfg::kDouble ? 2 : 1) * Cfg::kBufElems; i += NT) {
    const int tile_idx = i / TE, within = i % TE;
    const bool is_v = tile_idx % (NS + 1) == NS;
    lds[i] = (is_v && Sh::kSpareCol && within % RS == D) ? OneBits<T>::value : (uint16_t)0;
  }
  __syncthreads();

  int buf = 0;
  while (it.valid()) {
    uint16_t* bufp = lds + buf * Cfg::kBufElems;
    if constexpr (PRE) {
      if (tid < kTile) rowstat[tid] = srow_next;
      lds_barrier();
    } else {
    // ---- LayerNorm statistics, level 1: mean and centred sum of squares of every 8-channel chunk ----
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      float mean, m2;
      if constexpr (NS == 1) {
        // fp16: sums of (t - pivot) and its square, pivot = the chunk's first value, the difference in packed
        // half precision and the sums by the mixed-precision dot product (no cancellation: the deviations
        // inside a chunk are small next to a large common offset)
        const uint32_t p16 = tr[u][0] & 0xffffu;
        const f16x2 np = __builtin_bit_cast(f16x2, (p16 ^ 0x8000u) * 0x10001u);
        const f16x2 one = __builtin_bit_cast(f16x2, 0x3C003C00u);
        float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t word = tr[u][w];   // (by value: a bit cast applied to the vector element itself reads element 0)
          const f16x2 dd = __builtin_bit_cast(f16x2, word) + np;
          s1 = __builtin_amdgcn_fdot2(dd, one, s1, false);
          s2 = __builtin_amdgcn_fdot2(dd, dd, s2, false);
        }
        float pivot, unused;
        unpack2<T>(p16, pivot, unused);
        mean = __builtin_fmaf(s1, 0.125f, pivot);
        m2 = fmaxf(__builtin_fmaf(-0.125f * s1, s1, s2), 0.0f);
      } else {
        float tv[8];
        float sum = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          unpack2<T>(tr[u][w], tv[2 * w], tv[2 * w + 1]);
          sum += tv[2 * w] + tv[2 * w + 1];
        }
        mean = sum * 0.125f;
        m2 = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float dv = tv[e] - mean;
          m2 = __builtin_fmaf(dv, dv, m2);
        }
      }
      if (u * NT + tid < Cfg::kChunks) part[u * NT + tid] = f32x2{mean, m2};
    }
    lds_barrier();
    // ---- level 2: TPR threads per token row merge its PC chunks (all of 8 channels) -------------------
    {
      f32x2 mine[(PC + TPR - 1) / TPR];
      float s1 = 0.0f;
#pragma unroll
      for (int i = 0; i < (PC + TPR - 1) / TPR; ++i) {
        const int c = ssub + i * TPR;
        mine[i] = c < PC ? part[srow * PC + c] : f32x2{0.0f, 0.0f};
        s1 += mine[i][0];
      }
#pragma unroll
      for (int o = TPR / 2; o > 0; o >>= 1) s1 += __shfl_xor(s1, o);
      const float mu = s1 * (1.0f / (float)PC);
      float m2 = 0.0f;
#pragma unroll
      for (int i = 0; i < (PC + TPR - 1) / TPR; ++i) {
        if (ssub + i * TPR < PC) {
          const float dm = mine[i][0] - mu;
          m2 += mine[i][1] + 8.0f * dm * dm;
        }
      }
#pragma unroll
      for (int o = TPR / 2; o > 0; o >>= 1) m2 += __shfl_xor(m2, o);
      if (ssub == 0) {
        const float rstd = __builtin_amdgcn_rsqf(m2 * (1.0f / (float)(8 * PC)) + ln_eps);
        rowstat[srow] = f32x2{rstd, -mu * rstd};
      }
    }
    lds_barrier();
    }
    // ---- k = a + LeakyReLU(LayerNorm(t)) -> phi -> 16-bit (hi [, lo]) -> the owning head's tiles ; V ----
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (u * NT + tid < Cfg::kChunks) {
        const bool ok = trow[u] < lim;
        const f32x2 rsd = rowstat[ok ? trow[u] : 0];   // {rstd, -mean * rstd}: LayerNorm(t) = t * rsd[0] + rsd[1]
        u32x4 ph, pl;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float x0, x1, t0, t1;
          unpack2<T>(ar[u][w], x0, x1);
          unpack2<T>(tr[u][w], t0, t1);
          const f32x2 gg = *reinterpret_cast<const f32x2*>(affine + coff[u] + 2 * w);
          const f32x2 bb = *reinterpret_cast<const f32x2*>(affine + W * D + coff[u] + 2 * w);
          const float y0 = __builtin_fmaf(gg[0], __builtin_fmaf(t0, rsd[0], rsd[1]), bb[0]);
          const float y1 = __builtin_fmaf(gg[1], __builtin_fmaf(t1, rsd[0], rsd[1]), bb[1]);
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
    lim = next_lim;
  }

  // ---- each wave owns a whole partial (lane: rows 4 (l / 16) + i, column l % 16 of each 16 x 16 block) ----
  const long long head = PRE ? (b * gpb + grp) * W + wave : b * W + wave;   // (b * H + first head of the group + wave)
  float* dst = partials + ((head * gridDim.x) + blockIdx.x) * (long long)(D * D + D);
#pragma unroll
  for (int a = 0; a < MT; ++a) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = a * 16 + 4 * g4 + i;
      if (r < D) {
#pragma unroll
        for (int bb = 0; bb < MT; ++bb) {
          const int col = bb * 16 + j16;
          if (col < D) dst[r * D + col] = acc[a][bb][i];
          else if (Sh::kSpareCol && col == D) dst[D * D + r] = acc[a][bb][i];
        }
        if constexpr (!Sh::kSpareCol) {
          if (j16 == 0) dst[D * D + r] = accz[a][i];
        }
      }
    }
  }
}

// Apply on a group of W of a row's heads with the rows' statistics from an earlier kernel.  grid = (wgs, B * gpb),
// block = 64 W; `packed`: all heads' operand-ready states; `stats`: this branch's [B][n_pad] pairs.
template <typename T, int D>
constexpr int apply16_mlpg_lds_bytes(int waves) {
  return 2 * ApplyDmaCfg<D>::kRing * ApplyDmaCfg<D>::kSlotBytes * waves + ApplyDmaCfg<D>::kRing * 1024;
}

template <typename T, int D>
constexpr int apply16_mlp_lds_bytes(int waves) {
  return 2 * ApplyDmaCfg<D>::kRing * ApplyDmaCfg<D>::kSlotBytes * waves + waves * 2 * kTile * 8;
}

// Apply from the branch results of f'.  grid = (wgs, B), block = 64 W, H = W heads; `packed`: the heads'
// operand-ready states (pack_state16).  a_q and t_q share the token stride `row_q`; out has `row_o`.
template <typename T, int D, int FM, bool NORM, int W>
__global__ void __launch_bounds__(64 * W)
apply16_mlp(const u32x4* __restrict__ Aq, const u32x4* __restrict__ Tq, long long batch_q, int row_q,
            u32x4* __restrict__ O, long long batch_o, int row_o, const float* __restrict__ gamma,
            const float* __restrict__ beta, float ln_eps, float slope, const unsigned char* __restrict__ packed,
            float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long b = blockIdx.y;
  ApplyDma<T, D, FM, NORM, W, true> ap(Aq + b * batch_q, row_q, O + b * batch_o, row_o, N, tiles_per_block, blockIdx.x,
                                       gridDim.x, smem);
  ap.set_mlp(Tq + b * batch_q, gamma, beta, ln_eps, slope);
  ap.prefetch();
  ap.load_packed(packed + (b * W + wave) * Pack16<T, D>::kHeadBytes, eps);
  ap.stream();
}

template <typename T, int D, int FM, bool NORM, int W>
__global__ void __launch_bounds__(64 * W)
apply16_mlpg(const u32x4* __restrict__ Aq, const u32x4* __restrict__ Tq, long long batch_q, int row_q,
             u32x4* __restrict__ O, long long batch_o, int row_o, int gpb, const f32x2* __restrict__ stats,
             long long n_pad, const float* __restrict__ gamma, const float* __restrict__ beta, float slope,
             const unsigned char* __restrict__ packed, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long b = blockIdx.y / gpb;
  const int grp = (int)(blockIdx.y % gpb);
  const long long in_row = (long long)grp * (W * D / 8);   // the group's place inside a token row, 16-byte units
  ApplyDma<T, D, FM, NORM, W, true, D, true> ap(Aq + b * batch_q + in_row, row_q, O + b * batch_o + in_row, row_o, N,
                                               tiles_per_block, blockIdx.x, gridDim.x, smem);
  ap.set_mlp(Tq + b * batch_q + in_row, gamma + grp * (W * D), beta + grp * (W * D), 0.0f, slope);
  ap.set_stats(stats + b * n_pad);
  ap.prefetch();
  ap.load_packed(packed + ((b * gpb + grp) * W + wave) * Pack16<T, D>::kHeadBytes, eps);
  ap.stream();
}

}  // namespace lf
