// The two-branch module (lf_mlp16.hpp) for head widths above 64 (SD-v1.5's third level: 8 heads of 160): the wide
// kernels of lf_wide16.hpp with q and k formed per element from a, t, the rows' LayerNorm statistics (computed by
// mlp_rowstats16, lf_mlph16.hpp) and the head's gamma, beta.
#pragma once
#include "lf_wave16.hpp"

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

// ==========================================================================================
// apply16_wave (lf_wave16.hpp: a wave per tile, the head's whole operand-ready state in its registers, no
// workgroup barrier) on q = a + LeakyReLU(gamma (t rstd + cn) + beta).  apply16_wide_mlp shares
// every tile between eight waves behind two barriers and reached 2.7 TB/s at d = 160.  Two input tensors per tile
// would take 240 KB of ring at 32 tokens, so the tiles here hold 16 tokens (one block of matrix-core columns): per
// wave a ring of three slots of {a tile, t tile, the rows' statistics} (11 KiB at d = 160), 132 KiB per workgroup of
// four waves, and the head's gamma, beta behind it.  The query is formed where a lane reads its token's channels as
// B operands (a and t chunks from the slot, {rstd, cn} of its token from the slot's statistics deposit, gamma and
// beta of its channels from the table), phi applied, rounded to fp16 -- the arithmetic of apply16_wide_mlp's phi pass
// for fp16 tensors; the formed row of a bf16 tensor is scaled into fp16's range first, as apply16_wave does.
// Operands from pack_state_wave<D>.
// ==========================================================================================
template <int D> struct ApplyWaveMlpShape {
  using Sw = ApplyWaveShape<D>;
  static constexpr int kTok = 16;                              // tokens per tile
  static_assert((kTok * Sw::kCPR) % 64 == 0, "whole 1 KiB deposits per tile");
  static constexpr int kNL = kTok * Sw::kCPR / 64;             // deposits per tensor and tile
  static constexpr int kTensorBytes = kNL * 1024;
  static constexpr int kSlotBytes = 2 * kTensorBytes + 1024;   // a tile, t tile, the rows' statistics
  static constexpr int kRing = 3;
  static constexpr int kWaves = 4;
  static constexpr int kAffOffset = kRing * kWaves * kSlotBytes;   // gamma[D] then beta[D], fp32
  static constexpr int kLdsBytes = kAffOffset + 2 * D * 4;
  static_assert(kLdsBytes <= 160 * 1024, "workgroup LDS limit of the device");
};

template <typename T, int D, int FM, bool NORM>
struct ApplyWaveMlp {
  using TA = F16;   // the operands' type (bf16 tensors: the formed query row is scaled into fp16's range, as in apply16_wave)
  using Sw = ApplyWaveShape<D>;
  using Sm = ApplyWaveMlpShape<D>;
  static constexpr int CPR = Sw::kCPR, KS = Sw::kKS, RB = Sw::kRB, CB = Sw::kCB;
  static constexpr int NL = Sm::kNL, NLC = 2 * NL + 1, R = Sm::kRing, W = Sm::kWaves, TOK = Sm::kTok;
  static_assert(R == 3, "the wait counts below are written for a ring of three slots");
  static_assert(2 * NL + 2 * NLC <= 63, "the vector-memory counter has six bits");

  const u32x4* Ah;
  const u32x4* Th;
  const u32x4* St;
  u32x4* Oh;
  long long N;
  unsigned char* smem;
  int rs_q, rs_o;
  int lane, wave, g;
  float slope;
  int trow[NL], qoff[NL], ooff[NL], soff[NL];
  int rowb, x0;              // byte offset of this lane's token row in a tile image, its swizzle
  TileIter it, ahead;
  u32x4 A[RB][KS];
  float c1, eps_s;

  LF_DEV ApplyWaveMlp(const u32x4* Ah_, const u32x4* Th_, int rs_q_, u32x4* Oh_, int rs_o_, const void* stats,
                      float slope_, long long N_, int tiles_per_block, int wg, int nwg, unsigned char* smem_)
      : Ah(Ah_), Th(Th_), St(reinterpret_cast<const u32x4*>(stats)), Oh(Oh_), N(N_), smem(smem_), rs_q(rs_q_),
        rs_o(rs_o_), lane(threadIdx.x & 63), wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)), slope(slope_),
        it(wg, nwg, wave, tiles_per_block, (N_ + TOK - 1) / TOK, W), ahead(it) {
    g = lane >> 4;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int P = u * 64 + lane;             // position in the tile
      const int r = P / CPR, pos = P % CPR;
      const int c = pos ^ Sw::swz(r);          // position pos of row r holds chunk c (copy side and store side)
      trow[u] = r;
      qoff[u] = r * rs_q + c;
      ooff[u] = r * rs_o + pos;
      soff[u] = (r * CPR + c) * 16;
    }
    const int r = lane & 15;
    rowb = r * CPR * 16;
    x0 = Sw::swz(r);
  }

  // gamma, beta: this head's D values.  Whole workgroup (ends with a barrier).
  LF_DEV void set_affine(const float* gamma, const float* beta) {
    float* aff = reinterpret_cast<float*>(smem + Sm::kAffOffset);
    for (int i = threadIdx.x; i < 2 * D; i += 64 * W) aff[i] = i < D ? gamma[i] : beta[i - D];
    __syncthreads();
  }

  LF_DEV unsigned char* slot_ptr(int slot) const { return smem + (slot * W + wave) * Sm::kSlotBytes; }
  LF_DEV int chunk_off(int chunk) const { return rowb + ((chunk ^ x0) << 4); }

  // always issues exactly NLC vector memory instructions
  LF_DEV void issue_copy(long long tile, int slot) {
    long long rem = N - tile * TOK;
    const int lim = rem < TOK ? (int)rem : TOK;
    const u32x4* ap = Ah + tile * TOK * rs_q;
    const u32x4* tp = Th + tile * TOK * rs_q;
    unsigned char* sl = slot_ptr(slot);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int c = trow[u] < lim ? qoff[u] : 0;   // rows past N re-read chunk 0; never stored
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(ap + c),
                                       (LF_LDS void*)(sl + u * 1024), 16, 0, 2 /* nt */);
    }
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int c = trow[u] < lim ? qoff[u] : 0;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(tp + c),
                                       (LF_LDS void*)(sl + Sm::kTensorBytes + u * 1024), 16, 0, 2 /* nt */);
    }
    // the tile's 16 {rstd, cn} pairs, two per 16 bytes (the array is readable up to a whole last 32-token tile)
    const u32x4* sp = St + tile * (TOK / 2) + (lane & 7);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)sp,
                                     (LF_LDS void*)(sl + 2 * Sm::kTensorBytes), 16, 0, 0);
  }

  LF_DEV void prefetch() {
#pragma unroll
    for (int i = 0; i < R - 1; ++i) {
      if (ahead.valid()) issue_copy(ahead.t, i);
      ahead.next();
    }
  }

  LF_DEV void load_packed(const unsigned char* packed, float eps) {
    const u32x4* frag = reinterpret_cast<const u32x4*>(packed + PackWave<D>::kHeaderBytes);
#pragma unroll
    for (int b = 0; b < RB; ++b)
#pragma unroll
      for (int s = 0; s < KS; ++s) A[b][s] = frag[(b * KS + s) * 64 + lane];
    const float* scales = reinterpret_cast<const float*>(packed);
    c1 = scales[0];
    eps_s = eps * scales[1];
  }

  LF_DEV void store_tile(long long tile, int slot) {
    const unsigned char* sl = slot_ptr(slot);
    long long rem = N - tile * TOK;
    const int lim = rem < TOK ? (int)rem : TOK;
    u32x4* op = Oh + tile * TOK * rs_o;
    u32x4 w[NL];
#pragma unroll
    for (int u = 0; u < NL; ++u) w[u] = *reinterpret_cast<const u32x4*>(sl + soff[u]);
    if (lim == TOK) {   // (a branch per store would pull each read behind it, one LDS round trip each)
#pragma unroll
      for (int u = 0; u < NL; ++u) st_stream(op + ooff[u], w[u]);
    } else {
#pragma unroll
      for (int u = 0; u < NL; ++u)
        if (trow[u] < lim) st_stream(op + ooff[u], w[u]);
    }
  }

  // at most ns * NL + nc * NLC vector memory instructions outstanding (ns stores' groups, nc copies' groups)
  LF_DEV void wait_mix(int ns, int nc) {
    switch (ns * 3 + nc) {
      case 0: wait_vmcnt<0>(); break;
      case 1: wait_vmcnt<NLC>(); break;
      case 2: wait_vmcnt<2 * NLC>(); break;
      case 3: wait_vmcnt<NL>(); break;
      case 4: wait_vmcnt<NL + NLC>(); break;
      case 5: wait_vmcnt<NL + 2 * NLC>(); break;
      case 6: wait_vmcnt<2 * NL>(); break;
      case 7: wait_vmcnt<2 * NL + NLC>(); break;
      default: wait_vmcnt<2 * NL + 2 * NLC>(); break;
    }
  }

  // The tile in `slot` -> its outputs, over the a tile's rows.  All tile reads are issued before the first use.
  LF_DEV void compute_tile(int slot) {
    unsigned char* sl = slot_ptr(slot);
    u32x4 Ba[KS], Bt[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int o = chunk_off(4 * s + g);
      Ba[s] = *reinterpret_cast<const u32x4*>(sl + o);
      Bt[s] = *reinterpret_cast<const u32x4*>(sl + Sm::kTensorBytes + o);
    }
    const f32x2 rc = *reinterpret_cast<const f32x2*>(sl + 2 * Sm::kTensorBytes + (lane & 15) * 8);
    __builtin_amdgcn_sched_barrier(0);
    // ---- q = a + LeakyReLU(gamma (t rstd + cn) + beta), phi, fp16: the B operands ------------------------
    const float* aff = reinterpret_cast<const float*>(smem + Sm::kAffOffset);
    constexpr bool kScaled = !__is_same(T, TA);   // bf16 tensors: see ApplyWave::make_operands
    float x[kScaled ? 8 * KS : 2];
    float eps_tok = eps_s, post = 1.0f;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int ch0 = 32 * s + 8 * g;
      const f32x4 g0 = *reinterpret_cast<const f32x4*>(aff + ch0);
      const f32x4 g1 = *reinterpret_cast<const f32x4*>(aff + ch0 + 4);
      const f32x4 b0 = *reinterpret_cast<const f32x4*>(aff + D + ch0);
      const f32x4 b1 = *reinterpret_cast<const f32x4*>(aff + D + ch0 + 4);
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float a0, a1, t0, t1;
        unpack2<T>(Ba[s][w], a0, a1);
        unpack2<T>(Bt[s][w], t0, t1);
        const float ga = w < 2 ? g0[2 * w] : g1[2 * w - 4], gb = w < 2 ? g0[2 * w + 1] : g1[2 * w - 3];
        const float ba = w < 2 ? b0[2 * w] : b1[2 * w - 4], bb = w < 2 ? b0[2 * w + 1] : b1[2 * w - 3];
        const float y0 = __builtin_fmaf(ga, __builtin_fmaf(t0, rc[0], rc[1]), ba);
        const float y1 = __builtin_fmaf(gb, __builtin_fmaf(t1, rc[0], rc[1]), bb);
        a0 += fmaxf(y0, slope * y0);   // LeakyReLU for slopes up to one
        a1 += fmaxf(y1, slope * y1);
        if constexpr (kScaled) {
          x[8 * s + 2 * w] = a0;
          x[8 * s + 2 * w + 1] = a1;
        } else {
          Ba[s][w] = pack2<TA>(phi<FM>(a0), phi<FM>(a1));
        }
      }
    }
    if constexpr (kScaled) {
      constexpr float kLog2e = 1.44269504088896340736f;
      float m = FM == kPhiIdentity ? fabsf(x[0]) : x[0];
#pragma unroll
      for (int i = 1; i < 8 * KS; ++i) m = fmaxf(m, FM == kPhiIdentity ? fabsf(x[i]) : x[i]);
      m = fmaxf(m, __shfl_xor(m, 16));
      m = fmaxf(m, __shfl_xor(m, 32));
      float c = 0.0f, top;
      if constexpr (FM == kPhiEluPlusOne) {
        c = m < 0.0f ? fminf(-m * kLog2e, 3.0e38f) : 0.0f;
        top = m < 0.0f ? 1.0f : m + 1.0f;
      } else if constexpr (FM == kPhiRelu) {
        top = fmaxf(m, 0.0f);
      } else {
        top = m;
      }
      uint32_t f = (__builtin_bit_cast(uint32_t, top) >> 23) & 0xffu;
      f = f < 1u ? 1u : (f > 253u ? 253u : f);
      const float mult = __builtin_bit_cast(float, (254u - f) << 23);
#pragma unroll
      for (int s = 0; s < KS; ++s)
#pragma unroll
        for (int w = 0; w < 4; ++w)
          Ba[s][w] = pack2<TA>(phi_scaled<FM>(x[8 * s + 2 * w], c) * mult, phi_scaled<FM>(x[8 * s + 2 * w + 1], c) * mult);
      eps_tok = __builtin_amdgcn_exp2f(fminf(c, 190.0f) - 64.0f) * (eps_s * mult * 0x1p64f);
      post = __builtin_amdgcn_exp2f(-c) * __builtin_bit_cast(float, f << 23);
    }
    // ---- products, normalizer, outputs over the a tile's rows ---------------------------------------------
    f32x4 acc[RB];
#pragma unroll
    for (int b = 0; b < RB; ++b) acc[b] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
#pragma unroll
      for (int b = 0; b < RB; ++b) acc[b] = mfma_16x16x32<TA>(A[b][s], Ba[s], acc[b]);
    }
    float scale = c1 * post;
    if constexpr (NORM) {
      // rows d and d + 1 (the normalizer and what its rounding left) are rows 0 and 1 of the last block: lanes
      // 0-15 hold them for their tokens
      const float part = acc[RB - 1][0] + acc[RB - 1][1];
      const float den = __shfl(part, lane & 15) + eps_tok;
      scale = c1 * __builtin_amdgcn_rcpf(den);
    }
#pragma unroll
    for (int b = 0; b < CB; ++b) {
      const u32x2 w = {pack2<T>(acc[b][0] * scale, acc[b][1] * scale), pack2<T>(acc[b][2] * scale, acc[b][3] * scale)};
      // channels 16 b + 4 g .. + 3: chunk 2 b + g / 2, its first or second half
      *reinterpret_cast<u32x2*>(sl + chunk_off(2 * b + (g >> 1)) + 8 * (g & 1)) = w;
    }
  }

  // Issue order per wave:  C0 C1 [state] | C2 K0 | S0 C3 K1 | S1 C4 K2 | ...  Before tile j is touched its copies
  // must have landed: vector memory instructions issued after them are S(j-2), C(j+1) (previous round) and
  // S(j-1), C(j+2) (this round), where they exist.
  LF_DEV void stream() {
    int slot = 0, prev_slot = 0, j = 0;
    long long prev_tile = -1;
    bool next_copied = false;   // C(j+1) exists
    {
      TileIter second = it;
      second.next();
      next_copied = second.valid();
    }
    while (it.valid()) {
      const long long tile = it.t;
      const bool have_prev = prev_tile >= 0;
      if (have_prev) store_tile(prev_tile, prev_slot);
      const bool copied = ahead.valid();
      if (copied) issue_copy(ahead.t, have_prev ? prev_slot : R - 1);
      wait_mix(j >= 2 ? 2 : j, (next_copied ? 1 : 0) + (copied ? 1 : 0));
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      compute_tile(slot);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      it.next();
      ahead.next();
      next_copied = copied;
      prev_tile = tile;
      prev_slot = slot;
      slot = slot + 1 == R ? 0 : slot + 1;
      ++j;
    }
    if (prev_tile >= 0) store_tile(prev_tile, prev_slot);
  }
};

// grid = (wgs, B * H), block = 256 (four waves that share the gamma, beta table and nothing else); 16-token tiles
template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply16_wave_mlp(const u32x4* __restrict__ Aq, const u32x4* __restrict__ Tq, long long batch_q, int row_q,
                 u32x4* __restrict__ O, long long batch_o, int row_o, int H, const f32x2* __restrict__ stats,
                 long long n_pad, const float* __restrict__ gamma, const float* __restrict__ beta, float slope,
                 const unsigned char* __restrict__ packed, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.y;
  const long long b = bh / H;
  const int h = (int)(bh % H);
  const long long off_q = b * batch_q + (long long)h * (D / 8);
  ApplyWaveMlp<T, D, FM, NORM> ap(Aq + off_q, Tq + off_q, row_q, O + b * batch_o + (long long)h * (D / 8), row_o,
                               stats + b * n_pad, slope, N, tiles_per_block, blockIdx.x, gridDim.x, smem);
  ap.prefetch();
  ap.set_affine(gamma + h * D, beta + h * D);
  ap.load_packed(packed + bh * PackWave<D>::kHeadBytes, eps);
  ap.stream();
}

}  // namespace lf
