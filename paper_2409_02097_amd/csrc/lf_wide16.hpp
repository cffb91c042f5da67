// fp16 / bf16 kernels for head widths above 64 (d a multiple of 16 up to 160: the deeper levels of the
// SD-v1.5 UNet have d = 80 and d = 160).  Same mathematics as the narrow kernels (Prop. 2's g'(X)^T X state,
// Eq. 5's normalizer), other work split: the d x d fp32 state no longer fits one wave's accumulators, so
// the four waves of a workgroup share every 32-token tile and split the state between them --
//   state_reduce16_wide  by columns (value channels): wave w accumulates the 16-column blocks b = w mod 4;
//   apply16_wide         by output channels: wave w produces channels [w d/4, (w+1) d/4) of every token.
// Both move tiles as whole workgroups (coalesced over full token rows) and synchronise with workgroup
// barriers; both address memory through Layout, so every layout of the strided entry point works.
#pragma once
#include "lf_apply16_dma.hpp"

namespace lf {

template <int D> struct ShapeWide {
  static_assert(D % 16 == 0 && D > 64 && D <= 160, "wide kernels: head width a multiple of 16 in (64, 160]");
  static constexpr int kCPR = D / 8;                  // 16-byte chunks per token row
  static constexpr int kMT = D / 16;                  // 16-wide blocks across d
  static constexpr int kRS = D + 8;                   // LDS row stride of the reduction tiles (bank spread)
  static constexpr int kTileElems = kTile * kRS;
  static constexpr int kChunks = kTile * kCPR;        // chunks per tile
  static constexpr int kNLR = (kChunks + kThreads - 1) / kThreads;   // reduction: loads per thread per tensor
  static constexpr int kNBW = (kMT + kWavesPerWG - 1) / kWavesPerWG; // column blocks per wave (at most)
};

// apply: W waves per workgroup (4 or 8), wave w produces output channels [w d/W, (w+1) d/W)
template <int D, int W> struct ApplyWideShape {
  static_assert(kTile % W == 0 && D % (4 * W) == 0, "output channels split evenly, two per 32-bit word per half-wave");
  static constexpr int kCPR = D / 8;                  // 16-byte chunks per token row
  static constexpr int kDQ = D / W;                   // output channels per wave
  static constexpr int kHalf = kDQ / 2;               // ... per half-wave
  static constexpr int kMT2 = (kHalf + 2 + 15) / 16;  // 32-row output tiles incl. the two normalizer rows
  static constexpr int kKS = D / 16;                  // contraction steps of 16 channels
  static constexpr int kRPR = kTile / W;              // token rows per wave region
  static constexpr int kRegionChunks = kRPR * kCPR;
  static constexpr int kNLA = (kRegionChunks + 63) / 64;   // copies / stores per wave per tile
  static constexpr int kRegionBytes = kNLA * 1024;
  static constexpr int kRing = 3;
  static constexpr int kSlotBytes = W * kRegionBytes;
  // rotation of the chunks inside a token row that makes token-per-lane accesses bank-conflict free
  static constexpr int kG = (kCPR % 16 == 0) ? 16 : ((kCPR % 8 == 0) ? 8 : ((kCPR % 4 == 0) ? 4 : 2));
  static_assert(kCPR % 2 == 0 && kRPR * kG >= 16, "rotation classes must fit a region");
  static __device__ __forceinline__ int rot(int r) { return ((r * kG) >> 4) & (kG - 1); }
};

template <typename T, int D>
constexpr int reduce16_wide_lds_bytes() {
  return 2 * (NSplit<T>::value + 1) * ShapeWide<D>::kTileElems * 2;   // double-buffered phi(K) levels + V
}
// ring of tiles, plus (bf16) one slot-sized buffer for the low halves of phi(Q) of the current tile
template <typename T, int D, int W>
constexpr int apply16_wide_lds_bytes() {
  return (ApplyWideShape<D, W>::kRing + (NSplit<T>::value == 2 ? 1 : 0)) * ApplyWideShape<D, W>::kSlotBytes;
}

// ==========================================================================================
// State reduction.  grid = (splits, heads), block = 256.  Workgroup x walks blocks of tiles_per_block
// consecutive tiles (x, x + splits, ...; every wave visits every tile).  Per tile: all threads load K and V
// rows (coalesced), apply phi to K, write 16-bit operands into the LDS tiles of the current buffer; barrier;
// every wave reads all phi(K) operand blocks (transposing LDS reads) and the V blocks of its own columns
// and accumulates S[:, its columns]; z rows a = w mod 4 through a ones operand.  Two LDS buffers: the next
// tile is written while slower waves still multiply the previous one, one barrier per tile.
// Partial: S as [D][D] row-major then z, fp32; each wave writes its own columns.
// ==========================================================================================
template <typename T, int D, int FM>
__global__ void __launch_bounds__(kThreads, 2)   // two workgroups per CU: one multiplies while the other loads
state_reduce16_wide(const u32x4* __restrict__ K, Layout kl, const u32x4* __restrict__ V, Layout vl, HeadSubset hs,
                    float* __restrict__ partials, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Sw = ShapeWide<D>;
  constexpr int NS = NSplit<T>::value, RS = Sw::kRS, NL = Sw::kNLR, CPR = Sw::kCPR, MT = Sw::kMT, NBW = Sw::kNBW;
  constexpr int TE = Sw::kTileElems, BUF = (NS + 1) * TE;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const long long bh = hs.bh(blockIdx.y, kl.H);
  const u32x4* Kh = K + kl.slice(bh);
  const u32x4* Vh = V + vl.slice(bh);
  const int rs = kl.row, rsv = vl.row;   // the two tensors may be laid out differently (the backward pass pairs q with a dense temporary)
  uint16_t* lds = reinterpret_cast<uint16_t*>(smem);

  int goff[NL], goffv[NL], loff[NL], trow[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    const int p = u * kThreads + tid;
    const int r = p / CPR, c = p % CPR;
    const bool in = p < Sw::kChunks;
    trow[u] = in ? r : kTile;              // kTile: never below the row limit
    goff[u] = r * rs + c;
    goffv[u] = r * rsv + c;
    loff[u] = in ? r * RS + c * 8 : 0;
  }
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);

  const long long n_tiles = (N + kTile - 1) / kTile;

  f32x4 acc[MT][NBW];
  f32x4 accz[NBW];
  const uint32_t one2 = (uint32_t)OneBits<T>::value * 0x10001u;
  const u32x4 ones = {one2, one2, one2, one2};

  u32x4 kr[NL], vr[NL];
  auto issue_loads = [&](long long tile) {
    long long rem = N - tile * kTile;
    int lim = rem < kTile ? (int)rem : kTile;
    const u32x4* kp = Kh + tile * kTile * rs;
    const u32x4* vp = Vh + tile * kTile * rsv;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (trow[u] < lim) {
        kr[u] = ld_stream(kp + goff[u]);
        vr[u] = ld_stream(vp + goffv[u]);
      } else {
        kr[u] = u32x4{LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value};   // phi maps it to 0
        vr[u] = u32x4{0, 0, 0, 0};
      }
    }
    return lim;
  };

  // fp16 with elu + 1: phi(k) = exp(k) of keys far below zero leaves fp16's normal range (see reduce16_phase: the same
  // remedy here, decided by the workgroup as a whole since its waves share every tile): a stream whose normalizer sums
  // all stay below (tokens) 2^-11 is scanned for its largest key m and, if that is far below zero, summed again with
  // phi(k) = exp(k - m); the factor exp(m) is taken out of the fp32 sums afterwards.  Never taken for ordinary data.
  constexpr bool kRescan = NS == 1 && FM == kPhiEluPlusOne;
  constexpr float kRescanBelow = -5.0f, kShiftFloor = -64.0f, kLog2e = 1.44269504088896340736f;
  __shared__ float wgmax[kWavesPerWG];

  // The workgroup's whole stream, sums of phi(k) 2^kc (x) v into acc / accz; a second pass (fp16, elu + 1 only)
  // where the first one's normalizer sums call for it.
  float kc = 0.0f;
  for (int pass = 0;; ++pass) {
  TileIter it(blockIdx.x, gridDim.x, 0, tiles_per_block, n_tiles, 1);
#pragma unroll
  for (int i = 0; i < NBW; ++i) {
    accz[i] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int a = 0; a < MT; ++a) acc[a][i] = f32x4{0, 0, 0, 0};
  }
  long long tokens = 0;
  int lim = 0;
  if (it.valid()) lim = issue_loads(it.t);
  static_assert(BUF % 8 == 0, "16-byte fill");
  for (int i = tid; i < 2 * BUF / 8; i += kThreads) reinterpret_cast<u32x4*>(lds)[i] = u32x4{0, 0, 0, 0};   // pad columns stay zero
  __syncthreads();

  int buf = 0;
  while (it.valid()) {
    tokens += lim;
    uint16_t* bufp = lds + buf * BUF;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (u * kThreads + tid < Sw::kChunks) {
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
    lds_barrier();   // the tile is complete in this buffer; the other buffer is free to be rewritten

    const uint16_t* ldsV = bufp + NS * TE;
    u32x4 bfrag[NBW];
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
      const int b = wave + kWavesPerWG * i;
      bfrag[i] = u32x4{0, 0, 0, 0};
      if (b < MT) {
        u32x2 r0 = lds_read_tr16(ldsV + tr_base + 16 * b);
        u32x2 r1 = lds_read_tr16(ldsV + tr_base + 4 * RS + 16 * b);
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
  if constexpr (!kRescan) {
    break;
  } else {
    if (pass == 1) {
      const float back = __builtin_amdgcn_exp2f(-kc);      // the rescanned sums carry 2^kc
#pragma unroll
      for (int i = 0; i < NBW; ++i) {
        accz[i] *= back;
#pragma unroll
        for (int a = 0; a < MT; ++a) acc[a][i] *= back;
      }
      break;
    }
    // largest normalizer sum of the workgroup (accz: z of rows a = wave mod 4, every column holds it)
    float zm = 0.0f;
#pragma unroll
    for (int i = 0; i < NBW; ++i)
#pragma unroll
      for (int e = 0; e < 4; ++e) zm = fmaxf(zm, accz[i][e]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) zm = fmaxf(zm, __shfl_xor(zm, o));
    __syncthreads();   // (every wave has left the stream's last tile)
    if (lane == 0) wgmax[wave] = zm;
    __syncthreads();
    zm = 0.0f;
#pragma unroll
    for (int w = 0; w < kWavesPerWG; ++w) zm = fmaxf(zm, wgmax[w]);
    if (!(zm < (float)tokens * 0x1p-11f)) break;   // ordinary data, a workgroup without tiles (0 < 0), NaNs
    // the stream's largest key
    f16x2 kmax2 = __builtin_bit_cast(f16x2, LowestBits<F16>::value);
    {
      TileIter jt(blockIdx.x, gridDim.x, 0, tiles_per_block, n_tiles, 1);
      while (jt.valid()) {
        (void)issue_loads(jt.t);
#pragma unroll
        for (int u = 0; u < NL; ++u) {
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t word = kr[u][w];
            kmax2 = __builtin_elementwise_max(kmax2, __builtin_bit_cast(f16x2, word));
          }
        }
        jt.next();
      }
    }
    float m = fmaxf((float)kmax2[0], (float)kmax2[1]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    __syncthreads();
    if (lane == 0) wgmax[wave] = m;
    __syncthreads();
    m = wgmax[0];
#pragma unroll
    for (int w = 1; w < kWavesPerWG; ++w) m = fmaxf(m, wgmax[w]);
    // (not small after all -- many tokens of middling keys -- or nothing but the most negative value: keep the sums)
    if (!(m < kRescanBelow && m > -65504.0f)) break;
    kc = fmaxf(m, kShiftFloor) * -kLog2e;
  }
  }

  // ---- each wave writes its columns of the partial (lane: rows 4 (l / 16) + i, column l % 16 of a block) ----
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)(D * D + D);
#pragma unroll
  for (int a = 0; a < MT; ++a) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = a * 16 + 4 * g4 + i;
#pragma unroll
      for (int c = 0; c < NBW; ++c) {
        const int b = wave + kWavesPerWG * c;
        if (b < MT) st_agent(dst + row * D + b * 16 + j16, acc[a][c][i]);
      }
      if (a % kWavesPerWG == wave && j16 == 0) st_agent(dst + D * D + row, accz[a / kWavesPerWG][i]);
    }
  }
}

// ==========================================================================================
// Operand-ready state.  The apply kernel multiplies by S'^T = alpha_S S^T (and the normalizer rows
// alpha_z z) as 16-bit matrix-core A operands; building them from the fp32 state costs a pass over d*d + d
// floats, far too much to repeat in every apply workgroup at these widths.  pack_state_wide does it once
// per head: grid = (d / 16, heads), block = 64 W (W = the apply kernel's waves).  Every workgroup finds the maxima (power-of-two scales so
// that 16-bit storage neither overflows nor loses small entries), workgroup s then writes the operands of
// contraction step s for all W apply waves, in the order the apply lanes load them:
//   header  {c1 = alpha_z / alpha_S, alpha_z}, then  frag[level][wave][t][s][lane] (16 bytes each)
// Operand (wave w, tile t, step s), lane l: m = l % 32, kg = l / 32, element j:
//   contraction channel ch = 16 s + 8 kg + j;  slot = 16 t + 4 (m / 8) + m % 4,  half hv = (m / 4) % 2
//   h = d / (2 W):  slot < h -> S'[ch][w d/W + hv h + slot];   slot == h -> z'[ch] rounded to 16 bits;
//   slot == h+1 -> the remainder of z'[ch] after that rounding;  else 0.
// Level 1 (bf16 only) holds the remainders of the S' entries after rounding (hi + lo operands).
// ==========================================================================================
template <typename T, int D, int W> struct PackWide {
  using Sw = ApplyWideShape<D, W>;
  static constexpr int kHeaderBytes = 256;
  static constexpr int kFrags = NSplit<T>::value * W * Sw::kMT2 * Sw::kKS;   // per lane
  static constexpr int kHeadBytes = kHeaderBytes + kFrags * 64 * 16;
};

// Largest |S| and |z| among this thread's share of one head's fp32 state [D*D + D] (NT threads take it in float4
// pieces).  All of a thread's loads are issued before the first is used: as a loop of dependent round trips this
// scan took 12 of the 14 microseconds of the pack kernels at d = 160.
template <int D, int NT>
LF_DEV void state_maxima_share(const float* st, int tid, float& mS, float& mz) {
  constexpr int NE4 = (D * D + D) / 4, PER = (NE4 + NT - 1) / NT;   // D*D and D are multiples of 4
  const f32x4* st4 = reinterpret_cast<const f32x4*>(st);
  f32x4 x[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int e = tid + i * NT;
    x[i] = st4[e < NE4 ? e : NE4 - 1];   // past the end: the last piece once more (a maximum does not mind)
  }
  mS = 0.0f;
  mz = 0.0f;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int e = tid + i * NT;
    const float m = fmaxf(fmaxf(fabsf(x[i][0]), fabsf(x[i][1])), fmaxf(fabsf(x[i][2]), fabsf(x[i][3])));
    if (e < D * D / 4) mS = fmaxf(mS, m); else mz = fmaxf(mz, m);
  }
}

template <typename T, int D, int W>
__global__ void __launch_bounds__(64 * W)
pack_state_wide(const float* __restrict__ state, unsigned char* __restrict__ packed, int normalize) {
  using Sw = ApplyWideShape<D, W>;
  constexpr int NS = NSplit<T>::value, KS = Sw::kKS, MT2 = Sw::kMT2, HALF = Sw::kHalf, DQ = Sw::kDQ, NE = D * D + D;
  constexpr int kThreads = 64 * W, kWavesPerWG = W;   // this kernel's own workgroup shape
  __shared__ float redmax[2 * kWavesPerWG];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int s = blockIdx.x;
  const long long bh = blockIdx.y;
  const float* st = state + bh * NE;
  unsigned char* out = packed + bh * PackWide<T, D, W>::kHeadBytes;

  float mS, mz;
  state_maxima_share<D, kThreads>(st, tid, mS, mz);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    mS = fmaxf(mS, __shfl_xor(mS, o));
    mz = fmaxf(mz, __shfl_xor(mz, o));
  }
  if (lane == 0) { redmax[wave] = mS; redmax[kWavesPerWG + wave] = mz; }
  __syncthreads();
  mS = 0.0f; mz = 0.0f;
#pragma unroll
  for (int w = 0; w < kWavesPerWG; ++w) { mS = fmaxf(mS, redmax[w]); mz = fmaxf(mz, redmax[kWavesPerWG + w]); }
  const float aS = pow2_scale_for(mS);
  const float az = normalize ? pow2_scale_for(mz) : 1.0f;
  if (s == 0 && tid == 0) {
    float* scales = reinterpret_cast<float*>(out);
    scales[0] = az / aS;
    scales[1] = az;
  }

  u32x4* frag = reinterpret_cast<u32x4*>(out + PackWide<T, D, W>::kHeaderBytes);
  const int m = lane & 31, kg = lane >> 5;
  const int hv = (m >> 2) & 1;
#pragma unroll
  for (int t = 0; t < MT2; ++t) {
    const int slot = 16 * t + 4 * (m >> 3) + (m & 3);
    u32x4 hi4, lo4;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      float hi2[2], lo2[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        const int ch = 16 * s + 8 * kg + 2 * w + q;
        float x = 0.0f;
        bool zrem = false;
        if (slot < HALF) x = st[ch * D + wave * DQ + hv * HALF + slot] * aS;
        else if (normalize && slot == HALF) x = st[D * D + ch] * az;
        else if (normalize && slot == HALF + 1) { x = st[D * D + ch] * az; zrem = true; }
        float r0, r1;
        unpack2<T>(pack2<T>(x, 0.0f), r0, r1);   // x rounded once to 16 bits
        hi2[q] = zrem ? x - r0 : x;
        lo2[q] = (slot < HALF) ? x - r0 : 0.0f;
      }
      hi4[w] = pack2<T>(hi2[0], hi2[1]);
      lo4[w] = pack2<T>(lo2[0], lo2[1]);
    }
    frag[(((0 * kWavesPerWG + wave) * MT2 + t) * KS + s) * 64 + lane] = hi4;
    if constexpr (NS == 2) frag[(((1 * kWavesPerWG + wave) * MT2 + t) * KS + s) * 64 + lane] = lo4;
  }
}

// ==========================================================================================
// Apply + normalize.  grid = (wgs, heads), block = 64 W (W = 4 or 8 waves).  The LDS-DMA ring of apply16_dma with workgroup-wide
// slots: wave w copies in (and later stores) token rows (32/W) w .. of a tile, whole rows, and applies phi to
// them in place once they have landed (each element once per workgroup; bf16 keeps the low halves of the
// hi + lo operands in a buffer of their own).  Every wave then reads the whole tile as matrix-core B
// operands and -- after a barrier, since all waves read all channels -- overwrites its own d/W output
// channels of every token in place.  Per wave the
// products are those of apply16_dma for a head whose state has only this wave's d/W columns (plus the two
// normalizer rows, which every wave carries).  Pipelined as the row-piece kernel: store tile j-1, copy tile
// j+2, read tile j, barrier, compute and write back, wait for own rows of tile j+1 and apply phi to them,
// barrier.
// The state arrives operand-ready from pack_state_wide: the prologue is a handful of coalesced loads.
// MLP: the query is formed in that same pass over a wave's rows as  a + LeakyReLU(LayerNorm(t))  (the two-branch
// f' of Sec. 3.1 (Implementation Details)) from the tile of `a` in the ring, the tile of `t` in a second ring behind it (and behind the LO
// buffer), the rows' {rstd, -mean rstd} from an earlier kernel, which travel with each tile as one more 1 KiB
// deposit (256 bytes used; every wave brings the same 32 pairs to the same place and reads its own rows'), and
// the head's gamma, beta from a table in LDS.
// ==========================================================================================
template <typename T, int D, int FM, bool NORM, int W, bool MLP = false>
struct ApplyWide {
  using Sw = ApplyWideShape<D, W>;
  static constexpr int kWavesPerWG = W;   // this kernel's own workgroup shape
  static constexpr int NS = NSplit<T>::value;
  static constexpr int CPR = Sw::kCPR, KS = Sw::kKS, MT2 = Sw::kMT2, HALF = Sw::kHalf, DQ = Sw::kDQ;
  static constexpr int NL = Sw::kNLA, NE = D * D + D, R = Sw::kRing, RPR = Sw::kRPR;
  static_assert(R == 3, "the wait counts below are written for a ring of three slots");
  static constexpr int NLC = MLP ? 2 * NL + 1 : NL;                              // copy instructions per tile
  static constexpr int kTOffset = (R + (NS == 2 ? 1 : 0)) * Sw::kSlotBytes;      // MLP: ring of the t tiles
  static constexpr int kStatOffset = kTOffset + R * Sw::kSlotBytes;              // MLP: R deposits of statistics
  static constexpr int kAffOffset = kStatOffset + R * 1024;                      // MLP: gamma[D] then beta[D], fp32
  static constexpr int kLdsBytes = MLP ? kAffOffset + 2 * D * 4 : kTOffset;

  const u32x4* Qh;
  u32x4* Oh;
  long long N;
  unsigned char* smem;
  int rs_q, rs_o;
  int lane, wave, tok, kg, row_byte, trot;
  int trow[NL], qoff[NL], ooff[NL], soff[NL];
  // MLP: the t tensor, the statistics (two tokens per 16 bytes), the slope; and for the chunk this lane
  // transforms at deposit u of its wave's region: its token row in the tile and its first channel
  const u32x4* Th;
  const u32x4* St;
  float slope;
  int prow[MLP ? NL : 1], pch[MLP ? NL : 1];
  TileIter it, ahead;
  u32x4 A[NS][MT2][KS];
  float c1, eps_s;

  LF_DEV ApplyWide(const u32x4* Qh_, int rs_q_, u32x4* Oh_, int rs_o_, long long N_, int tiles_per_block, int wg,
                   int nwg, unsigned char* smem_)
      : Qh(Qh_), Oh(Oh_), N(N_), smem(smem_), rs_q(rs_q_), rs_o(rs_o_),
        lane(threadIdx.x & 63), wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)),
        it(wg, nwg, 0, tiles_per_block, (N_ + kTile - 1) / kTile, 1), ahead(it) {
    tok = lane & 31;
    kg = lane >> 5;
    row_byte = (tok / RPR) * Sw::kRegionBytes + (tok % RPR) * CPR * 16;
    trot = Sw::rot(tok);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int P = wave * Sw::kRegionChunks + u * 64 + lane;   // position in the tile
      const int r = P / CPR, pos = P % CPR;
      int spos = pos + Sw::rot(r);             // store side: this lane sends chunk pos, found at spos
      if (spos >= CPR) spos -= CPR;
      // copy side: position pos of row r receives chunk c; lanes past the region's chunks copy what the lane 32
      // below copies (same cache lines) and deposit it in the padding
      const int li = u * 64 + lane;            // chunk index inside the region; past its end: a valid stand-in
      const int lc = li < Sw::kRegionChunks ? li : (li - 32 < Sw::kRegionChunks ? li - 32 : li % Sw::kRegionChunks);
      const int Pc = wave * Sw::kRegionChunks + lc;
      const int rc = Pc / CPR;
      int c = Pc % CPR - Sw::rot(rc);
      if (c < 0) c += CPR;
      trow[u] = rc;
      qoff[u] = rc * rs_q + c;
      ooff[u] = r * rs_o + pos;
      soff[u] = ((r % RPR) * CPR + spos) * 16;
      if constexpr (MLP) {
        prow[u] = rc;
        pch[u] = c * 8;
      }
    }
  }

  // MLP: `Th_` addresses t like Qh addresses a; `stats`: the batch's pairs, readable up to a whole last tile;
  // gamma, beta: this head's D values.  Whole workgroup; call before prefetch() (ends with a barrier).
  LF_DEV void set_mlp(const u32x4* Th_, const void* stats, const float* gamma, const float* beta, float slope_) {
    Th = Th_;
    St = reinterpret_cast<const u32x4*>(stats);
    slope = slope_;
    float* aff = reinterpret_cast<float*>(smem + kAffOffset);
    for (int i = threadIdx.x; i < 2 * D; i += 64 * W) aff[i] = i < D ? gamma[i] : beta[i - D];
    __syncthreads();
  }

  LF_DEV unsigned char* region_ptr(int slot) const { return smem + slot * Sw::kSlotBytes + wave * Sw::kRegionBytes; }
  // where this lane finds 16-byte chunk `chunk` of its token's row in slot `slot`
  LF_DEV unsigned char* chunk_ptr(int slot, int chunk) const {
    int x = chunk + trot;
    if (x >= CPR) x -= CPR;
    return smem + slot * Sw::kSlotBytes + row_byte + (x << 4);
  }

  // always issues exactly NL vector memory instructions
  LF_DEV void issue_copy(long long tile, int slot) {
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    const u32x4* qp = Qh + tile * kTile * rs_q;
    unsigned char* sl = region_ptr(slot);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      // every lane issues every copy (see ApplyDma::issue_copy); lanes past the region's chunks deposit a valid
      // chunk in the region's padding
      const int c = trow[u] < lim ? qoff[u] : 0;   // rows past N re-read chunk 0; never stored
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(qp + c),
                                       (LF_LDS void*)(sl + u * 1024), 16, 0, 2 /* nt */);
    }
    if constexpr (MLP) {
      const u32x4* tp = Th + tile * kTile * rs_q;
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        const int c = trow[u] < lim ? qoff[u] : 0;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(tp + c),
                                         (LF_LDS void*)(sl + kTOffset + u * 1024), 16, 0, 2 /* nt */);
      }
      const u32x4* sp = St + tile * (kTile / 2) + (lane & 15);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)sp,
                                       (LF_LDS void*)(smem + kStatOffset + slot * 1024), 16, 0, 0);
    }
  }

  LF_DEV void prefetch() {
    if (ahead.valid()) issue_copy(ahead.t, 0);
    ahead.next();
    if (ahead.valid()) issue_copy(ahead.t, 1);
    ahead.next();
  }

  // `packed`: this head's operands as pack_state_wide wrote them
  LF_DEV void load_packed(const unsigned char* packed, float eps) {
    const u32x4* frag = reinterpret_cast<const u32x4*>(packed + PackWide<T, D, W>::kHeaderBytes);
#pragma unroll
    for (int l = 0; l < NS; ++l)
#pragma unroll
      for (int t = 0; t < MT2; ++t)
#pragma unroll
        for (int s = 0; s < KS; ++s)
          A[l][t][s] = frag[(((l * kWavesPerWG + wave) * MT2 + t) * KS + s) * 64 + lane];
    const float* scales = reinterpret_cast<const float*>(packed);
    c1 = scales[0];
    eps_s = eps * scales[1];
  }

  // phi on this wave's rows of ring slot `slot` (they have landed), in place; bf16: low halves to the LO buffer
  LF_DEV void phi_pass(int slot) {
    unsigned char* sl = region_ptr(slot);
    unsigned char* lo = smem + R * Sw::kSlotBytes + wave * Sw::kRegionBytes;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int at = u * 1024 + lane * 16;
      const u32x4 raw = *reinterpret_cast<const u32x4*>(sl + at);
      u32x4 traw;
      f32x2 rc;
      float gg[8], bb[8];
      if constexpr (MLP) {
        traw = *reinterpret_cast<const u32x4*>(sl + kTOffset + at);
        rc = *reinterpret_cast<const f32x2*>(smem + kStatOffset + slot * 1024 + prow[u] * 8);
        const float* aff = reinterpret_cast<const float*>(smem + kAffOffset);
        const f32x4 g0 = *reinterpret_cast<const f32x4*>(aff + pch[u]);
        const f32x4 g1 = *reinterpret_cast<const f32x4*>(aff + pch[u] + 4);
        const f32x4 b0 = *reinterpret_cast<const f32x4*>(aff + D + pch[u]);
        const f32x4 b1 = *reinterpret_cast<const f32x4*>(aff + D + pch[u] + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          gg[e] = g0[e];
          gg[4 + e] = g1[e];
          bb[e] = b0[e];
          bb[4 + e] = b1[e];
        }
      }
      u32x4 h4, l4;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float x0, x1;
        unpack2<T>(raw[w], x0, x1);
        if constexpr (MLP) {
          float t0, t1;
          unpack2<T>(traw[w], t0, t1);
          const float y0 = __builtin_fmaf(gg[2 * w], __builtin_fmaf(t0, rc[0], rc[1]), bb[2 * w]);
          const float y1 = __builtin_fmaf(gg[2 * w + 1], __builtin_fmaf(t1, rc[0], rc[1]), bb[2 * w + 1]);
          x0 += fmaxf(y0, slope * y0);   // LeakyReLU for slopes up to one
          x1 += fmaxf(y1, slope * y1);
        }
        if constexpr (NS == 1 && !MLP) {
          h4[w] = phi_pack2<T, FM>(raw[w]);
          continue;
        }
        const float r0 = phi<FM>(x0), r1 = phi<FM>(x1);
        if constexpr (NS == 1) {
          h4[w] = pack2<T>(r0, r1);
        } else {
          uint32_t h, l;
          pack2_split<T>(r0, r1, h, l);
          h4[w] = h;
          l4[w] = l;
        }
      }
      *reinterpret_cast<u32x4*>(sl + at) = h4;
      if constexpr (NS == 2) *reinterpret_cast<u32x4*>(lo + at) = l4;
    }
  }

  LF_DEV void store_tile(long long tile, int slot) {
    const unsigned char* sl = region_ptr(slot);
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    u32x4* op = Oh + tile * kTile * rs_o;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(sl + soff[u]);
      if (u * 64 + lane < Sw::kRegionChunks && trow[u] < lim) st_stream(op + ooff[u], w);
    }
  }

  // Issue order per wave:  C0 C1 [state] | C2 K0 w | S0 C3 K1 w | S1 C4 K2 w | ...  : after tile j+1's copies
  // come S(j-1) and C(j+2), where they exist.
  LF_DEV void stream() {
    {
      TileIter second = it;
      second.next();
      if (second.valid()) wait_vmcnt<NLC>();
      else wait_vmcnt<0>();
    }
    if (it.valid()) phi_pass(0);
    __syncthreads();
    int slot = 0, prev_slot = 0;
    long long prev_tile = -1;
    while (it.valid()) {
      const long long tile = it.t;
      const bool have_prev = prev_tile >= 0;
      if (have_prev) store_tile(prev_tile, prev_slot);
      const bool copied = ahead.valid();
      if (copied) issue_copy(ahead.t, have_prev ? prev_slot : R - 1);

      // ---- phi(q) of this lane's token, all channels: the B operands ---------------------------------
      u32x4 Bh[KS], Bl[NS == 2 ? KS : 1];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const unsigned char* p = chunk_ptr(slot, 2 * s + kg);
        Bh[s] = *reinterpret_cast<const u32x4*>(p);
        if constexpr (NS == 2) Bl[s] = *reinterpret_cast<const u32x4*>(p + (R - slot) * Sw::kSlotBytes);
      }
      lds_barrier();   // every wave holds its operands: the tile (and the LO buffer) may be overwritten

      f32x16 acc[MT2];
#pragma unroll
      for (int t = 0; t < MT2; ++t) {
        acc[t] = f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          acc[t] = mfma_32x32x16<T>(A[0][t][s], Bh[s], acc[t]);
          if constexpr (NS == 2) {
            acc[t] = mfma_32x32x16<T>(A[0][t][s], Bl[s], acc[t]);
            if (16 * t < HALF) acc[t] = mfma_32x32x16<T>(A[1][t][s], Bh[s], acc[t]);
          }
        }
      }
      float scale = c1;
      if constexpr (NORM) {
        const float den = acc[HALF / 16][HALF % 16] + acc[(HALF + 1) / 16][(HALF + 1) % 16] + eps_s;
        scale = c1 * __builtin_amdgcn_rcpf(den);
      }
      // ---- this lane's d/8 channels (wave quarter, half kg) -> 16 bits -> back into the row, in pieces
      //      that stay inside one 16-byte chunk -----------------------------------------------------------
      constexpr int PB = (HALF % 8 == 0) ? 16 : ((HALF % 4 == 0) ? 8 : 4);   // piece bytes
      const int byte0 = (wave * DQ + kg * HALF) * 2;
#pragma unroll
      for (int c = 0; c < HALF * 2 / PB; ++c) {
        uint32_t w[PB / 4];
#pragma unroll
        for (int e = 0; e < PB / 4; ++e) {
          const int s0 = c * (PB / 2) + 2 * e;
          w[e] = pack2<T>(acc[s0 / 16][s0 % 16] * scale, acc[(s0 + 1) / 16][(s0 + 1) % 16] * scale);
        }
        const int byte = byte0 + c * PB;
        unsigned char* p = chunk_ptr(slot, byte >> 4) + (byte & 15);
        if constexpr (PB == 16) *reinterpret_cast<u32x4*>(p) = u32x4{w[0], w[1], w[2], w[3]};
        else if constexpr (PB == 8) *reinterpret_cast<u32x2*>(p) = u32x2{w[0], w[1]};
        else *reinterpret_cast<uint32_t*>(p) = w[0];
      }

      it.next();
      ahead.next();
      if (it.valid()) {
        if (have_prev && copied) wait_vmcnt<NL + NLC>();
        else if (copied) wait_vmcnt<NLC>();
        else if (have_prev) wait_vmcnt<NL>();
        else wait_vmcnt<0>();
        phi_pass(slot + 1 == R ? 0 : slot + 1);
      }
      lds_barrier();   // tile j is finished by all waves; tile j+1 has landed and carries phi for all
      prev_tile = tile;
      prev_slot = slot;
      slot = slot + 1 == R ? 0 : slot + 1;
    }
    if (prev_tile >= 0) store_tile(prev_tile, prev_slot);
  }
};

template <typename T, int D, int FM, bool NORM, int W>
__global__ void __launch_bounds__(64 * W)
apply16_wide(const u32x4* __restrict__ Q, Layout lq, u32x4* __restrict__ O, Layout lo, HeadSubset hs,
             const unsigned char* __restrict__ packed, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = hs.bh(blockIdx.y, lq.H);
  ApplyWide<T, D, FM, NORM, W> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, tiles_per_block, blockIdx.x,
                               gridDim.x, smem);
  ap.prefetch();
  ap.load_packed(packed + bh * PackWide<T, D, W>::kHeadBytes, eps);
  ap.stream();
}

}  // namespace lf
