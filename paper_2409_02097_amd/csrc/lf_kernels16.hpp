// fp16 / bf16 kernels of the split-N path:
//   state_reduce16  S_p = sum_{j in chunk} phi(k_j)^T v_j,  z_p = sum phi(k_j)       (Prop. 2: g'(X)^T X)
//   combine_pack16  S = sum_p S_p, z = sum_p z_p in a fixed order; rescale; pack for apply
//   apply16         out_i = phi(q_i) S / (phi(q_i).z + eps)                            (Eq. 5 normalizer)
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

template <typename T, int D>
constexpr int reduce16_lds_bytes() {
  // per wave: NSplit tiles of phi(K) + one of V; reused by the cross-wave reduction
  int tiles = (NSplit<T>::value + 1) * Reduce16Cfg<D>::kTileElems * 2 * kWavesPerWG;
  int red = (D * D + D) * 4;
  return tiles > red ? tiles : red;
}

template <typename T, int D, int FM>
__global__ void __launch_bounds__(kThreads)
state_reduce16(const u32x4* __restrict__ K, const u32x4* __restrict__ V, float* __restrict__ partials,
               long long N, int tiles_per_block) {
  using Sh = Shape16<D>;
  using Cfg = Reduce16Cfg<D>;
  constexpr int NS = NSplit<T>::value;
  constexpr int RS = Cfg::kRS, NL = Cfg::kNL, CPR = Sh::kChunksPerRow, MT = Sh::kMT;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int split = blockIdx.x;
  const long long bh = blockIdx.y;

  uint16_t* wbase = reinterpret_cast<uint16_t*>(smem) + wave * (NS + 1) * Cfg::kTileElems;
  uint16_t* ldsP[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) ldsP[s] = wbase + s * Cfg::kTileElems;
  uint16_t* ldsV = wbase + NS * Cfg::kTileElems;

  // one-time fill of the wave's tiles: phi(K) pad columns zero; V pad columns zero except the
  // ones column at index D (when a spare column exists) which makes z fall out of the products
  for (int i = lane; i < Cfg::kTileElems; i += 64) {
#pragma unroll
    for (int s = 0; s < NS; ++s) ldsP[s][i] = 0;
    ldsV[i] = (Sh::kSpareCol && (i % RS) == D) ? OneBits<T>::value : (uint16_t)0;
  }

  // per-lane constants: which chunks of a tile this lane moves, and where they land in LDS
  int lds_off[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    int c = u * 64 + lane;
    lds_off[u] = (c / CPR) * RS + (c % CPR) * 8;
  }
  // transposing-read base: lane j of 16-lane group g reads row 8g + 4r + j/4, columns 4*(j%4)..
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);

  const long long n_tiles = (N + kTile - 1) / kTile;
  TileIter it(split, gridDim.x, wave, tiles_per_block, n_tiles);

  const u32x4* Kh = K + bh * N * CPR;
  const u32x4* Vh = V + bh * N * CPR;

  f32x4 acc[MT][MT];
  f32x4 accz[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    accz[a] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < MT; ++b) acc[a][b] = f32x4{0, 0, 0, 0};
  }
  const uint32_t one2 = (uint32_t)OneBits<T>::value * 0x10001u;
  const u32x4 ones = {one2, one2, one2, one2};

  u32x4 kr[NL], vr[NL];
  auto issue_loads = [&](long long tile) {
    // number of valid 16-byte chunks in this tile (ragged last tile of the head)
    long long rem = (N - tile * kTile) * CPR;
    int lim = rem < Cfg::kChunks ? (int)rem : Cfg::kChunks;
    const u32x4* kp = Kh + tile * Cfg::kChunks;
    const u32x4* vp = Vh + tile * Cfg::kChunks;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      int c = u * 64 + lane;
      if (c < lim) {
        kr[u] = ld_stream(kp + c);
        vr[u] = ld_stream(vp + c);
      } else {
        kr[u] = u32x4{0, 0, 0, 0};
        vr[u] = u32x4{0, 0, 0, 0};
      }
    }
    return lim;
  };

  int lim = 0;
  if (it.valid()) lim = issue_loads(it.t);

  while (it.valid()) {
    // ---- phi(K) -> 16-bit (hi [, lo]) -> LDS ; V -> LDS --------------------------------------
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      int c = u * 64 + lane;
      if (c < Cfg::kChunks) {
        const bool ok = c < lim;
        u32x4 ph, pl;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float x0, x1;
          unpack2<T>(kr[u][w], x0, x1);
          float p0 = ok ? phi<FM>(x0) : 0.0f;
          float p1 = ok ? phi<FM>(x1) : 0.0f;
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

  // ---- fixed-order cross-wave sum in LDS (wave 0, then 1, 2, 3), then one partial per WG -----
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);   // [D*D] S then [D] z
  for (int w = 0; w < kWavesPerWG; ++w) {
    if (wave == w) {
#pragma unroll
      for (int a = 0; a < MT; ++a) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = a * 16 + 4 * g4 + i;
          if (row < D) {
#pragma unroll
            for (int b = 0; b < MT; ++b) {
              const int col = b * 16 + j16;
              if (col < D) {
                float* p = red + row * D + col;
                *p = (w == 0) ? acc[a][b][i] : *p + acc[a][b][i];
              } else if (Sh::kSpareCol && col == D) {
                float* p = red + D * D + row;
                *p = (w == 0) ? acc[a][b][i] : *p + acc[a][b][i];
              }
            }
            if constexpr (!Sh::kSpareCol) {
              if (j16 == 0) {
                float* p = red + D * D + row;
                *p = (w == 0) ? accz[a][i] : *p + accz[a][i];
              }
            }
          }
        }
      }
    }
    __syncthreads();
  }
  float* dst = partials + (bh * gridDim.x + split) * (long long)(D * D + D);
  for (int i = threadIdx.x; i < D * D + D; i += kThreads) dst[i] = red[i];
}

// ==========================================================================================
// Combine.  grid = (ceil(NE / 64), B*H), block = 256, NE = d*d + d.  Thread (e, sg) sums element
// e of the head's partials over the sg-th quarter of the splits in split order; the four
// quarters are then added in order 0..3.  Fixed order => run-to-run identical.  Output: the
// fp32 state of the head, S as [d][d] row-major then z as [d].
// ==========================================================================================
constexpr int kCombineThreads = 256;
constexpr int kCombineElems = 64;

__global__ void __launch_bounds__(kCombineThreads)
combine_state(const float* __restrict__ partials, int splits, int NE, float* __restrict__ state) {
  __shared__ float part[4][kCombineElems];
  const int el = threadIdx.x & 63, sg = threadIdx.x >> 6;
  const int e = blockIdx.x * kCombineElems + el;
  const long long bh = blockIdx.y;
  const int per = (splits + 3) / 4;
  int p0 = sg * per, p1 = p0 + per;
  if (p1 > splits) p1 = splits;
  float s = 0.0f;
  if (e < NE) {
    const float* src = partials + (bh * splits) * (long long)NE + e;
    int p = p0;
    for (; p + 8 <= p1; p += 8) {   // eight loads in flight, added in split order
      float a[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) a[i] = src[(long long)(p + i) * NE];
#pragma unroll
      for (int i = 0; i < 8; ++i) s += a[i];
    }
    for (; p < p1; ++p) s += src[(long long)p * NE];
  }
  part[sg][el] = s;
  __syncthreads();
  if (sg == 0 && e < NE) state[bh * NE + e] = ((part[0][el] + part[1][el]) + part[2][el]) + part[3][el];
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

// ==========================================================================================
// Apply + normalize.  grid = (wgs_per_head, B*H), block = 256, dynamic LDS.
//
// Prologue (once per workgroup): the head's fp32 state is staged in LDS, rescaled by powers of
// two so that 16-bit storage neither overflows nor loses small entries (S' = alpha_S S,
// z' = alpha_z z), and every lane builds its matrix-core A operands (S'^T and the normalizer
// rows) in registers.  Fragment (T, s), lane l: output row m = l % 32, contraction group
// kg = l / 32, element j:
//   feature channel  ch   = (kg * KS + s) * 8 + j           (zero when that chunk is beyond d)
//   output slot      slot = 16 T + 4 (m / 8) + (m % 4),  half hv = (m / 4) % 2
//   slot <  d/2   -> S'[ch][hv * d/2 + slot];  slot == d/2 -> z' rounded to 16 bits;
//   slot == d/2+1 -> the remainder of z' after that rounding;  else 0.
// bf16 carries S' as hi + lo fragments (three products per step) to keep ~16 significant bits.
//
// Stream loop (per wave, 32-token tiles round-robin, no workgroup barrier): coalesced 128-bit
// loads of the contiguous tile -> phi -> 16-bit -> wave-private LDS tile -> each lane reads back
// the 8-channel pieces of its own token (lane % 32) as B operands -> 32x32x16 products: a lane's
// accumulators hold d/2 contiguous output channels of its token plus the two normalizer rows ->
// out = num * c1 / (den + eps') -> 16-bit -> LDS tile -> coalesced 128-bit stores.
// Q is read once, out is written once.
// ==========================================================================================
template <int D> struct Apply16Cfg {
  using Sh = Shape16<D>;
  static constexpr int kRowUnits = ((D * 2 / 16) % 2 == 0) ? D * 2 / 16 + 1 : D * 2 / 16;  // odd # of 16 B units
  static constexpr int kRS = kRowUnits * 8;                        // LDS row stride in 16-bit elements
  static constexpr int kTileElems = kTile * kRS;
  static constexpr int kChunks = kTile * Sh::kChunksPerRow;
  static constexpr int kNL = (kChunks + 63) / 64;
};

template <typename T, int D>
constexpr int apply16_lds_bytes() {
  int tiles = NSplit<T>::value * Apply16Cfg<D>::kTileElems * 2 * kWavesPerWG;
  int st = (D * D + D) * 4 + 64;
  return tiles > st ? tiles : st;
}

template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply16(const u32x4* __restrict__ Q, u32x4* __restrict__ O, const float* __restrict__ state, float eps,
        long long N, int tiles_per_block) {
  using Sh = Shape16<D>;
  using Cfg = Apply16Cfg<D>;
  constexpr int NS = NSplit<T>::value;
  constexpr int KS = Sh::kKS, MT2 = Sh::kMT2, CPR = Sh::kChunksPerRow, HALF = Sh::kHalf;
  constexpr int RS = Cfg::kRS, NL = Cfg::kNL, NE = D * D + D;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long bh = blockIdx.y;
  const int tok = lane & 31, kg = lane >> 5;

  // ---- prologue: state -> LDS, maxima, scales, A fragments ---------------------------------
  float* st = reinterpret_cast<float*>(smem);
  float* redmax = st + NE;                    // [2][kWavesPerWG]
  float mS = 0.0f, mz = 0.0f;
  for (int e = threadIdx.x; e < NE; e += kThreads) {
    float x = state[bh * NE + e];
    st[e] = x;
    if (e < D * D) mS = fmaxf(mS, fabsf(x)); else mz = fmaxf(mz, fabsf(x));
  }
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
  const float az = NORM ? pow2_scale_for(mz) : 1.0f;
  const float c1 = az / aS;
  const float eps_s = eps * az;

  u32x4 A[NS][MT2][KS];
  {
    const int m = lane & 31;
    const int hv = (m >> 2) & 1;
#pragma unroll
    for (int t = 0; t < MT2; ++t) {
      const int slot = 16 * t + 4 * (m >> 3) + (m & 3);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int chunk = kg * KS + s;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float hi2[2], lo2[2];
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int ch = chunk * 8 + 2 * w + q;
            float x = 0.0f;
            bool zrem = false;
            if (chunk < CPR) {
              if (slot < HALF) x = st[ch * D + hv * HALF + slot] * aS;
              else if (NORM && slot == HALF) x = st[D * D + ch] * az;
              else if (NORM && slot == HALF + 1) { x = st[D * D + ch] * az; zrem = true; }
            }
            float r0, r1;
            unpack2<T>(pack2<T>(x, 0.0f), r0, r1);     // x rounded once to 16 bits
            hi2[q] = zrem ? x - r0 : x;
            lo2[q] = (slot < HALF) ? x - r0 : 0.0f;    // S' remainder -> lo fragment (bf16 only)
          }
          A[0][t][s][w] = pack2<T>(hi2[0], hi2[1]);
          if constexpr (NS == 2) A[1][t][s][w] = pack2<T>(lo2[0], lo2[1]);
        }
      }
    }
  }
  __syncthreads();   // state in LDS no longer needed: the space becomes the waves' tiles

  // ---- stream loop ---------------------------------------------------------------------------------
  uint16_t* tileH = reinterpret_cast<uint16_t*>(smem) + wave * NS * Cfg::kTileElems;
  uint16_t* tileL = tileH + Cfg::kTileElems;   // only touched when NS == 2
  int lds_off[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    int c = u * 64 + lane;
    lds_off[u] = (c / CPR) * RS + (c % CPR) * 8;
  }
  const int row_off = tok * RS;

  const long long n_tiles = (N + kTile - 1) / kTile;
  TileIter it(blockIdx.x, gridDim.x, wave, tiles_per_block, n_tiles);
  const u32x4* Qh = Q + bh * N * CPR;
  u32x4* Oh = O + bh * N * CPR;

  u32x4 qr[NL];
  auto issue_loads = [&](long long tile) {
    long long rem = (N - tile * kTile) * CPR;
    int lim = rem < Cfg::kChunks ? (int)rem : Cfg::kChunks;
    const u32x4* qp = Qh + tile * Cfg::kChunks;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      int c = u * 64 + lane;
      if (c < lim) qr[u] = ld_stream(qp + c);
      else qr[u] = u32x4{0, 0, 0, 0};
    }
    return lim;
  };

  int lim = 0;
  if (it.valid()) lim = issue_loads(it.t);
  while (it.valid()) {
    // phi(Q) -> 16-bit -> LDS (coalesced layout in, token-per-lane layout out)
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      int c = u * 64 + lane;
      if (c < Cfg::kChunks) {
        u32x4 ph, pl;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float x0, x1;
          unpack2<T>(qr[u][w], x0, x1);
          float r0 = phi<FM>(x0), r1 = phi<FM>(x1);
          if constexpr (NS == 1) {
            ph[w] = pack2<T>(r0, r1);
          } else {
            uint32_t h, l;
            pack2_split<T>(r0, r1, h, l);
            ph[w] = h;
            pl[w] = l;
          }
        }
        *reinterpret_cast<u32x4*>(tileH + lds_off[u]) = ph;
        if constexpr (NS == 2) *reinterpret_cast<u32x4*>(tileL + lds_off[u]) = pl;
      }
    }
    const long long cur = it.t;
    const int cur_lim = lim;
    it.next();
    if (it.valid()) lim = issue_loads(it.t);

    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    u32x4 Bh[KS], Bl[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const bool ok = kg * KS + s < CPR;
      const int off = row_off + (kg * KS + s) * 8;
      Bh[s] = ok ? *reinterpret_cast<const u32x4*>(tileH + off) : u32x4{0, 0, 0, 0};
      if constexpr (NS == 2) Bl[s] = ok ? *reinterpret_cast<const u32x4*>(tileL + off) : u32x4{0, 0, 0, 0};
    }

    f32x16 acc[MT2];
#pragma unroll
    for (int t = 0; t < MT2; ++t) {
      acc[t] = f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        acc[t] = mfma_32x32x16<T>(A[0][t][s], Bh[s], acc[t]);
        if constexpr (NS == 2) {
          acc[t] = mfma_32x32x16<T>(A[0][t][s], Bl[s], acc[t]);
          if (16 * t < HALF) acc[t] = mfma_32x32x16<T>(A[1][t][s], Bh[s], acc[t]);   // lo rows are zero beyond S'
        }
      }
    }
    // normalizer: slots HALF (z' rounded) and HALF+1 (its remainder) of this lane's accumulators
    float scale = c1;
    if constexpr (NORM) {
      const float den = acc[HALF / 16][HALF % 16] + acc[(HALF + 1) / 16][(HALF + 1) % 16] + eps_s;
      scale = c1 * __builtin_amdgcn_rcpf(den);
    }
    // this lane's d/2 channels of its token -> 16-bit -> LDS row (rows that hold no token of the
    // ragged last tile are written too but never stored)
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    uint16_t* orow = tileH + row_off + kg * HALF;
    if constexpr ((HALF * 2) % 16 == 0) {
#pragma unroll
      for (int c = 0; c < HALF / 8; ++c) {
        u32x4 w;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int s0 = c * 8 + 2 * e;
          w[e] = pack2<T>(acc[s0 / 16][s0 % 16] * scale, acc[(s0 + 1) / 16][(s0 + 1) % 16] * scale);
        }
        *reinterpret_cast<u32x4*>(orow + c * 8) = w;
      }
    } else {
#pragma unroll
      for (int c = 0; c < HALF / 4; ++c) {
        u32x2 w;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int s0 = c * 4 + 2 * e;
          w[e] = pack2<T>(acc[s0 / 16][s0 % 16] * scale, acc[(s0 + 1) / 16][(s0 + 1) % 16] * scale);
        }
        *reinterpret_cast<u32x2*>(orow + c * 4) = w;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    u32x4* op = Oh + cur * Cfg::kChunks;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      int c = u * 64 + lane;
      if (c < cur_lim) st_stream(op + c, *reinterpret_cast<const u32x4*>(tileH + lds_off[u]));
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  }
}

}  // namespace lf
