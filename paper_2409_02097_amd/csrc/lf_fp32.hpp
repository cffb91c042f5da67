// fp32 kernels.  fp32 inputs never pass through 16-bit operands: the d x d contractions use the
// fp32 matrix-core instruction (16x16x4), whose operand layout holds one contraction index per
// lane, so no transposition and no LDS staging is needed anywhere.
//   state_reduce32  S_p, z_p over a workgroup's tiles          (Prop. 2: g'(X)^T X; Eq. 5: Z)
//   combine_state   (lf_reduce16.hpp) fixed-order sum of the partials
//   apply32         out_i = phi(q_i) S / (phi(q_i).z + eps)
#pragma once
#include "lf_common.hpp"
#include "lf_reduce16.hpp"   // kWavesPerWG, kThreads, combine_state

namespace lf {

constexpr int kTile32 = 16;   // tokens per tile: four 16x16x4 k-steps

template <int D> struct Shape32 {
  static constexpr int kChunks = D / 4;                     // float4 chunks per token row
  // apply: lane (token = lane % 16, kq = lane / 16) loads the kCS contiguous chunks kq*kCS + cs
  static constexpr int kCS = (kChunks + 3) / 4;
  static constexpr int kKSteps = kCS * 4;
  static constexpr int kQuarter = D / 4;                    // output channels per 16-lane group
  static constexpr int kMT = (kQuarter + 1 + 3) / 4;        // 16-row output tiles incl. normalizer row
};

template <int D> constexpr int reduce32_lds_bytes() { return 2 * (D * D + D) * 4; }

LF_DEV f32x4 mfma_16x16x4(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

// ------------------------------------------------------------------------------------------
// Lane (m = lane % 16, kq = lane / 16) holds channels 4m..4m+3 of token 4u + kq of the tile;
// element i of its K chunk (after phi) is the A operand and element j of its V chunk the B
// operand of product (i, j), whose accumulator tile is S[4*row + i][4*col + j].  z is summed
// on the vector ALU.  `smem`: reduce32_lds_bytes<D>() bytes; `dst`: this workgroup's partial;
// `Kh`, `Vh`: first token row of this head; `rs`: row stride in 16-byte units.
// ------------------------------------------------------------------------------------------
template <int D, int FM>
LF_DEV void reduce32_phase(const f32x4* __restrict__ Kh, const f32x4* __restrict__ Vh, int rs,
                           float* __restrict__ dst, long long N, int tiles_per_block, int split, int nsplit,
                           unsigned char* smem) {
  constexpr int CH = Shape32<D>::kChunks;
  constexpr int U = kTile32 / 4;
  float* red = reinterpret_cast<float*>(smem);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15, kq = lane >> 4;
  const bool lane_on = m < CH;

  const long long n_tiles = (N + kTile32 - 1) / kTile32;
  TileIter it(split, nsplit, wave, tiles_per_block, n_tiles);
  f32x4 acc[4][4];
  float zacc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0, 0, 0, 0};

  f32x4 kr[U], vr[U];
  bool okr[U];
  auto issue_loads = [&](long long tile) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long t = tile * kTile32 + 4 * u + kq;
      okr[u] = lane_on && t < N;
      if (okr[u]) {
        kr[u] = __builtin_nontemporal_load(Kh + t * rs + m);
        vr[u] = __builtin_nontemporal_load(Vh + t * rs + m);
      } else {
        kr[u] = f32x4{0, 0, 0, 0};
        vr[u] = f32x4{0, 0, 0, 0};
      }
    }
  };

  if (it.valid()) issue_loads(it.t);
  while (it.valid()) {
    f32x4 p[U], vv[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < 4; ++i) p[u][i] = okr[u] ? phi<FM, true>(kr[u][i]) : 0.0f;
      vv[u] = vr[u];
    }
    it.next();
    if (it.valid()) issue_loads(it.t);
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        zacc[i] += p[u][i];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = mfma_16x16x4(p[u][i], vv[u][j], acc[i][j]);
      }
    }
  }

  // cross-wave sum in a fixed order, (w0 + w2) + (w1 + w3): waves 0 and 1 park their accumulators in
  // two LDS copies, waves 2 and 3 add theirs on top (inside a wave the four token groups kq = 0..3 add
  // their z in order), then all threads add the two copies and write the partial
  constexpr int NE = D * D + D;
  float* mine = red + (wave & 1) * NE;
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if ((wave >> 1) == round) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = 4 * (4 * kq + r) + i;
          if (row < D) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int col = 4 * m + j;
              if (col < D) {
                float* q = mine + row * D + col;
                *q = (round == 0) ? acc[i][j][r] : *q + acc[i][j][r];
              }
            }
          }
        }
      for (int s = 0; s < 4; ++s) {
        if (kq == s && lane_on) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float* q = mine + D * D + 4 * m + i;
            *q = (round == 0 && s == 0) ? zacc[i] : *q + zacc[i];
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < NE; i += kThreads) st_agent(dst + i, red[i] + red[NE + i]);
}

// grid = (splits, B*H), block = 256
template <int D, int FM>
__global__ void __launch_bounds__(kThreads)
state_reduce32(const f32x4* __restrict__ K, const f32x4* __restrict__ V, Layout kv, float* __restrict__ partials,
               long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.y;
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)(D * D + D);
  const long long off = kv.slice(bh);
  reduce32_phase<D, FM>(K + off, V + off, kv.row, dst, N, tiles_per_block, blockIdx.x, gridDim.x, smem);
}

// ------------------------------------------------------------------------------------------
// Lane (token = lane % 16, kq = lane / 16) loads its kCS contiguous float4 chunks of the Q row;
// element e of chunk cs is the B operand of k-step 4*cs + e against S^T (A operand), which every
// lane gathers once from the head's fp32 state:
// lane l (output row mrow = l % 16, kq = l / 16), tile T, k-step 4*cs + e:
//   feature channel ch = 4*(kq*CS + cs) + e  (zero when that chunk is beyond d)
//   slot = 4*T + mrow % 4, group g = mrow / 4:  slot < d/4 -> S[ch][g*d/4 + slot];
//   slot == d/4 -> z[ch];  else 0.
// The accumulators of a lane hold d/4 contiguous output channels of its token and the
// normalizer phi(q).z.  `state`: this head's [D*D + D] floats; `Qh`, `Oh4`: first token row of this head;
// `rs_q`, `rs_o`: row strides in 16-byte units.
// ------------------------------------------------------------------------------------------
template <int D, int FM, bool NORM>
LF_DEV void apply32_phase(const f32x4* __restrict__ Qh, int rs_q, f32x4* __restrict__ Oh4, int rs_o,
                          const float* state, float eps, long long N, int tiles_per_block, int wg, int nwg) {
  using Sh = Shape32<D>;
  constexpr int CS = Sh::kCS, KST = Sh::kKSteps, MT = Sh::kMT, CH = Sh::kChunks, QT = Sh::kQuarter;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int tok = lane & 15, kq = lane >> 4;
  float A[MT][KST];
  {
    const int mrow = lane & 15, g = mrow >> 2;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int slot = 4 * t + (mrow & 3);
#pragma unroll
      for (int ks = 0; ks < KST; ++ks) {
        const int chunk = kq * CS + (ks >> 2);
        const int ch = 4 * chunk + (ks & 3);
        float x = 0.0f;
        if (chunk < CH) {
          if (slot < QT) x = ld_agent(state + ch * D + g * QT + slot);
          else if (NORM && slot == QT) x = ld_agent(state + D * D + ch);
        }
        A[t][ks] = x;
      }
    }
  }

  const long long n_tiles = (N + kTile32 - 1) / kTile32;
  TileIter it(wg, nwg, wave, tiles_per_block, n_tiles);

  f32x4 qr[CS];
  auto issue_loads = [&](long long tile) {
    const long long t = tile * kTile32 + tok;
#pragma unroll
    for (int cs = 0; cs < CS; ++cs) {
      if (t < N && kq * CS + cs < CH) qr[cs] = __builtin_nontemporal_load(Qh + t * rs_q + kq * CS + cs);
      else qr[cs] = f32x4{0, 0, 0, 0};
    }
  };
  if (it.valid()) issue_loads(it.t);
  while (it.valid()) {
    float r[KST];
#pragma unroll
    for (int cs = 0; cs < CS; ++cs)
#pragma unroll
      for (int e = 0; e < 4; ++e) r[4 * cs + e] = (kq * CS + cs < CH) ? phi<FM, true>(qr[cs][e]) : 0.0f;
    const long long cur = it.t;
    it.next();
    if (it.valid()) issue_loads(it.t);

    f32x4 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      acc[t] = f32x4{0, 0, 0, 0};
#pragma unroll
      for (int ks = 0; ks < KST; ++ks) acc[t] = mfma_16x16x4(A[t][ks], r[ks], acc[t]);
    }
    float scale = 1.0f;
    if constexpr (NORM) scale = 1.0f / (acc[QT / 4][QT % 4] + eps);
    const long long t = cur * kTile32 + tok;
    if (t < N) {
      float* orow = reinterpret_cast<float*>(Oh4 + t * rs_o) + kq * QT;
      if constexpr (QT % 4 == 0) {
#pragma unroll
        for (int c = 0; c < QT / 4; ++c) {
          f32x4 w = {acc[c][0] * scale, acc[c][1] * scale, acc[c][2] * scale, acc[c][3] * scale};
          __builtin_nontemporal_store(w, reinterpret_cast<f32x4*>(orow) + c);
        }
      } else {
#pragma unroll
        for (int c = 0; c < QT / 2; ++c) {
          const int s0 = 2 * c;
          f32x2 w = {acc[s0 / 4][s0 % 4] * scale, acc[(s0 + 1) / 4][(s0 + 1) % 4] * scale};
          __builtin_nontemporal_store(w, reinterpret_cast<f32x2*>(orow) + c);
        }
      }
    }
  }
}

// grid = (wgs_per_head, B*H), block = 256
template <int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply32(const f32x4* __restrict__ Q, Layout lq, f32x4* __restrict__ O, Layout lo, const float* __restrict__ state,
        float eps, long long N, int tiles_per_block) {
  const long long bh = blockIdx.y;
  apply32_phase<D, FM, NORM>(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, state + bh * (D * D + D), eps, N,
                             tiles_per_block, blockIdx.x, gridDim.x);
}

}  // namespace lf
