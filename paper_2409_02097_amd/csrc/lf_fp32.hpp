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

template <int D> constexpr int reduce32_lds_bytes(int waves = kWavesPerWG) { return reduce_copies(waves, D) * (D * D + D) * 4; }

LF_DEV f32x4 mfma_16x16x4(float a, float b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

// ------------------------------------------------------------------------------------------
// Lane (m = lane % 16, kq = lane / 16) holds channels 4m..4m+3 of token 4u + kq of the tile;
// element i of its K chunk (after phi) is the A operand and element j of its V chunk the B
// operand of product (i, j), whose accumulator tile is S[4*row + i][4*col + j].  z is summed
// on the vector ALU.  `smem`: reduce32_lds_bytes<D>(WAVES) bytes; `dst`: this workgroup's partial;
// `Kh`, `Vh`: first token row of this head; `rs`, `rsv`: their row strides in 16-byte units.  WAVES, TO_LDS: as reduce16_phase.
// ------------------------------------------------------------------------------------------
template <int D, int FM, int WAVES = kWavesPerWG, bool TO_LDS = false>
LF_DEV void reduce32_phase(const f32x4* __restrict__ Kh, const f32x4* __restrict__ Vh, int rs, int rsv,
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
  TileIter it(split, nsplit, wave, tiles_per_block, n_tiles, WAVES);
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
        if constexpr (TO_LDS) {      // every workgroup of the head reads these rows: keep them in the L2
          kr[u] = Kh[t * rs + m];
          vr[u] = Vh[t * rsv + m];
        } else {
          kr[u] = __builtin_nontemporal_load(Kh + t * rs + m);
          vr[u] = __builtin_nontemporal_load(Vh + t * rsv + m);
        }
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

  // cross-wave sum in a fixed order: wave w adds into LDS copy w % COPIES in round w / COPIES (round 0 stores;
  // inside a wave the four token groups kq = 0..3 add their z in order, by lane exchanges), then all threads add
  // the copies in order and write the partial.  Four waves: (w0 + w2) + (w1 + w3), with two copies or four (four:
  // every wave stores at once and no read-add-write round is needed).  A lane's four columns of a row leave as one
  // 16-byte store.
  constexpr int NE = D * D + D;
  constexpr int COPIES = reduce_copies(WAVES, D);
  static_assert(WAVES % COPIES == 0, "whole rounds");
  static_assert(D % 4 == 0, "rows of the state are moved four columns at a time");
  float* mine = red + (wave % COPIES) * NE;
  float zsum[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    float t = __shfl(zacc[i], m);
#pragma unroll
    for (int s = 1; s < 4; ++s) t += __shfl(zacc[i], m + 16 * s);
    zsum[i] = t;
  }
#pragma unroll
  for (int round = 0; round < WAVES / COPIES; ++round) {
    if (wave / COPIES == round) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = 4 * (4 * kq + r) + i;
          if (row < D && lane_on) {
            f32x4* q = reinterpret_cast<f32x4*>(mine + row * D + 4 * m);
            f32x4 x = f32x4{acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]};
            if (round != 0) x += *q;
            *q = x;
          }
        }
      if (kq == 0 && lane_on) {
        f32x4* q = reinterpret_cast<f32x4*>(mine + D * D + 4 * m);
        f32x4 x = f32x4{zsum[0], zsum[1], zsum[2], zsum[3]};
        if (round != 0) x += *q;
        *q = x;
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

// grid = (splits, B*H), block = 256
template <int D, int FM>
__global__ void __launch_bounds__(kThreads)
state_reduce32(const f32x4* __restrict__ K, Layout kl, const f32x4* __restrict__ V, Layout vl,
               float* __restrict__ partials, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.y;
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)(D * D + D);
  reduce32_phase<D, FM>(K + kl.slice(bh), V + vl.slice(bh), kl.row, vl.row, dst, N, tiles_per_block, blockIdx.x,
                        gridDim.x, smem);
}

// ------------------------------------------------------------------------------------------
// Apply + normalize, fp32.  out^T = S^T phi(Q)^T with 16x16x4 products: the A operands (one value per lane
// and k-step) are gathered once from the head's fp32 state:
//   lane l (output row mrow = l % 16, kq = l / 16), tile T, k-step 4*cs + e:
//   feature channel ch = 4*(kq*CS + cs) + e  (zero when that chunk is beyond d)
//   slot = 4*T + mrow % 4, group g = mrow / 4:  slot < d/4 -> S[ch][g*d/4 + slot];
//   slot == d/4 -> z[ch];  else 0.
// The accumulators of a lane (token = l % 16, quarter kq) hold d/4 contiguous output channels of its
// token and the normalizer phi(q).z.
// Q tiles (16 tokens, contiguous rows) travel as in apply16_dma: each wave owns a ring of three LDS slots
// filled by asynchronous global->LDS copies two tiles ahead, lanes read their own token's chunks from the
// slot, write their channels back into it, and the tile leaves with coalesced stores in memory order.
// The 16-byte chunks of a row are rotated by a row-dependent amount so that the token-per-lane accesses
// are bank-conflict free for every d (row r by (r * G / 16) mod G chunks, G = gcd(d / 4, 16)).
// ------------------------------------------------------------------------------------------
template <int D> struct Apply32Cfg {
  static constexpr int kCH = D / 4;
  static constexpr int kChunks = kTile32 * kCH;      // 16-byte chunks per tile
  static constexpr int kNL = (kChunks + 63) / 64;
  static constexpr int kSlotBytes = kNL * 1024;
  static constexpr int kRing = 3;
  static constexpr int kG = (kCH % 16 == 0) ? 16 : ((kCH % 8 == 0) ? 8 : ((kCH % 4 == 0) ? 4 : 2));
  static_assert(kCH % 2 == 0, "d is a multiple of 8");
  static __device__ __forceinline__ int rot(int r) { return ((r * kG) >> 4) & (kG - 1); }
};
template <int D> constexpr int apply32_lds_bytes(int waves = kWavesPerWG) { return Apply32Cfg<D>::kRing * waves * Apply32Cfg<D>::kSlotBytes; }

template <int N> LF_DEV void wait_vmcnt32() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// WPW: waves per workgroup (each wave streams on its own)
template <int D, int FM, bool NORM, int WPW = kWavesPerWG>
struct Apply32Dma {
  using Sh = Shape32<D>;
  using Cfg = Apply32Cfg<D>;
  static constexpr int CS = Sh::kCS, KST = Sh::kKSteps, MT = Sh::kMT, CH = Sh::kChunks, QT = Sh::kQuarter;
  static constexpr int NL = Cfg::kNL, R = Cfg::kRing;
  static_assert(R == 3, "the wait counts below are written for a ring of three slots");

  const f32x4* Qh;
  f32x4* Oh;
  long long N;
  unsigned char* smem;
  int rs_q, rs_o;
  int lane, wave, tok, kq, row_byte, trot;
  int trow[NL], qoff[NL], ooff[NL], soff[NL];
  TileIter it, ahead;
  float A[MT][KST];

  LF_DEV Apply32Dma(const f32x4* Qh_, int rs_q_, f32x4* Oh_, int rs_o_, long long N_, int tiles_per_block, int wg,
                    int nwg, unsigned char* smem_)
      : Qh(Qh_), Oh(Oh_), N(N_), smem(smem_), rs_q(rs_q_), rs_o(rs_o_), lane(threadIdx.x & 63),
        wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)),
        it(wg, nwg, wave, tiles_per_block, (N_ + kTile32 - 1) / kTile32, WPW), ahead(it) {
    tok = lane & 15;
    kq = lane >> 4;
    row_byte = tok * CH * 16;
    trot = Cfg::rot(tok);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int P = u * 64 + lane;
      const int r = P / CH, pos = P % CH;
      int c = pos - Cfg::rot(r);                 // copy side: position pos of row r receives chunk c
      if (c < 0) c += CH;
      int spos = pos + Cfg::rot(r);              // store side: this lane sends chunk pos, found at spos
      if (spos >= CH) spos -= CH;
      trow[u] = r;
      qoff[u] = r * rs_q + c;
      ooff[u] = r * rs_o + pos;
      soff[u] = (r * CH + spos) * 16;
    }
  }

  LF_DEV unsigned char* slot_ptr(int slot) const { return smem + (slot * WPW + wave) * Cfg::kSlotBytes; }
  LF_DEV unsigned char* chunk_ptr(int slot, int chunk) const {
    int x = chunk + trot;
    if (x >= CH) x -= CH;
    return slot_ptr(slot) + row_byte + (x << 4);
  }

  // always issues exactly NL vector memory instructions
  LF_DEV void issue_copy(long long tile, int slot) {
    long long rem = N - tile * kTile32;
    const int lim = rem < kTile32 ? (int)rem : kTile32;
    const f32x4* qp = Qh + tile * kTile32 * rs_q;
    unsigned char* sl = slot_ptr(slot);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      // every lane issues every copy (see ApplyDma::issue_copy); lanes past the tile deposit chunk 0 in the padding
      const int c = trow[u] < lim ? qoff[u] : 0;   // rows past N re-read chunk 0; never stored
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(qp + c),
                                       (LF_LDS void*)(sl + u * 1024), 16, 0, 2 /* nt */);
    }
  }
  LF_DEV void prefetch() {
    if (ahead.valid()) issue_copy(ahead.t, 0);
    ahead.next();
    if (ahead.valid()) issue_copy(ahead.t, 1);
    ahead.next();
  }

  // COHERENT: the state was written by other workgroups of the same launch (single-launch kernel)
  // Every lane loads all its operands from clamped, valid places first (the loads are independent and issued
  // back to back) and zeroes the unused ones afterwards; a test around each load would serialise them.
  template <bool COHERENT>
  LF_DEV void load_state(const float* state) {
    const int mrow = lane & 15, g = mrow >> 2;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int slot = 4 * t + (mrow & 3);
      const bool isS = slot < QT;
#pragma unroll
      for (int ks = 0; ks < KST; ++ks) {
        const int chunk = kq * CS + (ks >> 2);
        const int ch = 4 * (chunk < CH ? chunk : 0) + (ks & 3);
        const float* p = isS ? state + ch * D + g * QT + slot : state + D * D + ch;
        A[t][ks] = COHERENT ? ld_agent(p) : *p;
      }
    }
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int slot = 4 * t + (mrow & 3);
      const bool isS = slot < QT, isZ = NORM && slot == QT;
#pragma unroll
      for (int ks = 0; ks < KST; ++ks) {
        const bool used = (kq * CS + (ks >> 2) < CH) && (isS || isZ);
        A[t][ks] = used ? A[t][ks] : 0.0f;
      }
    }
  }

  LF_DEV void stream(float eps) {
    int slot = 0, iter = 0;
    while (it.valid()) {
      const long long tile = it.t;
      int aslot = slot + (R - 1);
      if (aslot >= R) aslot -= R;
      if (ahead.valid()) {
        issue_copy(ahead.t, aslot);
        // issue order  C0 C1 | C2 W0 S0 | C3 W1 S1 | ... : after tile j's copies come C(j+1), C(j+2), S(j-2), S(j-1)
        if (iter == 0) wait_vmcnt32<2 * NL>();
        else if (iter == 1) wait_vmcnt32<3 * NL>();
        else wait_vmcnt32<4 * NL>();
      } else {
        wait_vmcnt32<0>();
      }
      iter = iter < 2 ? iter + 1 : 2;

      float r[KST];
#pragma unroll
      for (int cs = 0; cs < CS; ++cs) {
        const int chunk = kq * CS + cs;
        f32x4 raw = f32x4{0, 0, 0, 0};
        if (chunk < CH) raw = *reinterpret_cast<const f32x4*>(chunk_ptr(slot, chunk));
#pragma unroll
        for (int e = 0; e < 4; ++e) r[4 * cs + e] = (chunk < CH) ? phi<FM, true>(raw[e]) : 0.0f;
      }
      f32x4 acc[MT];
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        acc[t] = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KST; ++ks) acc[t] = mfma_16x16x4(A[t][ks], r[ks], acc[t]);
      }
      float scale = 1.0f;
      if constexpr (NORM) scale = 1.0f / (acc[QT / 4][QT % 4] + eps);

      // ---- d/4 channels of this lane's token back into the slot, in pieces inside one chunk ----------
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      constexpr int PB = (QT % 4 == 0) ? 16 : 8;
#pragma unroll
      for (int c = 0; c < QT * 4 / PB; ++c) {
        const int byte = kq * QT * 4 + c * PB;
        unsigned char* p = chunk_ptr(slot, byte >> 4) + (byte & 15);
        const int s0 = c * (PB / 4);
        if constexpr (PB == 16) {
          *reinterpret_cast<f32x4*>(p) = f32x4{acc[s0 / 4][s0 % 4] * scale, acc[(s0 + 1) / 4][(s0 + 1) % 4] * scale,
                                               acc[(s0 + 2) / 4][(s0 + 2) % 4] * scale, acc[(s0 + 3) / 4][(s0 + 3) % 4] * scale};
        } else {
          *reinterpret_cast<f32x2*>(p) = f32x2{acc[s0 / 4][s0 % 4] * scale, acc[(s0 + 1) / 4][(s0 + 1) % 4] * scale};
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

      // ---- coalesced stores in memory order; always NL instructions ------------------------------------
      {
        const unsigned char* sl = slot_ptr(slot);
        long long rem = N - tile * kTile32;
        const int lim = rem < kTile32 ? (int)rem : kTile32;
        f32x4* op = Oh + tile * kTile32 * rs_o;
#pragma unroll
        for (int u = 0; u < NL; ++u) {
          const f32x4 w = *reinterpret_cast<const f32x4*>(sl + soff[u]);
          if (u * 64 + lane < Cfg::kChunks && trow[u] < lim) __builtin_nontemporal_store(w, op + ooff[u]);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      it.next();
      ahead.next();
      slot = slot + 1 == R ? 0 : slot + 1;
    }
  }
};

// grid = (wgs_per_head, B*H), block = 256, dynamic LDS apply32_lds_bytes<D>()
template <int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply32(const f32x4* __restrict__ Q, Layout lq, f32x4* __restrict__ O, Layout lo, const float* __restrict__ state,
        float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.y;
  Apply32Dma<D, FM, NORM> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, tiles_per_block, blockIdx.x,
                             gridDim.x, smem);
  ap.prefetch();
  ap.template load_state<false>(state + bh * (D * D + D));
  ap.stream(eps);
}

}  // namespace lf
