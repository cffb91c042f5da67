// Apply + normalize for fp16 / bf16 with asynchronous global->LDS tile loads.
//   out_i = phi(q_i) S / (phi(q_i).z + eps)                     (Eq. 5 normalizer on Prop. 2's form)
//
// grid = (wgs_per_head, B*H), block = 256, dynamic LDS.
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
// The output is computed transposed (out^T = S'^T phi(Q)^T, 32x32x16 products) so that a lane's
// accumulators hold d/2 contiguous output channels of its token plus the two normalizer rows:
// out = num * c1 / (den + eps'), c1 = alpha_z / alpha_S, eps' = eps alpha_z.
//
// Stream loop: how a Q tile reaches the lanes:
//   * each wave owns a ring of kRing LDS slots; a tile (32 tokens, contiguous in memory) is copied
//     into a slot by `global_load_lds_dwordx4` (lane l of load u deposits 16 bytes at slot + 1024 u
//     + 16 l), so tiles in flight occupy LDS, not registers, and kRing-1 tiles are always in flight;
//     the first two tiles are requested before the prologue, which hides their latency;
//   * a lane then reads the 8-channel pieces of its own token (lane % 32) straight from the slot as
//     matrix-core B operands and applies phi in registers;
//   * the finished rows go back into the same slot and leave with coalesced 128-bit stores.
// For head widths whose row is a power-of-two number of 16-byte chunks the chunk position inside a
// row is XOR-swizzled with the row index (both on the way in and on the way out) so that the
// token-per-lane LDS accesses are bank-conflict free; global accesses stay whole 128-byte rows.
//
// Completion of the asynchronous copies is tracked with the vector-memory counter: vector memory
// operations of a wave (these copies and the output stores alike) retire in issue order, so
// "at most n outstanding" with n = the number of vector memory instructions issued after the
// wanted tile's copies means that tile has landed.  Every instruction counted this way is issued
// unconditionally (partial lane masks, clamped addresses) so that n is a compile-time constant in
// the steady state; the last kRing-1 tiles of a wave simply wait for everything.  Other vector
// memory operations issued in between (the prologue's state loads) only make the wait stricter.
//
// LDS layout: slot s of wave w at (s * 4 + w) * kSlotBytes; the state staging area of the prologue
// starts at the third slot block (free until the stream loop starts) and may extend past the ring.
#pragma once
#include "lf_reduce16.hpp"

namespace lf {

template <int D> struct ApplyDmaCfg {
  using Sh = Shape16<D>;
  static constexpr int kCPR = Sh::kChunksPerRow;
  static constexpr int kRowBytes = D * 2;
  static constexpr int kChunks = kTile * kCPR;
  static constexpr int kNL = (kChunks + 63) / 64;
  static constexpr int kSlotBytes = kNL * 1024;          // whole 1 KiB deposits; >= the tile's bytes
  static constexpr int kRing = 3;
  static constexpr int kStageOffset = (kRing - 1) * kWavesPerWG * kSlotBytes;
  static constexpr int kStageBytes = (D * D + D) * 4 + 64;
  // XOR swizzle of the chunk position with the row index where rows are 64 or 128 bytes
  static constexpr int kSwzMask = (kCPR == 8) ? 7 : (kCPR == 4 ? 3 : 0);
  static constexpr int kSwzShift = (kCPR == 4) ? 2 : 0;
  static __device__ __forceinline__ int swz(int row) { return (row >> kSwzShift) & kSwzMask; }
};

template <typename T, int D>
constexpr int apply16_dma_lds_bytes() {
  int ring = ApplyDmaCfg<D>::kRing * ApplyDmaCfg<D>::kSlotBytes * kWavesPerWG;
  int st = ApplyDmaCfg<D>::kStageOffset + ApplyDmaCfg<D>::kStageBytes;
  return ring > st ? ring : st;
}

template <int N> LF_DEV void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// One workgroup's apply work: construct, prefetch(), run() -- or, with HG ("one head per wave": the four
// waves work on four different heads over the same tiles, every wave visiting all of the workgroup's
// tiles), construct with the wave's own pointers, prefetch(), load_state() once per head of the group,
// stream().  HG stores are ordinary cached stores: the waves of a group fill neighbouring pieces of
// the same memory rows, which the cache then writes back whole.
template <typename T, int D, int FM, bool NORM, bool HG = false>
struct ApplyDma {
  using Sh = Shape16<D>;
  using Cfg = ApplyDmaCfg<D>;
  static constexpr int NS = NSplit<T>::value;
  static constexpr int KS = Sh::kKS, MT2 = Sh::kMT2, CPR = Sh::kChunksPerRow, HALF = Sh::kHalf;
  static constexpr int NL = Cfg::kNL, NE = D * D + D, R = Cfg::kRing;
  static_assert(R == 3, "the wait counts below are written for a ring of three slots");

  const u32x4* Qh;
  u32x4* Oh;
  long long N;
  unsigned char* smem;
  int rs_q, rs_o;
  int lane, wave, tok, kg, row_byte, tsw;
  // LDS position p = 64 u + lane of a slot holds the chunk of token row trow[u] that lies qoff[u]
  // (in Q) / ooff[u] (in out) vector units after the tile's first row
  int trow[NL], qoff[NL], ooff[NL];
  TileIter it, ahead;
  u32x4 A[NSplit<T>::value][Shape16<D>::kMT2][Shape16<D>::kKS];   // this wave's state operands
  float c1, eps_s;

  // `Qh_`, `Oh_`: first token row of this head; `rs_q_`, `rs_o_`: row strides in 16-byte units
  LF_DEV ApplyDma(const u32x4* Qh_, int rs_q_, u32x4* Oh_, int rs_o_, long long N_, int tiles_per_block, int wg,
                  int nwg, unsigned char* smem_, bool active = true)
      : Qh(Qh_), Oh(Oh_), N(N_), smem(smem_), rs_q(rs_q_), rs_o(rs_o_),
        lane(threadIdx.x & 63), wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)),
        it(wg, nwg, HG ? 0 : wave, tiles_per_block, (HG && !active) ? 0 : (N_ + kTile - 1) / kTile,
           HG ? 1 : kWavesPerWG),
        ahead(it) {
    tok = lane & 31;
    kg = lane >> 5;
    row_byte = tok * Cfg::kRowBytes;
    tsw = Cfg::swz(tok);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int p = u * 64 + lane;
      const int r = p / CPR, pos = p % CPR;
      trow[u] = r;
      qoff[u] = r * rs_q + (pos ^ Cfg::swz(r));
      ooff[u] = r * rs_o + (pos ^ Cfg::swz(r));
    }
  }

  LF_DEV unsigned char* slot_ptr(int slot) const { return smem + (slot * kWavesPerWG + wave) * Cfg::kSlotBytes; }

  // copies tile `tile` into ring slot `slot`; always issues exactly NL vector memory instructions
  LF_DEV void issue_copy(long long tile, int slot) {
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;   // valid token rows
    const u32x4* qp = Qh + tile * kTile * rs_q;
    unsigned char* sl = slot_ptr(slot);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      if (u * 64 + lane < Cfg::kChunks) {          // lanes past the tile would deposit past the slot's rows
        const int c = trow[u] < lim ? qoff[u] : 0; // rows past N re-read chunk 0; their results are never stored
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(qp + c),
                                         (LF_LDS void*)(sl + u * 1024), 16, 0, 2 /* nt */);
      }
    }
  }

  // Requests the wave's first two tiles.  Ring slots 0 and 1 (the first 8 * kSlotBytes of `smem`) must
  // no longer be in use by anything else.
  LF_DEV void prefetch() {
    if (ahead.valid()) issue_copy(ahead.t, 0);
    ahead.next();
    if (ahead.valid()) issue_copy(ahead.t, 1);
    ahead.next();
  }

  // `state`: this head's [D*D + D] fp32 state.  The staging area (from kStageOffset) must be free.
  LF_DEV void run(const float* state, float eps) {
    load_state(state, eps, true);
    stream();
  }

  // Whole workgroup: stages one head's state in LDS; the waves with `keep` build their operands from it.
  LF_DEV void load_state(const float* state, float eps, bool keep) {
    // ---- prologue: state -> LDS, maxima, power-of-two scales, A fragments -------------------------
    float* st = reinterpret_cast<float*>(smem + Cfg::kStageOffset);
    float* redmax = st + NE;
    float mS = 0.0f, mz = 0.0f;
    for (int e = threadIdx.x; e < NE; e += kThreads) {
      float x = ld_agent(state + e);
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
    if (keep) {
      c1 = az / aS;
      eps_s = eps * az;
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
              unpack2<T>(pack2<T>(x, 0.0f), r0, r1);   // x rounded once to 16 bits
              hi2[q] = zrem ? x - r0 : x;
              lo2[q] = (slot < HALF) ? x - r0 : 0.0f;  // S' remainder -> lo fragment (bf16 only)
            }
            A[0][t][s][w] = pack2<T>(hi2[0], hi2[1]);
            if constexpr (NS == 2) A[1][t][s][w] = pack2<T>(lo2[0], lo2[1]);
          }
        }
      }
    }
    __syncthreads();   // the staged state is dead: the third slot block may be filled from here on
  }

  LF_DEV void stream() {
    int slot = 0;
    int iter = 0;
    while (it.valid()) {
      const long long tile = it.t;
      int aslot = slot + (R - 1);
      if (aslot >= R) aslot -= R;
      if (ahead.valid()) {
        issue_copy(ahead.t, aslot);
        // issue order is  C0 C1 | C2 W0 S0 | C3 W1 S1 | C4 W2 S2 | ...  (C copies, W wait, S stores, NL
        // instructions each): after tile j's copies come C(j+1), C(j+2) and the stores S(j-2), S(j-1)
        if (iter == 0) wait_vmcnt<2 * NL>();
        else if (iter == 1) wait_vmcnt<3 * NL>();
        else wait_vmcnt<4 * NL>();
      } else {
        wait_vmcnt<0>();
      }
      iter = iter < 2 ? iter + 1 : 2;
      unsigned char* sl = slot_ptr(slot);

      // ---- this lane's token row -> phi -> 16-bit B operands ----------------------------------------
      u32x4 Bh[KS], Bl[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int chunk = kg * KS + s;
        const bool ok = chunk < CPR;
        u32x4 raw = u32x4{0, 0, 0, 0};
        if (ok) raw = *reinterpret_cast<const u32x4*>(sl + row_byte + ((chunk ^ tsw) << 4));
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float x0, x1;
          unpack2<T>(raw[w], x0, x1);
          float r0 = ok ? phi<FM>(x0) : 0.0f;
          float r1 = ok ? phi<FM>(x1) : 0.0f;
          if constexpr (NS == 1) {
            Bh[s][w] = pack2<T>(r0, r1);
          } else {
            uint32_t h, l;
            pack2_split<T>(r0, r1, h, l);
            Bh[s][w] = h;
            Bl[s][w] = l;
          }
        }
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

      // ---- d/2 channels of this lane's token -> 16-bit -> back into the slot -------------------------
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      if constexpr (HALF % 8 == 0) {
#pragma unroll
        for (int c = 0; c < HALF / 8; ++c) {
          u32x4 w;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int s0 = c * 8 + 2 * e;
            w[e] = pack2<T>(acc[s0 / 16][s0 % 16] * scale, acc[(s0 + 1) / 16][(s0 + 1) % 16] * scale);
          }
          const int chunk = kg * (HALF / 8) + c;
          *reinterpret_cast<u32x4*>(sl + row_byte + ((chunk ^ tsw) << 4)) = w;
        }
      } else {
        static_assert(HALF % 8 == 0 || Cfg::kSwzMask == 0, "64-bit row pieces need an unswizzled row");
#pragma unroll
        for (int c = 0; c < HALF / 4; ++c) {
          u32x2 w;
#pragma unroll
          for (int e = 0; e < 2; ++e) {
            const int s0 = c * 4 + 2 * e;
            w[e] = pack2<T>(acc[s0 / 16][s0 % 16] * scale, acc[(s0 + 1) / 16][(s0 + 1) % 16] * scale);
          }
          *reinterpret_cast<u32x2*>(sl + row_byte + kg * (HALF * 2) + c * 8) = w;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");

      // ---- coalesced stores; always NL instructions (lanes without a valid chunk are masked) ------
      {
        long long rem = N - tile * kTile;
        const int lim = rem < kTile ? (int)rem : kTile;
        u32x4* op = Oh + tile * kTile * rs_o;
#pragma unroll
        for (int u = 0; u < NL; ++u) {
          const u32x4 w = *reinterpret_cast<const u32x4*>(sl + u * 1024 + lane * 16);
          if (u * 64 + lane < Cfg::kChunks && trow[u] < lim) {
            if constexpr (HG) op[ooff[u]] = w; else st_stream(op + ooff[u], w);
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      it.next();
      ahead.next();
      slot = slot + 1 == R ? 0 : slot + 1;
    }
  }
};

template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply16_dma(const u32x4* __restrict__ Q, Layout lq, u32x4* __restrict__ O, Layout lo,
            const float* __restrict__ state, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.y;
  ApplyDma<T, D, FM, NORM> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, tiles_per_block, blockIdx.x,
                              gridDim.x, smem);
  ap.prefetch();
  ap.run(state + bh * (D * D + D), eps);
}

// Apply with one head per wave.  grid = (wgs, B * ceil(H / 4)); same head assignment as state_reduce16_hg.
template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply16_dma_hg(const u32x4* __restrict__ Q, Layout lq, u32x4* __restrict__ O, Layout lo,
               const float* __restrict__ state, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int H = lq.H;
  const int gpb = (H + kWavesPerWG - 1) / kWavesPerWG;
  const int b = blockIdx.y / gpb;
  const int h0 = (blockIdx.y % gpb) * kWavesPerWG;
  const bool active = h0 + wave < H;
  const int h = active ? h0 + wave : H - 1;
  ApplyDma<T, D, FM, NORM, true> ap(Q + (b * lq.batch + h * lq.head), lq.row, O + (b * lo.batch + h * lo.head), lo.row,
                                    N, tiles_per_block, blockIdx.x, gridDim.x, smem, active);
  ap.prefetch();
  for (int w = 0; w < kWavesPerWG && h0 + w < H; ++w)
    ap.load_state(state + ((long long)b * H + h0 + w) * (D * D + D), eps, wave == w);
  ap.stream();
}

}  // namespace lf
