// Apply + normalize for head widths above 80 with one wave per tile (Eq. 5 applied to Prop. 2's state).
//
// The workgroup-shared apply of lf_wide16.hpp splits the output channels of every tile over the waves of a
// workgroup: all waves read the whole tile, so two workgroup barriers per tile separate "tile carries phi" ->
// "everyone holds its operands" -> "outputs are back", and with two workgroups per CU the barriers' bubbles
// bound the kernel well below the memory rate.  Here a wave keeps the WHOLE operand-ready state of its head in
// registers ((d + 2) x d 16-bit values: 220 registers at d = 160 fp16 -- one wave per SIMD, the 512-register file
// of a lone wave is what makes it fit) and streams tiles of its own through a ring of its own in LDS, exactly
// as the narrow per-head kernel does: copy in by LDS-DMA, phi in place, read the tile as matrix-core B operands,
// multiply, write the outputs over the tile, store.  No barrier anywhere; a wave waits only for its own copies.
//
// Products: v_mfma_f32_16x16x32 with A = S'^T row blocks (16 output channels, or the two normalizer rows, by 32
// contraction channels), B = phi(q) of 16 tokens.  Per tile and wave 2 token blocks x (d/16 + 1) row blocks x
// d/32 steps (110 at d = 160, 162 of 176 rows useful).  Lane l of a product: token l % 16, contraction channels
// 32 s + 8 (l / 16) .. + 7; afterwards it holds output channels 16 b + 4 (l / 16) .. + 3 of its token, four
// neighbours = one 8-byte piece of the output row.
//
// LDS: slot (ring position) of wave w at (slot * 4 + w) * kSlotBytes; a tile lies there row after row, the
// 16-byte chunks of row r swizzled (see ApplyWaveShape) so that token-per-lane accesses are bank-conflict free.
//
// The operands are fp16 for both storage types.  For bf16 tensors two levels of bf16 operands (hi + lo) would not
// fit the registers at d = 160 and would triple the products at every width, while fp16's 11 bits are what the
// fp16 path lives on and more than a bf16 output keeps.  What fp16 lacks is range, and that is given back per row:
// phi is applied when a lane reads its token's channels as B operands (no pass over the tile in place), and the
// row's largest channel m gives  phi~ = phi(q) 2^c / 2^e  with  2^c = exp(-m) for a row of negative channels under
// elu + 1 (1 otherwise) and 2^e the power of two at or below the row's largest phi 2^c.  Every row's largest operand
// then lies in [1, 2) -- a row at -300, at 1e30 or at 1e-20 alike -- and the factor cancels between numerator and
// denominator once eps carries it too.  fp16 tensors go the same way: a row far below zero (exp(q) subnormal or zero
// in fp16) or near the top of the range (phi = q + 1 above 65504) comes out as the definition gives it.
#pragma once
#include "lf_wide16.hpp"

namespace lf {

template <int D> struct ApplyWaveShape {
  static_assert(D % 32 == 0 && D > 64 && D <= 160, "one-wave-per-tile apply: head width a multiple of 32 in (64, 160]");
  static constexpr int kCPR = D / 8;                  // 16-byte chunks per token row
  static constexpr int kKS = D / 32;                  // contraction steps of 32 channels
  static constexpr int kCB = D / 16;                  // 16-row output blocks that hold channels
  static constexpr int kRB = kCB + 1;                 // ... and the block with the two normalizer rows
  static constexpr int kNL = kTile * kCPR / 64;       // 1 KiB deposits per tile (copies / stores per wave and tile)
  static constexpr int kSlotBytes = kNL * 1024;
  static constexpr int kWaves = 4;
  // Swizzle of the 16-byte chunks inside a token row: position p of row r holds chunk p ^ swz(r).  Token-per-lane
  // accesses to one chunk index then hit sixteen different groups of four banks (row starts are 16 r dwords apart
  // mod 64 where the row is not a multiple of 256 bytes: r % 4 picks the group of sixteen banks, (r / 4) % 4 the four
  // inside it; rows of 256 bytes all start at bank 0, so r % 16 picks), while every aligned group of four lanes of a
  // copy still reads one aligned 64-byte piece of memory (a rotation by single chunks would straddle two).
  static_assert(kCPR % 4 == 0, "four chunks per contraction step; the swizzle permutes inside aligned groups of four");
  static constexpr int kSwzMask = (kCPR % 16 == 0) ? 15 : 3;
  static constexpr int kSwzShift = (kCPR % 16 == 0) ? 0 : 2;
  static __device__ __forceinline__ int swz(int r) { return (r >> kSwzShift) & kSwzMask; }
};

// Ring slots per wave: the tile being worked on and two on their way.
constexpr int kApplyWaveRing = 3;
template <int D>
constexpr int apply16_wave_lds_bytes() { return ApplyWaveShape<D>::kWaves * kApplyWaveRing * ApplyWaveShape<D>::kSlotBytes; }

// The operand-ready state of one head for apply16_wave: {c1 = alpha_z / alpha_S, alpha_z} then frag[b][s][lane],
// 16 bytes each, fp16.  Lane l of fragment (b, s), element j:  output row m = 16 b + l % 16, contraction channel
// ch = 32 s + 8 (l / 16) + j;  m < d -> S'[ch][m] = alpha_S S[ch][m];  m == d -> z'[ch] = alpha_z z[ch] rounded to
// fp16;  m == d + 1 -> what that rounding left;  else 0.
template <int D> struct PackWave {
  using Sw = ApplyWaveShape<D>;
  static constexpr int kHeaderBytes = 256;
  static constexpr int kFrags = Sw::kRB * Sw::kKS;   // per lane
  static constexpr int kHeadBytes = kHeaderBytes + kFrags * 64 * 16;
};

// grid = (d / 32, heads), block = 256.  Every workgroup finds the maxima (power-of-two scales, as
// pack_state_wide); workgroup s writes the fragments of contraction step s, wave w those of row blocks w, w + 4, ..
template <int D>
__global__ void __launch_bounds__(kThreads)
pack_state_wave(const float* __restrict__ state, unsigned char* __restrict__ packed, int normalize) {
  using Sw = ApplyWaveShape<D>;
  constexpr int KS = Sw::kKS, RB = Sw::kRB, NE = D * D + D;
  __shared__ float redmax[2 * kWavesPerWG];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int s = blockIdx.x;
  const long long bh = blockIdx.y;
  const float* st = state + bh * NE;
  unsigned char* out = packed + bh * PackWave<D>::kHeadBytes;

  // this wave's row blocks b = wave, wave + 4, ..: their raw values are requested before the maxima are known, so that
  // the kernel waits for memory once
  constexpr int NB = (RB + kWavesPerWG - 1) / kWavesPerWG;
  const int g = lane >> 4;
  float raw[NB][8];
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int b = wave + kWavesPerWG * i;
    const int m = 16 * b + (lane & 15);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int ch = 32 * s + 8 * g + j;
      int at = ch * D;                                  // (rows past d + 1 and blocks past the end: a valid place, unused)
      if (m < D) at = ch * D + m;
      else if (m <= D + 1) at = D * D + ch;
      raw[i][j] = st[at];
    }
  }
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

  u32x4* frag = reinterpret_cast<u32x4*>(out + PackWave<D>::kHeaderBytes);
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    const int b = wave + kWavesPerWG * i;
    if (b < RB) {
      const int m = 16 * b + (lane & 15);
      u32x4 w4;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float v2[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          float x = 0.0f;
          bool zrem = false;
          if (m < D) x = raw[i][2 * w + q] * aS;
          else if (normalize && m == D) x = raw[i][2 * w + q] * az;
          else if (normalize && m == D + 1) { x = raw[i][2 * w + q] * az; zrem = true; }
          float r0, r1;
          unpack2<F16>(pack2<F16>(x, 0.0f), r0, r1);   // x rounded once to fp16
          v2[q] = zrem ? x - r0 : x;
        }
        w4[w] = pack2<F16>(v2[0], v2[1]);
      }
      frag[(b * KS + s) * 64 + lane] = w4;
    }
  }
}

// One wave's apply work on one head: construct, prefetch(), load_packed(), stream().  T: the tensors' storage type.
template <typename T, int D, int FM, bool NORM>
struct ApplyWave {
  using Sw = ApplyWaveShape<D>;
  using TA = F16;   // the operands' type
  static constexpr int CPR = Sw::kCPR, KS = Sw::kKS, RB = Sw::kRB, CB = Sw::kCB, NL = Sw::kNL;
  static constexpr int R = kApplyWaveRing;
  static constexpr int W = Sw::kWaves;
  static_assert(R == 3, "the wait counts below are written for a ring of three slots");
  static_assert(4 * NL <= 63, "the vector-memory counter has six bits");

  const u32x4* Qh;
  u32x4* Oh;
  long long N;
  unsigned char* smem;
  int rs_q, rs_o;
  int lane, wave, g;
  int trow[NL], qoff[NL], ooff[NL], soff[NL];
  int rowb[2], x0[2];        // per token block: byte offset of this lane's token row in a slot, its swizzle
  TileIter it, ahead;
  u32x4 A[RB][KS];
  float c1, eps_s;

  LF_DEV ApplyWave(const u32x4* Qh_, int rs_q_, u32x4* Oh_, int rs_o_, long long N_, int tiles_per_block, int wg,
                   int nwg, unsigned char* smem_)
      : Qh(Qh_), Oh(Oh_), N(N_), smem(smem_), rs_q(rs_q_), rs_o(rs_o_),
        lane(threadIdx.x & 63), wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)),
        it(wg, nwg, wave, tiles_per_block, (N_ + kTile - 1) / kTile, W), ahead(it) {
    g = lane >> 4;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int P = u * 64 + lane;             // position in the tile
      const int r = P / CPR, pos = P % CPR;
      const int c = pos ^ Sw::swz(r);          // copy side: position pos of row r receives chunk c
      const int spos = pos ^ Sw::swz(r);       // store side: this lane sends chunk pos, found at spos
      trow[u] = r;
      qoff[u] = r * rs_q + c;
      ooff[u] = r * rs_o + pos;
      soff[u] = (r * CPR + spos) * 16;
    }
#pragma unroll
    for (int tb = 0; tb < 2; ++tb) {
      const int r = 16 * tb + (lane & 15);
      rowb[tb] = r * CPR * 16;
      x0[tb] = Sw::swz(r);
    }
  }

  LF_DEV unsigned char* slot_ptr(int slot) const { return smem + (slot * W + wave) * Sw::kSlotBytes; }
  // where chunk `chunk` of this lane's token of block tb lies inside a slot
  LF_DEV int chunk_off(int tb, int chunk) const {
    return rowb[tb] + ((chunk ^ x0[tb]) << 4);
  }

  // always issues exactly NL vector memory instructions
  LF_DEV void issue_copy(long long tile, int slot) {
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    const u32x4* qp = Qh + tile * kTile * rs_q;
    unsigned char* sl = slot_ptr(slot);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int c = trow[u] < lim ? qoff[u] : 0;   // rows past N re-read chunk 0; never stored
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(qp + c),
                                       (LF_LDS void*)(sl + u * 1024), 16, 0, 2 /* nt */);
    }
  }

  LF_DEV void prefetch() {
#pragma unroll
    for (int i = 0; i < R - 1; ++i) {
      if (ahead.valid()) issue_copy(ahead.t, i);
      ahead.next();
    }
  }

  // `packed`: this head's operands as pack_state_wave wrote them
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

  // the finished tile in `slot` goes out; always NL vector memory instructions for a full tile (only the very
  // last tile of a head can be ragged, and nothing is counted after it)
  LF_DEV void store_tile(long long tile, int slot) {
    const unsigned char* sl = slot_ptr(slot);
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    u32x4* op = Oh + tile * kTile * rs_o;
    u32x4 w[NL];
#pragma unroll
    for (int u = 0; u < NL; ++u) w[u] = *reinterpret_cast<const u32x4*>(sl + soff[u]);
    if (lim == kTile) {   // (a branch per store would pull each read behind it, one LDS round trip each)
#pragma unroll
      for (int u = 0; u < NL; ++u) st_stream(op + ooff[u], w[u]);
    } else {
#pragma unroll
      for (int u = 0; u < NL; ++u)
        if (trow[u] < lim) st_stream(op + ooff[u], w[u]);
    }
  }

  // at most k * NL vector memory instructions outstanding
  LF_DEV void wait_groups(int k) {
    switch (k) {
      case 0: wait_vmcnt<0>(); break;
      case 1: wait_vmcnt<NL>(); break;
      case 2: wait_vmcnt<2 * NL>(); break;
      case 3: wait_vmcnt<3 * NL>(); break;
      default: wait_vmcnt<4 * NL>(); break;
    }
  }

  // this lane's 8 KS stored channels of its token of block tb of the tile at `sl`
  LF_DEV void read_block(const unsigned char* sl, int tb, u32x4 (&B)[KS]) {
#pragma unroll
    for (int s = 0; s < KS; ++s) B[s] = *reinterpret_cast<const u32x4*>(sl + chunk_off(tb, 4 * s + g));
  }

  // `B`: this lane's 8 KS stored channels of its token (lanes l, l + 16, l + 32, l + 48 hold one token between them)
  // -> the fp16 operands phi~ = phi(q) 2^c 2^-e, where 2^c = exp(-m) if the row's largest channel m is negative
  // under elu + 1 (else 1) and 2^e is the power of two at or below the row's largest phi 2^c, so the row's largest
  // operand lies in [1, 2) whatever the inputs' magnitude.  eps_tok = eps' 2^c 2^-e is what eps becomes in that
  // row's units (the factor cancels in Eq. 5's ratio), post = its inverse for the un-normalized form.  A row without
  // a positive phi (relu of non-positive channels) keeps operands 0 and gives 0, as the definition does; a NaN stays
  // in its own token's outputs (the row maximum skips it).
  LF_DEV void make_operands(u32x4 (&B)[KS], float& eps_tok, float& post) {
    constexpr float kLog2e = 1.44269504088896340736f;
    // (the channels are unpacked twice, for the maximum and for phi, rather than kept: 8 KS more live registers
    //  would not fit beside the head's operands at d = 160)
    float m = -__builtin_inff();
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float a, b;
        unpack2<T>(B[s][w], a, b);
        m = fmaxf(m, fmaxf(FM == kPhiIdentity ? fabsf(a) : a, FM == kPhiIdentity ? fabsf(b) : b));
      }
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
    float c = 0.0f, top;   // top: the row's largest |phi 2^c|
    if constexpr (FM == kPhiEluPlusOne) {
      c = m < 0.0f ? fminf(-m * kLog2e, 3.0e38f) : 0.0f;   // (finite: a row of -inf gives phi = 0, not inf - inf)
      top = m < 0.0f ? 1.0f : m + 1.0f;
    } else if constexpr (FM == kPhiRelu) {
      top = fmaxf(m, 0.0f);
    } else {
      top = m;
    }
    // 2^-e from top's exponent field f: (254 - f) as the field of the factor; f is kept inside [1, 253] so that the
    // factor is a normal number (top = 0: the operands are 0 whatever it is)
    uint32_t f = (__builtin_bit_cast(uint32_t, top) >> 23) & 0xffu;
    f = f < 1u ? 1u : (f > 253u ? 253u : f);
    const float mult = __builtin_bit_cast(float, (254u - f) << 23);
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float a, b;
        unpack2<T>(B[s][w], a, b);
        B[s][w] = pack2<TA>(phi_scaled<FM>(a, c) * mult, phi_scaled<FM>(b, c) * mult);
      }
    // eps' 2^c 2^-e in two finite factors (2^c alone leaves fp32's range from m = -88.7 on; the clamp only keeps
    // 0 * 2^c = 0 for eps = 0: beyond it the product is infinite anyway and the row's outputs are 0, as their true
    // size, below e^-131 / eps of the values', rounds to)
    eps_tok = __builtin_amdgcn_exp2f(fminf(c, 190.0f) - 64.0f) * (eps_s * mult * 0x1p64f);
    post = __builtin_amdgcn_exp2f(-c) * __builtin_bit_cast(float, f << 23);   // 2^-c 2^e
  }

  // multiply one block of 16 tokens and write its outputs over its rows of the tile at `sl`; `eps_tok`: eps in the
  // units of this lane's token's denominator, `post`: the row's scale taken out of its un-normalized outputs
  LF_DEV void multiply_block(unsigned char* sl, int tb, const u32x4 (&B)[KS], float eps_tok, float post) {
    f32x4 acc[RB];
#pragma unroll
    for (int b = 0; b < RB; ++b) acc[b] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
#pragma unroll
      for (int b = 0; b < RB; ++b) acc[b] = mfma_16x16x32<TA>(A[b][s], B[s], acc[b]);
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
      *reinterpret_cast<u32x2*>(sl + chunk_off(tb, 2 * b + (g >> 1)) + 8 * (g & 1)) = w;
    }
  }

  // The tile in `slot` (as stored) -> its outputs, in place.  All LDS reads are issued before the first use: a lone
  // wave per SIMD has nobody to hide an LDS round trip per contraction step behind.
  LF_DEV void compute_tile(int slot) {
    unsigned char* sl = slot_ptr(slot);
    u32x4 B0[KS], B1[KS];
    read_block(sl, 0, B0);
    read_block(sl, 1, B1);   // block 0's outputs land in other rows
    __builtin_amdgcn_sched_barrier(0);
    float eps_tok, post;
    make_operands(B0, eps_tok, post);
    multiply_block(sl, 0, B0, eps_tok, post);
    make_operands(B1, eps_tok, post);
    multiply_block(sl, 1, B1, eps_tok, post);
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
      wait_groups((j >= 2 ? 2 : j) + (next_copied ? 1 : 0) + (copied ? 1 : 0));
      compute_tile(slot);
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

// grid = (wgs, heads), block = 256 (four waves that share nothing but the workgroup); `packed` from pack_state_wave<D>
template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply16_wave(const u32x4* __restrict__ Q, Layout lq, u32x4* __restrict__ O, Layout lo, HeadSubset hs,
             const unsigned char* __restrict__ packed, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = hs.bh(blockIdx.y, lq.H);
  ApplyWave<T, D, FM, NORM> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, tiles_per_block, blockIdx.x,
                               gridDim.x, smem);
  ap.prefetch();
  ap.load_packed(packed + bh * PackWave<D>::kHeadBytes, eps);
  ap.stream();
}

}  // namespace lf
