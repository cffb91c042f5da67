// Row-piece forms of the two apply-shaped kernels of the backward pass (lf_backward16.hpp), for layouts in which
// the heads of a token are neighbours in memory (token-major [B, N, H*d]) and a head's row is no whole cache line:
// a workgroup of W waves takes a group of W heads, moves every tile as whole row pieces of W*d elements (both
// tensors, in and out) through a workgroup-wide LDS-DMA ring, and wave w computes head w exactly as the per-head
// kernel does -- same products, same operands.  bwd_kv16_rows (dK, dV) and bwd_q16_rows (dQ, per-token scalars)
// give the per-head kernels' bits; bwd_qs16_rows (dQ and the state gradient, fp16) sums a head's partial in one
// wave instead of four.  The ring, its
// rotation against bank conflicts and the pipeline with one workgroup barrier per tile are those of ApplyDma's
// row-piece mode (lf_apply16_dma.hpp), with two tensors per slot.
#pragma once
#include "lf_backward16.hpp"

namespace lf {

template <int D, int W> struct BwdRowsCfg {
  using Sh = Shape16<D>;
  static constexpr int kCPR = Sh::kChunksPerRow;
  static constexpr int kPC = W * kCPR;                          // chunks per row piece
  static constexpr int kRPR = kTile / W;                        // token rows per wave region
  static constexpr int kRegionChunks = kRPR * kPC;
  static constexpr int kNL = (kRegionChunks + 63) / 64;         // copies / stores per wave, tile and tensor
  static constexpr int kRegionBytes = kNL * 1024;
  static constexpr int kTileBytes = W * kRegionBytes;           // one tensor's tile
  static constexpr int kSlotBytes = 2 * kTileBytes;
  static constexpr int kRing = 3;
  static constexpr int kStageOffset = (kRing - 1) * kSlotBytes; // third slot: free before the stream loop
  static constexpr int kStageBytes = (D * D + D) * 4 + 64;
  static constexpr int kG = (kPC % 16 == 0) ? 16 : ((kPC % 8 == 0) ? 8 : 4);
  static_assert(kTile % W == 0 && kPC % 4 == 0 && kRPR * kG >= 16, "rotation classes must fit a region");
  static_assert(kRegionChunks % 32 == 0, "a region is whole half-waves of chunks");
  static_assert(kStageBytes <= kSlotBytes, "the state is staged in the third slot");
  // every wave its own head's state at once (behind the first slot, before the second tile is requested), where W
  // states fit the second and third slot; else one head after the other through the third slot
  static constexpr int kOwnBytes = (kStageBytes + 255) / 256 * 256;
  static constexpr bool kOwnStage = W * kOwnBytes <= 2 * kSlotBytes;
  static constexpr int kMTB = (Sh::kHalf + 15) / 16;
  static constexpr int lds_bytes() { return kRing * kSlotBytes; }
  static __device__ __forceinline__ int rot(int r) { return ((r * kG) >> 4) & (kG - 1); }
};

template <typename T, int D, int W>
struct Ring2Rows {
  using Sh = Shape16<D>;
  using C = BwdRowsCfg<D, W>;
  static constexpr int NS = NSplit<T>::value;
  static constexpr int KS = Sh::kKS, CPR = C::kCPR, PC = C::kPC, RPR = C::kRPR, HALF = Sh::kHalf, MTB = C::kMTB;
  static constexpr int NL = C::kNL, NE = D * D + D, R = C::kRing, TB = C::kTileBytes;
  static_assert(R == 3, "the wait counts are written for a ring of three slots");

  const u32x4 *Xh, *Yh;   // first token row of the group's row piece in the two tensors
  int rsx, rsy;           // token strides, 16-byte units
  long long N;
  unsigned char* smem;
  int lane, wave, tok, kg, row_byte, tsw;
  int trow[NL], xoff[NL], yoff[NL];     // copy side: token row and offsets of the chunk this lane brings
  int trow_o[NL], ooff[NL], soff[NL];   // store side: token row, chunk inside the row piece, byte in the region
  TileIter it, ahead;
  const float* stage;                    // where the state this wave builds its operands from is staged

  LF_DEV Ring2Rows(const u32x4* Xh_, int rsx_, const u32x4* Yh_, int rsy_, long long N_, int tiles_per_block, int wg,
                   int nwg, unsigned char* smem_)
      : Xh(Xh_), Yh(Yh_), rsx(rsx_), rsy(rsy_), N(N_), smem(smem_), lane(threadIdx.x & 63),
        wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)),
        it(wg, nwg, 0, tiles_per_block, (N_ + kTile - 1) / kTile, 1), ahead(it),
        stage(reinterpret_cast<const float*>(smem_ + C::kStageOffset)) {
    tok = lane & 31;
    kg = lane >> 5;
    row_byte = (tok / RPR) * C::kRegionBytes + (tok % RPR) * PC * 16;
    tsw = wave * CPR + C::rot(tok);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int P = wave * C::kRegionChunks + u * 64 + lane;   // position in the tile of row pieces
      // lanes past the region's chunks copy what the lane 32 below copies and deposit it in the padding
      const int Pc = (u * 64 + lane < C::kRegionChunks) ? P : P - 32;
      const int rc = Pc / PC;
      int cc = Pc % PC - C::rot(rc);
      if (cc < 0) cc += PC;
      trow[u] = rc;
      xoff[u] = rc * rsx + cc;
      yoff[u] = rc * rsy + cc;
      const int r = P / PC, cs = P % PC;   // store side: this lane sends chunk cs of row r ...
      int pos = cs + C::rot(r);            // ... which sits at this rotated position of the row piece
      if (pos >= PC) pos -= PC;
      trow_o[u] = r;
      ooff[u] = cs;
      soff[u] = ((r % RPR) * PC + pos) * 16;
    }
  }

  LF_DEV unsigned char* tile_ptr(int slot, int which) const { return smem + slot * C::kSlotBytes + which * TB; }
  // where this lane finds (and overwrites) chunk `chunk` of its token's row of this wave's head
  LF_DEV unsigned char* chunk_ptr(int slot, int which, int chunk) const {
    int x = tsw + chunk;
    if (x >= PC) x -= PC;
    return tile_ptr(slot, which) + row_byte + (x << 4);
  }
  LF_DEV unsigned char* byte_ptr(int slot, int which, int byte) const {
    return chunk_ptr(slot, which, byte >> 4) + (byte & 15);
  }
  // address of the four 16-bit elements (row, col .. col + 3) of this wave's head in tile part `which`, col a
  // multiple of 4: what one lane names in a transposing LDS read
  LF_DEV const uint16_t* tr_ptr(int slot, int which, int row, int col) const {
    int x = wave * CPR + C::rot(row) + (col >> 3);
    if (x >= PC) x -= PC;
    return reinterpret_cast<const uint16_t*>(tile_ptr(slot, which) + (row / RPR) * C::kRegionBytes +
                                             (row % RPR) * PC * 16 + (x << 4) + (col & 7) * 2);
  }

  // this wave's rows of tile `tile` of both tensors into ring slot `slot`: always 2 NL vector memory instructions,
  // issued by every lane as straight-line code (see ApplyDma::issue_copy)
  LF_DEV void issue_copy(long long tile, int slot) {
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
      const u32x4* gp = which ? Yh + tile * kTile * rsy : Xh + tile * kTile * rsx;
      unsigned char* sl = tile_ptr(slot, which) + wave * C::kRegionBytes;
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        const int c = trow[u] < lim ? (which ? yoff[u] : xoff[u]) : 0;   // rows past N re-read chunk 0; never stored
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gp + c),
                                         (LF_LDS void*)(sl + u * 1024), 16, 0, 2 /* nt */);
      }
    }
  }
  // the first two tiles; in two steps where the states are staged behind the first slot (kOwnStage)
  LF_DEV void prefetch_first() {
    if (ahead.valid()) issue_copy(ahead.t, 0);
    ahead.next();
  }
  LF_DEV void prefetch_second() {
    if (ahead.valid()) issue_copy(ahead.t, 1);
    ahead.next();
  }
  // This wave alone: stages its head's fp32 state in its own piece of LDS (kOwnStage) and returns the power-of-two
  // scale for the matrix.  A workgroup barrier must follow before prefetch_second().
  LF_DEV float stage_state_own(const float* state) {
    float* st = reinterpret_cast<float*>(smem + C::kSlotBytes + wave * C::kOwnBytes);
    float mS = 0.0f;
    for (int e = lane; e < NE / 4; e += 64) {
      const f32x4 x = reinterpret_cast<const f32x4*>(state)[e];
      reinterpret_cast<f32x4*>(st)[e] = x;
      if (e < D * D / 4) mS = fmaxf(mS, fmaxf(fmaxf(fabsf(x[0]), fabsf(x[1])), fmaxf(fabsf(x[2]), fabsf(x[3]))));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mS = fmaxf(mS, __shfl_xor(mS, o));
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the wave's LDS writes before its reads of them
    stage = st;
    return pow2_scale_for(mS);
  }
  // this wave's rows of tile part `which` of slot `slot`, in memory order, to the group's row pieces of `Oh`
  LF_DEV void store_tile(long long tile, int slot, int which, u32x4* Oh, int rso) {
    const unsigned char* sl = tile_ptr(slot, which) + wave * C::kRegionBytes;
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    u32x4* op = Oh + tile * kTile * rso;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(sl + soff[u]);
      if (u * 64 + lane < C::kRegionChunks && trow_o[u] < lim) st_stream(op + trow_o[u] * rso + ooff[u], w);
    }
  }

  // Whole workgroup: stages one head's fp32 state ([D*D] matrix then [D] vector) in the third slot and returns
  // the power-of-two scale for the matrix.
  LF_DEV float stage_state(const float* state) {
    float* st = reinterpret_cast<float*>(smem + C::kStageOffset);
    float* redmax = st + NE;
    float mS = 0.0f;
    for (int e = threadIdx.x; e < NE / 4; e += 64 * W) {
      const f32x4 x = reinterpret_cast<const f32x4*>(state)[e];
      reinterpret_cast<f32x4*>(st)[e] = x;
      if (e < D * D / 4) mS = fmaxf(mS, fmaxf(fmaxf(fabsf(x[0]), fabsf(x[1])), fmaxf(fabsf(x[2]), fabsf(x[3]))));
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mS = fmaxf(mS, __shfl_xor(mS, o));
    if (lane == 0) redmax[wave] = mS;
    __syncthreads();
    mS = 0.0f;
#pragma unroll
    for (int w = 0; w < W; ++w) mS = fmaxf(mS, redmax[w]);
    return pow2_scale_for(mS);
  }
  // A operands of the staged matrix (see Ring2::build_A)
  template <bool TRANSPOSED>
  LF_DEV void build_A(float aS, u32x4 (&A)[NS][MTB][KS]) const {
    const float* st = stage;
    const int m = lane & 31;
    const int hv = (m >> 2) & 1;
#pragma unroll
    for (int t = 0; t < MTB; ++t) {
      const int slot = 16 * t + 4 * (m >> 3) + (m & 3);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int chunk = kg * KS + s;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float hi2[2], lo2[2];
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            const int c = chunk * 8 + 2 * w + q;
            const int o = hv * HALF + slot;
            float x = 0.0f;
            if (chunk < CPR && slot < HALF) x = (TRANSPOSED ? st[c * D + o] : st[o * D + c]) * aS;
            float r0, r1;
            unpack2<T>(pack2<T>(x, 0.0f), r0, r1);
            hi2[q] = x;
            lo2[q] = x - r0;
          }
          A[0][t][s][w] = pack2<T>(hi2[0], hi2[1]);
          if constexpr (NS == 2) A[1][t][s][w] = pack2<T>(lo2[0], lo2[1]);
        }
      }
    }
  }
  LF_DEV void load_vec(float (&v)[HALF]) const {
    const float* st = stage + D * D;
#pragma unroll
    for (int i = 0; i < HALF; ++i) v[i] = st[kg * HALF + i];
  }
  LF_DEV void read_half_row(int slot, int which, float (&x)[HALF]) const {
    constexpr int PB = (HALF % 8 == 0) ? 16 : 8;
#pragma unroll
    for (int c = 0; c < HALF * 2 / PB; ++c) {
      const unsigned char* p = byte_ptr(slot, which, kg * HALF * 2 + c * PB);
      uint32_t w[PB / 4];
      if constexpr (PB == 16) {
        const u32x4 t = *reinterpret_cast<const u32x4*>(p);
        w[0] = t[0]; w[1] = t[1]; w[2] = t[2]; w[3] = t[3];
      } else {
        const u32x2 t = *reinterpret_cast<const u32x2*>(p);
        w[0] = t[0]; w[1] = t[1];
      }
#pragma unroll
      for (int e = 0; e < PB / 4; ++e) unpack2<T>(w[e], x[c * (PB / 2) + 2 * e], x[c * (PB / 2) + 2 * e + 1]);
    }
  }
  LF_DEV void write_half_row(int slot, int which, const float (&x)[HALF]) const {
    constexpr int PB = (HALF % 8 == 0) ? 16 : 8;
#pragma unroll
    for (int c = 0; c < HALF * 2 / PB; ++c) {
      unsigned char* p = byte_ptr(slot, which, kg * HALF * 2 + c * PB);
      uint32_t w[PB / 4];
#pragma unroll
      for (int e = 0; e < PB / 4; ++e) w[e] = pack2<T>(x[c * (PB / 2) + 2 * e], x[c * (PB / 2) + 2 * e + 1]);
      if constexpr (PB == 16) *reinterpret_cast<u32x4*>(p) = u32x4{w[0], w[1], w[2], w[3]};
      else *reinterpret_cast<u32x2*>(p) = u32x2{w[0], w[1]};
    }
  }
  LF_DEV void read_B_raw(int slot, int which, u32x4 (&B)[KS]) const {
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int chunk = kg * KS + s;
      B[s] = u32x4{0, 0, 0, 0};
      if (chunk < CPR) B[s] = *reinterpret_cast<const u32x4*>(chunk_ptr(slot, which, chunk));
    }
  }
  LF_DEV void products(const u32x4 (&A)[NS][MTB][KS], const u32x4 (&Bh)[KS], const u32x4* Bl, f32x16 (&acc)[MTB]) const {
#pragma unroll
    for (int t = 0; t < MTB; ++t) {
      acc[t] = f32x16{0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        acc[t] = mfma_32x32x16<T>(A[0][t][s], Bh[s], acc[t]);
        if constexpr (NS == 2) {
          acc[t] = mfma_32x32x16<T>(A[1][t][s], Bh[s], acc[t]);
          if (Bl) acc[t] = mfma_32x32x16<T>(A[0][t][s], Bl[s], acc[t]);
        }
      }
    }
  }
};

// ==========================================================================================
// bwd_kv16_rows: dK and dV of a group of W neighbouring heads.  grid = (wgs, B * gpb), block = 64 W: workgroup
// (x, y) takes heads W (y % gpb) .. + W - 1 of batch y / gpb.  `kv`, `dkv`: layouts of k / v and dk / dv (heads
// neighbours: head stride = d); `dstate`: [B*H][D*D + D].
// Per iteration j: store tile j-1 (finished since the last barrier), copy tile j+2 into the slot that frees, compute
// tile j in place, wait for this wave's rows of tile j+1, barrier.
// ==========================================================================================
template <typename T, int D, int FM, int W>
__global__ void __launch_bounds__(64 * W)
bwd_kv16_rows(const u32x4* __restrict__ K, const u32x4* __restrict__ V, Layout lkv, u32x4* __restrict__ dK,
              u32x4* __restrict__ dV, Layout ldkv, int gpb, const float* __restrict__ dstate, long long N,
              int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using RG = Ring2Rows<T, D, W>;
  constexpr int NS = RG::NS, KS = RG::KS, MTB = RG::MTB, HALF = RG::HALF, NL = RG::NL, R = RG::R, CPR = RG::CPR;
  const long long b = blockIdx.y / gpb;
  const long long h0 = (long long)(blockIdx.y % gpb) * W;
  const long long in_off = b * lkv.batch + h0 * lkv.head, out_off = b * ldkv.batch + h0 * ldkv.head;
  RG rg(K + in_off, lkv.row, V + in_off, lkv.row, N, tiles_per_block, blockIdx.x, gridDim.x, smem);
  u32x4* dKg = dK + out_off;
  u32x4* dVg = dV + out_off;
  rg.prefetch_first();

  // every wave its own head's operands
  u32x4 A1[NS][MTB][KS], A2[NS][MTB][KS];
  float dzo[HALF];
  float inv_aS = 1.0f;
  if constexpr (BwdRowsCfg<D, W>::kOwnStage) {
    const float aS = rg.stage_state_own(dstate + (b * lkv.H + h0 + rg.wave) * (D * D + D));
    rg.template build_A<true>(aS, A1);    // dv = dS^T p
    rg.template build_A<false>(aS, A2);   // dp = dS v (+ dz)
    rg.load_vec(dzo);
    inv_aS = 1.0f / aS;
    __syncthreads();   // the staged states are dead: the second slot may be filled
    rg.prefetch_second();
  } else {
    rg.prefetch_second();
    for (int h = 0; h < W; ++h) {   // the heads' states pass through the third slot one after the other
      const float aS = rg.stage_state(dstate + (b * lkv.H + h0 + h) * (D * D + D));
      if (rg.wave == h) {
        rg.template build_A<true>(aS, A1);
        rg.template build_A<false>(aS, A2);
        rg.load_vec(dzo);
        inv_aS = 1.0f / aS;
      }
      __syncthreads();
    }
  }

  {   // this wave's rows of the first tile: only the second tile's copies were issued after them
    TileIter second = rg.it;
    second.next();
    if (second.valid()) wait_vmcnt<2 * NL>();
    else wait_vmcnt<0>();
  }
  lds_barrier();
  int slot = 0, prev_slot = 0;
  long long prev_tile = -1;
  while (rg.it.valid()) {
    const long long tile = rg.it.t;
    const bool have_prev = prev_tile >= 0;
    if (have_prev) {
      rg.store_tile(prev_tile, prev_slot, 0, dKg, ldkv.row);
      rg.store_tile(prev_tile, prev_slot, 1, dVg, ldkv.row);
    }
    const bool copied = rg.ahead.valid();
    if (copied) rg.issue_copy(rg.ahead.t, have_prev ? prev_slot : R - 1);

    // phi(k) of this lane's input chunks -> B operands (hi [, lo]); v raw
    u32x4 Bp[KS], Bpl[NS == 2 ? KS : 1], Bv[KS];
    rg.read_B_raw(slot, 0, Bp);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const bool ok = rg.kg * KS + s < CPR;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float x0, x1;
        unpack2<T>(Bp[s][w], x0, x1);
        const float r0 = ok ? phi<FM>(x0) : 0.0f, r1 = ok ? phi<FM>(x1) : 0.0f;
        if constexpr (NS == 1) {
          Bp[s][w] = pack2<T>(r0, r1);
        } else {
          uint32_t hh, ll;
          pack2_split<T>(r0, r1, hh, ll);
          Bp[s][w] = hh;
          Bpl[s][w] = ll;
        }
      }
    }
    rg.read_B_raw(slot, 1, Bv);
    f32x16 acc1[MTB], acc2[MTB];
    rg.products(A1, Bp, NS == 2 ? Bpl : nullptr, acc1);
    rg.products(A2, Bv, nullptr, acc2);
    float x[HALF], o[HALF];
    rg.read_half_row(slot, 0, x);             // k at this lane's output channels
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const float pk = phi<FM>(x[i]);
      x[i] = (acc2[i / 16][i % 16] * inv_aS + dzo[i]) * phi_prime_from<FM>(x[i], pk);   // dk
      o[i] = acc1[i / 16][i % 16] * inv_aS;                                              // dv
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // both half-waves have read the row before it changes
    rg.write_half_row(slot, 0, x);
    rg.write_half_row(slot, 1, o);

    rg.it.next();
    rg.ahead.next();
    if (rg.it.valid()) {
      // after the copies of tile j+1 came the stores of tile j-1 and the copies of tile j+2, where they exist
      if (have_prev && copied) wait_vmcnt<4 * NL>();
      else if (have_prev || copied) wait_vmcnt<2 * NL>();
      else wait_vmcnt<0>();
    }
    lds_barrier();   // tile j is finished by all waves; tile j+1 has landed for all
    prev_tile = tile;
    prev_slot = slot;
    slot = slot + 1 == R ? 0 : slot + 1;
  }
  if (prev_tile >= 0) {
    rg.store_tile(prev_tile, prev_slot, 0, dKg, ldkv.row);
    rg.store_tile(prev_tile, prev_slot, 1, dVg, ldkv.row);
  }
}

// ==========================================================================================
// bwd_qs16_rows (fp16): bwd_qs16 on a group of W neighbouring heads -- dQ, and the group's share of the state
// gradient.  grid = (wgs, B * gpb), block = 64 W.  Wave w works on head w of the group for every token of the
// workgroup's tiles, so its accumulators are that head's whole partial: written (divided by beta) without a sum
// across waves, as [B*H][gridDim.x][D*D + D] for combine_state.  (The order in which tiles enter a partial differs
// from the per-head kernel's, so dS, dz and what follows from them -- dK, dV -- agree with it up to fp32 summation
// order, not bit for bit; dQ does not depend on them.)  LDS: BwdRowsCfg<D, W>::lds_bytes() + 64 W.
// ==========================================================================================
template <typename T, int D, int FM, bool NORM, int W>
__global__ void __launch_bounds__(64 * W)
bwd_qs16_rows(const u32x4* __restrict__ Q, Layout lq, const u32x4* __restrict__ G, Layout lg, u32x4* __restrict__ dQ,
              Layout ldq, int gpb, const float* __restrict__ state, float* __restrict__ partials, float eps,
              long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using RG = Ring2Rows<T, D, W>;
  using Sh = Shape16<D>;
  using C = BwdRowsCfg<D, W>;
  static_assert(NSplit<T>::value == 1, "single-level operands only (fp16)");
  constexpr int NS = 1, KS = RG::KS, MTB = RG::MTB, HALF = RG::HALF, NL = RG::NL, R = RG::R, CPR = RG::CPR;
  constexpr int MT = Sh::kMT, NE = D * D + D;
  const long long b = blockIdx.y / gpb;
  const long long h0 = (long long)(blockIdx.y % gpb) * W;
  RG rg(Q + (b * lq.batch + h0 * lq.head), lq.row, G + (b * lg.batch + h0 * lg.head), lg.row, N, tiles_per_block,
        blockIdx.x, gridDim.x, smem);
  u32x4* dQg = dQ + (b * ldq.batch + h0 * ldq.head);
  uint16_t* ecol = reinterpret_cast<uint16_t*>(smem + C::lds_bytes()) + rg.wave * 32;
  rg.prefetch_first();

  // every wave its own head's operands
  u32x4 A[NS][MTB][KS];
  float zo[HALF];
  float inv_aS = 1.0f, beta = 1.0f, inv_beta = 1.0f;
  auto build = [&](float aS) {
    rg.template build_A<false>(aS, A);
    rg.load_vec(zo);
    inv_aS = 1.0f / aS;
    if constexpr (NORM) {   // power of two near the typical denominator (see bwd_state16)
      const float* z = rg.stage + D * D;
      float zs = 0.0f;
      for (int i = 0; i < D; ++i) zs += z[i];
      if (zs > 0.0f && zs < 3.0e38f) {
        int ex;
        (void)__builtin_frexpf(zs, &ex);
        ex = ex > 100 ? 100 : (ex < -100 ? -100 : ex);
        beta = __builtin_ldexpf(1.0f, ex);
        inv_beta = __builtin_ldexpf(1.0f, -ex);
      }
    }
  };
  if constexpr (C::kOwnStage) {
    build(rg.stage_state_own(state + (b * lq.H + h0 + rg.wave) * NE));
    __syncthreads();   // the staged states are dead: the second slot may be filled
    rg.prefetch_second();
  } else {
    rg.prefetch_second();
    for (int h = 0; h < W; ++h) {   // the heads' states pass through the third slot one after the other
      const float aS = rg.stage_state(state + (b * lq.H + h0 + h) * NE);
      if (rg.wave == h) build(aS);
      __syncthreads();
    }
  }

  f32x4 accS[MT][MT], accZ[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    accZ[a] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int bb = 0; bb < MT; ++bb) accS[a][bb] = f32x4{0, 0, 0, 0};
  }
  const int j16 = rg.lane & 15, g4 = rg.lane >> 4;
  const int tr_row = 8 * g4 + (j16 >> 2), tr_col = 4 * (j16 & 3);

  {   // this wave's rows of the first tile: only the second tile's copies were issued after them
    TileIter second = rg.it;
    second.next();
    if (second.valid()) wait_vmcnt<2 * NL>();
    else wait_vmcnt<0>();
  }
  lds_barrier();
  int slot = 0, prev_slot = 0;
  long long prev_tile = -1;
  while (rg.it.valid()) {
    const long long tile = rg.it.t;
    const bool have_prev = prev_tile >= 0;
    if (have_prev) rg.store_tile(prev_tile, prev_slot, 0, dQg, ldq.row);
    const bool copied = rg.ahead.valid();
    if (copied) rg.issue_copy(rg.ahead.t, have_prev ? prev_slot : R - 1);
    long long rem = N - tile * kTile;
    const bool ok = rg.tok < (rem < kTile ? (int)rem : kTile);

    u32x4 Bg[KS];
    rg.read_B_raw(slot, 1, Bg);
    f32x16 acc[MTB];
    rg.products(A, Bg, nullptr, acc);
    float x[HALF], dr[HALF], rr[HALF];
    rg.read_half_row(slot, 0, x);
    float denp = 0.0f, rup = 0.0f;
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const float r = phi<FM>(x[i]);
      const float u = acc[i / 16][i % 16] * inv_aS;
      denp = __builtin_fmaf(r, zo[i], denp);
      rup = __builtin_fmaf(r, u, rup);
      dr[i] = u;
      rr[i] = ok ? r : 0.0f;
      x[i] = phi_prime_from<FM>(x[i], r);
    }
    float gsc = ok ? 1.0f : 0.0f, e = 0.0f;
    if constexpr (NORM) {
      const float den = denp + __shfl_xor(denp, 32) + eps;
      const float ru = rup + __shfl_xor(rup, 32);
      const float invden = 1.0f / den;
      const float go = ru * invden;
#pragma unroll
      for (int i = 0; i < HALF; ++i) dr[i] = (dr[i] - go * zo[i]) * invden * x[i];
      gsc = ok ? invden * beta : 0.0f;
      e = ok ? -go * invden * beta : 0.0f;
    } else {
#pragma unroll
      for (int i = 0; i < HALF; ++i) dr[i] *= x[i];
    }
    // ---- phi(q), g beta / den and e beta take the places of this head's columns ----------------------
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.write_half_row(slot, 0, rr);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int chunk = rg.kg * KS + s;
      if (chunk < CPR) {
        u32x4 w;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          float g0, g1;
          unpack2<T>(Bg[s][c], g0, g1);
          w[c] = pack2<T>(g0 * gsc, g1 * gsc);
        }
        *reinterpret_cast<u32x4*>(rg.chunk_ptr(slot, 1, chunk)) = w;
      }
    }
    if (rg.kg == 0) ecol[rg.tok] = (uint16_t)pack2<T>(e, 0.0f);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // ---- dS, dz: token-major operands by transposing reads --------------------------------------------
    {
      u32x4 bfrag[MT], bfe = u32x4{0, 0, 0, 0};
      if (j16 == 0) bfe = *reinterpret_cast<const u32x4*>(ecol + 8 * g4);
#pragma unroll
      for (int bb = 0; bb < MT; ++bb) {
        const u32x2 r0 = lds_read_tr16(rg.tr_ptr(slot, 1, tr_row, 16 * bb + tr_col));
        const u32x2 r1 = lds_read_tr16(rg.tr_ptr(slot, 1, tr_row + 4, 16 * bb + tr_col));
        bfrag[bb] = u32x4{r0[0], r0[1], r1[0], r1[1]};
      }
#pragma unroll
      for (int a = 0; a < MT; ++a) {
        const u32x2 r0 = lds_read_tr16(rg.tr_ptr(slot, 0, tr_row, 16 * a + tr_col));
        const u32x2 r1 = lds_read_tr16(rg.tr_ptr(slot, 0, tr_row + 4, 16 * a + tr_col));
        const u32x4 afrag = u32x4{r0[0], r0[1], r1[0], r1[1]};
#pragma unroll
        for (int bb = 0; bb < MT; ++bb) accS[a][bb] = mfma_16x16x32<T>(afrag, bfrag[bb], accS[a][bb]);
        accZ[a] = mfma_16x16x32<T>(afrag, bfe, accZ[a]);
      }
    }
    // ---- dq takes the place of this head's columns of the Q tile --------------------------------------
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.write_half_row(slot, 0, dr);

    rg.it.next();
    rg.ahead.next();
    if (rg.it.valid()) {
      // after the copies of tile j+1 came the stores of tile j-1 (dq only) and the copies of tile j+2
      if (have_prev && copied) wait_vmcnt<3 * NL>();
      else if (copied) wait_vmcnt<2 * NL>();
      else if (have_prev) wait_vmcnt<NL>();
      else wait_vmcnt<0>();
    }
    lds_barrier();   // tile j is finished by all waves; tile j+1 has landed for all
    prev_tile = tile;
    prev_slot = slot;
    slot = slot + 1 == R ? 0 : slot + 1;
  }
  if (prev_tile >= 0) rg.store_tile(prev_tile, prev_slot, 0, dQg, ldq.row);

  // ---- this wave's accumulators are its head's partial ----------------------------------------------------
  float* dst = partials + (((b * lq.H + h0 + rg.wave) * gridDim.x) + blockIdx.x) * (long long)NE;
#pragma unroll
  for (int a = 0; a < MT; ++a) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = a * 16 + 4 * g4 + i;
      if (row < D) {
#pragma unroll
        for (int bb = 0; bb < MT; ++bb) {
          const int col = bb * 16 + j16;
          if (col < D) dst[row * D + col] = accS[a][bb][i] * inv_beta;
        }
        if (j16 == 0) dst[D * D + row] = accZ[a][i] * inv_beta;
      }
    }
  }
}

// ==========================================================================================
// bwd_q16_rows: bwd_q16 (dQ and the per-token scalars {1 / den, e} for bwd_state16) on a group of W neighbouring
// heads.  grid = (wgs, B * gpb), block = 64 W.  `scal`: [B*H][N] pairs.  Same values as the per-head kernel.
// ==========================================================================================
template <typename T, int D, int FM, bool NORM, int W>
__global__ void __launch_bounds__(64 * W)
bwd_q16_rows(const u32x4* __restrict__ Q, Layout lq, const u32x4* __restrict__ G, Layout lg, u32x4* __restrict__ dQ,
             Layout ldq, int gpb, const float* __restrict__ state, f32x2* __restrict__ scal, float eps, long long N,
             int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using RG = Ring2Rows<T, D, W>;
  using C = BwdRowsCfg<D, W>;
  constexpr int NS = RG::NS, KS = RG::KS, MTB = RG::MTB, HALF = RG::HALF, NL = RG::NL, R = RG::R;
  constexpr int NE = D * D + D;
  const long long b = blockIdx.y / gpb;
  const long long h0 = (long long)(blockIdx.y % gpb) * W;
  RG rg(Q + (b * lq.batch + h0 * lq.head), lq.row, G + (b * lg.batch + h0 * lg.head), lg.row, N, tiles_per_block,
        blockIdx.x, gridDim.x, smem);
  u32x4* dQg = dQ + (b * ldq.batch + h0 * ldq.head);
  f32x2* sh = scal + (b * lq.H + h0 + rg.wave) * N;
  rg.prefetch_first();

  u32x4 A[NS][MTB][KS];
  float zo[HALF];
  float inv_aS = 1.0f;
  if constexpr (C::kOwnStage) {
    const float aS = rg.stage_state_own(state + (b * lq.H + h0 + rg.wave) * NE);
    rg.template build_A<false>(aS, A);       // u = S g
    rg.load_vec(zo);
    inv_aS = 1.0f / aS;
    __syncthreads();   // the staged states are dead: the second slot may be filled
    rg.prefetch_second();
  } else {
    rg.prefetch_second();
    for (int h = 0; h < W; ++h) {   // the heads' states pass through the third slot one after the other
      const float aS = rg.stage_state(state + (b * lq.H + h0 + h) * NE);
      if (rg.wave == h) {
        rg.template build_A<false>(aS, A);
        rg.load_vec(zo);
        inv_aS = 1.0f / aS;
      }
      __syncthreads();
    }
  }

  {   // this wave's rows of the first tile: only the second tile's copies were issued after them
    TileIter second = rg.it;
    second.next();
    if (second.valid()) wait_vmcnt<2 * NL>();
    else wait_vmcnt<0>();
  }
  lds_barrier();
  int slot = 0, prev_slot = 0;
  long long prev_tile = -1;
  while (rg.it.valid()) {
    const long long tile = rg.it.t;
    const bool have_prev = prev_tile >= 0;
    if (have_prev) rg.store_tile(prev_tile, prev_slot, 0, dQg, ldq.row);
    const bool copied = rg.ahead.valid();
    if (copied) rg.issue_copy(rg.ahead.t, have_prev ? prev_slot : R - 1);

    u32x4 Bg[KS];
    rg.read_B_raw(slot, 1, Bg);
    f32x16 acc[MTB];
    rg.products(A, Bg, nullptr, acc);
    float x[HALF];
    rg.read_half_row(slot, 0, x);             // q at this lane's output channels
    float denp = 0.0f, rup = 0.0f;
    float dr[HALF];
#pragma unroll
    for (int i = 0; i < HALF; ++i) {
      const float r = phi<FM>(x[i]);
      const float u = acc[i / 16][i % 16] * inv_aS;
      denp = __builtin_fmaf(r, zo[i], denp);
      rup = __builtin_fmaf(r, u, rup);
      dr[i] = u;
      x[i] = phi_prime_from<FM>(x[i], r);     // x now holds phi'(q)
    }
    if constexpr (NORM) {
      const float den = denp + __shfl_xor(denp, 32) + eps;
      const float ru = rup + __shfl_xor(rup, 32);
      const float invden = 1.0f / den;
      const float go = ru * invden;
#pragma unroll
      for (int i = 0; i < HALF; ++i) dr[i] = (dr[i] - go * zo[i]) * invden * x[i];
      long long rem = N - tile * kTile;
      const int lim = rem < kTile ? (int)rem : kTile;
      if (rg.kg == 0 && rg.tok < lim) sh[tile * kTile + rg.tok] = f32x2{invden, -go * invden};
    } else {
#pragma unroll
      for (int i = 0; i < HALF; ++i) dr[i] *= x[i];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // both half-waves have read the row before it changes
    rg.write_half_row(slot, 0, dr);

    rg.it.next();
    rg.ahead.next();
    if (rg.it.valid()) {
      // after the copies of tile j+1 came the stores of tile j-1 and the copies of tile j+2 (and up to two stores of
      // scalars, which these counts leave out: a stricter wait, never a laxer one)
      if (have_prev && copied) wait_vmcnt<3 * NL>();
      else if (copied) wait_vmcnt<2 * NL>();
      else if (have_prev) wait_vmcnt<NL>();
      else wait_vmcnt<0>();
    }
    lds_barrier();   // tile j is finished by all waves; tile j+1 has landed for all
    prev_tile = tile;
    prev_slot = slot;
    slot = slot + 1 == R ? 0 : slot + 1;
  }
  if (prev_tile >= 0) rg.store_tile(prev_tile, prev_slot, 0, dQg, ldq.row);
}

}  // namespace lf
