// Backward pass of the token mixer for fp16 / bf16, head widths up to 80 (training by distillation, Sec. 2.5 (Training Objectives),
// Eq. 8, needs it; the paper gives no formula -- these are the derivatives of Eq. 5 on Prop. 2's form).
// With P = phi(K), R = phi(Q), S = P^T V, z = P^T 1, den = R z + eps, out = R S / den and g = dL/d out:
//     u_i  = S g_i                      (d-vector per token)
//     go_i = (r_i . u_i) / den_i        (= g_i . out_i, recomputed in fp32 instead of read back in 16 bits)
//     dr_i = (u_i - go_i z) / den_i ,   dq = dr * phi'(q)
//     e_i  = -go_i / den_i ,            dS = R^T (g / den) ,  dz = R^T e
//     dp_j = dS v_j + dz ,              dk = dp * phi'(k) ,   dv_j = dS^T p_j
// (un-normalized: den = 1, go = e = 0).  Launches:
//     state_reduce16 + combine_state    S, z                         (the forward kernels; skipped when the
//                                                                      forward pass's state is handed in)
//     bwd_qs16 + combine_state          reads Q, g: writes dQ, and dS, dz as split partials
//     bwd_kv16                          reads K, V: writes dK, dV    (large fp16 problems: bwd_pack_kv16 +
//                                                                      bwd_kv16_packed, short-lived workgroups)
// The merged bwd_qs16 has no row-piece form for bf16 and d > 48; token-major tensors whose head rows are no whole
// cache lines take two kernels in its place there (and bf16 at d = 80 everywhere, where that measured faster):
//     bwd_q16                           reads Q, g: writes dQ and per token {1 / den_i, e_i}
//     bwd_state16 + combine_state       reads Q, g and those scalars: dS, dz
// The two apply-shaped kernels use the LDS-DMA ring of apply16_dma with two tensors per slot; the
// reduction is state_reduce16 with phi(Q) in the place of phi(K), g / den in the place of V and e_i in the
// place of the ones column.  Every tensor is addressed through a Layout (contiguous or strided views); the
// row-piece forms of the two apply-shaped kernels for token-major tensors are in lf_backward16_rows.hpp.
#pragma once
#include "lf_apply16_dma.hpp"

namespace lf {

template <int FM>
LF_DEV float phi_prime_from(float x, float phi_x) {   // d phi / dx given x and phi(x)
  if constexpr (FM == kPhiEluPlusOne) return x > 0.0f ? 1.0f : phi_x;
  else if constexpr (FM == kPhiRelu) return x > 0.0f ? 1.0f : 0.0f;
  else return 1.0f;
}

// RING: slots of the per-wave ring (RING - 1 tiles in flight); three where two workgroups share a CU
template <int D, int RING = 3> struct BwdCfg {
  using Sh = Shape16<D>;
  using AC = ApplyDmaCfg<D>;
  static constexpr int kNL = AC::kNL;
  static constexpr int kTileBytes = AC::kSlotBytes;              // one tensor's tile (whole 1 KiB deposits)
  static constexpr int kSlotBytes = 2 * kTileBytes;              // two tensors per ring slot
  static constexpr int kRing = RING;
  static constexpr int kStageOffset = (kRing - 1) * kWavesPerWG * kSlotBytes;
  static constexpr int kStageBytes = (D * D + D) * 4 + 64;
  static constexpr int kMTB = (Sh::kHalf + 15) / 16;            // 32-row output tiles (no normalizer rows)
  static constexpr int lds_bytes() {
    int ring = kRing * kWavesPerWG * kSlotBytes, st = kStageOffset + kStageBytes;
    return ring > st ? ring : st;
  }
};

// ---- two-tensor LDS-DMA ring, one wave per tile (see apply16_dma for the mechanism) -----------------
template <typename T, int D, int RING = 3>
struct Ring2 {
  using Sh = Shape16<D>;
  using AC = ApplyDmaCfg<D>;
  using BC = BwdCfg<D, RING>;
  static constexpr int NS = NSplit<T>::value;
  static constexpr int KS = Sh::kKS, CPR = Sh::kChunksPerRow, HALF = Sh::kHalf, MTB = BC::kMTB;
  static constexpr int NL = BC::kNL, NE = D * D + D, R = BC::kRing, TB = BC::kTileBytes;
  static_assert(R >= 3 && R <= 5, "ring depths the wait counts are written out for");

  const u32x4 *Xh, *Yh;
  int rsx, rsy;   // token strides of the two tensors, in 16-byte units (CPR when the rows are dense)
  long long N;
  unsigned char* smem;
  int lane, wave, tok, kg, row_byte, tsw;
  int trow[NL], gpos[NL];   // LDS position 64 u + lane holds chunk gpos[u] of token row trow[u]
  TileIter it, ahead;

  LF_DEV Ring2(const u32x4* Xh_, int rsx_, const u32x4* Yh_, int rsy_, long long N_, int tiles_per_block, int wg,
               int nwg, unsigned char* smem_)
      : Xh(Xh_), Yh(Yh_), rsx(rsx_), rsy(rsy_), N(N_), smem(smem_), lane(threadIdx.x & 63),
        wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)),
        it(wg, nwg, wave, tiles_per_block, (N_ + kTile - 1) / kTile), ahead(it) {
    tok = lane & 31;
    kg = lane >> 5;
    row_byte = tok * AC::kRowBytes;
    tsw = AC::swz(tok);
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int p = u * 64 + lane;
      const int r = p / CPR, pos = p % CPR;
      trow[u] = r;
      gpos[u] = pos ^ AC::swz(r);
    }
  }

  LF_DEV unsigned char* tile_ptr(int slot, int which) const {
    return smem + (slot * kWavesPerWG + wave) * BC::kSlotBytes + which * TB;
  }
  LF_DEV unsigned char* chunk_ptr(int slot, int which, int chunk) const {
    return tile_ptr(slot, which) + row_byte + ((chunk ^ tsw) << 4);
  }
  // pointer to byte `byte` of this lane's token row (pieces never straddle a 16-byte chunk)
  LF_DEV unsigned char* byte_ptr(int slot, int which, int byte) const {
    return chunk_ptr(slot, which, byte >> 4) + (byte & 15);
  }

  // address of the four 16-bit elements (row, col .. col + 3) of tile part `which`, col a multiple of 4: what
  // one lane names in a transposing LDS read
  LF_DEV const uint16_t* tr_ptr(int slot, int which, int row, int col) const {
    const int chunk = col >> 3;
    return reinterpret_cast<const uint16_t*>(tile_ptr(slot, which) + row * AC::kRowBytes +
                                             ((chunk ^ AC::swz(row)) << 4) + (col & 7) * 2);
  }

  // copies tile `tile` of both tensors into ring slot `slot`: always 2 NL vector memory instructions
  LF_DEV void issue_copy(long long tile, int slot) {
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
      const int rs = which ? rsy : rsx;
      const u32x4* gp = (which ? Yh : Xh) + tile * kTile * rs;
      unsigned char* sl = tile_ptr(slot, which);
#pragma unroll
      for (int u = 0; u < NL; ++u) {   // every lane issues every copy; lanes past the tile deposit chunk 0 in the padding
        const int c = trow[u] < lim ? trow[u] * rs + gpos[u] : 0;
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(gp + c),
                                         (LF_LDS void*)(sl + u * 1024), 16, 0, 2 /* nt */);
      }
    }
  }
  LF_DEV void prefetch() {
#pragma unroll
    for (int s = 0; s < R - 1; ++s) {
      if (ahead.valid()) issue_copy(ahead.t, s);
      ahead.next();
    }
  }
  // coalesced stores of tile part `which` of slot `slot` to head tensor `Oh` (token stride `rso`): always NL
  // instructions
  LF_DEV void store_tile(long long tile, int slot, int which, u32x4* Oh, int rso) {
    const unsigned char* sl = tile_ptr(slot, which);
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    u32x4* op = Oh + tile * kTile * rso;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const u32x4 w = *reinterpret_cast<const u32x4*>(sl + u * 1024 + lane * 16);
      if (u * 64 + lane < AC::kChunks && trow[u] < lim) st_stream(op + trow[u] * rso + gpos[u], w);
    }
  }
  // waits until the copies of the tile that is about to be used have landed; `iter` = tiles done so far
  // (0 ... R - 1 = that many or more), `more` = a copy was issued this iteration, SN = store instructions per
  // tile.  Issued after the wanted tile's copies: those of the R - 1 tiles behind it and the stores of the up to
  // R - 1 tiles finished since.
  template <int SN>
  LF_DEV void wait_tile(int iter, bool more) {
    constexpr int C = (R - 1) * 2 * NL;
    static_assert(C + (R - 1) * SN <= 63, "the counter of outstanding vector memory operations has six bits");
    if (!more) { wait_vmcnt<0>(); return; }
    constexpr int M = R - 1;   // `iter` never exceeds it
    if (iter == 0) wait_vmcnt<C>();
    else if (iter == 1) wait_vmcnt<C + SN>();
    else if (iter == 2) wait_vmcnt<C + 2 * SN>();
    else if (iter == 3) wait_vmcnt<C + (M < 3 ? M : 3) * SN>();
    else wait_vmcnt<C + (M < 4 ? M : 4) * SN>();
  }

  // Stages one head's fp32 state ([D*D] matrix then [D] vector) in LDS and returns the power-of-two scale
  // for the matrix.  The staging area starts at the third slot block (free before the stream loop).
  LF_DEV float stage_state(const float* state) {
    float* st = reinterpret_cast<float*>(smem + BC::kStageOffset);
    float* redmax = st + NE;
    float mS = 0.0f;
    for (int e = threadIdx.x; e < NE / 4; e += kThreads) {
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
    for (int w = 0; w < kWavesPerWG; ++w) mS = fmaxf(mS, redmax[w]);
    return pow2_scale_for(mS);
  }
  // A operands of the staged matrix M scaled by aS, for products  out[o] = sum_c M'[.][.] b[c]  over the
  // contraction index c = input channel of the B operand and o = this lane-half's output channels:
  //   TRANSPOSED = false: element M[o][c]   (out = M b);   TRANSPOSED = true: element M[c][o]  (out = M^T b)
  template <bool TRANSPOSED>
  LF_DEV void build_A(float aS, u32x4 (&A)[NS][MTB][KS]) const {
    const float* st = reinterpret_cast<const float*>(smem + BC::kStageOffset);
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
  // the staged vector at this lane-half's output channels
  LF_DEV void load_vec(float (&v)[HALF]) const {
    const float* st = reinterpret_cast<const float*>(smem + BC::kStageOffset) + D * D;
#pragma unroll
    for (int i = 0; i < HALF; ++i) v[i] = st[kg * HALF + i];
  }
  // this lane's HALF channels (lane-half kg) of its token's row in tile part `which`, widened to fp32
  LF_DEV void read_half_row(int slot, int which, float (&x)[HALF]) const {
    constexpr int PB = (HALF % 8 == 0) ? 16 : 8;   // piece bytes (HALF is a multiple of 4)
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
  // the same from words already packed (element 2 i in the low half of word i)
  LF_DEV void write_half_row_words(int slot, int which, const uint32_t (&w)[HALF / 2]) const {
    constexpr int PB = (HALF % 8 == 0) ? 16 : 8;
#pragma unroll
    for (int c = 0; c < HALF * 2 / PB; ++c) {
      unsigned char* p = byte_ptr(slot, which, kg * HALF * 2 + c * PB);
      if constexpr (PB == 16) *reinterpret_cast<u32x4*>(p) = u32x4{w[4 * c], w[4 * c + 1], w[4 * c + 2], w[4 * c + 3]};
      else *reinterpret_cast<u32x2*>(p) = u32x2{w[2 * c], w[2 * c + 1]};
    }
  }
  // B operands: this lane's input chunks of its token's row, raw 16-bit values
  LF_DEV void read_B_raw(int slot, int which, u32x4 (&B)[KS]) const {
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int chunk = kg * KS + s;
      B[s] = u32x4{0, 0, 0, 0};
      if (chunk < CPR) B[s] = *reinterpret_cast<const u32x4*>(chunk_ptr(slot, which, chunk));
    }
  }
  // acc[t] = sum_s A[.][t][s] * B[s]   (b_lo: low halves of a split B operand, or null)
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
// bwd_q16: dQ and the per-token scalars.  grid = (wgs, B*H), block = 256, dynamic LDS BwdCfg<D>::lds_bytes().
// `scal`: [B*H][N] pairs {1 / den_i, e_i} (written only when NORM).
// ==========================================================================================
template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
bwd_q16(const u32x4* __restrict__ Q, Layout lq, const u32x4* __restrict__ G, Layout lg, u32x4* __restrict__ dQ,
        Layout ldq, const float* __restrict__ state, f32x2* __restrict__ scal, float eps, long long N,
        int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using RG = Ring2<T, D>;
  constexpr int NS = RG::NS, KS = RG::KS, MTB = RG::MTB, HALF = RG::HALF, NL = RG::NL, R = RG::R;
  constexpr int SN = NL + (NORM ? 1 : 0);
  const long long bh = blockIdx.y;
  RG rg(Q + lq.slice(bh), lq.row, G + lg.slice(bh), lg.row, N, tiles_per_block, blockIdx.x, gridDim.x, smem);
  u32x4* dQh = dQ + ldq.slice(bh);
  f32x2* sh = scal + bh * N;
  rg.prefetch();

  const float aS = rg.stage_state(state + bh * (D * D + D));
  u32x4 A[NS][MTB][KS];
  rg.template build_A<false>(aS, A);       // u = S g
  float zo[HALF];
  rg.load_vec(zo);
  const float inv_aS = 1.0f / aS;
  __syncthreads();                          // the staged state is dead

  int slot = 0, iter = 0;
  while (rg.it.valid()) {
    const long long tile = rg.it.t;
    int aslot = slot + (R - 1);
    if (aslot >= R) aslot -= R;
    const bool more = rg.ahead.valid();
    if (more) rg.issue_copy(rg.ahead.t, aslot);
    rg.template wait_tile<SN>(iter, more);
    iter = iter < 2 ? iter + 1 : 2;

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
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.write_half_row(slot, 0, dr);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.store_tile(tile, slot, 0, dQh, ldq.row);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.it.next();
    rg.ahead.next();
    slot = slot + 1 == R ? 0 : slot + 1;
  }
}

// ==========================================================================================
// bwd_qs16: bwd_q16 and bwd_state16 in one pass over Q and g.  After a tile's dq is known, the wave
// overwrites the Q tile in its LDS slot with phi(q) and the g tile with g beta / den (16-bit), keeps
// e_i beta in a 32-entry column, and accumulates dS += phi(q)^T (g beta / den), dz += phi(q)^T (e beta) with
// transposing LDS reads exactly as the reductions do; then dq takes the Q tile's place and leaves.
// bf16 needs two 8-bit levels of each of the three: the rounded values go first and are read into operands,
// then the remainders take the same places (no LDS beyond the ring), and three products per block follow
// (rounded x rounded, remainder x rounded, rounded x remainder).
// At the end the four waves' accumulators are summed in a fixed order and written (divided by beta) as
// this workgroup's partial: [B*H][gridDim.x][D*D + D], for combine_state.  No per-token scalars in memory,
// two tensor passes fewer.  LDS: qs_lds_bytes<T, D>().
// ==========================================================================================
// Ring depth of the merged kernel: three slots and two workgroups per CU where the kernel fits 256 registers;
// beyond that a lone workgroup per CU (512 registers per lane) with a deeper ring, as LDS allows.
template <typename T, int D> constexpr bool qs_two_per_cu() { return NSplit<T>::value == 1 ? D <= 48 : D <= 32; }
template <typename T, int D> constexpr int qs_ring() {
  if (qs_two_per_cu<T, D>()) return 3;
  return D <= 48 ? 5 : (D <= 64 ? 4 : 3);
}
template <typename T, int D> constexpr int qs_lds_bytes() { return BwdCfg<D, qs_ring<T, D>()>::lds_bytes() + 512; }

template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
bwd_qs16(const u32x4* __restrict__ Q, Layout lq, const u32x4* __restrict__ G, Layout lg, u32x4* __restrict__ dQ,
         Layout ldq, const float* __restrict__ state, float* __restrict__ partials, float eps, long long N,
         int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using RG = Ring2<T, D, qs_ring<T, D>()>;
  using BC = typename RG::BC;
  using Sh = Shape16<D>;
  constexpr int NS = RG::NS, KS = RG::KS, MTB = RG::MTB, HALF = RG::HALF, NL = RG::NL, R = RG::R, CPR = RG::CPR;
  constexpr int MT = Sh::kMT, NE = D * D + D;
  const long long bh = blockIdx.y;
  RG rg(Q + lq.slice(bh), lq.row, G + lg.slice(bh), lg.row, N, tiles_per_block, blockIdx.x, gridDim.x, smem);
  u32x4* dQh = dQ + ldq.slice(bh);
  uint16_t* ecol = reinterpret_cast<uint16_t*>(smem + BC::lds_bytes()) + rg.wave * 32;
  rg.prefetch();

  const float aS = rg.stage_state(state + bh * NE);
  u32x4 A[NS][MTB][KS];
  rg.template build_A<false>(aS, A);
  // z at this lane-half's output channels: in registers (fp16) or, where registers are short (bf16), in a copy
  // of its own in LDS behind the e column, read per use
  float zo[NS == 1 ? HALF : 1];
  float* zlds = reinterpret_cast<float*>(smem + BC::lds_bytes() + 256);
  if constexpr (NS == 1) {
    rg.load_vec(zo);
  } else {
    const float* z = reinterpret_cast<const float*>(smem + BC::kStageOffset) + D * D;
    for (int i = threadIdx.x; i < D; i += kThreads) zlds[i] = z[i];
  }
  auto zv = [&](int i) -> float {
    if constexpr (NS == 1) return zo[i];
    else return zlds[rg.kg * HALF + i];
  };
  const float inv_aS = 1.0f / aS;
  float beta = 1.0f, inv_beta = 1.0f;
  if constexpr (NORM) {   // power of two near the typical denominator (see bwd_state16)
    const float* z = reinterpret_cast<const float*>(smem + BC::kStageOffset) + D * D;
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
  __syncthreads();

  f32x4 accS[MT][MT], accZ[MT];
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    accZ[a] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < MT; ++b) accS[a][b] = f32x4{0, 0, 0, 0};
  }
  const int j16 = rg.lane & 15, g4 = rg.lane >> 4;
  const int tr_row = 8 * g4 + (j16 >> 2), tr_col = 4 * (j16 & 3);

  int slot = 0, iter = 0;
  while (rg.it.valid()) {
    const long long tile = rg.it.t;
    int aslot = slot + (R - 1);
    if (aslot >= R) aslot -= R;
    const bool more = rg.ahead.valid();
    if (more) rg.issue_copy(rg.ahead.t, aslot);
    rg.template wait_tile<NL>(iter, more);
    iter = iter < R - 1 ? iter + 1 : R - 1;
    long long rem = N - tile * kTile;
    const bool ok = rg.tok < (rem < kTile ? (int)rem : kTile);

    u32x4 Bg[KS];
    rg.read_B_raw(slot, 1, Bg);
    f32x16 acc[MTB];
    rg.products(A, Bg, nullptr, acc);
    // dq and phi(q) leave this block as the 16-bit words that go to LDS (bf16: phi(q) as a rounded value plus the
    // remainder).  bf16 is short of registers: it keeps phi'(q) as one sign bit per element and takes the value
    // back from the two levels of phi(q) (16 significant bits; elu + 1 and relu have phi' = 1 where q > 0, else phi
    // resp. 0, the identity map 1 everywhere).
    uint32_t dqw[HALF / 2], rw[NS][HALF / 2];
    float gsc = ok ? 1.0f : 0.0f, e = 0.0f;
    {
      float x[HALF], dr[HALF];
      rg.read_half_row(slot, 0, x);
      float denp = 0.0f, rup = 0.0f;
      uint64_t pos = 0;   // bit i: q at output channel i is positive
#pragma unroll
      for (int i = 0; i < HALF; i += 2) {
        float r[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          r[q] = phi<FM>(x[i + q]);
          const float u = acc[(i + q) / 16][(i + q) % 16] * inv_aS;
          denp = __builtin_fmaf(r[q], zv(i + q), denp);
          rup = __builtin_fmaf(r[q], u, rup);
          dr[i + q] = u;
          if constexpr (NS == 1) x[i + q] = phi_prime_from<FM>(x[i + q], r[q]);
          else pos |= (uint64_t)(x[i + q] > 0.0f ? 1u : 0u) << (i + q);
          r[q] = ok ? r[q] : 0.0f;
        }
        if constexpr (NS == 1) rw[0][i / 2] = pack2<T>(r[0], r[1]);
        else pack2_split<T>(r[0], r[1], rw[0][i / 2], rw[1][i / 2]);
      }
      auto phi_prime = [&](int i) -> float {
        if constexpr (NS == 1) {
          return x[i];
        } else if constexpr (FM == kPhiIdentity) {
          return 1.0f;
        } else {
          float h[2], l[2];
          unpack2<T>(rw[0][i / 2], h[0], h[1]);
          unpack2<T>(rw[1][i / 2], l[0], l[1]);
          const float below = FM == kPhiRelu ? 0.0f : h[i & 1] + l[i & 1];
          return (pos >> i) & 1u ? 1.0f : below;
        }
      };
      if constexpr (NORM) {
        const float den = denp + __shfl_xor(denp, 32) + eps;
        const float ru = rup + __shfl_xor(rup, 32);
        const float invden = 1.0f / den;
        const float go = ru * invden;
#pragma unroll
        for (int i = 0; i < HALF; ++i) dr[i] = (dr[i] - go * zv(i)) * invden * phi_prime(i);
        gsc = ok ? invden * beta : 0.0f;
        e = ok ? -go * invden * beta : 0.0f;
      } else {
#pragma unroll
        for (int i = 0; i < HALF; ++i) dr[i] *= phi_prime(i);
      }
#pragma unroll
      for (int i = 0; i < HALF / 2; ++i) dqw[i] = pack2<T>(dr[2 * i], dr[2 * i + 1]);
    }
    // ---- phi(q), g beta / den and e beta take the tiles' places --------------------------------------
    // bf16 carries each as two 8-bit levels.  The remainders take the same places once the rounded values have
    // been read into operands (a wave's LDS operations retire in order), so no LDS beyond the ring is needed.
    u32x4 glo[NS == 2 ? KS : 1];
    uint32_t elo = 0;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.write_half_row_words(slot, 0, rw[0]);
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int chunk = rg.kg * KS + s;
      if (chunk < CPR) {
        u32x4 w;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          float g0, g1;
          unpack2<T>(Bg[s][c], g0, g1);
          if constexpr (NS == 1) {
            w[c] = pack2<T>(g0 * gsc, g1 * gsc);
          } else {
            uint32_t h, l;
            pack2_split<T>(g0 * gsc, g1 * gsc, h, l);
            w[c] = h;
            glo[s][c] = l;
          }
        }
        *reinterpret_cast<u32x4*>(rg.chunk_ptr(slot, 1, chunk)) = w;
      }
    }
    if constexpr (NS == 1) {
      if (rg.kg == 0) ecol[rg.tok] = (uint16_t)pack2<T>(e, 0.0f);
    } else {
      uint32_t eh;
      pack2_split<T>(e, 0.0f, eh, elo);
      if (rg.kg == 0) ecol[rg.tok] = (uint16_t)eh;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    // ---- dS, dz: token-major operands by transposing reads --------------------------------------------
    auto read_a = [&](int a) {
      const u32x2 r0 = lds_read_tr16(rg.tr_ptr(slot, 0, tr_row, 16 * a + tr_col));
      const u32x2 r1 = lds_read_tr16(rg.tr_ptr(slot, 0, tr_row + 4, 16 * a + tr_col));
      return u32x4{r0[0], r0[1], r1[0], r1[1]};
    };
    auto read_b = [&](int b) {
      const u32x2 r0 = lds_read_tr16(rg.tr_ptr(slot, 1, tr_row, 16 * b + tr_col));
      const u32x2 r1 = lds_read_tr16(rg.tr_ptr(slot, 1, tr_row + 4, 16 * b + tr_col));
      return u32x4{r0[0], r0[1], r1[0], r1[1]};
    };
    auto read_e = [&]() {
      u32x4 w = u32x4{0, 0, 0, 0};
      if (j16 == 0) w = *reinterpret_cast<const u32x4*>(ecol + 8 * g4);
      return w;
    };
    if constexpr (NS == 1) {
      u32x4 bfrag[MT];
      const u32x4 bfe = read_e();
#pragma unroll
      for (int b = 0; b < MT; ++b) bfrag[b] = read_b(b);
#pragma unroll
      for (int a = 0; a < MT; ++a) {
        const u32x4 afrag = read_a(a);
#pragma unroll
        for (int b = 0; b < MT; ++b) accS[a][b] = mfma_16x16x32<T>(afrag, bfrag[b], accS[a][b]);
        accZ[a] = mfma_16x16x32<T>(afrag, bfe, accZ[a]);
      }
    } else {
      // rounded x rounded, remainder x rounded, rounded x remainder; the remainders' operands live one at a time
      u32x4 ah[MT], bh[MT];
      const u32x4 beh = read_e();
#pragma unroll
      for (int b = 0; b < MT; ++b) bh[b] = read_b(b);
#pragma unroll
      for (int a = 0; a < MT; ++a) ah[a] = read_a(a);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      rg.write_half_row_words(slot, 0, rw[NS - 1]);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int chunk = rg.kg * KS + s;
        if (chunk < CPR) *reinterpret_cast<u32x4*>(rg.chunk_ptr(slot, 1, chunk)) = glo[s];
      }
      if (rg.kg == 0) ecol[rg.tok] = (uint16_t)elo;
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
#pragma unroll
      for (int a = 0; a < MT; ++a) {
#pragma unroll
        for (int b = 0; b < MT; ++b) accS[a][b] = mfma_16x16x32<T>(ah[a], bh[b], accS[a][b]);
        accZ[a] = mfma_16x16x32<T>(ah[a], beh, accZ[a]);
      }
#pragma unroll
      for (int a = 0; a < MT; ++a) {
        const u32x4 al = read_a(a);
#pragma unroll
        for (int b = 0; b < MT; ++b) accS[a][b] = mfma_16x16x32<T>(al, bh[b], accS[a][b]);
        accZ[a] = mfma_16x16x32<T>(al, beh, accZ[a]);
      }
#pragma unroll
      for (int b = 0; b < MT; ++b) {
        const u32x4 bl = read_b(b);
#pragma unroll
        for (int a = 0; a < MT; ++a) accS[a][b] = mfma_16x16x32<T>(ah[a], bl, accS[a][b]);
      }
      const u32x4 bel = read_e();
#pragma unroll
      for (int a = 0; a < MT; ++a) accZ[a] = mfma_16x16x32<T>(ah[a], bel, accZ[a]);
    }
    // ---- dq takes the Q tile's place and leaves -----------------------------------------------------------
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.write_half_row_words(slot, 0, dqw);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.store_tile(tile, slot, 0, dQh, ldq.row);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.it.next();
    rg.ahead.next();
    slot = slot + 1 == R ? 0 : slot + 1;
  }

  // ---- cross-wave sum in a fixed order, (w0 + w2) + (w1 + w3), then the partial ---------------------------
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);
  float* mine = red + (rg.wave & 1) * NE;
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if ((rg.wave >> 1) == round) {
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
                float* p = mine + row * D + col;
                *p = (round == 0) ? accS[a][b][i] : *p + accS[a][b][i];
              }
            }
            if (j16 == 0) {
              float* p = mine + D * D + row;
              *p = (round == 0) ? accZ[a][i] : *p + accZ[a][i];
            }
          }
        }
      }
    }
    __syncthreads();
  }
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)NE;
  for (int i = threadIdx.x; i < NE; i += kThreads) dst[i] = (red[i] + red[NE + i]) * inv_beta;
}

// ==========================================================================================
// bwd_kv16: dK and dV.  grid = (wgs, B*H), block = 256.  `dstate`: [B*H][D*D + D], dS row-major then dz.
// bwd_kv16_packed: the same stream from operands that bwd_pack_kv16 prepared once per head, so that a
// workgroup's start-up is a few coalesced loads and a launch can use many short-lived workgroups (see
// apply16_packed: the chip then reads and writes one narrow moving window of memory).
// ==========================================================================================
// What bwd_pack_kv16 leaves per head: {1 / scale} and dz in a 1 KiB header, then the lanes' operands of dS^T and dS
template <typename T, int D> struct PackKV16 {
  static constexpr int kHeaderBytes = 1024;
  static constexpr int kDzOffset = 256;   // bytes; D floats
  static constexpr int kFrags = NSplit<T>::value * BwdCfg<D>::kMTB * Shape16<D>::kKS;   // per lane and matrix
  static constexpr int kHeadBytes = kHeaderBytes + 2 * kFrags * 64 * 16;
  static_assert(kDzOffset + D * 4 <= kHeaderBytes, "dz fits the header");
};

template <typename T, int D, int FM>
LF_DEV void bwd_kv_stream(Ring2<T, D>& rg, const u32x4 (&A1)[NSplit<T>::value][BwdCfg<D>::kMTB][Shape16<D>::kKS],
                          const u32x4 (&A2)[NSplit<T>::value][BwdCfg<D>::kMTB][Shape16<D>::kKS],
                          const float (&dzo)[Shape16<D>::kHalf], float inv_aS, u32x4* dKh, u32x4* dVh, int rso) {
  using RG = Ring2<T, D>;
  constexpr int NS = RG::NS, KS = RG::KS, MTB = RG::MTB, HALF = RG::HALF, NL = RG::NL, R = RG::R, CPR = RG::CPR;
  constexpr int SN = 2 * NL;
  int slot = 0, iter = 0;
  while (rg.it.valid()) {
    const long long tile = rg.it.t;
    int aslot = slot + (R - 1);
    if (aslot >= R) aslot -= R;
    const bool more = rg.ahead.valid();
    if (more) rg.issue_copy(rg.ahead.t, aslot);
    rg.template wait_tile<SN>(iter, more);
    iter = iter < 2 ? iter + 1 : 2;

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
          uint32_t h, l;
          pack2_split<T>(r0, r1, h, l);
          Bp[s][w] = h;
          Bpl[s][w] = l;
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
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.write_half_row(slot, 0, x);
    rg.write_half_row(slot, 1, o);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.store_tile(tile, slot, 0, dKh, rso);
    rg.store_tile(tile, slot, 1, dVh, rso);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    rg.it.next();
    rg.ahead.next();
    slot = slot + 1 == R ? 0 : slot + 1;
  }
}

template <typename T, int D, int FM>
__global__ void __launch_bounds__(kThreads)
bwd_kv16(const u32x4* __restrict__ K, const u32x4* __restrict__ V, Layout lkv, u32x4* __restrict__ dK,
         u32x4* __restrict__ dV, Layout ldkv, const float* __restrict__ dstate, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using RG = Ring2<T, D>;
  constexpr int NS = RG::NS, KS = RG::KS, MTB = RG::MTB, HALF = RG::HALF;
  const long long bh = blockIdx.y;
  RG rg(K + lkv.slice(bh), lkv.row, V + lkv.slice(bh), lkv.row, N, tiles_per_block, blockIdx.x, gridDim.x, smem);
  rg.prefetch();

  const float aS = rg.stage_state(dstate + bh * (D * D + D));
  u32x4 A1[NS][MTB][KS], A2[NS][MTB][KS];
  rg.template build_A<true>(aS, A1);        // dv = dS^T p
  rg.template build_A<false>(aS, A2);       // dp = dS v (+ dz)
  float dzo[HALF];
  rg.load_vec(dzo);
  __syncthreads();
  bwd_kv_stream<T, D, FM>(rg, A1, A2, dzo, 1.0f / aS, dK + ldkv.slice(bh), dV + ldkv.slice(bh), ldkv.row);
}

// grid = (B*H), block = 256, dynamic LDS BwdCfg<D>::lds_bytes(): the operands of bwd_kv16 for one head, built with
// that kernel's own prologue and written by wave 0 in lane order.
template <typename T, int D>
__global__ void __launch_bounds__(kThreads)
bwd_pack_kv16(const float* __restrict__ dstate, unsigned char* __restrict__ packed) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using RG = Ring2<T, D>;
  using PK = PackKV16<T, D>;
  constexpr int NS = RG::NS, KS = RG::KS, MTB = RG::MTB;
  const long long bh = blockIdx.x;
  RG rg(nullptr, 0, nullptr, 0, 0, kWavesPerWG, 0, 1, smem);
  const float aS = rg.stage_state(dstate + bh * (D * D + D));
  u32x4 A1[NS][MTB][KS], A2[NS][MTB][KS];
  rg.template build_A<true>(aS, A1);
  rg.template build_A<false>(aS, A2);
  unsigned char* dst = packed + bh * PK::kHeadBytes;
  if (rg.wave == 0) {
    u32x4* frag = reinterpret_cast<u32x4*>(dst + PK::kHeaderBytes);
#pragma unroll
    for (int l = 0; l < NS; ++l)
#pragma unroll
      for (int t = 0; t < MTB; ++t)
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          frag[((l * MTB + t) * KS + s) * 64 + rg.lane] = A1[l][t][s];
          frag[(PK::kFrags + (l * MTB + t) * KS + s) * 64 + rg.lane] = A2[l][t][s];
        }
    const float* st = reinterpret_cast<const float*>(smem + BwdCfg<D>::kStageOffset) + D * D;
    float* dz = reinterpret_cast<float*>(dst + PK::kDzOffset);
    for (int i = rg.lane; i < D; i += 64) dz[i] = st[i];
    if (rg.lane == 0) *reinterpret_cast<float*>(dst) = 1.0f / aS;
  }
}

// grid = (wgs, B*H), block = 256, dynamic LDS = the ring (BwdCfg<D>::kRing slots); no staging, no workgroup barrier
template <typename T, int D, int FM>
__global__ void __launch_bounds__(kThreads)
bwd_kv16_packed(const u32x4* __restrict__ K, const u32x4* __restrict__ V, Layout lkv, u32x4* __restrict__ dK,
                u32x4* __restrict__ dV, Layout ldkv, const unsigned char* __restrict__ packed, long long N,
                int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using RG = Ring2<T, D>;
  using PK = PackKV16<T, D>;
  constexpr int NS = RG::NS, KS = RG::KS, MTB = RG::MTB, HALF = RG::HALF;
  const long long bh = blockIdx.y;
  RG rg(K + lkv.slice(bh), lkv.row, V + lkv.slice(bh), lkv.row, N, tiles_per_block, blockIdx.x, gridDim.x, smem);
  rg.prefetch();
  const unsigned char* src = packed + bh * PK::kHeadBytes;
  const u32x4* frag = reinterpret_cast<const u32x4*>(src + PK::kHeaderBytes);
  u32x4 A1[NS][MTB][KS], A2[NS][MTB][KS];
#pragma unroll
  for (int l = 0; l < NS; ++l)
#pragma unroll
    for (int t = 0; t < MTB; ++t)
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        A1[l][t][s] = frag[((l * MTB + t) * KS + s) * 64 + rg.lane];
        A2[l][t][s] = frag[(PK::kFrags + (l * MTB + t) * KS + s) * 64 + rg.lane];
      }
  const float* dz = reinterpret_cast<const float*>(src + PK::kDzOffset);
  float dzo[HALF];
#pragma unroll
  for (int i = 0; i < HALF; ++i) dzo[i] = dz[rg.kg * HALF + i];
  const float inv_aS = *reinterpret_cast<const float*>(src);
  bwd_kv_stream<T, D, FM>(rg, A1, A2, dzo, inv_aS, dK + ldkv.slice(bh), dV + ldkv.slice(bh), ldkv.row);
}

// ==========================================================================================
// bwd_state16: dS = sum_i phi(q_i)^T (g_i / den_i),  dz = sum_i phi(q_i) e_i, as split-N partials (then
// combine_state).  grid = (splits, B*H), block = 256.  state_reduce16's stream with the B tile built from
// g and the scalars; the tile carries one extra 16-column block whose first column holds e_i.
// `state`: the forward state (only z is read, for the scale beta below).
// Partial: dS as [D][D] row-major (row = feature index of phi(q), column = channel of g), then dz.
// ==========================================================================================
template <int D> struct BwdReduceCfg {
  using Sh = Shape16<D>;
  static constexpr int kRS = Sh::kDP + 24;                       // one more 16-column block, 8 columns of padding
  static constexpr int kTileElems = kTile * kRS;
  static constexpr int kChunks = kTile * Sh::kChunksPerRow;
  static constexpr int kNL = (kChunks + 63) / 64;
};
template <typename T, int D>
constexpr int bwd_state_lds_bytes() {
  int tiles = 2 * NSplit<T>::value * BwdReduceCfg<D>::kTileElems * 2 * kWavesPerWG;
  int red = 2 * (D * D + D) * 4;
  return tiles > red ? tiles : red;
}

template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
bwd_state16(const u32x4* __restrict__ Q, Layout lq, const u32x4* __restrict__ G, Layout lg,
            const f32x2* __restrict__ scal, const float* __restrict__ state, float* __restrict__ partials, long long N,
            int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using Sh = Shape16<D>;
  using Cfg = BwdReduceCfg<D>;
  constexpr int NS = NSplit<T>::value;
  constexpr int RS = Cfg::kRS, NL = Cfg::kNL, CPR = Sh::kChunksPerRow, MT = Sh::kMT, TE = Cfg::kTileElems;
  constexpr int NE = D * D + D;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long bh = blockIdx.y;
  const u32x4* Qh = Q + lq.slice(bh);
  const u32x4* Gh = G + lg.slice(bh);
  const f32x2* sh = scal + bh * N;
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)NE;

  // g / den and e are of the order 1 / (N d): far below the fp16 normal range for large N.  Both are
  // carried times beta, a power of two near the typical denominator (sum of z, as phi(q) is of order one),
  // and the partial is divided by beta again (exactly) at the end.
  float beta = 1.0f, inv_beta = 1.0f;
  if constexpr (NORM) {
    const float* z = state + bh * NE + D * D;
    float zs = 0.0f;
    for (int i = lane; i < D; i += 64) zs += z[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) zs += __shfl_xor(zs, o);
    if (zs > 0.0f && zs < 3.0e38f) {
      int ex;
      (void)__builtin_frexpf(zs, &ex);
      ex = ex > 100 ? 100 : (ex < -100 ? -100 : ex);
      beta = __builtin_ldexpf(1.0f, ex);
      inv_beta = __builtin_ldexpf(1.0f, -ex);
    }
  }

  // per wave: NS tiles of phi(Q) then NS tiles of g / den (with the e column)
  uint16_t* wbase = reinterpret_cast<uint16_t*>(smem) + wave * 2 * NS * TE;
  int lds_off[NL], trow[NL], goff[NL];
#pragma unroll
  for (int u = 0; u < NL; ++u) {
    const int c = u * 64 + lane;
    trow[u] = c / CPR;
    goff[u] = c % CPR;
    lds_off[u] = trow[u] * RS + (c % CPR) * 8;
  }
  const int j16 = lane & 15, g4 = lane >> 4;
  const int tr_base = (8 * g4 + (j16 >> 2)) * RS + 4 * (j16 & 3);

  TileIter it(blockIdx.x, gridDim.x, wave, tiles_per_block, (N + kTile - 1) / kTile);

  f32x4 acc[MT][MT + 1];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b <= MT; ++b) acc[a][b] = f32x4{0, 0, 0, 0};

  u32x4 qr[NL], gr[NL];
  f32x2 sc[NL];
  auto issue_loads = [&](long long tile) {
    long long rem = N - tile * kTile;
    int lim = rem < kTile ? (int)rem : kTile;
    const u32x4* qp = Qh + tile * kTile * lq.row;
    const u32x4* gp = Gh + tile * kTile * lg.row;
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      qr[u] = u32x4{0, 0, 0, 0};
      gr[u] = u32x4{0, 0, 0, 0};
      sc[u] = f32x2{1.0f, 0.0f};
      if (u * 64 + lane < Cfg::kChunks && trow[u] < lim) {
        qr[u] = ld_stream(qp + trow[u] * lq.row + goff[u]);
        gr[u] = ld_stream(gp + trow[u] * lg.row + goff[u]);
        if constexpr (NORM) {
          sc[u] = sh[tile * kTile + trow[u]];
          sc[u][0] *= beta;
          sc[u][1] *= beta;
        }
      }
    }
    return lim;
  };

  int lim = 0;
  if (it.valid()) lim = issue_loads(it.t);
  for (int i = lane; i < 2 * NS * TE; i += 64) wbase[i] = 0;   // pad columns and the unused part of the extra block

  while (it.valid()) {
#pragma unroll
    for (int u = 0; u < NL; ++u) {
      const int c = u * 64 + lane;
      if (c < Cfg::kChunks) {
        const bool ok = trow[u] < lim;
        u32x4 ph, pl, gh, gl;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float x0, x1, g0, g1;
          unpack2<T>(qr[u][w], x0, x1);
          unpack2<T>(gr[u][w], g0, g1);
          const float p0 = ok ? phi<FM>(x0) : 0.0f, p1 = ok ? phi<FM>(x1) : 0.0f;
          g0 *= sc[u][0];
          g1 *= sc[u][0];
          if constexpr (NS == 1) {
            ph[w] = pack2<T>(p0, p1);
            gh[w] = pack2<T>(g0, g1);
          } else {
            uint32_t h, l;
            pack2_split<T>(p0, p1, h, l);
            ph[w] = h; pl[w] = l;
            pack2_split<T>(g0, g1, h, l);
            gh[w] = h; gl[w] = l;
          }
        }
        *reinterpret_cast<u32x4*>(wbase + lds_off[u]) = ph;
        *reinterpret_cast<u32x4*>(wbase + NS * TE + lds_off[u]) = gh;
        if constexpr (NS == 2) {
          *reinterpret_cast<u32x4*>(wbase + TE + lds_off[u]) = pl;
          *reinterpret_cast<u32x4*>(wbase + 3 * TE + lds_off[u]) = gl;
        }
        if (NORM && c % CPR == 0) {   // this lane holds the first chunk of its row: it also writes e_i
          const float e = ok ? sc[u][1] : 0.0f;
          if constexpr (NS == 1) {
            wbase[NS * TE + trow[u] * RS + Sh::kDP] = (uint16_t)pack2<T>(e, 0.0f);
          } else {
            uint32_t h, l;
            pack2_split<T>(e, 0.0f, h, l);
            wbase[2 * TE + trow[u] * RS + Sh::kDP] = (uint16_t)h;
            wbase[3 * TE + trow[u] * RS + Sh::kDP] = (uint16_t)l;
          }
        }
      }
    }
    it.next();
    int next_lim = 0;
    if (it.valid()) next_lim = issue_loads(it.t);

    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    u32x4 bfrag[NS][MT + 1];
#pragma unroll
    for (int s = 0; s < NS; ++s)
#pragma unroll
      for (int b = 0; b <= MT; ++b) {
        const uint16_t* base = wbase + (NS + s) * TE;
        u32x2 r0 = lds_read_tr16(base + tr_base + 16 * b);
        u32x2 r1 = lds_read_tr16(base + tr_base + 4 * RS + 16 * b);
        bfrag[s][b] = u32x4{r0[0], r0[1], r1[0], r1[1]};
      }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
#pragma unroll
      for (int a = 0; a < MT; ++a) {
        u32x2 r0 = lds_read_tr16(wbase + s * TE + tr_base + 16 * a);
        u32x2 r1 = lds_read_tr16(wbase + s * TE + tr_base + 4 * RS + 16 * a);
        const u32x4 afrag = u32x4{r0[0], r0[1], r1[0], r1[1]};
#pragma unroll
        for (int b = 0; b <= MT; ++b) {
          acc[a][b] = mfma_16x16x32<T>(afrag, bfrag[0][b], acc[a][b]);              // hi * hi, lo * hi
          if (NS == 2 && s == 0) acc[a][b] = mfma_16x16x32<T>(afrag, bfrag[NS - 1][b], acc[a][b]);   // hi * lo
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    lim = next_lim;
  }

  // ---- cross-wave sum in a fixed order, (w0 + w2) + (w1 + w3), as in state_reduce16 ----------------
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);
  float* mine = red + (wave & 1) * NE;
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if ((wave >> 1) == round) {
#pragma unroll
      for (int a = 0; a < MT; ++a) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = a * 16 + 4 * g4 + i;
          if (row < D) {
#pragma unroll
            for (int b = 0; b <= MT; ++b) {
              const int col = b * 16 + j16;
              float* p = nullptr;
              if (b < MT && col < D) p = mine + row * D + col;
              else if (b == MT && j16 == 0) p = mine + D * D + row;
              if (p) *p = (round == 0) ? acc[a][b][i] : *p + acc[a][b][i];
            }
          }
        }
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < NE; i += kThreads) dst[i] = (red[i] + red[NE + i]) * inv_beta;
}

}  // namespace lf
