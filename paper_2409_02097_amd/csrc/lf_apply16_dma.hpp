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

// D: width of the query rows that come in; DV: width of the value / output rows that leave (Prop. 3 allows a
// feature width other than the value width; DV = D everywhere else).
template <int D, int DV = D> struct ApplyDmaCfg {
  using Sh = Shape16<D>;
  static constexpr int kCPR = Sh::kChunksPerRow;
  static constexpr int kRowBytes = D * 2;
  static constexpr int kChunks = kTile * kCPR;
  static constexpr int kNL = (kChunks + 63) / 64;
  static constexpr int kCPRO = DV / 8;                   // the same four for the tile that is stored
  static constexpr int kRowBytesO = DV * 2;
  static constexpr int kChunksO = kTile * kCPRO;
  static constexpr int kNLO = (kChunksO + 63) / 64;
  static constexpr int kSlotBytes = (kNL > kNLO ? kNL : kNLO) * 1024;   // whole 1 KiB deposits; >= either tile's bytes
  static constexpr int kRing = 3;
  static constexpr int kStageOffset = (kRing - 1) * kWavesPerWG * kSlotBytes;
  static constexpr int kStageBytes = (D * DV + D) * 4 + 256;   // the state and two maxima per wave
  // XOR swizzle of the chunk position with the row index where rows are 64 or 128 bytes
  static constexpr int kSwzMask = (kCPR == 8) ? 7 : (kCPR == 4 ? 3 : 0);
  static constexpr int kSwzShift = (kCPR == 4) ? 2 : 0;
  static __device__ __forceinline__ int swz(int row) { return (row >> kSwzShift) & kSwzMask; }
  static constexpr int kSwzMaskO = (kCPRO == 8) ? 7 : (kCPRO == 4 ? 3 : 0);
  static constexpr int kSwzShiftO = (kCPRO == 4) ? 2 : 0;
  static __device__ __forceinline__ int swzo(int row) { return (row >> kSwzShiftO) & kSwzMaskO; }
};

// `waves`: waves per workgroup (4, or 8 for the row-piece kernel on groups of eight heads)
template <typename T, int D, int DV = D>
constexpr int apply16_dma_lds_bytes(int waves = kWavesPerWG) {
  int ring = ApplyDmaCfg<D, DV>::kRing * ApplyDmaCfg<D, DV>::kSlotBytes * waves;
  int st = (ApplyDmaCfg<D, DV>::kRing - 1) * ApplyDmaCfg<D, DV>::kSlotBytes * waves + ApplyDmaCfg<D, DV>::kStageBytes;
  return ring > st ? ring : st;
}

// The state of one head as the apply lanes' matrix-core A operands (see the header comment), written once
// per head by pack_state16 for the kernels whose workgroups would otherwise rebuild it for several heads:
// {c1, alpha_z} then frag[level][t][s][lane], 16 bytes each.
template <typename T, int D> struct Pack16 {
  static constexpr int kHeaderBytes = 256;
  static constexpr int kFrags = NSplit<T>::value * Shape16<D>::kMT2 * Shape16<D>::kKS;   // per lane
  static constexpr int kHeadBytes = kHeaderBytes + kFrags * 64 * 16;
};

template <int N> LF_DEV void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// One workgroup's apply work on one head: construct, prefetch(), run().
//
// ROWS_W = W > 0 (4 or 8; for layouts in which the W heads h0..h0+W-1 of a token are neighbours in memory,
// so that a token row of the group is one contiguous piece of W d elements): a workgroup of W waves works
// on the W heads at once, wave w computing head h0 + w, and all waves walk the same tiles.  A ring slot
// then spans the waves' regions and holds a tile of whole row pieces: wave w copies in (and later stores)
// token rows (32 / W) w .. + 32 / W - 1 of the tile, all heads of them -- contiguous W d-element pieces
// instead of W scattered d-element ones -- and two workgroup barriers per tile separate "pieces have
// landed" -> "each wave reads and overwrites its head's columns" -> "pieces leave".  Inside a row piece
// the 16-byte chunks are rotated by a row-dependent amount (both ways) so that the token-per-lane
// accesses to one head's columns are bank-conflict free.  Use: construct with the group's pointers,
// prefetch(), load_packed() with the wave's own head (operands prepared by pack_state16), stream().
//
// MLP (row-piece mode with the workgroup covering whole token rows, C = W D channels): the query is not read
// but formed per element as  a + LeakyReLU(LayerNorm_C(t)),  the sum of the two branches of f' (Sec. 3.1 (Implementation Details)), from
// the branch results `a` (through the ring at offset 0) and `t` (through a second ring behind it).  The row
// statistics come from the tile in LDS: every lane reduces the channels it holds of its token (mean and
// centred sum of squares, exact in two passes over registers), the 2 W pieces per token meet in LDS and are
// merged with the pairwise-variance formula -- one more workgroup barrier per tile, no extra memory pass.
// MLP with PRE (for shapes whose token rows do not fit one workgroup; per-head mode, or row-piece mode on a group of
// W of the row's heads): the row statistics were computed by an earlier kernel, {rstd, -mean rstd} per token; a
// tile's 32 pairs travel with its copies as one more deposit (256 bytes used) into a third ring (row-piece mode:
// every wave brings the same pairs to the same place, one deposit per slot).
// WPW: waves per workgroup in per-head mode (each wave streams on its own, so any count works; 4 where the
// workgroup stages the fp32 state together, fewer for the short-lived workgroups of apply16_packed).
template <typename T, int D, int FM, bool NORM, int ROWS_W = 0, bool MLP = false, int DV = D, bool PRE = false,
          int WPW = kWavesPerWG>
struct ApplyDma {
  static constexpr bool ROWS = ROWS_W > 0;
  static_assert(!MLP || ROWS || PRE, "the two-branch input needs whole token rows in one workgroup, or their statistics");
  static_assert(!PRE || (MLP && DV == D), "precomputed row statistics serve the two-branch kernels");
  static_assert(DV == D || !ROWS, "unequal query and value widths run on the per-head kernel only");
  static constexpr int W = ROWS ? ROWS_W : WPW;   // waves per workgroup
  static constexpr int NT = 64 * W;
  using Sh = Shape16<D>;
  using Cfg = ApplyDmaCfg<D, DV>;
  static constexpr int NS = NSplit<T>::value;
  // fp16 + elu+1 on stored queries: rows whose channels are all very negative are shifted (see compute_tile)
  static constexpr bool kShiftRows = NSplit<T>::value == 1 && FM == kPhiEluPlusOne && !MLP;
  static constexpr float kSmallDen = 64.0f * D;   // see compute_tile
  // k-steps and chunks follow the query width D, output tiles and channels per half-wave the value width DV
  static constexpr int KS = Sh::kKS, MT2 = Shape16<DV>::kMT2, CPR = Sh::kChunksPerRow, HALF = Shape16<DV>::kHalf;
  static constexpr int NL = Cfg::kNL, NLO = Cfg::kNLO, NE = D * DV + D, R = Cfg::kRing;
  static_assert(R == 3, "the wait counts below are written for a ring of three slots");
  // ROWS: chunks per row piece, and the rotation that spreads 16 consecutive tokens over the 16
  // sixteen-byte bank groups: row r is rotated by (r * G >> 4) % G chunks, G = gcd(PC, 16)
  static constexpr int PC = W * CPR;
  static constexpr int G = (PC % 16 == 0) ? 16 : ((PC % 8 == 0) ? 8 : 4);
  static constexpr int RPR = kTile / W;   // token rows per wave region
  static_assert(!ROWS || (PC % 4 == 0 && RPR * G >= 16 && kTile % W == 0), "rotation classes must fit a region");
  static constexpr int kStageOffset = (R - 1) * W * Cfg::kSlotBytes;
  static constexpr int NLC = MLP ? 2 * NL + (PRE ? 1 : 0) : NL;  // copy instructions per tile
  static constexpr int kTOffset = R * W * Cfg::kSlotBytes;        // MLP: ring of the LayerNorm branch's tiles
  static constexpr int kPartOffset = 2 * R * W * Cfg::kSlotBytes; // MLP: (mean, M2) per (wave, half, token)
  static constexpr int kStatOffset = 2 * R * W * Cfg::kSlotBytes; // PRE: ring of 1 KiB deposits, {rstd, cn} per token
  static __device__ __forceinline__ int rot(int r) { return ((r * G) >> 4) & (G - 1); }

  const u32x4* Qh;
  u32x4* Oh;
  long long N;
  unsigned char* smem;
  int rs_q, rs_o;
  int lane, wave, tok, kg, row_byte, tsw;   // ROWS: row_byte = byte offset of the token's piece in a slot block,
                                            //       tsw = first chunk of this wave's head + the row's rotation
  int row_byte_o, tsw_o;                    // the same two for the row that leaves (differ when DV != D)
  // LDS position p = 64 u + lane of a slot holds the chunk of token row trow[u] that lies qoff[u]
  // (in Q) / ooff[u] (in out) vector units after the tile's first row
  int trow[NL], qoff[NL], ooff[NLO], trow_o[NLO];
  // ROWS: stores go out in memory order (whole 128-byte lines per instruction); lane (u, l) then fetches its
  // chunk from byte soff[u] of the wave's slot region
  int soff[ROWS ? NL : 1];
  TileIter it, ahead;
  u32x4 A[NSplit<T>::value][Shape16<DV>::kMT2][Shape16<D>::kKS];   // this wave's state operands
  float c1, eps_s, c1_az;   // c1_az: alpha_z, kept for save_packed
  // MLP: the LayerNorm branch's tensor, the affine of this lane's channels, and the two scalars
  const u32x4* Th;
  const u32x4* St;   // PRE: the batch's row statistics, two tokens per 16 bytes (readable up to a whole last tile)
  float gam[MLP ? Shape16<D>::kKS * 8 : 1], bet[MLP ? Shape16<D>::kKS * 8 : 1];
  float ln_eps, slope;

  // `Qh_`, `Oh_`: first token row of this head; `rs_q_`, `rs_o_`: row strides in 16-byte units
  LF_DEV ApplyDma(const u32x4* Qh_, int rs_q_, u32x4* Oh_, int rs_o_, long long N_, int tiles_per_block, int wg,
                  int nwg, unsigned char* smem_)
      : Qh(Qh_), Oh(Oh_), N(N_), smem(smem_), rs_q(rs_q_), rs_o(rs_o_),
        lane(threadIdx.x & 63), wave(__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)),
        it(wg, nwg, ROWS ? 0 : wave, tiles_per_block, (N_ + kTile - 1) / kTile, ROWS ? 1 : WPW),
        ahead(it) {
    tok = lane & 31;
    kg = lane >> 5;
    if constexpr (ROWS) {
      row_byte = (tok / RPR) * Cfg::kSlotBytes + (tok % RPR) * PC * 16;
      tsw = wave * CPR + rot(tok);
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        const int P = wave * Cfg::kChunks + u * 64 + lane;   // position in the tile of row pieces
        const int r = P / PC;
        int c = P % PC - rot(r);
        if (c < 0) c += PC;
        // lanes past the region's chunks copy what the lane 32 below copies (same cache lines, no extra request:
        // re-reading one fixed chunk instead measured 5 % slower) and deposit it in the padding; never stored
        static_assert(Cfg::kChunks % 32 == 0, "a region is whole half-waves of chunks");
        const int Pc = (u * 64 + lane < Cfg::kChunks) ? P : P - 32;
        const int rc = Pc / PC;
        int cc = Pc % PC - rot(rc);
        if (cc < 0) cc += PC;
        trow[u] = rc;
        qoff[u] = rc * rs_q + cc;
        const int cs = P % PC;               // store side: this lane takes chunk cs of row r ...
        int pos = cs + rot(r);               // ... which sits at this rotated position of the row piece
        if (pos >= PC) pos -= PC;
        ooff[u] = r * rs_o + cs;
        trow_o[u] = r;
        soff[u] = ((r % RPR) * PC + pos) * 16;
      }
      row_byte_o = row_byte;
      tsw_o = tsw;
    } else {
      row_byte = tok * Cfg::kRowBytes;
      tsw = Cfg::swz(tok);
      row_byte_o = tok * Cfg::kRowBytesO;
      tsw_o = Cfg::swzo(tok);
#pragma unroll
      for (int u = 0; u < NL; ++u) {
        const int p = u * 64 + lane;
        const int r = p / CPR, pos = p % CPR;
        trow[u] = r;
        qoff[u] = r * rs_q + (pos ^ Cfg::swz(r));
      }
#pragma unroll
      for (int u = 0; u < NLO; ++u) {
        const int p = u * 64 + lane;
        const int r = p / Cfg::kCPRO, pos = p % Cfg::kCPRO;
        trow_o[u] = r;
        ooff[u] = r * rs_o + (pos ^ Cfg::swzo(r));
      }
    }
  }

  // MLP: `Th_` addresses the LayerNorm branch like Qh the linear one (same row stride); gamma, beta: the
  // affine of the group's W D channels.  Call before prefetch().
  LF_DEV void set_mlp(const u32x4* Th_, const float* gamma, const float* beta, float ln_eps_, float slope_) {
    Th = Th_;
    ln_eps = ln_eps_;
    slope = slope_;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const int chunk = kg * KS + s;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int ch = (ROWS ? wave * D : 0) + chunk * 8 + e;
        gam[s * 8 + e] = chunk < CPR ? gamma[ch] : 0.0f;
        bet[s * 8 + e] = chunk < CPR ? beta[ch] : 0.0f;
      }
    }
  }

  LF_DEV void set_stats(const void* stats) { St = reinterpret_cast<const u32x4*>(stats); }

  // this wave's region of ring slot `slot`: what it copies in and stores from
  LF_DEV unsigned char* slot_ptr(int slot) const { return smem + (slot * W + wave) * Cfg::kSlotBytes; }
  // where this lane finds (and overwrites) 16-byte chunk `chunk` of its token's head row in slot `slot`
  LF_DEV unsigned char* chunk_ptr(int slot, int chunk) const {
    if constexpr (ROWS) {
      int x = tsw + chunk;
      if (x >= PC) x -= PC;
      return smem + slot * W * Cfg::kSlotBytes + row_byte + (x << 4);
    } else {
      return slot_ptr(slot) + row_byte + ((chunk ^ tsw) << 4);
    }
  }
  // the same for the row that leaves (the finished tile takes the place of the tile that came in)
  LF_DEV unsigned char* out_chunk_ptr(int slot, int chunk) const {
    if constexpr (DV == D) return chunk_ptr(slot, chunk);
    else return slot_ptr(slot) + row_byte_o + ((chunk ^ tsw_o) << 4);
  }

  // copies tile `tile` into ring slot `slot`; always issues exactly NLC vector memory instructions
  LF_DEV void issue_copy(long long tile, int slot) {
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;   // valid token rows
    const u32x4* qp = Qh + tile * kTile * rs_q;
    unsigned char* sl = slot_ptr(slot);
#pragma unroll
    // Every lane issues every copy, as straight-line code.  (A lane-masked copy is a branch to the compiler,
    // which may sink two masked copies into one instruction whose scalar LDS base then depends on the lane --
    // wrong deposits -- and which changes the number of instructions a wave issues, on which the wait counts
    // below rely.)  Lanes past the tile's chunks re-read chunk 0 and deposit it in the slot's padding (slots
    // are whole 1 KiB deposits); rows past N re-read chunk 0 and are never stored.
    for (int u = 0; u < NL; ++u) {
      const int c = trow[u] < lim ? qoff[u] : 0;
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
    }
    if constexpr (PRE) {
      // lanes 0..15 bring the tile's 32 pairs, the others repeat them into the deposit's unused part
      const u32x4* sp = St + tile * (kTile / 2) + (lane & 15);
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)sp,
                                       (LF_LDS void*)(smem + kStatOffset + (ROWS ? slot : slot * W + wave) * 1024), 16, 0, 0);
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
  // COHERENT: the state was written by other workgroups of the same launch (single-launch kernel) and
  // must be read past this XCD's L2; otherwise an earlier kernel wrote it and plain wide loads do.
  template <bool COHERENT = false>
  LF_DEV void run(const float* state, float eps) {
    load_state<COHERENT>(state, eps, true);
    stream();
  }

  // This wave's operands from what pack_state16 wrote for its head.
  LF_DEV void load_packed(const unsigned char* packed, float eps) {
    const u32x4* frag = reinterpret_cast<const u32x4*>(packed + Pack16<T, D>::kHeaderBytes);
#pragma unroll
    for (int l = 0; l < NS; ++l)
#pragma unroll
      for (int t = 0; t < MT2; ++t)
#pragma unroll
        for (int s = 0; s < KS; ++s) A[l][t][s] = frag[((l * MT2 + t) * KS + s) * 64 + lane];
    const float* scales = reinterpret_cast<const float*>(packed);
    c1 = scales[0];
    eps_s = eps * scales[1];
  }

  // Writes this wave's operands where load_packed finds them (`out`: one head's Pack16 record).
  LF_DEV void save_packed(unsigned char* out, bool header) const {
    u32x4* frag = reinterpret_cast<u32x4*>(out + Pack16<T, D>::kHeaderBytes);
#pragma unroll
    for (int l = 0; l < NS; ++l)
#pragma unroll
      for (int t = 0; t < MT2; ++t)
#pragma unroll
        for (int s = 0; s < KS; ++s) frag[((l * MT2 + t) * KS + s) * 64 + lane] = A[l][t][s];
    if (header && lane == 0) {
      float* scales = reinterpret_cast<float*>(out);
      scales[0] = c1;
      scales[1] = c1_az;
    }
  }

  // Whole workgroup: stages one head's state in LDS; the waves with `keep` build their operands from it.
  // STAGED: the state already lies in the staging area (the workgroup computed it itself), S row-major as in
  // memory; `state` is not read.  Otherwise S is staged transposed -- st[col * D + ch], then z[ch] -- so that the
  // eight consecutive feature channels of one output column that make up a lane's operand are two 16-byte LDS
  // reads, all of them issued before the first is used (read one by one, row-major, with the slot tests around
  // each read, the operand build took 3-5 us per workgroup: a fifth of a small call).
  template <bool COHERENT = false, bool STAGED = false>
  LF_DEV void load_state(const float* state, float eps, bool keep) {
    // ---- prologue: state -> LDS, maxima, power-of-two scales, A fragments -------------------------
    float* st = reinterpret_cast<float*>(smem + kStageOffset);
    float* redmax = st + NE;
    float mS = 0.0f, mz = 0.0f;
    static_assert(NE % 4 == 0 && (D * DV) % 4 == 0 && DV % 4 == 0, "the state is moved four floats of one row at a time");
    for (int e = threadIdx.x; e < NE / 4; e += NT) {
      f32x4 x;
      if constexpr (STAGED) {
        x = reinterpret_cast<const f32x4*>(st)[e];
      } else if constexpr (COHERENT) {
        x = f32x4{ld_agent(state + 4 * e), ld_agent(state + 4 * e + 1), ld_agent(state + 4 * e + 2),
                  ld_agent(state + 4 * e + 3)};
      } else {
        x = reinterpret_cast<const f32x4*>(state)[e];
      }
      if constexpr (!STAGED) {
        if (e < D * DV / 4) {
          const int ch = (4 * e) / DV, col = (4 * e) % DV;
#pragma unroll
          for (int i = 0; i < 4; ++i) st[(col + i) * D + ch] = x[i];
        } else {
          reinterpret_cast<f32x4*>(st)[e] = x;
        }
      }
      const float m4 = fmaxf(fmaxf(fabsf(x[0]), fabsf(x[1])), fmaxf(fabsf(x[2]), fabsf(x[3])));
      if (e < D * DV / 4) mS = fmaxf(mS, m4); else mz = fmaxf(mz, m4);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      mS = fmaxf(mS, __shfl_xor(mS, o));
      mz = fmaxf(mz, __shfl_xor(mz, o));
    }
    if (lane == 0) { redmax[wave] = mS; redmax[W + wave] = mz; }
    __syncthreads();
    mS = 0.0f; mz = 0.0f;
#pragma unroll
    for (int w = 0; w < W; ++w) { mS = fmaxf(mS, redmax[w]); mz = fmaxf(mz, redmax[W + w]); }
    const float aS = pow2_scale_for(mS);
    const float az = NORM ? pow2_scale_for(mz) : 1.0f;
    if (keep) {
      c1 = az / aS;
      eps_s = eps * az;
      c1_az = az;
      const int m = lane & 31;
      const int hv = (m >> 2) & 1;
      // per output tile: the raw fp32 values of its fragments first (unconditional reads from clamped, valid
      // places), then the arithmetic
#pragma unroll
      for (int t = 0; t < MT2; ++t) {
        const int slot = 16 * t + 4 * (m >> 3) + (m & 3);
        const bool isS = slot < HALF;
        const bool isZ = NORM && slot == HALF, zrem = NORM && slot == HALF + 1;
        const int col = isS ? hv * HALF + slot : 0;
        const float sc = isS ? aS : az;
        float raw[KS][8];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const int chunk = kg * KS + s;
          const int ch0 = (chunk < CPR ? chunk : 0) * 8;
          if constexpr (STAGED) {
#pragma unroll
            for (int j = 0; j < 8; ++j) raw[s][j] = isS ? st[(ch0 + j) * DV + col] : st[D * DV + ch0 + j];
          } else {
            const float* src = isS ? st + col * D + ch0 : st + D * DV + ch0;
            const f32x4 lo4 = *reinterpret_cast<const f32x4*>(src);
            const f32x4 hi4 = *reinterpret_cast<const f32x4*>(src + 4);
#pragma unroll
            for (int j = 0; j < 4; ++j) { raw[s][j] = lo4[j]; raw[s][4 + j] = hi4[j]; }
          }
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const bool used = (kg * KS + s < CPR) && (isS || isZ || zrem);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            float hi2[2], lo2[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
              const float x = used ? raw[s][2 * w + q] * sc : 0.0f;
              float r0, r1;
              unpack2<T>(pack2<T>(x, 0.0f), r0, r1);   // x rounded once to 16 bits
              hi2[q] = zrem ? x - r0 : x;
              lo2[q] = isS ? x - r0 : 0.0f;            // S' remainder -> lo fragment (bf16 only)
            }
            A[0][t][s][w] = pack2<T>(hi2[0], hi2[1]);
            if constexpr (NS == 2) A[1][t][s][w] = pack2<T>(lo2[0], lo2[1]);
          }
        }
      }
    }
    __syncthreads();   // the staged state is dead: the third slot block may be filled from here on
  }

  // Per-head mode: each wave streams on its own.
  LF_DEV void stream() {
    if constexpr (ROWS) { stream_rows(); return; }
    int slot = 0;
    int iter = 0;
    while (it.valid()) {
      const long long tile = it.t;
      int aslot = slot + (R - 1);
      if (aslot >= R) aslot -= R;
      if (ahead.valid()) {
        issue_copy(ahead.t, aslot);
        // issue order is  C0 C1 | C2 W0 S0 | C3 W1 S1 | C4 W2 S2 | ...  (C copies of NLC, S stores of NLO
        // instructions, W wait): after tile j's copies come C(j+1), C(j+2) and the stores S(j-2), S(j-1)
        if (iter == 0) wait_vmcnt<2 * NLC>();
        else if (iter == 1) wait_vmcnt<2 * NLC + NLO>();
        else wait_vmcnt<2 * NLC + 2 * NLO>();
      } else {
        wait_vmcnt<0>();
      }
      iter = iter < 2 ? iter + 1 : 2;
      compute_tile(slot);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      store_tile(tile, slot);
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      it.next();
      ahead.next();
      slot = slot + 1 == R ? 0 : slot + 1;
    }
  }

  // Row-piece mode: the waves move in step, one workgroup barrier per tile.  Iteration j: store tile
  // j-1 (complete since the last barrier), copy tile j+2 into the slot that frees, compute tile j,
  // wait for this wave's rows of tile j+1, barrier ("tile j computed by all, tile j+1 landed for all").
  // Issue order per wave:  C0 C1 [state] | C2 K0 w | S0 C3 K1 w | S1 C4 K2 w | ...  so after tile j+1's
  // copies come S(j-1) and C(j+2), where they exist.
  LF_DEV void stream_rows() {
    {   // this wave's rows of the first tile: only the second tile's copies were issued after them
      TileIter second = it;
      second.next();
      if (second.valid()) wait_vmcnt<NLC>();
      else wait_vmcnt<0>();
    }
    lds_barrier();
    int slot = 0, prev_slot = 0;
    long long prev_tile = -1;
    while (it.valid()) {
      const long long tile = it.t;
      const bool have_prev = prev_tile >= 0;
      if (have_prev) store_tile(prev_tile, prev_slot);
      const bool copied = ahead.valid();
      if (copied) issue_copy(ahead.t, have_prev ? prev_slot : R - 1);
      compute_tile(slot);
      it.next();
      ahead.next();
      if (it.valid()) {
        if (have_prev && copied) wait_vmcnt<NL + NLC>();
        else if (copied) wait_vmcnt<NLC>();
        else if (have_prev) wait_vmcnt<NL>();
        else wait_vmcnt<0>();
      }
      lds_barrier();
      prev_tile = tile;
      prev_slot = slot;
      slot = slot + 1 == R ? 0 : slot + 1;
    }
    if (prev_tile >= 0) store_tile(prev_tile, prev_slot);
  }

  // B operands of this lane's token from ring slot `slot`, products with the state operands, normalizer,
  // and the finished channels back into the same places of the slot
  LF_DEV void compute_tile(int slot) {
    // ---- this lane's token row -> phi -> 16-bit B operands ----------------------------------------
    u32x4 Bh[KS], Bl[KS];
    u32x4 traw[MLP ? KS : 1];      // MLP: this lane's chunks of t, raw
    float rstd = 0.0f, cn = 0.0f;   // MLP: LayerNorm(t) = t * rstd + cn
    if constexpr (PRE) {
      const f32x2 rc =
          *reinterpret_cast<const f32x2*>(smem + kStatOffset + (ROWS ? slot : slot * W + wave) * 1024 + tok * 8);
      rstd = rc[0];
      cn = rc[1];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        traw[s] = u32x4{0, 0, 0, 0};
        if (kg * KS + s < CPR) traw[s] = *reinterpret_cast<const u32x4*>(chunk_ptr(slot, kg * KS + s) + kTOffset);
      }
    } else if constexpr (MLP) {
      // ---- LayerNorm statistics of this lane's token over all W D channels: sums of (t - pivot) and of its
      //      square, the pivot being the token's channel 0 (the same for all lanes of the token, so the
      //      pieces simply add; deviations are small next to a large common offset, so nothing cancels) ----
      const uint16_t pv16 = *reinterpret_cast<const uint16_t*>(smem + slot * W * Cfg::kSlotBytes + kTOffset +
                                                               row_byte + (rot(tok) << 4));
      float pivot, pivot_unused;
      unpack2<T>((uint32_t)pv16, pivot, pivot_unused);
      float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const bool ok = kg * KS + s < CPR;
        u32x4 raw = u32x4{0, 0, 0, 0};
        if (ok) raw = *reinterpret_cast<const u32x4*>(chunk_ptr(slot, kg * KS + s) + kTOffset);
        traw[s] = raw;
        if constexpr (NS == 1) {
          // fp16: for the two sums the difference is taken in packed half precision (its rounding is relative
          // to the deviation and averages out) and accumulated by the mixed-precision dot product
          const f16x2 np = __builtin_bit_cast(f16x2, (uint32_t)(pv16 ^ 0x8000u) * 0x10001u);
          const f16x2 one = __builtin_bit_cast(f16x2, 0x3C003C00u);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t word = raw[w];   // (by value: a bit cast applied to the vector element itself reads element 0)
            const f16x2 dd = __builtin_bit_cast(f16x2, word) + np;   // feeds the statistics only
            if (ok) {
              s1 = __builtin_amdgcn_fdot2(dd, one, s1, false);
              s2 = __builtin_amdgcn_fdot2(dd, dd, s2, false);
            }
          }
        } else {
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            float t0, t1;
            unpack2<T>(raw[w], t0, t1);
            t0 -= pivot;
            t1 -= pivot;
            if (ok) {
              s1 += t0 + t1;
              s2 = __builtin_fmaf(t0, t0, __builtin_fmaf(t1, t1, s2));
            }
          }
        }
      }
      f32x2* part = reinterpret_cast<f32x2*>(smem + kPartOffset);
      part[(wave * 2 + kg) * kTile + tok] = f32x2{s1, s2};
      lds_barrier();
      s1 = 0.0f;
      s2 = 0.0f;
#pragma unroll
      for (int i = 0; i < 2 * W; ++i) {
        const f32x2 pp = part[i * kTile + tok];
        s1 += pp[0];
        s2 += pp[1];
      }
      const float mu = s1 * (1.0f / (float)(W * D));           // mean of t - pivot
      const float var = fmaxf(__builtin_fmaf(-mu, mu, s2 * (1.0f / (float)(W * D))), 0.0f);
      rstd = __builtin_amdgcn_rsqf(var + ln_eps);
      cn = -(pivot + mu) * rstd;
    }
    // fp16, elu+1: a token whose channels are all far below zero has phi(q) = exp(q) below fp16's normal range
    // (bits are lost below -10, everything below -17), although only the ratios between its channels matter.
    // Such a token shows in its (scaled) denominator, which is then tiny: z' is scaled to about 2^14, so every row
    // whose largest phi(q) is below 2^-8 has den' < 64 d.  Where a tile holds such a row the wave goes through the
    // tile a second time and evaluates those rows as exp(q - m), m = the row's largest channel: the factor exp(-m)
    // cancels between numerator and denominator once eps carries it too.  Ordinary tiles take one round and pay a
    // compare.  (Without the normalizer nothing signals the case, so there every row is treated that way and the
    // factor is taken out again at the end.)
    float qc = 0.0f;   // this lane's row is evaluated times 2^qc
    auto row_shift = [&](const u32x4* raw) {      // -log2(e) * min(largest channel of the lane's token, 0)
      f16x2 m2 = __builtin_bit_cast(f16x2, LowestBits<F16>::value);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        if (kg * KS + s < CPR) {
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t word = raw[s][w];
            m2 = __builtin_elementwise_max(m2, __builtin_bit_cast(f16x2, word));
          }
        }
      }
      float m = fmaxf((float)m2[0], (float)m2[1]);
      m = fmaxf(m, __shfl_xor(m, 32));          // the token's other half of the channels
      return fminf(m, 0.0f) * -1.44269504088896340736f;
    };
    f32x16 acc[MT2];
    float den = 0.0f;
    // B operands of the lane's token (each row times 2^c) and the products with the state operands
    auto products = [&](const bool shift, const bool only_small) {
      u32x4 qraw[KS];
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        qraw[s] = u32x4{0, 0, 0, 0};
        if (kg * KS + s < CPR) qraw[s] = *reinterpret_cast<const u32x4*>(chunk_ptr(slot, kg * KS + s));
      }
      if (shift) {
        const float sh = row_shift(qraw);      // (all lanes take part: it exchanges values between them)
        qc = (!only_small || den < kSmallDen) ? sh : 0.0f;
      }
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int chunk = kg * KS + s;
        const bool ok = chunk < CPR;
        const u32x4 raw = qraw[s];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          float x0, x1;
          unpack2<T>(raw[w], x0, x1);
          if constexpr (MLP) {
            float t0, t1;
            unpack2<T>(traw[s][w], t0, t1);
            const float y0 = __builtin_fmaf(gam[s * 8 + 2 * w], __builtin_fmaf(t0, rstd, cn), bet[s * 8 + 2 * w]);
            const float y1 = __builtin_fmaf(gam[s * 8 + 2 * w + 1], __builtin_fmaf(t1, rstd, cn), bet[s * 8 + 2 * w + 1]);
            x0 += fmaxf(y0, slope * y0);   // LeakyReLU for slopes up to one
            x1 += fmaxf(y1, slope * y1);
          }
          if constexpr (NS == 1 && !MLP) {
            const uint32_t r = shift ? phi_pack2_scaled<T, FM>(raw[w], qc) : phi_pack2<T, FM>(raw[w]);
            Bh[s][w] = ok ? r : 0u;
            continue;
          }
          float r0 = ok ? (shift ? phi_scaled<FM>(x0, qc) : phi<FM>(x0)) : 0.0f;
          float r1 = ok ? (shift ? phi_scaled<FM>(x1, qc) : phi<FM>(x1)) : 0.0f;
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
      if constexpr (NORM) den = acc[HALF / 16][HALF % 16] + acc[(HALF + 1) / 16][(HALF + 1) % 16];
    };
    if constexpr (kShiftRows && !NORM) {
      products(true, false);
    } else {
      products(false, false);
      if constexpr (kShiftRows) {
        if (__builtin_amdgcn_ballot_w64(den < kSmallDen) != 0) products(true, true);   // rare: a second round
      }
    }
    float scale = c1;
    if constexpr (NORM) {
      float eps_row = eps_s;
      if constexpr (kShiftRows) eps_row = eps_s * __builtin_amdgcn_exp2f(qc);   // (inf for a row of -65504s: out = 0)
      scale = c1 * __builtin_amdgcn_rcpf(den + eps_row);
    } else if constexpr (kShiftRows) {
      scale = c1 * __builtin_amdgcn_exp2f(-qc);   // nothing cancels without the normalizer: take the factor out again
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
        *reinterpret_cast<u32x4*>(out_chunk_ptr(slot, chunk)) = w;
      }
    } else {
      static_assert(HALF % 8 == 0 || Cfg::kSwzMaskO == 0, "64-bit pieces assume whole chunks stay together");
#pragma unroll
      for (int c = 0; c < HALF / 4; ++c) {
        u32x2 w;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int s0 = c * 4 + 2 * e;
          w[e] = pack2<T>(acc[s0 / 16][s0 % 16] * scale, acc[(s0 + 1) / 16][(s0 + 1) % 16] * scale);
        }
        const int byte = kg * (HALF * 2) + c * 8;   // offset inside the head's row
        *reinterpret_cast<u32x2*>(out_chunk_ptr(slot, byte >> 4) + (byte & 15)) = w;
      }
    }
  }

  // coalesced stores of a finished tile; always NLO instructions (lanes without a valid chunk are masked)
  LF_DEV void store_tile(long long tile, int slot) {
    const unsigned char* sl = slot_ptr(slot);
    long long rem = N - tile * kTile;
    const int lim = rem < kTile ? (int)rem : kTile;
    u32x4* op = Oh + tile * kTile * rs_o;
#pragma unroll
    for (int u = 0; u < NLO; ++u) {
      int from = u * 1024 + lane * 16;
      if constexpr (ROWS) from = soff[u];
      const u32x4 w = *reinterpret_cast<const u32x4*>(sl + from);
      if (u * 64 + lane < Cfg::kChunksO && trow_o[u] < lim) st_stream(op + ooff[u], w);
    }
  }
};

template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply16_dma(const u32x4* __restrict__ Q, Layout lq, u32x4* __restrict__ O, Layout lo, HeadSubset hs,
            const float* __restrict__ state, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = hs.bh(blockIdx.y, lq.H);
  ApplyDma<T, D, FM, NORM> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N, tiles_per_block, blockIdx.x,
                              gridDim.x, smem);
  ap.prefetch();
  ap.run(state + bh * (D * D + D), eps);
}

// apply16_dma with the head's operands prepared by pack_state16: a workgroup's start-up is a few coalesced
// loads instead of staging and packing the fp32 state, so a launch can use many short-lived workgroups
// (each a few tiles), which the hardware deals out in order: the chip then reads and writes one narrow
// moving window of memory, which the write stream in particular rewards.
template <typename T, int D, int FM, bool NORM, int WPW>
__global__ void __launch_bounds__(64 * WPW)
apply16_packed(const u32x4* __restrict__ Q, Layout lq, u32x4* __restrict__ O, Layout lo, HeadSubset hs,
               const unsigned char* __restrict__ packed, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = hs.bh(blockIdx.y, lq.H);
  ApplyDma<T, D, FM, NORM, 0, false, D, false, WPW> ap(Q + lq.slice(bh), lq.row, O + lo.slice(bh), lo.row, N,
                                                       tiles_per_block, blockIdx.x, gridDim.x, smem);
  ap.prefetch();
  ap.load_packed(packed + bh * Pack16<T, D>::kHeadBytes, eps);
  ap.stream();
}

// Apply on groups of W (4 or 8) neighbouring heads (see ROWS_W above).  grid = (wgs, B * groups_per_batch),
// block = 64 W: workgroup (x, y) takes heads W (y % gpb) .. + W - 1 of batch y / gpb.  Heads beyond the last
// whole group are left to apply16_dma.
template <typename T, int D, int FM, bool NORM, int W>
__global__ void __launch_bounds__(64 * W)
apply16_rows(const u32x4* __restrict__ Q, Layout lq, u32x4* __restrict__ O, Layout lo, int groups_per_batch,
             const unsigned char* __restrict__ packed, float eps, long long N, int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long b = blockIdx.y / groups_per_batch;
  const long long h0 = (long long)(blockIdx.y % groups_per_batch) * W;
  ApplyDma<T, D, FM, NORM, W> ap(Q + (b * lq.batch + h0 * lq.head), lq.row, O + (b * lo.batch + h0 * lo.head), lo.row,
                                 N, tiles_per_block, blockIdx.x, gridDim.x, smem);
  ap.prefetch();
  ap.load_packed(packed + (b * lq.H + h0 + wave) * Pack16<T, D>::kHeadBytes, eps);
  ap.stream();
}

// Operand-ready state for apply16_rows.  grid = (B*H), block = 256: the workgroup builds the head's operands
// with the per-head kernel's own prologue (one wave's registers hold them all) and wave 0 writes them out.
template <typename T, int D, bool NORM>
__global__ void __launch_bounds__(kThreads)
pack_state16(const float* __restrict__ state, unsigned char* __restrict__ packed) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.x;
  ApplyDma<T, D, 0, NORM> ap(nullptr, 0, nullptr, 0, 0, kWavesPerWG, 0, 1, smem);
  ap.load_state(state + bh * (D * D + D), 0.0f, ap.wave == 0);
  if (ap.wave == 0) ap.save_packed(packed + bh * Pack16<T, D>::kHeadBytes, true);
}

}  // namespace lf
