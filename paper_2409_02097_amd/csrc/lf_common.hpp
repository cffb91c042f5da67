// Shared device-side helpers for the gfx950 LinFusion kernels: vector types, 16-bit
// conversions, the feature map phi (Sec. 2.3: non-negative activation on Q and K), and the
// shape constants that the state-reduction, combine and apply kernels must agree on.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lf {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kPhiEluPlusOne = 0;
constexpr int kPhiRelu = 1;
constexpr int kPhiIdentity = 2;

struct F16 {};   // tag: IEEE binary16 storage
struct BF16 {};  // tag: bfloat16 storage

#define LF_DEV __device__ __forceinline__
#define LF_LDS __attribute__((address_space(3)))

// ---- feature map -------------------------------------------------------------------------
// elu(x)+1 = x+1 for x > 0, exp(x) otherwise.  exp(x) = 2^(x*log2 e) on the hardware exp2
// unit; `Precise` adds the rounding error of the product back as a first-order correction
// (used on the fp32 path, whose tolerance is 1e-5).
template <int FM, bool Precise = false>
LF_DEV float phi(float x) {
  if constexpr (FM == kPhiEluPlusOne) {
    constexpr float kLog2e = 1.44269504088896340736f;
    float t = x * kLog2e;
    float e = __builtin_amdgcn_exp2f(t);
    if constexpr (Precise) {
      // t_err = x*log2e - t (exactly, via fma) plus the part of log2e that fp32 drops.
      float terr = __builtin_fmaf(x, kLog2e, -t) + x * 1.92596299112661746e-8f;
      e = __builtin_fmaf(e, terr * 0.69314718055994530942f, e);
    }
    return x > 0.0f ? x + 1.0f : e;
  } else if constexpr (FM == kPhiRelu) {
    return x > 0.0f ? x : 0.0f;   // NaN maps to 0 like fmax(x, 0)
  } else {
    return x;
  }
}

// elu(x)+1 of a value whose exponential branch is evaluated as exp(x + c / log2 e), i.e. scaled by 2^c: used
// where a whole row (or a whole stream) of inputs is negative and so small that exp(x) itself would leave the
// normal range of fp16; the caller divides the factor out again (or it cancels in a ratio).  c = 0: phi itself.
template <int FM>
LF_DEV float phi_scaled(float x, float c) {
  if constexpr (FM == kPhiEluPlusOne) {
    constexpr float kLog2e = 1.44269504088896340736f;
    const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(x, kLog2e, c));
    return x > 0.0f ? x + 1.0f : e;
  } else {
    return phi<FM>(x);
  }
}

// ---- 16-bit storage <-> fp32 ----------------------------------------------------------------
template <typename T> LF_DEV void unpack2(uint32_t w, float& lo, float& hi);
template <> LF_DEV void unpack2<F16>(uint32_t w, float& lo, float& hi) {
  f16x2 h = __builtin_bit_cast(f16x2, w);
  lo = (float)h[0];
  hi = (float)h[1];
}
template <> LF_DEV void unpack2<BF16>(uint32_t w, float& lo, float& hi) {
  lo = __builtin_bit_cast(float, w << 16);
  hi = __builtin_bit_cast(float, w & 0xffff0000u);
}

// round-to-nearest-even pack of two floats into one 32-bit word (element 0 in the low half)
template <typename T> LF_DEV uint32_t pack2(float lo, float hi);
template <> LF_DEV uint32_t pack2<F16>(float lo, float hi) {
  f16x2 h = {(_Float16)lo, (_Float16)hi};
  return __builtin_bit_cast(uint32_t, h);
}
template <> LF_DEV uint32_t pack2<BF16>(float lo, float hi) {
  bf16x2 h = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, h);
}

// phi of a stored pair, rounded to the storage type again: the word a matrix-core operand takes; the _scaled form
// is phi_scaled on both halves.  fp16 elu(x)+1 goes a shorter way to the same bits: x + 1 in packed fp16 arithmetic
// (the exact sum rounded once, as the fp32 sum rounded to fp16 is: it is exact in fp32 wherever it is not 1 anyway),
// the exponential through fp32 as in phi(), and the choice between them by the sign bit (both give 1 at +-0, and
// callers scale by 2^c only rows or streams without a non-negative element; a NaN stays a NaN on either side) --
// 6 + 2 instructions per pair instead of 11 + 2.
template <typename T, int FM> struct PhiPack2 {
  static LF_DEV uint32_t run(uint32_t w) {
    float x0, x1;
    unpack2<T>(w, x0, x1);
    return pack2<T>(phi<FM>(x0), phi<FM>(x1));
  }
  static LF_DEV uint32_t run_scaled(uint32_t w, float c) {
    float x0, x1;
    unpack2<T>(w, x0, x1);
    return pack2<T>(phi_scaled<FM>(x0, c), phi_scaled<FM>(x1, c));
  }
};
template <> struct PhiPack2<F16, kPhiEluPlusOne> {
  static LF_DEV uint32_t run_scaled(uint32_t w, float c) {
    const float kLog2e = 1.44269504088896340736f;
    const f16x2 x = __builtin_bit_cast(f16x2, w);
    const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
    const uint32_t lin = __builtin_bit_cast(uint32_t, x + one);
    // (written out: left to itself the compiler turns the mask into two compares and selects, and converts before
    //  it multiplies)  t = fma(half, log2 e, c) in one rounding, as the fp32 fma of the converted half is
    float t0, t1;
    uint32_t neg;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel_hi:[1,0,0]" : "=v"(t0) : "v"(w), "v"(kLog2e), "v"(c));
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(t1) : "v"(w), "v"(kLog2e), "v"(c));
    // 0xffff in every negative half (op_sel_hi: the upper half takes its shift count from the constant's lower half too)
    asm("v_pk_ashrrev_i16 %0, 15, %1 op_sel_hi:[0,1]" : "=v"(neg) : "v"(w));
    const uint32_t e = pack2<F16>(__builtin_amdgcn_exp2f(t0), __builtin_amdgcn_exp2f(t1));
    return (e & neg) | (lin & ~neg);
  }
  static LF_DEV uint32_t run(uint32_t w) { return run_scaled(w, 0.0f); }
};
template <typename T, int FM> LF_DEV uint32_t phi_pack2(uint32_t w) { return PhiPack2<T, FM>::run(w); }
template <typename T, int FM> LF_DEV uint32_t phi_pack2_scaled(uint32_t w, float c) { return PhiPack2<T, FM>::run_scaled(w, c); }

// value of a packed pair after rounding, back in fp32 (for hi/lo operand splitting)
template <typename T> LF_DEV void pack2_split(float lo, float hi, uint32_t& w_hi, uint32_t& w_lo) {
  w_hi = pack2<T>(lo, hi);
  float rl, rh;
  unpack2<T>(w_hi, rl, rh);
  w_lo = pack2<T>(lo - rl, hi - rh);
}

// ---- matrix-core wrappers (operands carried as raw 128-bit words) ---------------------------
template <typename T> LF_DEV f32x4 mfma_16x16x32(u32x4 a, u32x4 b, f32x4 c);
template <> LF_DEV f32x4 mfma_16x16x32<F16>(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <> LF_DEV f32x4 mfma_16x16x32<BF16>(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
template <typename T> LF_DEV f32x16 mfma_32x32x16(u32x4 a, u32x4 b, f32x16 c);
template <> LF_DEV f32x16 mfma_32x32x16<F16>(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}
template <> LF_DEV f32x16 mfma_32x32x16<BF16>(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// LDS transposing read: the 16 lanes of a group each name 8 bytes (4 x 16-bit, lane i = row
// i/4, columns 4*(i%4)..+3 of a 4 x 16 block); afterwards lane j of the group holds column j
// of the 4 rows.  Two of them give the 8 contraction-index elements a 16x16x32 operand needs.
LF_DEV u32x2 lds_read_tr16(const uint16_t* p) {
  s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LF_LDS s16x4*)(p));
  return __builtin_bit_cast(u32x2, r);
}

// Workgroup barrier that orders LDS traffic only: the wave's LDS operations are complete before it arrives,
// while its outstanding global loads, stores and LDS copies stay in flight (before __syncthreads() the
// compiler drains every memory counter, which would expose the latency of loads issued just before it).
LF_DEV void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// streaming 128-bit global load / store (non-temporal: the tensors are touched once)
LF_DEV u32x4 ld_stream(const u32x4* p) { return __builtin_nontemporal_load(p); }
LF_DEV void st_stream(u32x4* p, u32x4 v) { __builtin_nontemporal_store(v, p); }
LF_DEV void st_stream(u32x2* p, u32x2 v) { __builtin_nontemporal_store(v, p); }

// Loads / stores of the small fp32 partial states and states that other workgroups (on other XCDs,
// each with its own L2) consume inside the same launch: device-scope relaxed atomics, which go
// through to the device-coherent level instead of staying in the issuing XCD's L2.
LF_DEV void st_agent(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
LF_DEV float ld_agent(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// ---- shape constants of the 16-bit path ---------------------------------------------------
// State reduction tiles the d x d state in 16 x 16 blocks; apply tiles the output in 32-row
// blocks with the two normalizer rows (z hi, z lo) appended after each half of the channels.
template <int D> struct Shape16 {
  static_assert(D % 8 == 0 && D >= 8 && D <= 80, "head width must be a multiple of 8 up to 80");
  static constexpr int kChunksPerRow = D / 8;          // 16-byte chunks per token row
  static constexpr int kMT = (D + 15) / 16;            // 16-wide tiles across d
  static constexpr int kDP = kMT * 16;
  static constexpr bool kSpareCol = (D % 16) != 0;     // a free padded column carries the ones
  // apply: k-steps of 16 channels (lanes 0-31 supply the first 8, lanes 32-63 the second 8)
  static constexpr int kKS = (kChunksPerRow + 1) / 2;
  static constexpr int kHalf = D / 2;                  // output channels held by one half-wave
  static constexpr int kMT2 = (kHalf + 2 + 15) / 16;   // 32-row output tiles incl. normalizer rows
};

// ---- where a (batch, head) slice of a tensor starts and how far apart its token rows are ------
// All in units of one vector access (16 bytes): [B, H, N, d] contiguous has row = d * s / 16,
// head = N * row, batch = H * head; the token-major [B, N, H * d] layout of the UNet has
// row = H * d * s / 16, head = d * s / 16, batch = N * row.  Inside a row the d channels are contiguous.
struct Layout {
  long long batch, head;   // strides between batches / heads
  int row;                 // stride between consecutive tokens of one head
  int H;                   // heads per batch
  LF_DEV long long slice(long long bh) const { return (bh / H) * batch + (bh % H) * head; }
};

// Heads [first, first + count) of every batch: grid row y of a per-head kernel works on
// head first + y % count of batch y / count.  {0, H} = all heads.
struct HeadSubset {
  int first, count;
  LF_DEV long long bh(int y, int H) const { return (long long)(y / count) * H + first + y % count; }
};

// ---- which tiles a wave processes -----------------------------------------------------------
// The tiles of a head are cut into blocks of `blk` consecutive tiles (blk a multiple of the
// waves per workgroup); workgroup g of G takes blocks g, g + G, g + 2G, ... and inside a block its
// waves take tiles round-robin.  blk = ceil(n_tiles / G) gives every workgroup one contiguous
// chunk; a small blk keeps all workgroups of the chip inside one moving window of memory.
// `stride` = 4 with `wave_` = the wave's index is that round-robin; `stride` = 1 with `wave_` = 0 makes a
// wave visit every tile of the workgroup's blocks (used when each wave of a workgroup works on a
// different head over the same token range).
struct TileIter {
  long long t, blk_end, blk_first, n_tiles, step;
  int blk, wave, stride;
  LF_DEV TileIter(int g, int G, int wave_, int blk_, long long n_tiles_, int stride_ = 4)
      : n_tiles(n_tiles_), step((long long)G * blk_), blk(blk_), wave(wave_), stride(stride_) {
    blk_first = (long long)g * blk;
    t = blk_first + wave;
    blk_end = blk_first + blk < n_tiles ? blk_first + blk : n_tiles;
  }
  LF_DEV bool valid() const { return t < n_tiles; }
  LF_DEV void next() {
    t += stride;
    if (t >= blk_end) {
      blk_first += step;
      t = blk_first + wave;
      blk_end = blk_first + blk < n_tiles ? blk_first + blk : n_tiles;
    }
  }
};

template <typename T> struct NSplit;                 // operand levels needed to hold an fp32 value
template <> struct NSplit<F16> { static constexpr int value = 1; };
template <> struct NSplit<BF16> { static constexpr int value = 2; };

// Bit pattern of the most negative finite value of the storage type.  Rows past the end of a head are given this
// value instead of a per-element mask: elu(x)+1 and relu map it to exactly 0 (exp underflows), so such rows add
// nothing to the state; only the identity map (a test aid) still needs the mask.
template <typename T> struct LowestBits;
template <> struct LowestBits<F16> { static constexpr uint32_t value = 0xFBFFFBFFu; };    // -65504
template <> struct LowestBits<BF16> { static constexpr uint32_t value = 0xFF7FFF7Fu; };   // -3.39e38
template <int FM> constexpr bool kPhiKillsLowest = FM != kPhiIdentity;

template <typename T> struct OneBits;                // bit pattern of 1.0 in the storage type
template <> struct OneBits<F16> { static constexpr uint16_t value = 0x3C00; };
template <> struct OneBits<BF16> { static constexpr uint16_t value = 0x3F80; };

}  // namespace lf
