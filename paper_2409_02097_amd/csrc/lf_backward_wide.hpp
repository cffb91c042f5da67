// Backward pass composed of the forward's state reduction and apply kernels and the small kernels below: fp16 at
// head widths above 80 (on the wide kernels) and fp32 at every width it has (on the fp32 kernels).  Same derivative as lf_backward16.hpp (of Eq. 5 applied to Prop. 2's state; Sec. 2.5 (Training Objectives)
// differentiates through every module), evaluated in units of a power of two beta near sum(z) so that every 16-bit
// intermediate is of order one whatever N is:
//   S' = S / beta, z' = z / beta, eps' = eps / beta            (fp32, exact)
//   u'_i  = S' g_i                                             apply(state S'^T, input g, identity map, no normalizer)
//   den'_i = phi(q_i) . z' + eps',  go_i = phi(q_i) . u'_i / den'_i
//   dq_i  = (u'_i - go_i z') / den'_i * phi'(q_i),   gp_i = g_i / den'_i,   e'_i = -go_i / den'_i     (bwdw_q_finish)
//   dS' = sum_i phi(q_i)^T gp_i                                state reduction(K := q, V := gp)
//   dz' = sum_i phi(q_i) e'_i                                  (bwdw_dz)
//   dS = dS' / beta, dz = dz' / beta                           (bwdw_finish_state; fp32, exact)
//   dv_j = dS^T phi(k_j)                                       apply(state dS, input k, phi, no normalizer)
//   t_j  = dS v_j                                              apply(state dS^T, input v, identity map, no normalizer)
//   dk_j = (t_j + dz) * phi'(k_j)                              (bwdw_k_finish)
// Without the normalizer: den' = 1, go = e' = 0, beta = 1.  The temporaries u', gp, t have the tensors' type (fp32
// needs no beta for range, but takes the same route).  At the sizes the wide widths occur in training (the innermost
// UNet levels: tens to a few thousand tokens) the pass is bound by its sixteen launches, not by its fourteen tensor
// passes; it is there so that every level of the UNet, and the fp32 type, has a gradient, not for speed.
#pragma once
#include <type_traits>

#include "lf_backward16.hpp"

namespace lf {

constexpr int kBwdWideThreads = 256;

struct F32 {};   // tag: fp32 storage

// A 16-byte chunk of a token row as floats
template <typename T> struct RowChunk {
  static constexpr int kPer = 8;   // elements per chunk
  using Elem = uint16_t;
  static LF_DEV void load(const u32x4* p, float (&x)[8]) {
    const u32x4 w = *p;
#pragma unroll
    for (int i = 0; i < 4; ++i) unpack2<T>(w[i], x[2 * i], x[2 * i + 1]);
  }
  static LF_DEV void store(u32x4* p, const float (&x)[8]) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = pack2<T>(x[2 * i], x[2 * i + 1]);
    *p = w;
  }
  static LF_DEV float elem(Elem e) {
    float x, unused;
    unpack2<T>((uint32_t)e, x, unused);
    return x;
  }
};
template <> struct RowChunk<F32> {
  static constexpr int kPer = 4;
  using Elem = float;
  static LF_DEV void load(const u32x4* p, float (&x)[4]) {
    const u32x4 w = *p;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t e = w[i];   // (a bit cast applied to the vector element itself read element 0 four times)
      x[i] = __builtin_bit_cast(float, e);
    }
  }
  static LF_DEV void store(u32x4* p, const float (&x)[4]) {
    u32x4 w;
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = __builtin_bit_cast(uint32_t, x[i]);
    *p = w;
  }
  static LF_DEV float elem(Elem e) { return e; }
};
template <typename T, int FM> LF_DEV float bw_phi(float x) {
  if constexpr (std::is_same<T, F32>::value) return phi<FM, true>(x);
  else return phi<FM>(x);
}
constexpr int kBwdStrip = 8;   // rows of the state per workgroup of the two state kernels

// grid = (D / 8, heads), block = 256.  st: {S [D][D], z [D]} fp32 of the head.  Workgroup x writes rows 8 x ..
// 8 x + 7 of tS = {S^T / beta, z / beta} (x = 0: z and aux[bh] = {beta, 1 / beta} too); every workgroup finds beta.
template <int D, bool NORM>
__global__ void __launch_bounds__(kBwdWideThreads)
bwdw_prep_state(const float* __restrict__ state, float* __restrict__ tstate, float* __restrict__ aux) {
  constexpr int NE = D * D + D;
  __shared__ float red[kBwdWideThreads / 64];
  const long long bh = blockIdx.y;
  const float* st = state + bh * NE;
  float* ts = tstate + bh * NE;
  float beta = 1.0f, inv_beta = 1.0f;
  if constexpr (NORM) {
    float zs = 0.0f;
    for (int i = threadIdx.x; i < D; i += kBwdWideThreads) zs += st[D * D + i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) zs += __shfl_xor(zs, o);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = zs;
    __syncthreads();
    zs = 0.0f;
#pragma unroll
    for (int w = 0; w < kBwdWideThreads / 64; ++w) zs += red[w];
    if (zs > 0.0f && zs < 3.0e38f) {
      int ex;
      (void)__builtin_frexpf(zs, &ex);
      ex = ex > 100 ? 100 : (ex < -100 ? -100 : ex);
      beta = __builtin_ldexpf(1.0f, ex);
      inv_beta = __builtin_ldexpf(1.0f, -ex);
    }
  }
  const int a0 = kBwdStrip * blockIdx.x;
  for (int e = threadIdx.x; e < kBwdStrip * D; e += kBwdWideThreads) {
    const int a = a0 + e % kBwdStrip, b = e / kBwdStrip;   // ts[a][b] = S[b][a] / beta: eight neighbours of a row of S per read
    ts[a * D + b] = st[b * D + a] * inv_beta;
  }
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i < D; i += kBwdWideThreads) ts[D * D + i] = st[D * D + i] * inv_beta;
    if (threadIdx.x == 0) {
      aux[2 * bh] = beta;
      aux[2 * bh + 1] = inv_beta;
    }
  }
}

// One wave per token, lane l < (chunks per row) holds the channels of chunk l.  grid = (ceil(N / 4), heads),
// block = 256.  q, g: the call's tensors; u: S' g (dense [B, H, N, D]); tstate: its z' is read.  Writes dq, gp
// (dense) and scal[bh][token] = e'.
template <typename T, int D, int FM, bool NORM>
__global__ void __launch_bounds__(kBwdWideThreads)
bwdw_q_finish(const u32x4* __restrict__ Q, Layout lq, const u32x4* __restrict__ G, Layout lg,
              const u32x4* __restrict__ U, const float* __restrict__ tstate, const float* __restrict__ aux,
              u32x4* __restrict__ DQ, Layout ldq, u32x4* __restrict__ GP, float* __restrict__ scal, float eps,
              long long N) {
  using RC = RowChunk<T>;
  constexpr int PER = RC::kPer, CPR = D / PER, NE = D * D + D;
  static_assert(CPR <= 32, "a token row fits half a wave");
  const int lane = threadIdx.x & 63;
  const long long bh = blockIdx.y;
  const long long t = (long long)blockIdx.x * (kBwdWideThreads / 64) + (threadIdx.x >> 6);
  if (t >= N) return;
  const bool on = lane < CPR;
  const int c = on ? lane : 0;
  const long long dense = (bh * N + t) * CPR + c;
  float x[PER], gg[PER], uu[PER], r[PER], z[PER];
  RC::load(Q + lq.slice(bh) + t * lq.row + c, x);
  RC::load(G + lg.slice(bh) + t * lg.row + c, gg);
  RC::load(U + dense, uu);
  const float* zp = tstate + bh * NE + D * D + PER * c;
  float s_rz = 0.0f, s_ru = 0.0f;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    r[i] = bw_phi<T, FM>(x[i]);
    z[i] = NORM ? zp[i] : 0.0f;
    if (on) {
      s_rz = __builtin_fmaf(r[i], z[i], s_rz);
      s_ru = __builtin_fmaf(r[i], uu[i], s_ru);
    }
  }
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) {
    s_rz += __shfl_xor(s_rz, o);
    s_ru += __shfl_xor(s_ru, o);
  }
  float invden = 1.0f, go = 0.0f;
  if constexpr (NORM) {
    invden = 1.0f / (s_rz + eps * aux[2 * bh + 1]);
    go = s_ru * invden;
  }
  if (lane == 0) scal[bh * N + t] = -go * invden;
  if (!on) return;
  float o2[PER], p2[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    o2[i] = (uu[i] - go * z[i]) * invden * phi_prime_from<FM>(x[i], r[i]);
    p2[i] = gg[i] * invden;
  }
  RC::store(DQ + ldq.slice(bh) + t * ldq.row + c, o2);
  RC::store(GP + dense, p2);
}

// dz' partials: grid = (splits, heads), block = 256; thread c < D sums phi(q_t[c]) e'_t over the split's tokens in
// token order.  part[bh][split][c].
template <typename T, int D, int FM>
__global__ void __launch_bounds__(kBwdWideThreads)
bwdw_dz(const typename RowChunk<T>::Elem* __restrict__ Q, Layout lq, const float* __restrict__ scal,
        float* __restrict__ part, long long N) {
  using RC = RowChunk<T>;
  using Elem = typename RC::Elem;
  constexpr int PER = RC::kPer;
  const long long bh = blockIdx.y;
  const int c = threadIdx.x;
  const long long per = (N + gridDim.x - 1) / gridDim.x;
  const long long t0 = blockIdx.x * per, t1 = t0 + per < N ? t0 + per : N;
  float acc = 0.0f;
  if (c < D) {
    const Elem* qh = Q + lq.slice(bh) * PER;     // Layout counts 16-byte units
    long long t = t0;
    for (; t + 4 <= t1; t += 4) {   // four independent loads in flight; summed in token order all the same
      Elem w[4];
      float e[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        w[i] = qh[(t + i) * lq.row * PER + c];
        e[i] = scal[bh * N + t + i];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) acc = __builtin_fmaf(bw_phi<T, FM>(RC::elem(w[i])), e[i], acc);
    }
    for (; t < t1; ++t) acc = __builtin_fmaf(bw_phi<T, FM>(RC::elem(qh[t * lq.row * PER + c])), scal[bh * N + t], acc);
    part[(bh * gridDim.x + blockIdx.x) * D + c] = acc;
  }
}

// grid = (D / 8, heads), block = 256.  raw: {dS' [D][D], (unused) [D]} as the reduction left it; part: dz' partials.
// Workgroup x writes rows 8 x .. 8 x + 7 of dstate = {dS, dz} and of tdstate = {dS^T, 0} (x = 0: the vectors too),
// all divided by beta.
template <int D>
__global__ void __launch_bounds__(kBwdWideThreads)
bwdw_finish_state(const float* __restrict__ raw, float* __restrict__ dstate, float* __restrict__ tdstate,
                  const float* __restrict__ part, int splits, const float* __restrict__ aux) {
  constexpr int NE = D * D + D;
  const long long bh = blockIdx.y;
  const float* rw = raw + bh * NE;
  float* ds = dstate + bh * NE;
  float* td = tdstate + bh * NE;
  const float inv_beta = aux[2 * bh + 1];
  const int a0 = kBwdStrip * blockIdx.x;
  for (int e = threadIdx.x; e < kBwdStrip * D; e += kBwdWideThreads) ds[a0 * D + e] = rw[a0 * D + e] * inv_beta;
  for (int e = threadIdx.x; e < kBwdStrip * D; e += kBwdWideThreads) {
    const int a = a0 + e % kBwdStrip, b = e / kBwdStrip;
    td[a * D + b] = rw[b * D + a] * inv_beta;
  }
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i < D; i += kBwdWideThreads) {
      float s = 0.0f;
      for (int p = 0; p < splits; ++p) s += part[(bh * splits + p) * D + i];
      ds[D * D + i] = s * inv_beta;
      td[D * D + i] = 0.0f;
    }
  }
}

// dk = (t + dz) phi'(k): one wave per token as bwdw_q_finish.  Tk: dS v (dense).
template <typename T, int D, int FM>
__global__ void __launch_bounds__(kBwdWideThreads)
bwdw_k_finish(const u32x4* __restrict__ K, Layout lk, const u32x4* __restrict__ Tk, const float* __restrict__ dstate,
              u32x4* __restrict__ DK, Layout ldk, long long N) {
  using RC = RowChunk<T>;
  constexpr int PER = RC::kPer, CPR = D / PER, NE = D * D + D;
  const int lane = threadIdx.x & 63;
  const long long bh = blockIdx.y;
  const long long t = (long long)blockIdx.x * (kBwdWideThreads / 64) + (threadIdx.x >> 6);
  if (t >= N || lane >= CPR) return;
  float x[PER], tt[PER], o[PER];
  RC::load(K + lk.slice(bh) + t * lk.row + lane, x);
  RC::load(Tk + (bh * N + t) * CPR + lane, tt);
  const float* dz = dstate + bh * NE + D * D + PER * lane;
#pragma unroll
  for (int i = 0; i < PER; ++i) o[i] = (tt[i] + dz[i]) * phi_prime_from<FM>(x[i], bw_phi<T, FM>(x[i]));
  RC::store(DK + ldk.slice(bh) + t * ldk.row + lane, o);
}

}  // namespace lf
