// Feature width DK of the queries and keys different from the value width DV (Prop. 3: the attention
// weights may be vector valued, f', g' then map to d' r channels while X keeps its own): the state is
// DK x DV, S = sum_j phi(k_j)^T v_j, z = sum_j phi(k_j) has DK entries, out_i = phi(q_i) S / (phi(q_i) . z + eps)
// has DV.  fp16 / bf16, contiguous [B, H, N, DK] (q, k) and [B, H, N, DV] (v, out), three-kernel path:
// state_reduce16_qv -> combine_state -> apply16_qv.  The reduction is state_reduce16 with the two tile
// shapes told apart; the apply kernel is ApplyDma with its output geometry taken from DV.
#pragma once
#include "lf_apply16_dma.hpp"

namespace lf {

template <typename T, int DK, int DV>
constexpr int reduce16_qv_lds_bytes() {
  int tiles = (NSplit<T>::value * Reduce16Cfg<DK>::kTileElems + Reduce16Cfg<DV>::kTileElems) * 2 * kWavesPerWG;
  int red = 2 * (DK * DV + DK) * 4;
  return tiles > red ? tiles : red;
}

// grid = (splits, B*H), block = 256; partial per workgroup: S as [DK][DV] row-major then z as [DK], fp32.
template <typename T, int DK, int DV, int FM>
__global__ void __launch_bounds__(kThreads)
state_reduce16_qv(const u32x4* __restrict__ K, const u32x4* __restrict__ V, float* __restrict__ partials, long long N,
                  int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  using ShK = Shape16<DK>;
  using ShV = Shape16<DV>;
  using CK = Reduce16Cfg<DK>;
  using CV = Reduce16Cfg<DV>;
  constexpr int NS = NSplit<T>::value;
  constexpr int RSK = CK::kRS, RSV = CV::kRS, NLK = CK::kNL, NLV = CV::kNL, MTK = ShK::kMT, MTV = ShV::kMT;
  constexpr int CPRK = ShK::kChunksPerRow, CPRV = ShV::kChunksPerRow;
  constexpr int NE = DK * DV + DK;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long long bh = blockIdx.y;
  const u32x4* Kh = K + bh * N * CPRK;
  const u32x4* Vh = V + bh * N * CPRV;
  float* dst = partials + (bh * gridDim.x + blockIdx.x) * (long long)NE;

  uint16_t* wbase = reinterpret_cast<uint16_t*>(smem) + wave * (NS * CK::kTileElems + CV::kTileElems);
  uint16_t* ldsP[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) ldsP[s] = wbase + s * CK::kTileElems;
  uint16_t* ldsV = wbase + NS * CK::kTileElems;

  int offk[NLK], rowk[NLK], offv[NLV], rowv[NLV];
#pragma unroll
  for (int u = 0; u < NLK; ++u) {
    const int c = u * 64 + lane;
    rowk[u] = c / CPRK;
    offk[u] = rowk[u] * RSK + (c % CPRK) * 8;
  }
#pragma unroll
  for (int u = 0; u < NLV; ++u) {
    const int c = u * 64 + lane;
    rowv[u] = c / CPRV;
    offv[u] = rowv[u] * RSV + (c % CPRV) * 8;
  }
  const int j16 = lane & 15, g4 = lane >> 4;
  const int trk = (8 * g4 + (j16 >> 2)) * RSK + 4 * (j16 & 3);
  const int trv = (8 * g4 + (j16 >> 2)) * RSV + 4 * (j16 & 3);

  const long long n_tiles = (N + kTile - 1) / kTile;
  TileIter it(blockIdx.x, gridDim.x, wave, tiles_per_block, n_tiles);

  f32x4 acc[MTK][MTV];
  f32x4 accz[MTK];
#pragma unroll
  for (int a = 0; a < MTK; ++a) {
    accz[a] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int b = 0; b < MTV; ++b) acc[a][b] = f32x4{0, 0, 0, 0};
  }
  const uint32_t one2 = (uint32_t)OneBits<T>::value * 0x10001u;
  const u32x4 ones = {one2, one2, one2, one2};

  u32x4 kr[NLK], vr[NLV];
  auto issue_loads = [&](long long tile) {
    long long rem = N - tile * kTile;
    int lim = rem < kTile ? (int)rem : kTile;
    const u32x4* kp = Kh + tile * kTile * CPRK;   // rows are contiguous: chunk c of the tile is the c-th vector
    const u32x4* vp = Vh + tile * kTile * CPRV;
#pragma unroll
    for (int u = 0; u < NLK; ++u)
      kr[u] = (u * 64 + lane < CK::kChunks && rowk[u] < lim) ? ld_stream(kp + u * 64 + lane)
                                                             : u32x4{LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value, LowestBits<T>::value};   // phi maps it to 0
#pragma unroll
    for (int u = 0; u < NLV; ++u)
      vr[u] = (u * 64 + lane < CV::kChunks && rowv[u] < lim) ? ld_stream(vp + u * 64 + lane) : u32x4{0, 0, 0, 0};
    return lim;
  };

  int lim = 0;
  if (it.valid()) lim = issue_loads(it.t);

  // one-time fill: pad columns zero; the ones column at index DV of the V tile (when a spare column exists)
  for (int i = lane; i < CK::kTileElems; i += 64) {
#pragma unroll
    for (int s = 0; s < NS; ++s) ldsP[s][i] = 0;
  }
  for (int i = lane; i < CV::kTileElems; i += 64)
    ldsV[i] = (ShV::kSpareCol && (i % RSV) == DV) ? OneBits<T>::value : (uint16_t)0;

  while (it.valid()) {
#pragma unroll
    for (int u = 0; u < NLK; ++u) {
      if (u * 64 + lane < CK::kChunks) {
        const bool ok = rowk[u] < lim;
        u32x4 ph, pl;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          if constexpr (NS == 1 && kPhiKillsLowest<FM>) {
            ph[w] = phi_pack2<T, FM>(kr[u][w]);
            continue;
          }
          float x0, x1;
          unpack2<T>(kr[u][w], x0, x1);
          float p0 = phi<FM>(x0), p1 = phi<FM>(x1);
          if constexpr (!kPhiKillsLowest<FM>) {
            p0 = ok ? p0 : 0.0f;
            p1 = ok ? p1 : 0.0f;
          }
          if constexpr (NS == 1) {
            ph[w] = pack2<T>(p0, p1);
          } else {
            uint32_t h, l;
            pack2_split<T>(p0, p1, h, l);
            ph[w] = h;
            pl[w] = l;
          }
        }
        *reinterpret_cast<u32x4*>(ldsP[0] + offk[u]) = ph;
        if constexpr (NS == 2) *reinterpret_cast<u32x4*>(ldsP[1] + offk[u]) = pl;
      }
    }
#pragma unroll
    for (int u = 0; u < NLV; ++u)
      if (u * 64 + lane < CV::kChunks) *reinterpret_cast<u32x4*>(ldsV + offv[u]) = vr[u];
    it.next();
    int next_lim = 0;
    if (it.valid()) next_lim = issue_loads(it.t);

    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    u32x4 bfrag[MTV];
#pragma unroll
    for (int b = 0; b < MTV; ++b) {
      u32x2 r0 = lds_read_tr16(ldsV + trv + 16 * b);
      u32x2 r1 = lds_read_tr16(ldsV + trv + 4 * RSV + 16 * b);
      bfrag[b] = u32x4{r0[0], r0[1], r1[0], r1[1]};
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
#pragma unroll
      for (int a = 0; a < MTK; ++a) {
        u32x2 r0 = lds_read_tr16(ldsP[s] + trk + 16 * a);
        u32x2 r1 = lds_read_tr16(ldsP[s] + trk + 4 * RSK + 16 * a);
        u32x4 afrag = u32x4{r0[0], r0[1], r1[0], r1[1]};
#pragma unroll
        for (int b = 0; b < MTV; ++b) acc[a][b] = mfma_16x16x32<T>(afrag, bfrag[b], acc[a][b]);
        if constexpr (!ShV::kSpareCol) accz[a] = mfma_16x16x32<T>(afrag, ones, accz[a]);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    lim = next_lim;
  }

  // cross-wave sum in a fixed order, (w0 + w2) + (w1 + w3), through two LDS copies of the partial
  __syncthreads();
  float* red = reinterpret_cast<float*>(smem);
  float* mine = red + (wave & 1) * NE;
#pragma unroll
  for (int round = 0; round < 2; ++round) {
    if ((wave >> 1) == round) {
#pragma unroll
      for (int a = 0; a < MTK; ++a) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int row = a * 16 + 4 * g4 + i;
          if (row < DK) {
#pragma unroll
            for (int b = 0; b < MTV; ++b) {
              const int col = b * 16 + j16;
              float* p = nullptr;
              if (col < DV) p = mine + row * DV + col;
              else if (ShV::kSpareCol && col == DV) p = mine + DK * DV + row;
              if (p) *p = (round == 0) ? acc[a][b][i] : *p + acc[a][b][i];
            }
            if constexpr (!ShV::kSpareCol) {
              if (j16 == 0) {
                float* p = mine + DK * DV + row;
                *p = (round == 0) ? accz[a][i] : *p + accz[a][i];
              }
            }
          }
        }
      }
    }
    __syncthreads();
  }
  for (int i = threadIdx.x; i < NE; i += kThreads) dst[i] = red[i] + red[NE + i];
}

// grid = (wgs, B*H), block = 256.  `state`: [B*H][DK*DV + DK] fp32 from combine_state.
template <typename T, int DK, int DV, int FM, bool NORM>
__global__ void __launch_bounds__(kThreads)
apply16_qv(const u32x4* __restrict__ Q, u32x4* __restrict__ O, const float* __restrict__ state, float eps, long long N,
           int tiles_per_block) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const long long bh = blockIdx.y;
  ApplyDma<T, DK, FM, NORM, 0, false, DV> ap(Q + bh * N * (DK / 8), DK / 8, O + bh * N * (DV / 8), DV / 8, N,
                                            tiles_per_block, blockIdx.x, gridDim.x, smem);
  ap.prefetch();
  ap.run(state + bh * (DK * DV + DK), eps);
}

}  // namespace lf
