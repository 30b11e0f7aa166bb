// Transposition of a tile-major bit matrix into per-row pair lists, as a device function so that it
// can run as one role of a larger launch.
#pragma once
#include "slide_internal.h"

namespace slide {

// One workgroup per call and tile of TS bitmap words, all samples: the tile's touched rows, in row order,
// each with the ascending list of the samples that touch it.  Row slots of tile t are
// [t*TS*32, t*TS*32 + tile_nu[t]).  FEAT = false: the active bit matrix; a pair's coefficient
// index is its slot in the sample-major arrays, and the tile's first pair position is the sum over
// the samples of their in-sample ranks at the tile start (no atomics: the layout is a pure function
// of the bit matrix).  FEAT = true: the feature bit matrix of the batch; the coefficient index is the
// position in the CSR value array (the features of a sample are ascending, so it is the position of
// the tile's first feature plus the rank inside the tile), pair space is handed out per workgroup, and the matrix is cleared
// behind the read so that it is all-zero again for the next batch.
template <bool FEAT>
__device__ void transpose_tile(const TransposeArgs& ta, int tileno, uint32_t* lds) {
  // TW = words per record of the bit matrix (the unit ranks are kept for), TS = words handled here
  const int B = ta.B, Bpad = ta.Bpad, TW = ta.TW, TS = ta.TS;
  const int per = TW / TS, rec = tileno / per, w0 = (tileno - rec * per) * TS;
  uint32_t* bits = ta.bits;
  const uint32_t* __restrict__ rankT = ta.rankT;
  const int32_t* __restrict__ as_base = ta.as_base;
  const int32_t* __restrict__ x_indptr = ta.x_indptr;
  const int32_t* __restrict__ x_indices = ta.x_indices;
  const PairsDev& pd = ta.pd;
  const int nwaves = blockDim.x >> 6;
  uint32_t* tile = lds;                                  // [TS][Bpad]
  uint32_t* sb = tile + (size_t)TS * Bpad;                // [Bpad] slot of the sample's first pair in this tile
  uint32_t* wu = sb + Bpad;                              // [32] union word
  uint32_t* wnp = wu + 32;                               // [32] pairs per word, then exclusive prefix
  uint32_t* wou = wnp + 32;                              // [32] rows before the word
  uint32_t* blk = wou + 32;                              // [2] pair base of the tile, sum of ranks
  uint16_t* rk = (uint16_t*)(blk + 2);                   // [TS][Bpad] rank inside this tile before the word
  const int tid = threadIdx.x;
  if (tid == 0) { blk[0] = 0; blk[1] = 0; }
  __syncthreads();
  uint32_t ranksum = 0;
  for (int i = tid; i < Bpad; i += blockDim.x) {
    uint32_t* src = bits + ((size_t)rec * B + i) * TW;
    // the whole record in a few vector loads (a scalar load per word would wait for each in turn)
    uint32_t x[32];
    if (TW >= 4) {
#pragma unroll
      for (int v = 0; v < 8; ++v) {
        const uint4 q = (i < B && v * 4 < TW) ? ((const uint4*)src)[v] : make_uint4(0u, 0u, 0u, 0u);
        x[4 * v] = q.x; x[4 * v + 1] = q.y; x[4 * v + 2] = q.z; x[4 * v + 3] = q.w;
      }
    } else {
#pragma unroll
      for (int w = 0; w < 32; ++w) x[w] = (i < B && w < TW) ? src[w] : 0u;
    }
    uint32_t before = 0, run = 0, any = 0;             // before: active neurons of the record before this tile
#pragma unroll
    for (int w = 0; w < 32; ++w) {
      if (w < w0) {
        before += __popc(x[w]);
      } else if (w < w0 + TS) {
        tile[(w - w0) * Bpad + i] = x[w];
        rk[(w - w0) * Bpad + i] = (uint16_t)run;
        run += __popc(x[w]);
        any |= x[w];
      }
    }
    if (FEAT && any)                                   // leave the feature matrix all-zero behind
      for (int w = 0; w < TS; ++w) src[w0 + w] = 0u;
    if (!FEAT) {
      const uint32_t r0 = i < B ? rankT[(size_t)rec * B + i] + before : 0u;
      sb[i] = i < B ? (uint32_t)as_base[i] + r0 : 0u;
      ranksum += r0;
    } else {
      // position in the CSR arrays of the sample's first feature inside this tile (one search per
      // sample and tile, all samples at once; indices are ascending)
      uint32_t a = 0;
      if (any) {
        const int first = (rec * TW + w0) * 32;
        int lo_ = x_indptr[i], hi_ = x_indptr[i + 1];
        while (lo_ < hi_) { const int mid = (lo_ + hi_) >> 1; if (x_indices[mid] < first) lo_ = mid + 1; else hi_ = mid; }
        a = (uint32_t)lo_;
      }
      sb[i] = a;
    }
  }
  if (!FEAT) atomicAdd(&blk[1], ranksum);                // integer sum: order does not matter
  __syncthreads();
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int groups = Bpad >> 6;
  for (int w = wave; w < TS; w += nwaves) {
    uint32_t u = 0, np = 0;
    for (int k = 0; k < groups; ++k) { const uint32_t x = tile[w * Bpad + k * 64 + lane]; u |= x; np += __popc(x); }
    for (int d = 32; d > 0; d >>= 1) { u |= __shfl_xor(u, d); np += __shfl_xor(np, d); }
    if (lane == 0) { wu[w] = u; wnp[w] = np; }
  }
  __syncthreads();
  if (tid == 0) {
    uint32_t nu = 0, np = 0;
    for (int w = 0; w < TS; ++w) { wou[w] = nu; nu += __popc(wu[w]); const uint32_t c = wnp[w]; wnp[w] = np; np += c; }
    pd.tile_nu[tileno] = (int32_t)nu;
    if (nu > *(volatile uint32_t*)pd.max_nu) atomicMax(pd.max_nu, nu);   // few workgroups ever get here
    blk[0] = FEAT ? (np ? atomicAdd(pd.pcount, np) : 0u) : blk[1];
  }
  __syncthreads();
  const uint32_t slot0 = (uint32_t)tileno * (uint32_t)(TS * 32);
  constexpr int KG = 4;                                  // sample groups held in registers
  for (int w = wave; w < TS; w += nwaves) {
    uint32_t u = __builtin_amdgcn_readfirstlane(wu[w]);
    if (u == 0) continue;
    uint32_t us = slot0 + __builtin_amdgcn_readfirstlane(wou[w]);
    uint32_t po = __builtin_amdgcn_readfirstlane(blk[0] + wnp[w]);
    uint32_t xr[KG], sr[KG];
#pragma unroll
    for (int k = 0; k < KG; ++k) {
      const int i = k * 64 + lane;
      xr[k] = k < groups ? tile[w * Bpad + i] : 0u;
      sr[k] = k < groups ? sb[i] + rk[w * Bpad + i] : 0u;
    }
    while (u) {
      const int b = __ffs(u) - 1;
      u &= u - 1;
      const int row = (rec * TW + w0 + w) * 32 + b;
      uint32_t cntj = 0;
      auto take = [&](int k, uint32_t x, uint32_t sbase) {
        const int i = k * 64 + lane;
        const bool has = (x >> b) & 1u;
        const unsigned long long mk = __ballot(has);
        if (has) {
          const uint32_t p = po + cntj + __popcll(mk & ((1ull << lane) - 1ull));
          pd.pairs[p] = make_int2(i, (int)(sbase + __popc(x & ((1u << b) - 1u))));
        }
        cntj += (uint32_t)__popcll(mk);
      };
#pragma unroll
      for (int k = 0; k < KG; ++k)
        if (k < groups) take(k, xr[k], sr[k]);
      for (int k = KG; k < groups; ++k) {
        const int i = k * 64 + lane;
        take(k, tile[w * Bpad + i], sb[i] + rk[w * Bpad + i]);
      }
      if (lane == 0) {
        pd.umeta[us] = make_int4(row, (int)po, (int)cntj, 0);
        if ((int)cntj > kLongRow) {
          const uint32_t l = atomicAdd(pd.nlong, 1u);
          if (l < (uint32_t)pd.long_cap) pd.longlist[l] = (int32_t)us;
        }
      }
      ++us;
      po += cntj;
    }
  }
}

inline size_t transpose_lds(int TS, int Bpad) { return (size_t)TS * Bpad * 6 + (size_t)Bpad * 4 + 98 * 4; }

}  // namespace slide
