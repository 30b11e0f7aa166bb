// Transposition of a tile-major bit matrix into per-row pair lists, as a device function so that it
// can run as one role of a larger launch.
#pragma once
#include "slide_internal.h"
#include "wave_ops.h"

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
  const int groups = Bpad >> 6;                          // 64-sample groups
  uint32_t* tile = lds;                                  // [TS][Bpad]
  uint32_t* sb = tile + (size_t)TS * Bpad;                // [Bpad] slot of the sample's first pair in this tile
  uint32_t* wug = sb + Bpad;                             // [TS][groups] union of the word over a sample group
  uint32_t* wu = wug + (size_t)TS * groups;              // [TS] union over all samples
  uint32_t* wnp = wu + TS;                               // [TS] pairs per word, then exclusive prefix
  uint32_t* wou = wnp + TS;                              // [TS] rows before the word
  uint32_t* blk = wou + TS;                              // [2] pair base of the tile, sum of ranks
  uint16_t* rk = (uint16_t*)(blk + 2);                   // [TS][Bpad] rank inside this tile before the word
  const int tid = threadIdx.x, lane = tid & 63;
  for (int q = tid; q < TS * groups + 3 * TS + 2; q += blockDim.x) wug[q] = 0;   // wug, wu, wnp, wou, blk
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
        // union and pair count of the word over this wave's 64 samples: LDS atomics from the few
        // lanes that hold anything, or one register reduction when many do
        const int holders = __popcll(__ballot(x[w] != 0u));
        if (holders > 8) {
          const uint32_t o = wave_or(x[w]), c = wave_sum((uint32_t)__popc(x[w]));
          if (lane == 0) { wug[(w - w0) * groups + (i >> 6)] = o; atomicAdd(&wnp[w - w0], c); }
        } else if (x[w]) {
          atomicOr(&wug[(w - w0) * groups + (i >> 6)], x[w]);
          atomicAdd(&wnp[w - w0], (uint32_t)__popc(x[w]));
        }
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
  if (!FEAT && ranksum) atomicAdd(&blk[1], ranksum);     // integer sum: order does not matter
  __syncthreads();
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (wave == 0) {                                       // per word: union, rows and pairs before it
    uint32_t u = 0;
    if (lane < TS) for (int k = 0; k < groups; ++k) u |= wug[lane * groups + k];
    const uint32_t c = __popc(u), np = lane < TS ? wnp[lane] : 0u;
    const uint32_t cin = wave_incl_scan_add(c), pin = wave_incl_scan_add(np);
    if (lane < TS) { wu[lane] = u; wou[lane] = cin - c; wnp[lane] = pin - np; }
    if (lane == 63) {
      pd.tile_nu[tileno] = (int32_t)cin;
      if (cin > *(volatile uint32_t*)pd.max_nu) atomicMax(pd.max_nu, cin);   // few workgroups ever get here
      blk[0] = FEAT ? (pin ? atomicAdd(pd.pcount, pin) : 0u) : blk[1];
    }
  }
  __syncthreads();
  const uint32_t slot0 = (uint32_t)tileno * (uint32_t)(TS * 32);
  constexpr int KG = 4;                                  // sample groups held in registers
  for (int w = wave; w < TS; w += nwaves) {
    uint32_t u = __builtin_amdgcn_readfirstlane(wu[w]);
    if (u == 0) continue;
    uint32_t us = slot0 + __builtin_amdgcn_readfirstlane(wou[w]);
    uint32_t po = __builtin_amdgcn_readfirstlane(blk[0] + wnp[w]);
    uint32_t xr[KG], sr[KG], ug[KG];                     // ug: union of the word over the 64 samples
#pragma unroll
    for (int k = 0; k < KG; ++k) {
      const int i = k * 64 + lane;
      xr[k] = k < groups ? tile[w * Bpad + i] : 0u;
      sr[k] = k < groups ? sb[i] + rk[w * Bpad + i] : 0u;
      ug[k] = k < groups ? __builtin_amdgcn_readfirstlane(wug[w * groups + k]) : 0u;
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
        if ((ug[k] >> b) & 1u) take(k, xr[k], sr[k]);     // skip sample groups without this row
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

inline size_t transpose_lds(int TS, int Bpad) {
  return (size_t)TS * Bpad * 6 + (size_t)Bpad * 4 + ((size_t)TS * (Bpad >> 6) + 3 * TS + 2) * 4;
}

}  // namespace slide
