// Transposition of a tile-major bit matrix into per-row pair lists, as a device function so that it
// can run as one role of a larger launch.
#pragma once
#include "slide_internal.h"
#include "wave_ops.h"

namespace slide {

// One workgroup per call and tile (TW bitmap words = TW*32 rows, all samples): the tile's touched
// rows, in row order, each with the ascending list of the samples that touch it.  Row slots of tile
// t are [t*TW*32, t*TW*32 + tile_nu[t]).
//   FEAT = false: the active bit matrix; a pair's coefficient index is its slot in the sample-major
//     arrays, and the tile's first pair position is the sum over the samples of their in-sample
//     ranks at the tile start (the layout is a pure function of the bit matrix).
//   FEAT = true: the feature bit matrix of the batch; the coefficient index is the position in the
//     CSR value array (the features of a sample are ascending, so it is the position of the
//     sample's first feature inside the tile, recorded by the hidden-layer kernel, plus the rank
//     inside the tile); pair space is handed out per workgroup, and the matrix is cleared behind
//     the read so that it is all-zero again for the next batch.
// WT = min(TW, 8) words of a record per thread, TW/WT adjacent threads per sample.  Pass 1 builds
// the transposed tile in LDS: one bit per (row, sample), set with LDS atomics from the (few)
// non-zero bits of the records.  Lane = row then gives every row's pair count, the touched rows,
// every row's position in the pair space and, inside it, where each group of 64 samples starts.
// Pass 2 reads the records again (from cache); for each of its bits a thread finds the pair's place
// in the row's list as the number of lower samples in the row's LDS mask, so every pair is written
// straight to its final position -- ascending samples per row, no sort -- and a store instruction
// carries one pair for every lane that still has a bit in its word, not one row.
template <bool FEAT, int TW>
__device__ __forceinline__ void transpose_tile_t(const TransposeArgs& ta, int tileno, uint32_t* lds) {
  constexpr int ROWS = TW * 32;
  constexpr int WT = TW < 8 ? TW : 8;                    // words per thread
  constexpr int SUB = TW / WT;                           // threads per sample (1, 2 or 4)
  const int B = ta.B, Bpad = ta.Bpad;
  const PairsDev& pd = ta.pd;
  const int groups = Bpad >> 6, GW = Bpad >> 5;
  uint32_t* T = lds;                                     // [GW][ROWS] bit (i & 31) of word i >> 5: sample i holds the row
  uint32_t* rowoff = T + (size_t)GW * ROWS;              // [ROWS] pairs of the word's lower rows
  uint32_t* wu = rowoff + ROWS;                          // [TW] touched rows of the word (bit mask)
  uint32_t* wnp = wu + TW;                               // [TW] pairs of the word, then pairs before it
  uint32_t* wou = wnp + TW;                              // [TW] rows before the word
  uint32_t* blk = wou + TW;                              // [2] pair base of the tile, sum of ranks
  uint16_t* rowcnt = (uint16_t*)(blk + 2);               // [ROWS] pairs of the row
  uint16_t* rowgrp = rowcnt + ROWS;                      // [groups][ROWS] pairs of the row in lower sample groups
  const int tid = threadIdx.x, lane = tid & 63, b31 = tid & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t below = (1u << b31) - 1u;
  const int nwork = Bpad * SUB;

  for (int q = tid; q < GW * ROWS; q += blockDim.x) T[q] = 0;
  if (tid == 0) blk[1] = 0;
  __syncthreads();

  // The loaded words (and `extra`, a value loaded beside them) are forced to arrive before the
  // call returns: left to the first use inside the branching word loops, the compiler's wait would
  // be a wait for every outstanding memory operation, the loop's own stores included.
  auto load_words = [&](int i, int sub, uint32_t* x, bool clear, uint32_t& extra) {
    uint32_t* src = ta.bits + ((size_t)tileno * B + i) * TW + sub * WT;
    uint32_t any = 0;
    if (WT >= 4) {
#pragma unroll
      for (int v = 0; v < WT / 4; ++v) {
        const uint4 q = i < B ? ((const uint4*)src)[v] : make_uint4(0u, 0u, 0u, 0u);
        x[4 * v] = q.x; x[4 * v + 1] = q.y; x[4 * v + 2] = q.z; x[4 * v + 3] = q.w;
        any |= q.x | q.y | q.z | q.w;
      }
      asm volatile("" : "+v"(any), "+v"(extra));
      if (clear && any) {
#pragma unroll
        for (int v = 0; v < WT / 4; ++v) ((uint4*)src)[v] = make_uint4(0u, 0u, 0u, 0u);
      }
    } else {
#pragma unroll
      for (int w = 0; w < WT; ++w) { x[w] = i < B ? src[w] : 0u; any |= x[w]; }
      asm volatile("" : "+v"(any), "+v"(extra));
      if (clear && any) {
#pragma unroll
        for (int w = 0; w < WT; ++w) src[w] = 0u;
      }
    }
  };

  // ---- pass 1: transposed tile -------------------------------------------------------------------
  for (int t = tid; t < nwork; t += blockDim.x) {
    const int i = t / SUB, sub = t % SUB;
    uint32_t x[WT];
    uint32_t rank0 = (!FEAT && sub == 0 && i < B) ? ta.rankT[(size_t)tileno * B + i] : 0u;
    load_words(i, sub, x, false, rank0);
    uint32_t* tc = T + (size_t)(i >> 5) * ROWS + sub * WT * 32;
    const uint32_t ibit = 1u << (i & 31);
#pragma unroll
    for (int w = 0; w < WT; ++w) {
      uint32_t y = x[w];
      while (y) {
        const int b = __ffs(y) - 1;
        y &= y - 1u;
        atomicOr(&tc[w * 32 + b], ibit);
      }
    }
    if (!FEAT) {
      const uint32_t s = wave_sum(rank0);
      if (lane == 0 && s) atomicAdd(&blk[1], s);         // integer sum: order does not matter
    }
  }
  __syncthreads();

  // ---- rows: pairs per row and per sample group, prefix inside the word (lane = bit of the word) ---
  for (int r0 = 0; r0 < ROWS; r0 += blockDim.x) {
    const int r = r0 + tid;
    const bool ok = r < ROWS;
    uint32_t c = 0;
    if (ok) {
      for (int g = 0; g < groups; ++g) {
        rowgrp[(size_t)g * ROWS + r] = (uint16_t)c;
        c += __popc(T[(size_t)(2 * g) * ROWS + r]) + __popc(T[(size_t)(2 * g + 1) * ROWS + r]);
      }
    }
    const unsigned long long touched = __ballot(c != 0u);
    const uint32_t incl = half_incl_scan_add(c);
    if (ok) {
      rowoff[r] = incl - c;
      rowcnt[r] = (uint16_t)c;
      if (b31 == 31) { wu[r >> 5] = (uint32_t)(touched >> (lane & 32)); wnp[r >> 5] = incl; }
    }
  }
  __syncthreads();

  // ---- rows and pairs before each word -----------------------------------------------------------
  uint32_t nu_tile = 0;
  if (wave == 0) {
    const uint32_t u = lane < TW ? wu[lane] : 0u, np = lane < TW ? wnp[lane] : 0u;
    const uint32_t c = __popc(u);
    const uint32_t cin = wave_incl_scan_add(c), pin = wave_incl_scan_add(np);
    if (lane < TW) { wou[lane] = cin - c; wnp[lane] = pin - np; }
    if (lane == 63) {
      nu_tile = cin;
      pd.tile_nu[tileno] = (int32_t)cin;
      blk[0] = FEAT ? (pin ? atomicAdd(pd.pcount, pin) : 0u) : blk[1];
    }
  }
  __syncthreads();
  const uint32_t blk0 = blk[0];
  const uint32_t slot0 = (uint32_t)tileno * (uint32_t)ROWS;

  // ---- row headers ---------------------------------------------------------------------------------
  for (int r = tid; r < ROWS; r += blockDim.x) {
    const uint32_t c = rowcnt[r];
    if (c) {
      const int w = r >> 5;
      const uint32_t us = slot0 + wou[w] + __popc(wu[w] & below);
      pd.umeta[us] = make_int4(tileno * ROWS + r, (int)(blk0 + wnp[w] + rowoff[r]), (int)c, 0);
      if ((int)c > kLongRow) {
        const uint32_t l = atomicAdd(pd.nlong, 1u);
        if (l < (uint32_t)pd.long_cap) pd.longlist[l] = (int32_t)us;
      }
    }
  }

  // ---- pass 2: emit ----------------------------------------------------------------------------------
  const uint32_t cmax = FEAT ? (uint32_t)(ta.x_nnz > 0 ? ta.x_nnz - 1 : 0) : 0xffffffffu;
  for (int t = tid; t < nwork; t += blockDim.x) {
    const int i = t / SUB, sub = t % SUB;
    uint32_t x[WT];
    uint32_t cbase = 0;                                  // coefficient index of the sample's first pair here
    if (i < B) cbase = FEAT ? (uint32_t)ta.xfirst[(size_t)tileno * B + i]
                            : (uint32_t)ta.as_base[i] + ta.rankT[(size_t)tileno * B + i];
    load_words(i, sub, x, FEAT, cbase);
    uint32_t mine = 0;
#pragma unroll
    for (int w = 0; w < WT; ++w) mine += __popc(x[w]);
    uint32_t run = 0;                                    // bits of the sample in the words of its lower threads
    if (SUB > 1) {
      const uint32_t p0 = dpp_u32<0x00>(0u, mine), p1 = dpp_u32<0x55>(0u, mine), p2 = dpp_u32<0xAA>(0u, mine);
      run = (sub > 0 ? p0 : 0u) + (sub > 1 ? p1 : 0u) + (sub > 2 ? p2 : 0u);
      if (SUB == 2) run = (sub & 1) ? ((lane & 2) ? p2 : p0) : 0u;
    }
    if (!mine) continue;
    const int g = i >> 6;
    const uint32_t lo_mask = (i & 32) ? 0xffffffffu : ((1u << (i & 31)) - 1u);
    const uint32_t hi_mask = (i & 32) ? ((1u << (i & 31)) - 1u) : 0u;
    const uint32_t* t_lo = T + (size_t)(2 * g) * ROWS;
    const uint32_t* t_hi = t_lo + ROWS;
    const uint16_t* grp = rowgrp + (size_t)g * ROWS;
#pragma unroll
    for (int w = 0; w < WT; ++w) {
      uint32_t y = x[w];
      if (!y) continue;
      const int W = sub * WT + w;
      const uint32_t wbase = blk0 + wnp[W];
      while (y) {
        const int b = __ffs(y) - 1;
        y &= y - 1u;
        const int row = W * 32 + b;
        const uint32_t place = wbase + rowoff[row] + grp[row] + __popc(t_lo[row] & lo_mask) + __popc(t_hi[row] & hi_mask);
        const uint32_t ci = cbase + run + __popc(x[w] & ((1u << b) - 1u));
        pd.pairs[place] = make_int2(i, (int)min(ci, cmax));
      }
      run += __popc(x[w]);
    }
  }
  // few workgroups ever raise the maximum; the read is off the critical path here
  if (wave == 0 && lane == 63 && nu_tile > *(volatile uint32_t*)pd.max_nu) atomicMax(pd.max_nu, nu_tile);
}

template <bool FEAT>
__device__ __forceinline__ void transpose_tile(const TransposeArgs& ta, int tileno, uint32_t* lds) {
  switch (ta.TW) {
    case 32: transpose_tile_t<FEAT, 32>(ta, tileno, lds); break;
    case 16: transpose_tile_t<FEAT, 16>(ta, tileno, lds); break;
    case 8: transpose_tile_t<FEAT, 8>(ta, tileno, lds); break;
    case 4: transpose_tile_t<FEAT, 4>(ta, tileno, lds); break;
    case 2: transpose_tile_t<FEAT, 2>(ta, tileno, lds); break;
    default: transpose_tile_t<FEAT, 1>(ta, tileno, lds); break;
  }
}

inline size_t transpose_lds(int TW, int Bpad) {
  const size_t rows = (size_t)TW * 32, GW = (size_t)Bpad >> 5, groups = (size_t)Bpad >> 6;
  return (rows * GW + rows + (size_t)TW * 3 + 2) * 4 + rows * 2 + groups * rows * 2;
}

}  // namespace slide
