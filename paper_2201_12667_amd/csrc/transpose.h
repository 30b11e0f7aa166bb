// Transposition of sample-major id lists into per-row pair lists, as a device function so that it
// can run as one role of a larger launch.
#pragma once
#include "slide_internal.h"
#include "wave_ops.h"

namespace slide {

// One workgroup per call and tile of ROWS = TW*32 consecutive rows, all samples: the tile's touched
// rows, in row order, each with the ascending list of the samples that touch it.  Row slots of tile
// t are [t*ROWS, t*ROWS + tile_nu[t]).
// The input is sample-major: every sample has an ascending id list, and the part of it that falls
// into a tile is a known segment [lo, hi) of the id array.
//   FEAT = false: active sets; ids = the compact active-set lists, segment = the sample's slice
//     start plus its ranks at the tile's two ends (kept per tile by the lookup), and the tile's
//     first pair position is the sum of the lower ranks over the samples (a pure function of the
//     sets).  A pair's coefficient index is the id's slot in the sample-major arrays.
//   FEAT = true: features of the batch; ids = the CSR index array, segments recorded per (tile,
//     sample) by the hidden-layer kernel and cleared here behind the read (all-zero = empty, ready
//     for the next batch); pair space is handed out per workgroup.  The coefficient index is the
//     position in the CSR arrays.
// A thread owns a sample (or, when the workgroup has more threads than samples, an interleaved
// share of a sample's segment).  Pass 1 builds the transposed tile in LDS: one bit per (row, sample), set
// with LDS atomics.  Lane = row then gives every row's pair count, the touched rows, every row's
// position in the pair space and, inside it, where each group of 64 samples starts.  Pass 2 walks
// the segments again; a pair's place in the row's list is the number of lower samples in the row's
// LDS mask, so every pair is written straight to its final position: ascending samples per row,
// no sort, no global atomics on the data.
constexpr int kInFlight = 4;    // ids a thread requests before it uses the first
constexpr int kTilesPerWave = 2; // feature tiles a wave takes, one after the other, when the waves take tiles

template <bool FEAT, int TW, bool BITS = false>
__device__ __forceinline__ void transpose_tile_t(const TransposeArgs& ta, int tileno, uint32_t* lds) {
  constexpr int ROWS = TW * 32;
  const int B = ta.B, Bpad = ta.Bpad;
  const PairsDev& pd = ta.pd;
  const int32_t* __restrict__ ids = ta.ids;
  const int groups = Bpad >> 6, GW = Bpad >> 5;
  uint32_t* T = lds;                                     // [GW][ROWS] bit (i & 31) of word i >> 5: sample i holds the row
  uint32_t* rowoff = T + (size_t)GW * ROWS;              // [ROWS] pairs of the word's lower rows
  uint32_t* wu = rowoff + ROWS;                          // [TW] touched rows of each 32-row word (bit mask)
  uint32_t* wnp = wu + TW;                               // [TW] pairs of the word, then pairs before it
  uint32_t* wou = wnp + TW;                              // [TW] rows before the word
  uint32_t* blk = wou + TW;                              // [4] pair base of the tile, sum of ranks, long rows, their queue base
  uint32_t* lq = blk + 4;                                // [ROWS] slots of the tile's long rows (queued together at the end)
  uint16_t* rowcnt = (uint16_t*)(lq + ROWS);             // [ROWS] pairs of the row
  uint16_t* rowgrp = rowcnt + ROWS;                      // [groups][ROWS] pairs of the row in lower sample groups
  const int tid = threadIdx.x, lane = tid & 63, b31 = tid & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const uint32_t below = (1u << b31) - 1u;
  const int row0 = tileno * ROWS;

  if (FEAT) {
    // Most tiles of a wide input layer hold few features of the batch, or none: one look at the
    // segments settles it.  None: nothing to do.  At most 64: one wave sorts the (row, sample) keys in
    // its lanes and writes the tile's lists, without the transposed bit tile.
    if (tid == 0) { blk[1] = 0; blk[2] = 0; }
    __syncthreads();
    uint32_t mine = 0;
    for (int i = tid; i < B; i += blockDim.x) {
      const int2 v = ta.xse[(size_t)tileno * B + i];
      const int lo = max(v.x, 0), hi = min(v.y, ta.x_nnz);
      mine += hi > lo ? (uint32_t)(hi - lo) : 0u;
    }
    mine = wave_sum(mine);
    if (lane == 0 && mine) atomicAdd(&blk[1], mine);
    __syncthreads();
    const uint32_t total = blk[1];
    if (total <= 64u) {
      uint32_t* skey = T;                                // [64] row in tile << 16 | sample
      uint32_t* spos = T + 64;                           // [64] position in the batch's feature arrays
      if (total) {
        for (int i = tid; i < B; i += blockDim.x) {
          const int2 v = ta.xse[(size_t)tileno * B + i];
          const int lo = max(v.x, 0), hi = min(v.y, ta.x_nnz);
          for (int p = lo; p < hi; ++p) {
            const int r = ids[p] - row0;
            if ((unsigned)r < (unsigned)ROWS) {
              const uint32_t at = atomicAdd(&blk[2], 1u);
              if (at < 64u) { skey[at] = ((uint32_t)r << 16) | (uint32_t)i; spos[at] = (uint32_t)p; }
            }
          }
        }
      }
      __syncthreads();
      const uint32_t n = min(blk[2], 64u);
      if (wave == 0) {
        uint32_t key = (uint32_t)lane < n ? skey[lane] : 0xffffffffu;
        uint32_t pos = (uint32_t)lane < n ? spos[lane] : 0u;
#pragma unroll
        for (int k = 2; k <= 64; k <<= 1)                 // bitonic sort across the lanes, ascending keys
#pragma unroll
          for (int j = k >> 1; j > 0; j >>= 1) {
            const uint32_t okey = __shfl_xor(key, j), opos = __shfl_xor(pos, j);
            const bool up = (lane & k) == 0, lower = (lane & j) == 0;
            const bool take = (lower == up) ? okey < key : okey > key;
            if (take) { key = okey; pos = opos; }
          }
        const uint32_t prev = __shfl_up(key, 1);
        const bool head = (uint32_t)lane < n && (lane == 0 || (prev >> 16) != (key >> 16));
        const unsigned long long heads = __ballot(head);
        const uint32_t nu = (uint32_t)__popcll(heads);
        uint32_t base = 0;
        if (lane == 0) {
          pd.tile_nu[tileno] = (int32_t)nu;
          base = n ? pd.region0 + (uint32_t)(tileno % kPairRegions) * pd.region_pairs + atomicAdd(&pd.pcount[tileno % kPairRegions], n) : 0u;
          if (nu > *(volatile uint32_t*)pd.max_nu) atomicMax(pd.max_nu, nu);
        }
        base = (uint32_t)__builtin_amdgcn_readfirstlane((int)base);
        if ((uint32_t)lane < n) pd.pairs[base + lane] = make_int2((int)(key & 0xffffu), (int)pos);
        if (head) {
          const unsigned long long above = lane < 63 ? heads >> (lane + 1) : 0ull;
          const uint32_t c = above ? (uint32_t)__ffsll((long long)above) : n - (uint32_t)lane;
          const uint32_t us = (uint32_t)tileno * (uint32_t)ROWS + (uint32_t)__popcll(heads & ((1ull << lane) - 1ull));
          pd.umeta[us] = make_int4(row0 + (int)(key >> 16), (int)(base + lane), (int)c, 0);
          if (ta.touched) ta.touched[row0 + (int)(key >> 16)] = 1;
          if ((int)c > kLongRow) {
            const uint32_t l = atomicAdd(pd.nlong, 1u);
            if (l < (uint32_t)pd.long_cap) pd.longlist[l] = (int32_t)us;
          }
        }
      }
      for (int i = tid; i < B; i += blockDim.x) {        // leave the segments all-zero for the next batch
        int2* se = ta.xse + (size_t)tileno * B + i;
        const int2 v = *se;
        if (v.x | v.y) *se = make_int2(0, 0);
      }
      return;
    }
    __syncthreads();                                     // (blk is set up again below)
  }
  for (int q = tid; q < GW * ROWS; q += blockDim.x) T[q] = 0;
  if (tid == 0) { blk[1] = 0; blk[2] = 0; }
  __syncthreads();

  // segment of sample i inside this tile; rank0 = the sample's rank at the tile start (active sets)
  auto segment = [&](int i, int& lo, int& hi, uint32_t& rank0) {
    lo = 0; hi = 0; rank0 = 0;
    if (i >= B) return;
    if (FEAT) {
      const int2 v = ta.xse[(size_t)tileno * B + i];
      lo = max(v.x, 0); hi = min(v.y, ta.x_nnz);
    } else {
      const int base = ta.as_base[i];
      rank0 = ta.rankT[(size_t)tileno * B + i];
      lo = base + (int)rank0; hi = base + (int)ta.rankT[(size_t)(tileno + 1) * B + i];
    }
  };

  // ---- pass 1: transposed tile -------------------------------------------------------------------
  // A thread's first kKeep ids of each segment stay in registers (as rows of the tile) together with the
  // segment's ends: the second pass then needs no memory read at all for them.
  constexpr int kKeep = 8, kSegs = 4;                    // (kSegs >= Bpad * shares / blockDim: batches up to 2048)
  const int shares = max(1, (int)blockDim.x / Bpad);     // threads per sample
  int klo[kSegs], khi[kSegs], krow[kSegs][kKeep];
#pragma unroll
  for (int j = 0; j < kSegs; ++j) {
    const int idx = tid + j * (int)blockDim.x;
    klo[j] = 0; khi[j] = 0;
#pragma unroll
    for (int k = 0; k < kKeep; ++k) krow[j][k] = -1;
    if (idx >= Bpad * shares) continue;
    const int i = idx % Bpad, share = idx / Bpad;
    int lo, hi;
    uint32_t rank0;
    segment(i, lo, hi, rank0);
    if (share) rank0 = 0;
    klo[j] = lo; khi[j] = hi;
    uint32_t* tc = T + (size_t)(i >> 5) * ROWS;
    const uint32_t ibit = 1u << (i & 31);
    if (BITS && !FEAT && TW >= 4) {
      // from the sample's bitmap of the tile (TW words, one coalesced read): the thread's share of the words
      if (i < B) {
        const uint32_t* sw = ta.act + ((size_t)tileno * B + i) * TW;
        const int w0 = share * TW / shares, w1 = (share + 1) * TW / shares;
#pragma unroll
        for (int w4 = 0; w4 < TW; w4 += 4) {
          if (w4 + 4 <= w0 || w4 >= w1) continue;
          const uint4 q = *(const uint4*)(sw + w4);
          const uint32_t ww[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            uint32_t word = (w4 + k >= w0 && w4 + k < w1) ? ww[k] : 0u;
            while (word) {
              const int b = __ffs(word) - 1;
              word &= word - 1;
              atomicOr(&tc[(w4 + k) * 32 + b], ibit);
            }
          }
        }
      }
      if (!FEAT) {
        const uint32_t s = wave_sum(rank0);
        if (lane == 0 && s) atomicAdd(&blk[1], s);
      }
      continue;
    }
    // this thread's ids: lo + 4*share + (0..3), then every 4*shares further on
#pragma unroll
    for (int k = 0; k < kKeep; ++k) {
      const int p = lo + 4 * share + (k >> 2) * 4 * shares + (k & 3);
      krow[j][k] = p < hi ? ids[p] - row0 : -1;
    }
#pragma unroll
    for (int k = 0; k < kKeep; ++k)
      if ((unsigned)krow[j][k] < (unsigned)ROWS) atomicOr(&tc[krow[j][k]], ibit);
    for (int p = lo + 4 * share + (kKeep / 4) * 4 * shares; p < hi; p += 4 * shares) {   // longer segments
      int r[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) r[k] = p + k < hi ? ids[p + k] - row0 : -1;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if ((unsigned)r[k] < (unsigned)ROWS) atomicOr(&tc[r[k]], ibit);
    }
    if (!FEAT) {
      const uint32_t s = wave_sum(rank0);
      if (lane == 0 && s) atomicAdd(&blk[1], s);         // integer sum: order does not matter
    }
  }
  __syncthreads();

  // ---- rows: pairs per row and per sample group, prefix inside each 32-row word (lane = row) -------
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
      blk[0] = FEAT ? (pin ? pd.region0 + (uint32_t)(tileno % kPairRegions) * pd.region_pairs + atomicAdd(&pd.pcount[tileno % kPairRegions], pin) : 0u)
                    : blk[1];
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
      pd.umeta[us] = make_int4(row0 + r, (int)(blk0 + wnp[w] + rowoff[r]), (int)c, 0);
      if (ta.touched) ta.touched[row0 + r] = 1;
      if ((int)c > kLongRow) lq[atomicAdd(&blk[2], 1u)] = us;   // (one update of the global queue per tile, below)
    }
  }

  // ---- pass 2: emit ----------------------------------------------------------------------------------
#pragma unroll
  for (int j = 0; j < kSegs; ++j) {
    const int idx = tid + j * (int)blockDim.x;
    if (idx >= Bpad * shares) continue;
    const int i = idx % Bpad, share = idx / Bpad;
    const int lo = klo[j], hi = khi[j];
    const int g = i >> 6;
    const uint32_t lo_mask = (i & 32) ? 0xffffffffu : ((1u << (i & 31)) - 1u);
    const uint32_t hi_mask = (i & 32) ? ((1u << (i & 31)) - 1u) : 0u;
    const uint32_t* t_lo = T + (size_t)(2 * g) * ROWS;
    const uint32_t* t_hi = t_lo + ROWS;
    const uint16_t* grp = rowgrp + (size_t)g * ROWS;
    auto emit = [&](int row, int pos) {
      const uint32_t place = blk0 + wnp[row >> 5] + rowoff[row] + grp[row] + __popc(t_lo[row] & lo_mask) +
                             __popc(t_hi[row] & hi_mask);
      pd.pairs[place] = make_int2(i, pos);
    };
    if (BITS && !FEAT && TW >= 4) {
      // the bitmap again: a set bit's coefficient index is the segment's start plus the bits below it
      if (i < B) {
        const uint32_t* sw = ta.act + ((size_t)tileno * B + i) * TW;
        const int w0 = share * TW / shares, w1 = (share + 1) * TW / shares;
        int pos = lo;
#pragma unroll
        for (int w4 = 0; w4 < TW; w4 += 4) {
          if (w4 >= w1) continue;
          const uint4 q = *(const uint4*)(sw + w4);
          const uint32_t ww[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            uint32_t word = ww[k];
            if (w4 + k < w0 || w4 + k >= w1) { pos += __popc(word); continue; }
            while (word) {
              const int b = __ffs(word) - 1;
              word &= word - 1;
              emit((w4 + k) * 32 + b, pos++);
            }
          }
        }
      }
      continue;
    }
#pragma unroll
    for (int k = 0; k < kKeep; ++k)
      if ((unsigned)krow[j][k] < (unsigned)ROWS) emit(krow[j][k], lo + 4 * share + (k >> 2) * 4 * shares + (k & 3));
    for (int p = lo + 4 * share + (kKeep / 4) * 4 * shares; p < hi; p += 4 * shares) {
      int r[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) r[k] = p + k < hi ? ids[p + k] - row0 : -1;
#pragma unroll
      for (int k = 0; k < 4; ++k)
        if ((unsigned)r[k] < (unsigned)ROWS) emit(r[k], p + k);
    }
  }
  __syncthreads();
  {                                                      // the tile's long rows join the queue as one stretch
    const uint32_t nl = blk[2];
    if (nl) {
      if (tid == 0) blk[3] = atomicAdd(pd.nlong, nl);
      __syncthreads();
      const uint32_t base = blk[3];
      for (uint32_t q = tid; q < nl; q += blockDim.x)
        if (base + q < (uint32_t)pd.long_cap) pd.longlist[base + q] = (int32_t)lq[q];
    }
  }
  if (FEAT) {                                            // leave the segments all-zero for the next batch
    for (int i = tid; i < B; i += blockDim.x) {
      int2* se = ta.xse + (size_t)tileno * B + i;
      const int2 v = *se;
      if (v.x | v.y) *se = make_int2(0, 0);
    }
  }
  // few workgroups ever raise the maximum; the read is off the critical path here
  if (wave == 0 && lane == 63 && nu_tile > *(volatile uint32_t*)pd.max_nu) atomicMax(pd.max_nu, nu_tile);
}

// Feature tiles of a very wide input layer: nearly every tile holds a handful of the batch's features,
// or none, and a workgroup per tile would spend its time on fixed latencies.  Here a workgroup takes
// as many consecutive tiles as it has waves, a wave per tile: the wave counts the tile's entries,
// gathers up to 64 of them in its own corner of the LDS, sorts the (row, sample) keys across its lanes
// and writes the tile's lists.  Tiles with more entries are left to the whole workgroup afterwards.
template <int TW>
__device__ __forceinline__ int feature_tile_group_t(const TransposeArgs& ta, int group, uint32_t* lds, int* big) {
  constexpr int ROWS = TW * 32;
  const int B = ta.B;
  const PairsDev& pd = ta.pd;
  const int32_t* __restrict__ ids = ta.ids;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = (int)blockDim.x >> 6;
  int& nbig = big[16];                                   // big[0 .. 15]: tiles left to the workgroup
  if (tid == 0) nbig = 0;
  __syncthreads();
  for (int rep = 0; rep < kTilesPerWave; ++rep) {
  const int tileno = (group * kTilesPerWave + rep) * nw + wave;
  if (tileno < ta.ntiles) {
    const int row0 = tileno * ROWS;
    uint32_t* skey = lds + wave * 132;                   // [64] row in tile << 16 | sample
    uint32_t* spos = skey + 64;                          // [64] position in the batch's feature arrays
    uint32_t* cnt = spos + 64;                           // [1]
    // the tile's segments, four per lane at a time with their reads in flight together (a batch of up to
    // 256 samples: the registers of the count serve the gather as well)
    int2 v[4];
    auto load_chunk = [&](int i0) {
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int i = i0 + k * 64 + lane;
        v[k] = i < B ? ta.xse[(size_t)tileno * B + i] : make_int2(0, 0);
      }
    };
    const int nchunk = (B + 255) >> 8;
    uint32_t total = 0;
    for (int ch = 0; ch < nchunk; ++ch) {
      load_chunk(ch << 8);
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const int lo = max(v[k].x, 0), hi = min(v[k].y, ta.x_nnz);
        total += hi > lo ? (uint32_t)(hi - lo) : 0u;
      }
    }
    total = wave_sum(total);
    if (total > 64u) {
      if (lane == 0) big[atomicAdd(&nbig, 1)] = tileno;
    } else {
      if (lane == 0) *cnt = 0;
      __builtin_amdgcn_wave_barrier();
      for (int ch = 0; ch < nchunk; ++ch) {              // (an empty tile still clears what bad data may have left)
          if (nchunk > 1) load_chunk(ch << 8);
          int first[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) {                   // (nearly every segment holds one feature)
            const int lo = max(v[k].x, 0), hi = min(v[k].y, ta.x_nnz);
            first[k] = hi > lo ? ids[lo] : -1;
          }
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int i = (ch << 8) + k * 64 + lane;
            const int lo = max(v[k].x, 0), hi = min(v[k].y, ta.x_nnz);
            for (int p = lo; p < hi; ++p) {
              const int r = (p == lo ? first[k] : ids[p]) - row0;
              if ((unsigned)r < (unsigned)ROWS) {
                const uint32_t at = atomicAdd(cnt, 1u);
                if (at < 64u) { skey[at] = ((uint32_t)r << 16) | (uint32_t)i; spos[at] = (uint32_t)p; }
              }
            }
            if (v[k].x | v[k].y) ta.xse[(size_t)tileno * B + i] = make_int2(0, 0);   // all-zero again for the next batch
          }
        }
      __builtin_amdgcn_wave_barrier();
      const uint32_t n = min(*cnt, 64u);
      uint32_t key = (uint32_t)lane < n ? skey[lane] : 0xffffffffu;
      uint32_t pos = (uint32_t)lane < n ? spos[lane] : 0u;
#pragma unroll
      for (int k = 2; k <= 64; k <<= 1)                   // bitonic sort across the lanes, ascending keys
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
          const uint32_t okey = __shfl_xor(key, j), opos = __shfl_xor(pos, j);
          const bool up = (lane & k) == 0, lower = (lane & j) == 0;
          const bool take = (lower == up) ? okey < key : okey > key;
          if (take) { key = okey; pos = opos; }
        }
      const uint32_t prev = __shfl_up(key, 1);
      const bool head = (uint32_t)lane < n && (lane == 0 || (prev >> 16) != (key >> 16));
      const unsigned long long heads = __ballot(head);
      const uint32_t nu = (uint32_t)__popcll(heads);
      if (lane == 0) {
        pd.tile_nu[tileno] = (int32_t)nu;
        if (nu > *(volatile uint32_t*)pd.max_nu) atomicMax(pd.max_nu, nu);
      }
      const uint32_t base = (uint32_t)tileno * 64u;      // (these tiles have 64 pairs of room each, ahead of the regions)
      if ((uint32_t)lane < n) pd.pairs[base + lane] = make_int2((int)(key & 0xffffu), (int)pos);
      if (head) {
        const unsigned long long above = lane < 63 ? heads >> (lane + 1) : 0ull;
        const uint32_t c = above ? (uint32_t)__ffsll((long long)above) : n - (uint32_t)lane;
        const uint32_t us = (uint32_t)tileno * (uint32_t)ROWS + (uint32_t)__popcll(heads & ((1ull << lane) - 1ull));
        pd.umeta[us] = make_int4(row0 + (int)(key >> 16), (int)(base + lane), (int)c, 0);
        if (ta.touched) ta.touched[row0 + (int)(key >> 16)] = 1;
        if ((int)c > kLongRow) {
          const uint32_t l = atomicAdd(pd.nlong, 1u);
          if (l < (uint32_t)pd.long_cap) pd.longlist[l] = (int32_t)us;
        }
      }
    }
  }
  }
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(nbig);
}

// The feature tiles of workgroup role `role` of a launch: its own tile, or -- in grouped mode -- the
// tiles of its group that its waves could not finish alone.
template <int TW>
__device__ __forceinline__ void feature_tile_role_t(const TransposeArgs& ta, int role, uint32_t* lds) {
  __shared__ int big[17];                                // [0 .. 15] tiles left to the whole workgroup, [16] their number
  static_assert(kTilesPerWave * 8 <= 16, "one slot per tile of a group of eight waves");
  int nb = 1;
  if (ta.grouped) nb = feature_tile_group_t<TW>(ta, role, lds, big);
#pragma unroll 1
  for (int q = 0; q < nb; ++q) {
    const int t = ta.grouped ? __builtin_amdgcn_readfirstlane(big[q]) : role;
    __syncthreads();
    transpose_tile_t<true, TW, false>(ta, t, lds);
  }
}

// (the choice of the tile size stays outside the loop above: one copy of the tile code per loop)
__device__ __forceinline__ void feature_tile_role(const TransposeArgs& ta, int role, uint32_t* lds) {
  switch (ta.TW) {
    case 32: feature_tile_role_t<32>(ta, role, lds); break;
    case 16: feature_tile_role_t<16>(ta, role, lds); break;
    case 8: feature_tile_role_t<8>(ta, role, lds); break;
    case 4: feature_tile_role_t<4>(ta, role, lds); break;
    case 2: feature_tile_role_t<2>(ta, role, lds); break;
    default: feature_tile_role_t<1>(ta, role, lds); break;
  }
}

template <bool FEAT, bool BITS>
__device__ __forceinline__ void transpose_tile(const TransposeArgs& ta, int tileno, uint32_t* lds) {
  switch (ta.TW) {
    case 32: transpose_tile_t<FEAT, 32, BITS>(ta, tileno, lds); break;
    case 16: transpose_tile_t<FEAT, 16, BITS>(ta, tileno, lds); break;
    case 8: transpose_tile_t<FEAT, 8, BITS>(ta, tileno, lds); break;
    case 4: transpose_tile_t<FEAT, 4, BITS>(ta, tileno, lds); break;
    case 2: transpose_tile_t<FEAT, 2, BITS>(ta, tileno, lds); break;
    default: transpose_tile_t<FEAT, 1, BITS>(ta, tileno, lds); break;
  }
}

// Workgroups a launch spends on the tiles of `t` (workgroups of `threads` threads).
__host__ __device__ inline int transpose_roles(const TransposeArgs& t, int threads) {
  const int per = (threads >> 6) * kTilesPerWave;
  return t.grouped ? (t.ntiles + per - 1) / per : t.ntiles;
}

inline size_t transpose_lds(int TW, int Bpad) {
  const size_t rows = (size_t)TW * 32, GW = (size_t)Bpad >> 5, groups = (size_t)Bpad >> 6;
  const size_t tile = (rows * GW + rows + (size_t)TW * 3 + 4 + rows) * 4 + rows * 2 + groups * rows * 2;
  const size_t waves = 16 * 132 * 4;                     // a corner per wave when the waves take a tile each
  return tile > waves ? tile : waves;
}

}  // namespace slide
