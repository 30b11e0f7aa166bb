// Active-set retrieval (paper Algorithm 1, the retrieval step of the loop body; Figure 1: the union of the
// neurons returned by every table) and the index structures the float kernels consume.
//
//  lookup_union : one workgroup per sample.  Reads one bucket per table, sets one bit per candidate
//                 and per label in an LDS bitmap over the neuron ids (deduplication and sorting
//                 are free: the bitmap is swept in id order), writes per-tile population counts
//                 (their prefix splits the sample's id list into one segment per tile of rows).
//                 It also emits the compact ascending id list per sample + the labels' slots and hands
//                 the sample its forward work items (chunks of kChunk active neurons).
#include "slide_internal.h"
#include "spmm.h"
#include "wave_ops.h"

namespace slide {

constexpr int kSelWords = 264;     // 256 histogram bins + counters of the sampling-budget selection

// Counter-based random numbers of the sampling budget (Section 3.7): the 32-bit finaliser of
// MurmurHash3, a bijection, keyed by (seed, step, sample) and then by neuron or draw number.
__device__ __forceinline__ uint32_t sample_mix(uint32_t x) {
  x ^= x >> 16; x *= 0x85EBCA6Bu; x ^= x >> 13; x *= 0xC2B2AE35u; x ^= x >> 16;
  return x;
}
__device__ __forceinline__ uint32_t sample_prio(uint32_t base, uint32_t j) { return sample_mix(base + 0x9E3779B1u * (j + 1u)); }
__device__ __forceinline__ uint32_t sample_draw(uint32_t base, uint32_t d, uint32_t N) {
  return __umulhi(sample_mix((base ^ 0xA5A5A5A5u) + 0x632BE5ABu * (d + 1u)), N);
}

// Exclusive scan over a workgroup of up to 1024 threads; sm: 17 words of LDS.
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* sm, uint32_t& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const uint32_t inc = wave_incl_scan_add(v);
  __syncthreads();
  if (lane == 63) sm[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
  for (int w = 0; w < nw; ++w) { const uint32_t x = sm[w]; if (w < wave) base += x; tot += x; }
  total = tot;
  return base + inc - v;
}

// Position of bitmap word w of sample i in the spill copy of the bitmaps (used only when a bitmap
// does not fit the LDS in one piece): tile-major, [tile][sample][TW
// words], so that the transposition reads one contiguous block per tile; the per-sample writer
// pays the stride instead (full 4*TW-byte records).
__device__ __forceinline__ size_t act_index(const ActiveDev& ad, int i, int w) {
  const int tws = __ffs(ad.TW) - 1;
  return ((size_t)(w >> tws) * ad.B + i) * ad.TW + (w & (ad.TW - 1));
}

// Hash codes of one vector held in LDS, one thread per elementary hash (same arithmetic, in the
// same order, as the row-tile kernel in hash.hip).  raw[e]: DWTA winner position or -1, SimHash bit.
__device__ void sample_hash_codes(const HashDev& hd, const float* hvec, int8_t* raw, uint32_t* codes_out,
                                  uint32_t* __restrict__ codes_global) {
  const int tid = threadIdx.x, nthr = blockDim.x;
  if (hd.kind == SLIDE_HASH_SIMHASH) {
    const int half = hd.Spad / 2;
    for (int e = tid; e < hd.NH; e += nthr) {
      const uint32_t* __restrict__ sw = hd.words + (size_t)e * half;
      float acc = 0.0f;
      for (int s2 = 0; s2 < half; ++s2) {
        const uint32_t w = sw[s2];
        const float x0 = hvec[w & 0x7fffu];
        acc = (w & 0x8000u) ? acc - x0 : acc + x0;
        if (2 * s2 + 1 < hd.S) {
          const float x1 = hvec[(w >> 16) & 0x7fffu];
          acc = (w & 0x80000000u) ? acc - x1 : acc + x1;
        }
      }
      raw[e] = acc > 0.0f ? 1 : 0;
    }
    __syncthreads();
    for (int t = tid; t < hd.L; t += nthr) {
      uint32_t c = 0;
      for (int k = 0; k < hd.K; ++k) c |= (uint32_t)raw[t * hd.K + k] << k;
      codes_out[t] = c;
      codes_global[t] = c;
    }
  } else {
    const int half = hd.m / 2;
    for (int e = tid; e < hd.NH; e += nthr) {
      int best_p = -1;
      float best = 0.0f;
      for (int p2 = 0; p2 < half; ++p2) {
        const uint32_t w = hd.words[(size_t)e * half + p2];
        const float x0 = hvec[w & 0xffffu], x1 = hvec[w >> 16];
        if (x0 != 0.0f && x0 == x0 && (best_p < 0 || x0 > best)) { best_p = 2 * p2; best = x0; }
        if (x1 != 0.0f && x1 == x1 && (best_p < 0 || x1 > best)) { best_p = 2 * p2 + 1; best = x1; }
      }
      raw[e] = (int8_t)best_p;
    }
    __syncthreads();
    for (int t = tid; t < hd.L; t += nthr) {
      uint32_t c = 0;
      for (int k = 0; k < hd.K; ++k) {
        const int e = t * hd.K + k;
        int val = raw[e];
        if (val < 0) {                                   // empty bin: borrow from the probe sequence
          val = 0;
          for (uint32_t tr = 1; tr <= 100; ++tr) {
            const uint32_t u = hd.dens_a * (uint32_t)(e + 1) + hd.dens_b * tr;
            const int r2 = raw[(u >> 8) % (uint32_t)hd.NH];
            if (r2 >= 0) { val = r2; break; }
          }
        }
        c |= (uint32_t)val << (k * hd.lgm);
      }
      codes_out[t] = c;
      codes_global[t] = c;
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(1024) void lookup_union_kernel(
    ActiveDev ad, HashDev hd, const float* __restrict__ h, SpmmArgs sp, const uint32_t* __restrict__ off,
    const int32_t* __restrict__ ids, uint32_t nb, uint32_t* __restrict__ codes,
    const int32_t* __restrict__ y_indptr, const int32_t* __restrict__ y_indices, int include_labels,
    int32_t* __restrict__ ncand, Ctrl* ctrl, int segw) {
  extern __shared__ uint32_t lds[];
  uint32_t* bm = lds;                    // [segw] bitmap segment
  uint32_t* o0s = bm + segw;             // [L] bucket start inside its table (first: the table codes)
  uint32_t* pos = o0s + ad.L;            // [L+1] exclusive prefix of the bucket lengths
  uint32_t* sm = pos + ad.L + 1;         // [20] scan scratch + counters
  float* hvec = (float*)(sm + 20);       // [H] the sample's hidden activations
  uint32_t* tcnt = (uint32_t*)(hvec + hd.H);   // [NT] active neurons per tile, then their exclusive prefix
  uint32_t* sel = tcnt + ad.NT;          // [kSelWords] sampling budget: digit histogram + counters
  int8_t* raw = (int8_t*)(sel + kSelWords);    // [NH] elementary hash values
  const int i = blockIdx.x, tid = threadIdx.x, nthr = blockDim.x;
  const int lane = tid & 63;
  if (tid == 0) { sm[17] = 0; sm[18] = 0; }
  if (i == 0 && tid == 0) {                              // consumed after this kernel
    ctrl->nlong2 = 0; ctrl->max_nu2 = 0;
    if (sp.W1) { ctrl->p1 = 0; ctrl->nlong1 = 0; ctrl->max_nu1 = 0; }
    for (int r = 0; r < kPairRegions; ++r) ctrl->p1r[r] = 0;
  }

  // the sample's slice of the sample-major arrays: room for every candidate plus its labels
  int y0 = 0, nlab = 0;
  if (include_labels) {
    y0 = min(max(y_indptr[i], 0), ad.num_labels);
    nlab = min(max(y_indptr[i + 1], y0), ad.num_labels) - y0;
  }
  const int base_i = i * ad.PS + y0;
  const int tws = __ffs(ad.TW) - 1;                      // TW is a power of two >= 4
  const int LT = ad.TW >> 2;                             // lanes per tile in the sweeps (four words per lane)

  const bool budgeted = ad.budget > 0 && include_labels;  // (then the whole bitmap is one segment)
  // The labels of bitmap segment [seg0, seg0 + sw) words (their "new bit" test counts the distinct
  // labels, so they go in before any candidate; under a sampling budget they go in after it).
  auto segment_labels = [&](int seg0, int sw) {
    if (budgeted) return;
    const int64_t lo = (int64_t)seg0 * 32, hi = lo + (int64_t)sw * 32;
    for (int q = tid; q < nlab; q += nthr) {
      const int y = y_indices[y0 + q];
      if (y < 0 || y >= ad.N) { if (seg0 == 0) atomicOr(&ctrl->status, SLIDE_FLAG_BAD_LABEL); continue; }
      if (y >= lo && y < hi) {
        const uint32_t bit = 1u << (y & 31);
        const uint32_t old = atomicOr(&bm[(y - lo) >> 5], bit);
        if (!(old & bit)) atomicAdd(&sm[17], 1u);       // distinct labels
      }
    }
  };
  auto clear_segment = [&](int sw) {
    for (int q = tid; q < sw / 4; q += nthr) ((uint4*)bm)[q] = make_uint4(0u, 0u, 0u, 0u);
  };

  // a1 (sparse-input mode): the sample's hidden activations, by the first waves of the workgroup;
  // the first bitmap segment is cleared meanwhile.  Dense-hidden mode: the activations are read.
  if (sp.W1 && hd.H <= nthr && spmm_stage_rows(segw, hd.H, nthr) >= 32) {
    spmm_sample_staged(sp, i, ad.B, (float*)bm, segw, hvec, ctrl);   // (the bitmap's room is free until it is cleared)
    clear_segment(min(segw, ad.NWpad));
  } else {
    clear_segment(min(segw, ad.NWpad));
    if (sp.W1) {
      const int wave = tid >> 6;
      if (wave * 128 < hd.H) spmm_sample(sp, i, ad.B, wave, lane, hvec, ctrl);
    } else {
      for (int c = tid; c < hd.H; c += nthr) hvec[c] = h[(size_t)i * hd.H + c];
    }
  }
  __syncthreads();                                       // (also orders the counters' reset before the labels)
  segment_labels(0, min(segw, ad.NWpad));
  // a2: hash codes of the hidden activations
  sample_hash_codes(hd, hvec, raw, o0s, codes + (size_t)i * ad.L);

  uint32_t carry = 0;
  for (int base = 0; base < ad.L; base += nthr) {
    const int t = base + tid;
    uint32_t len = 0;
    if (t < ad.L) {
      const uint32_t code = o0s[t];
      const uint32_t a = off[(size_t)t * (nb + 1) + code];
      const uint32_t b = off[(size_t)t * (nb + 1) + code + 1];
      len = min(b - a, (uint32_t)ad.C);
      o0s[t] = a;
    }
    uint32_t total;
    const uint32_t ex = block_excl_scan(len, sm, total);
    if (t < ad.L) pos[t] = carry + ex;
    carry += total;
    __syncthreads();
  }
  if (tid == 0) pos[ad.L] = carry;
  __syncthreads();
  const uint32_t T = pos[ad.L];

  // Sampling budget: the bitmap holds the retrieved neurons.  The labels do not count (their bits are
  // taken out first and put back at the end); more than `budget` left: keep the `budget` of smallest
  // priority (a radix selection over the 32-bit priorities, which are distinct); fewer, with the fill
  // option: draws d = 0, 1, 2, ... accepted when new, in rounds that cannot overshoot.
  auto apply_budget = [&]() {
    uint32_t* hist = sel;                                // [256]
    uint32_t* misc = sel + 256;                          // [0] count, [1] prefix, [2] still to take, [3] new bits
    const uint32_t base = sample_mix(ad.sample_seed + 0x9E3779B9u * ad.step + 0x7F4A7C15u * (uint32_t)i);
    const int nq = ad.NWpad / 4;
    for (int q = tid; q < nlab; q += nthr) {
      const int y = y_indices[y0 + q];
      if (y >= 0 && y < ad.N) atomicAnd(&bm[y >> 5], ~(1u << (y & 31)));
    }
    if (tid == 0) { misc[0] = 0; misc[1] = 0; misc[2] = (uint32_t)ad.budget; }
    __syncthreads();
    uint32_t c = 0;
    for (int q = tid; q < nq; q += nthr) {
      const uint4 wd = ((const uint4*)bm)[q];
      c += __popc(wd.x) + __popc(wd.y) + __popc(wd.z) + __popc(wd.w);
    }
    c = wave_sum(c);
    if (lane == 0 && c) atomicAdd(&misc[0], c);
    __syncthreads();
    const uint32_t have = misc[0];
    if (have > (uint32_t)ad.budget) {
      for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        for (int b = tid; b < 256; b += nthr) hist[b] = 0;
        __syncthreads();
        const uint32_t prefix = misc[1];
        for (int q = tid; q < nq; q += nthr) {
          const uint4 wd = ((const uint4*)bm)[q];
          const uint32_t ww[4] = {wd.x, wd.y, wd.z, wd.w};
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            uint32_t word = ww[k];
            while (word) {
              const int b = __ffs(word) - 1;
              word &= word - 1;
              const uint32_t p = sample_prio(base, (uint32_t)((4 * q + k) * 32 + b));
              const uint32_t upper = pass == 0 ? 0u : p >> ((shift + 8) & 31);   // the digits fixed so far
              if (upper == prefix) atomicAdd(&hist[(p >> shift) & 255u], 1u);
            }
          }
        }
        __syncthreads();
        if (tid < 64) {                                  // the digit that holds the misc[2]-th smallest: wave 0,
          const uint32_t h0 = hist[4 * lane], h1 = hist[4 * lane + 1], h2 = hist[4 * lane + 2], h3 = hist[4 * lane + 3];
          const uint32_t four = h0 + h1 + h2 + h3;       // four bins per lane
          const uint32_t inc = wave_incl_scan_add(four);
          const uint32_t take = misc[2];
          const unsigned long long reached = __ballot(inc >= take);
          if (reached && lane == __ffsll(reached) - 1) {
            uint32_t cum = inc - four;
            int bin = 4 * lane;
            if (cum + h0 < take) { cum += h0; ++bin;
              if (cum + h1 < take) { cum += h1; ++bin;
                if (cum + h2 < take) { cum += h2; ++bin; } } }
            misc[1] = (prefix << 8) | (uint32_t)bin;
            misc[2] = take - cum;
          }
        }
        __syncthreads();
      }
      const uint32_t last = misc[1];                     // the largest priority that stays
      for (int q = tid; q < nq; q += nthr) {
        const uint4 wd = ((const uint4*)bm)[q];
        if (!(wd.x | wd.y | wd.z | wd.w)) continue;
        uint32_t ww[4] = {wd.x, wd.y, wd.z, wd.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          uint32_t word = ww[k];
          while (word) {
            const int b = __ffs(word) - 1;
            word &= word - 1;
            if (sample_prio(base, (uint32_t)((4 * q + k) * 32 + b)) > last) ww[k] &= ~(1u << b);
          }
        }
        ((uint4*)bm)[q] = make_uint4(ww[0], ww[1], ww[2], ww[3]);
      }
    } else if (ad.fill && have < (uint32_t)ad.budget) {
      uint32_t need = (uint32_t)ad.budget - have, drawn = 0;
      const uint32_t dmax = 4u * (uint32_t)ad.budget + 64u;
      while (need > 0 && drawn < dmax) {                 // (uniform: both come from LDS values read after barriers)
        const uint32_t n = min(need, dmax - drawn);
        if (tid == 0) misc[3] = 0;
        __syncthreads();
        for (uint32_t d = tid; d < n; d += nthr) {
          const uint32_t j = sample_draw(base, drawn + d, (uint32_t)ad.N);
          bool is_label = false;
          for (int q = 0; q < nlab; ++q) is_label |= y_indices[y0 + q] == (int)j;
          if (!is_label) {
            const uint32_t bit = 1u << (j & 31);
            if (!(atomicOr(&bm[j >> 5], bit) & bit)) atomicAdd(&misc[3], 1u);
          }
        }
        __syncthreads();
        need -= misc[3];
        drawn += n;
        __syncthreads();
      }
    }
    __syncthreads();
    for (int q = tid; q < nlab; q += nthr) {             // the labels, counted once each
      const int y = y_indices[y0 + q];
      if (y < 0 || y >= ad.N) { atomicOr(&ctrl->status, SLIDE_FLAG_BAD_LABEL); continue; }
      const uint32_t bit = 1u << (y & 31);
      if (!(atomicOr(&bm[y >> 5], bit) & bit)) atomicAdd(&sm[17], 1u);
    }
    __syncthreads();
  };

  uint32_t my_cnt = 0;
  for (int seg0 = 0; seg0 < ad.NWpad; seg0 += segw) {
    const int sw = min(segw, ad.NWpad - seg0);
    const int64_t lo = (int64_t)seg0 * 32, hi = lo + (int64_t)sw * 32;
    if (seg0 > 0) { clear_segment(sw); __syncthreads(); segment_labels(seg0, sw); __syncthreads(); }
    auto candidate = [&](uint32_t c) -> int {           // the c-th of the sample's T bucket entries
      int a = 0, b = ad.L;                              // last t with pos[t] <= c
      while (b - a > 1) { const int mid = (a + b) >> 1; if (pos[mid] <= c) a = mid; else b = mid; }
      return ids[(size_t)a * ad.N + o0s[a] + (c - pos[a])];
    };
    for (uint32_t c0 = 0; c0 < T; c0 += 4 * nthr) {     // four entries per thread in flight
      int j[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { const uint32_t c = c0 + u * nthr + tid; j[u] = c < T ? candidate(c) : -1; }
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (j[u] >= lo && j[u] < hi) atomicOr(&bm[(j[u] - lo) >> 5], 1u << (j[u] & 31));
    }
    __syncthreads();
    if (budgeted) apply_budget();
    // sweep, four words per lane: population per tile (the last lane of a tile holds its count)
    for (int qb = 0; qb < sw / 4; qb += nthr) {
      const int q = qb + tid;
      const uint4 wd = q < sw / 4 ? ((const uint4*)bm)[q] : make_uint4(0u, 0u, 0u, 0u);
      uint32_t c = __popc(wd.x) + __popc(wd.y) + __popc(wd.z) + __popc(wd.w);
      my_cnt += c;
      if (q < sw / 4 && (segw < ad.NWpad || ad.write_act)) {   // spill: re-read by the id sweep / by the row lists
        uint32_t* dst = &ad.act[act_index(ad, i, seg0 + 4 * q)];
        *(uint4*)dst = wd;
      }
      c = small_group_incl_scan_add(c, LT);
      if (q < sw / 4 && (lane & (LT - 1)) == LT - 1) tcnt[(seg0 + 4 * q) >> tws] = c;
    }
    __syncthreads();
  }
  for (int d = 32; d > 0; d >>= 1) my_cnt += __shfl_xor(my_cnt, d);
  if (lane == 0) atomicAdd(&sm[18], my_cnt);
  __syncthreads();
  const int n = (int)sm[18];
  const uint32_t nch = ((uint32_t)n + kChunk - 1) / kChunk;
  if (tid == 0) {
    ad.cnt[i] = n; ad.ny[i] = (int32_t)sm[17]; ncand[i] = (int32_t)T; ad.as_base[i] = base_i;
    // forward work items of this sample: the partial results of its chunk c go to slot
    // base_i / kChunk + i + c (the samples' slices of the sample-major arrays do not overlap, so neither
    // do these), and the largest number of items of any sample bounds the forward launch's enumeration
    // (most samples find the maximum already there: only a larger count updates it)
    ad.chunk_ptr[i] = base_i / kChunk + i;
    if (nch > *(volatile uint32_t*)&ctrl->max_nch[ad.par]) atomicMax(&ctrl->max_nch[ad.par], nch);
    if (i == 0) ctrl->max_nch[ad.par ^ 1] = 0;           // the previous call's: clear for the next call
  }

  // per-tile counts -> exclusive prefix inside the sample (rank of the tile's first active neuron)
  uint32_t* rk = tcnt;
  carry = 0;
  for (int base = 0; base < ad.NT; base += nthr) {
    const int t = base + tid;
    const uint32_t v = t < ad.NT ? rk[t] : 0u;
    uint32_t total;
    const uint32_t ex = block_excl_scan(v, sm, total);
    if (t < ad.NT) { rk[t] = carry + ex; ad.rankT[(size_t)t * ad.B + i] = carry + ex; }
    carry += total;
    __syncthreads();
  }
  if (tid == 0) ad.rankT[(size_t)ad.NT * ad.B + i] = carry;   // closes the last tile's segment
  // compact ascending id list: sweep the bitmap (still in LDS if it fitted in one segment)
  const bool in_lds = segw >= ad.NWpad;
  for (int qb = 0; qb < ad.NWpad / 4; qb += nthr) {
    const int q = qb + tid;
    uint4 wd = make_uint4(0u, 0u, 0u, 0u);
    if (q < ad.NWpad / 4) wd = in_lds ? ((const uint4*)bm)[q] : *(const uint4*)&ad.act[act_index(ad, i, 4 * q)];
    const uint32_t c = __popc(wd.x) + __popc(wd.y) + __popc(wd.z) + __popc(wd.w);
    const uint32_t inc = small_group_incl_scan_add(c, LT);
    if (c) {
      int slot = base_i + (int)(rk[(4 * q) >> tws] + inc - c);
      const uint32_t ww[4] = {wd.x, wd.y, wd.z, wd.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        uint32_t word = ww[k];
        while (word) {
          const int b = __ffs(word) - 1;
          ad.as_ids[slot] = (4 * q + k) * 32 + b;
          ++slot;
          word &= word - 1;
        }
      }
    }
  }
  if (!in_lds) __syncthreads();                      // (the labels are then looked up in the list just written)
  // for every label entry its slot (-1 for invalid or repeated entries): these slots are the label flags
  for (int q = tid; q < nlab; q += nthr) {
    const int y = y_indices[y0 + q];
    int slot = -1;
    if (y >= 0 && y < ad.N) {
      int a = 0;
      bool found;
      if (in_lds) {                                      // rank of the label in the bitmap = its slot
        const int w = y >> 5, w0 = w & ~(ad.TW - 1);
        a = (int)rk[w >> tws] + __popc(bm[w] & ((1u << (y & 31)) - 1u));
        for (int q = w0; q < w; ++q) a += __popc(bm[q]);
        found = (bm[w] >> (y & 31)) & 1u;
      } else {
        int b = n;
        while (a < b) { const int mid = (a + b) >> 1; if (ad.as_ids[base_i + mid] < y) a = mid + 1; else b = mid; }
        found = a < n && ad.as_ids[base_i + a] == y;
      }
      if (found) {
        slot = base_i + a;
        for (int q2 = 0; q2 < q; ++q2) if (y_indices[y0 + q2] == y) { slot = -1; break; }
      }
    }
    ad.ylist[y0 + q] = slot;
  }
}

size_t lookup_fixed_lds(int L, int H, int NT, int NH) {
  return ((size_t)2 * L + 1 + 20 + H + NT + kSelWords) * 4 + (((size_t)NH + 3) & ~(size_t)3);
}

bool lookup_bitmap_fits(int NWpad, int NT, int L, int H, int NH, size_t lds_limit) {
  return lookup_fixed_lds(L, H, NT, NH) + (size_t)NWpad * 4 <= lds_limit;
}

hipError_t active_setup_attributes(size_t* lds_limit_out) {
  int dev = 0, lim = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  e = hipDeviceGetAttribute(&lim, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
  if (e != hipSuccess) return e;
  if (lim > 160 * 1024) lim = 160 * 1024;
  e = hipFuncSetAttribute((const void*)lookup_union_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
  if (e != hipSuccess) return e;
  *lds_limit_out = (size_t)lim;
  return hipSuccess;
}

hipError_t launch_lookup_union(const ActiveDev& ad, const HashDev& hd, const float* h, const SpmmArgs& sp,
                               const TablesDev& td, uint32_t* codes, const int32_t* y_indptr,
                               const int32_t* y_indices, int include_labels, int32_t* ncand, Ctrl* ctrl,
                               size_t lds_limit, hipStream_t s) {
  const size_t fixed = lookup_fixed_lds(ad.L, hd.H, ad.NT, hd.NH);
  // (slide_init has refused configurations whose fixed part leaves less than kLookupMinSegment words:
  // with a tiny segment the kernel would sweep all candidates once per few hundred neurons)
  if (fixed + (size_t)kLookupMinSegment * 4 > lds_limit) return hipErrorInvalidValue;
  size_t avail = (lds_limit - fixed) / 4;
  int segw = (int)(avail / 32 * 32);
  if (segw > ad.NWpad) segw = ad.NWpad;
  const size_t bytes = (size_t)segw * 4 + fixed;
  hipLaunchKernelGGL(lookup_union_kernel, dim3(ad.B), dim3(1024), bytes, s, ad, hd, h, sp, td.off, td.ids, td.nb,
                     codes, y_indptr, y_indices, include_labels, ncand, ctrl, segw);
  return hipGetLastError();
}

}  // namespace slide
