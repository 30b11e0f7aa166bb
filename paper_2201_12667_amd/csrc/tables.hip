// Hash-table build / rebuild (paper Algorithm 1 "hash weights to hash tables", rebuilt on a
// schedule, Section 3.1).  Layout: per table a CSR over the 2^bits codes -- off[t][code] is the
// start of the bucket inside ids[t][0..N).  A bucket's first min(size, C) ids are its kept members,
// ascending by id; which members are kept when size > C is decided by the smallest
// (priority, id) keys.
//
// The build is a two-level counting sort with every counter in LDS (no global atomics on the
// tables): (1) hash every row of W2, codes stored table-major; (2) split each table's rows by the
// high bits of the code: per-slab LDS histograms, a scan over slabs and digits, and a scatter of
// (code, id) entries into their partition; (3) one workgroup per (table, partition) counts the low
// bits in LDS, writes that partition's offsets, places the ids, and sorts the small buckets in
// place; (4) buckets that are long or over capacity are queued and handled by one workgroup each.
#include "slide_internal.h"
#include "wave_ops.h"

namespace slide {

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t step = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = v;
}

// Plain streaming copy, 16 bytes per thread per step: the yardstick the HBM counters and the
// achievable bandwidth are calibrated against.
__global__ void copy_kernel(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t step = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += step) dst[i] = src[i];
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (uint4*)dst, (const uint4*)src, n16);
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
  return hipGetLastError();
}

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t t = __shfl_up(v, d);
    if (lane >= d) v += t;
  }
  return v;
}

constexpr int kSlab = 16384;       // rows per workgroup in the partition passes

__global__ __launch_bounds__(1024) void part_hist_kernel(const uint32_t* __restrict__ codes_t, int64_t N, int lb,
                                                         int nbins, uint32_t* __restrict__ bh, int nslab) {
  extern __shared__ uint32_t hst[];
  const int slab = blockIdx.x, tid = threadIdx.x;
  const size_t t = blockIdx.y;
  for (int b = tid; b < nbins; b += 1024) hst[b] = 0;
  __syncthreads();
  const int64_t j0 = (int64_t)slab * kSlab;
  for (int k = 0; k < kSlab / 1024; ++k) {
    const int64_t j = j0 + k * 1024 + tid;
    if (j < N) atomicAdd(&hst[codes_t[t * N + j] >> lb], 1u);
  }
  __syncthreads();
  for (int b = tid; b < nbins; b += 1024) bh[(t * nslab + slab) * nbins + b] = hst[b];
}

// Exclusive scan over a workgroup of 1024 threads; sm: 17 words of LDS.
__device__ uint32_t block_excl_scan1024(uint32_t v, uint32_t* sm, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_incl_scan(v);
  __syncthreads();
  if (lane == 63) sm[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
  for (int w = 0; w < 16; ++w) { const uint32_t x = sm[w]; if (w < wave) base += x; tot += x; }
  *total = tot;
  return base + inc - v;
}

// One workgroup per table: bh[t][slab][d] becomes the number of rows of digit d in earlier slabs,
// pbase[t][d] the start of partition d.
__global__ __launch_bounds__(1024) void part_scan_kernel(uint32_t* bh, int nslab, int nbins, uint32_t* pbase,
                                                         Ctrl* ctrl) {
  __shared__ uint32_t sm[20];
  const size_t t = blockIdx.x;
  const int tid = threadIdx.x;
  uint32_t carry = 0;
  for (int base = 0; base < nbins; base += 1024) {
    const int d = base + tid;
    uint32_t run = 0;
    if (d < nbins)
      for (int slab = 0; slab < nslab; ++slab) {
        uint32_t* p = bh + (t * nslab + slab) * nbins + d;
        const uint32_t v = *p;
        *p = run;
        run += v;
      }
    uint32_t total;
    const uint32_t ex = block_excl_scan1024(run, sm, &total);
    if (d < nbins) pbase[t * (nbins + 1) + d] = carry + ex;
    carry += total;
    __syncthreads();
  }
  if (tid == 0) pbase[t * (nbins + 1) + nbins] = carry;
  if (t == 0 && tid == 0) { ctrl->wl_count = 0; ctrl->overflowed = 0; }
}

// An entry of the partitioned list: (code, row), or -- PACKED, when the low digit and the row index fit
// 32 bits together -- (low digit << rowbits) | row, which halves what the two passes below move.
template <bool PACKED> struct Entry { typedef uint2 type; };
template <> struct Entry<true> { typedef uint32_t type; };

// One workgroup per (slab, table): the slab's entries are first grouped by partition in
// LDS (a local counting sort), then written out, so that every partition receives one contiguous
// run per slab instead of single entries.
template <bool PACKED>
__global__ __launch_bounds__(1024) void part_scatter_kernel(const uint32_t* __restrict__ codes_t, int64_t N, int lb,
                                                            int rowbits, int nbins, const uint32_t* __restrict__ bh,
                                                            int nslab, const uint32_t* __restrict__ pbase,
                                                            typename Entry<PACKED>::type* __restrict__ entries) {
  typedef typename Entry<PACKED>::type E;
  extern __shared__ uint32_t lds[];
  E* stage = (E*)lds;                              // [kSlab] entries grouped by partition
  uint16_t* stage_p = (uint16_t*)(lds + kSlab);    // [kSlab] PACKED: their partitions (the entry no longer says)
  uint32_t* lstart = lds + 2 * kSlab;              // [nbins] first staged entry of the partition
  uint32_t* cur = lstart + nbins;                  // [nbins] counters, then cursors
  uint32_t* gbase = cur + nbins;                   // [nbins] where the partition's run goes in the table's entries
  uint32_t* sm = gbase + nbins;                    // [20]
  const int slab = blockIdx.x, tid = threadIdx.x;
  const size_t t = blockIdx.y;
  for (int b = tid; b < nbins; b += 1024) {
    cur[b] = 0;
    gbase[b] = pbase[t * (nbins + 1) + b] + bh[(t * nslab + slab) * nbins + b];
  }
  __syncthreads();
  const int64_t j0 = (int64_t)slab * kSlab;
  const int nvalid = (int)(N - j0 < kSlab ? N - j0 : kSlab);
  uint32_t code[kSlab / 1024];
#pragma unroll
  for (int k = 0; k < kSlab / 1024; ++k) {
    const int r = k * 1024 + tid;
    code[k] = r < nvalid ? codes_t[t * N + j0 + r] : 0u;
    if (r < nvalid) atomicAdd(&cur[code[k] >> lb], 1u);
  }
  __syncthreads();
  uint32_t carry = 0;
  for (int base = 0; base < nbins; base += 1024) {
    const int b = base + tid;
    const uint32_t v = b < nbins ? cur[b] : 0u;
    uint32_t total;
    const uint32_t ex = block_excl_scan1024(v, sm, &total);
    if (b < nbins) lstart[b] = carry + ex;
    carry += total;
    __syncthreads();
  }
  for (int b = tid; b < nbins; b += 1024) cur[b] = lstart[b];
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kSlab / 1024; ++k) {
    const int r = k * 1024 + tid;
    if (r < nvalid) {
      const uint32_t pos = atomicAdd(&cur[code[k] >> lb], 1u);
      if constexpr (PACKED) {
        stage[pos] = ((code[k] & ((1u << lb) - 1u)) << rowbits) | (uint32_t)(j0 + r);
        stage_p[pos] = (uint16_t)(code[k] >> lb);
      } else {
        stage[pos] = make_uint2(code[k], (uint32_t)(j0 + r));
      }
    }
  }
  __syncthreads();
  E* out = entries + t * N;
  for (int k = tid; k < nvalid; k += 1024) {
    const E e = stage[k];
    uint32_t p;
    if constexpr (PACKED) p = stage_p[k]; else p = e.x >> lb;
    out[gbase[p] + ((uint32_t)k - lstart[p])] = e;
  }
}

constexpr int kStageIds = 4096;    // ids of a partition staged in LDS by part_buckets (larger partitions go through memory)
constexpr int kLdsSort = 32;       // buckets up to this size are sorted by one thread while staged in LDS

// One workgroup per (partition d, table t): buckets (d << lb) .. (d << lb) + 2^lb - 1.  Counts the
// low digit, writes the partition's offsets, groups the ids by bucket -- in LDS when the partition
// fits, so that the table receives whole lines -- and sorts the small buckets; long and
// over-capacity buckets are queued.
template <bool PACKED>
__global__ __launch_bounds__(256) void part_buckets_kernel(const typename Entry<PACKED>::type* __restrict__ entries,
                                                           const uint32_t* __restrict__ pbase, int nbins, int lb,
                                                           int rowbits, uint32_t nb, int64_t N, int C,
                                                           uint32_t* __restrict__ off,
                                                           int32_t* ids, uint64_t* worklist, uint32_t wl_cap,
                                                           Ctrl* ctrl) {
  extern __shared__ uint32_t lds[];
  const int nlo = 1 << lb, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nchunk = (nlo + 63) >> 6;    // 64 buckets per scan chunk
  uint32_t* cur = lds;                   // [nlo] counters, then bucket starts, then (after placing) bucket ends
  uint32_t* csum = cur + nlo;            // [nchunk] ids in the chunk, then in the chunks before it
  int32_t* idl = (int32_t*)(csum + nchunk);   // [kStageIds] the partition's ids grouped by bucket
  const uint32_t d = blockIdx.x;
  const size_t t = blockIdx.y;
  const uint32_t s0 = pbase[t * (nbins + 1) + d], s1 = pbase[t * (nbins + 1) + d + 1];
  const uint32_t mask = (uint32_t)nlo - 1u;
  const typename Entry<PACKED>::type* ent = entries + t * N;
  auto low_digit = [&](typename Entry<PACKED>::type e) -> uint32_t {
    if constexpr (PACKED) return e >> rowbits; else return e.x & mask;
  };
  auto row_of = [&](typename Entry<PACKED>::type e) -> int32_t {
    if constexpr (PACKED) return (int32_t)(e & ((1u << rowbits) - 1u)); else return (int32_t)e.y;
  };
  const bool staged = s1 - s0 <= (uint32_t)kStageIds;
  for (int b = tid; b < nlo; b += 256) cur[b] = 0;
  __syncthreads();
  for (uint32_t e = s0 + tid; e < s1; e += 256) atomicAdd(&cur[low_digit(ent[e])], 1u);
  __syncthreads();
  // exclusive scan of the counters: every wave scans chunks of 64 in registers, wave 0 the chunk sums
  for (int c = wave; c < nchunk; c += 4) {
    const int b = c * 64 + lane;
    const uint32_t v = b < nlo ? cur[b] : 0u;
    const uint32_t inc = wave_incl_scan_add(v);
    if (b < nlo) cur[b] = inc - v;
    if (lane == 63) csum[c] = inc;
  }
  __syncthreads();
  if (wave == 0) {
    uint32_t carry = 0;
    for (int c0 = 0; c0 < nchunk; c0 += 64) {
      const int c = c0 + lane;
      const uint32_t v = c < nchunk ? csum[c] : 0u;
      const uint32_t inc = wave_incl_scan_add(v);
      if (c < nchunk) csum[c] = carry + inc - v;
      carry += (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
    }
  }
  __syncthreads();
  uint32_t* orow = off + t * (nb + 1) + ((size_t)d << lb);
  for (int b = tid; b < nlo; b += 256) {
    const uint32_t st = cur[b] + csum[b >> 6];
    cur[b] = st;
    orow[b] = s0 + st;
  }
  if (d == (uint32_t)nbins - 1 && tid == 0) off[t * (nb + 1) + nb] = (uint32_t)N;
  __syncthreads();
  int32_t* seg = ids + t * N + s0;
  int32_t* place = staged ? idl : seg;
  for (uint32_t e = s0 + tid; e < s1; e += 256) {
    const auto x = ent[e];
    place[atomicAdd(&cur[low_digit(x)], 1u)] = row_of(x);
  }
  __syncthreads();                                  // cur[b] is now the end of bucket b = the start of bucket b + 1
  const uint32_t small = staged ? (uint32_t)kLdsSort : (uint32_t)kSmallBucket;
  uint32_t over = 0;
  for (int b = tid; b < nlo; b += 256) {
    const uint32_t a = b ? cur[b - 1] : 0u, sz = cur[b] - a;
    if (sz > (uint32_t)C) ++over;
    if (sz < 2) continue;
    if (sz <= small && sz <= (uint32_t)C) {
      int32_t* p = place + a;                     // arrival order is arbitrary: restore ascending ids
      for (uint32_t i = 1; i < sz; ++i) {
        const int32_t key = p[i];
        int q = (int)i - 1;
        while (q >= 0 && p[q] > key) { p[q + 1] = p[q]; --q; }
        p[q + 1] = key;
      }
    } else {
      const uint32_t slot = atomicAdd(&ctrl->wl_count, 1u);
      if (slot < wl_cap) worklist[slot] = ((uint64_t)t << 32) | ((d << lb) + (uint32_t)b);
    }
  }
  if (over) atomicAdd(&ctrl->overflowed, over);
  if (staged) {
    __syncthreads();
    for (uint32_t k = tid; k < s1 - s0; k += 256) seg[k] = idl[k];
  }
}

__device__ void bitonic_sort_u64(uint64_t* keys, int n) {
  for (int k = 2; k <= n; k <<= 1)
    for (int j = k >> 1; j > 0; j >>= 1) {
      for (int i = threadIdx.x; i < n / 2; i += 256) {
        const int a = 2 * j * (i / j) + (i % j), b = a + j;
        const bool up = (a & k) == 0;
        const uint64_t x = keys[a], y = keys[b];
        if ((x > y) == up) { keys[a] = y; keys[b] = x; }
      }
      __syncthreads();
    }
}

__device__ __forceinline__ uint32_t overflow_prio(uint32_t j, uint32_t t, uint32_t r, uint32_t pa, uint32_t pb) {
  uint32_t u = pa * (j + 1u) + pb * (t * 65537u + r + 1u);
  u ^= u >> 15; u *= pa; u ^= u >> 13;
  return u;
}

// One workgroup per queued bucket.  size <= C: sort by id.  size > C: stream the members through
// LDS keeping the C smallest (priority, id) keys, then sort the survivors by id.
__global__ __launch_bounds__(256) void big_buckets_kernel(const uint32_t* __restrict__ off, int32_t* ids,
                                                          uint32_t nb, int64_t N, int C, int policy, uint32_t r,
                                                          uint32_t pa, uint32_t pb,
                                                          const uint64_t* __restrict__ worklist,
                                                          uint32_t wl_cap, const Ctrl* ctrl) {
  __shared__ uint64_t keys[kSortCap];
  uint32_t n_items = ctrl->wl_count;
  if (n_items > wl_cap) n_items = wl_cap;
  int capp = 1;
  while (capp < C) capp <<= 1;
  for (uint32_t item = blockIdx.x; item < n_items; item += gridDim.x) {
    const uint64_t w = worklist[item];
    const uint64_t t = w >> 32;
    const uint32_t c = (uint32_t)w;
    const uint32_t o0 = off[t * (nb + 1) + c];
    const uint32_t s = off[t * (nb + 1) + c + 1] - o0;
    int32_t* p = ids + t * N + o0;
    if (s <= (uint32_t)C) {
      int n2 = 2;
      while ((uint32_t)n2 < s) n2 <<= 1;
      for (int i = threadIdx.x; i < n2; i += 256) keys[i] = (uint32_t)i < s ? (uint64_t)(uint32_t)p[i] : ~0ull;
      __syncthreads();
      bitonic_sort_u64(keys, n2);
      for (uint32_t i = threadIdx.x; i < s; i += 256) p[i] = (int32_t)(uint32_t)keys[i];
    } else {
      const uint32_t chunk = kSortCap - capp;
      for (int i = threadIdx.x; i < capp; i += 256) keys[i] = ~0ull;
      for (uint32_t base = 0; base < s; base += chunk) {
        for (uint32_t i = threadIdx.x; i < chunk; i += 256) {
          uint64_t k = ~0ull;
          if (base + i < s) {
            const uint32_t j = (uint32_t)p[base + i];
            const uint32_t pr = policy == SLIDE_KEEP_LOWEST_ID ? 0u : overflow_prio(j, (uint32_t)t, r, pa, pb);
            k = ((uint64_t)pr << 32) | j;
          }
          keys[capp + i] = k;
        }
        __syncthreads();
        bitonic_sort_u64(keys, kSortCap);
      }
      uint64_t mine[kSortCap / 512];            // capp <= 1024: at most 4 per thread
      for (int i = threadIdx.x, q = 0; i < capp; i += 256, ++q)
        mine[q] = i < C ? (uint64_t)(uint32_t)keys[i] : ~0ull;
      __syncthreads();
      for (int i = threadIdx.x, q = 0; i < capp; i += 256, ++q) keys[i] = mine[q];
      __syncthreads();
      bitonic_sort_u64(keys, capp);
      for (int i = threadIdx.x; i < C; i += 256) p[i] = (int32_t)(uint32_t)keys[i];
    }
    __syncthreads();
  }
}

// Split of the code into partition digit (high hb bits) and in-partition digit (low lb bits).
void tables_split(int bits, int64_t N, int* hb, int* lb) {
  int want = 0;
  while (want < 11 && ((int64_t)4096 << want) < N) ++want;     // about 2048 to 4096 rows per partition
  int h = want < bits ? want : bits;
  if (bits - h > 13) h = bits - 13;                            // low digit counters must fit in LDS
  *hb = h;
  *lb = bits - h;
}

size_t tables_bh_words(int bits, int64_t N, int L) {
  int hb, lb;
  tables_split(bits, N, &hb, &lb);
  const int64_t nslab = (N + kSlab - 1) / kSlab;
  return (size_t)L * (size_t)(nslab > 0 ? nslab : 1) * ((size_t)1 << hb);
}

size_t tables_pbase_words(int bits, int64_t N, int L) {
  int hb, lb;
  tables_split(bits, N, &hb, &lb);
  return (size_t)L * (((size_t)1 << hb) + 1);
}

static size_t part_buckets_lds(int lb) {
  const size_t nlo = (size_t)1 << lb;
  return (nlo + ((nlo + 63) >> 6) + kStageIds) * 4;
}
static size_t part_scatter_lds(int nbins) { return ((size_t)2 * kSlab + 3 * (size_t)nbins + 20) * 4; }

// Rows of W2 touched since the last build (one byte each, set by the training step) -> a list of
// their ids and its length; the marks are cleared.  One thread per row, one counter update per
// workgroup (ascending ids within a workgroup's stretch; stretches in arrival order).
__global__ __launch_bounds__(1024) void collect_touched_kernel(uint8_t* __restrict__ touched, int64_t N,
                                                               int32_t* __restrict__ rows, uint32_t* count) {
  __shared__ uint32_t wsum[17];
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool hit = j < N && touched[j] != 0;
  const uint64_t m = __ballot(hit);
  if (lane == 0) wsum[wave] = (uint32_t)__popcll(m);
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t run = 0;
    for (int w = 0; w < 16; ++w) { const uint32_t c = wsum[w]; wsum[w] = run; run += c; }
    wsum[16] = run ? atomicAdd(count, run) : 0u;
  }
  __syncthreads();
  if (hit) {
    rows[wsum[16] + wsum[wave] + __popcll(m & ((1ull << lane) - 1))] = (int32_t)j;
    touched[j] = 0;
  }
}

// When most rows were touched, hashing all of them in place is cheaper than hashing them through
// the list (whole lines of codes instead of scattered words): the count becomes N, which the hash
// kernel takes as "no list".
__global__ void settle_touched_kernel(uint32_t* count, uint32_t N) {
  if (threadIdx.x == 0 && blockIdx.x == 0 && (uint64_t)*count * 4 > (uint64_t)N * 3) *count = N;
}

hipError_t tables_setup_attributes() {
  hipError_t e;
#define SLIDE_SET(K, BYTES) \
  e = hipFuncSetAttribute((const void*)&K, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(BYTES)); \
  if (e != hipSuccess) return e;
  SLIDE_SET(part_buckets_kernel<false>, part_buckets_lds(13))
  SLIDE_SET(part_buckets_kernel<true>, part_buckets_lds(13))
  SLIDE_SET(part_scatter_kernel<false>, part_scatter_lds(2048))
  SLIDE_SET(part_scatter_kernel<true>, part_scatter_lds(2048))
#undef SLIDE_SET
  return hipSuccess;
}

hipError_t launch_build_tables(const HashDev& hd, const TablesDev& td, const float* W2, uint32_t* codes_t,
                               uint2* entries, uint32_t* bh, uint32_t* pbase, uint64_t* worklist,
                               uint32_t wl_cap, Ctrl* ctrl, int policy, uint32_t r, uint32_t prio_a,
                               uint32_t prio_b, uint8_t* touched, int32_t* touched_rows, bool only_touched,
                               hipStream_t s) {
  hipError_t e;
  int bits = 0, hb, lb;
  while ((1u << bits) < td.nb) ++bits;
  tables_split(bits, td.N, &hb, &lb);
  const int nbins = 1 << hb;
  const int nslab = td.N > 0 ? (int)((td.N + kSlab - 1) / kSlab) : 1;
  // (1) codes of every row, or -- when codes_t still holds the codes of the last build -- only of the
  // rows whose weights changed since; the grouping below always runs in full, so the tables are the
  // same either way.
  if (only_touched) {
    if ((e = launch_fill_u32(&ctrl->rehashed, 1, 0u, s)) != hipSuccess) return e;
    hipLaunchKernelGGL(collect_touched_kernel, dim3((unsigned)ceil_div(td.N, 1024)), dim3(1024), 0, s, touched, td.N,
                       touched_rows, &ctrl->rehashed);
    hipLaunchKernelGGL(settle_touched_kernel, dim3(1), dim3(64), 0, s, &ctrl->rehashed, (uint32_t)td.N);
    if ((e = launch_hash(hd, W2, td.N, codes_t, 1, td.N, touched_rows, &ctrl->rehashed, hd.L, s)) != hipSuccess) return e;
  } else {
    if ((e = launch_fill_u32(&ctrl->rehashed, 1, (uint32_t)td.N, s)) != hipSuccess) return e;
    if (touched && (e = launch_fill_u32((uint32_t*)touched, (size_t)ceil_div(td.N, 4), 0u, s)) != hipSuccess) return e;
    if ((e = launch_hash(hd, W2, td.N, codes_t, 1, td.N, nullptr, nullptr, hd.L, s)) != hipSuccess) return e;
  }
  hipLaunchKernelGGL(part_hist_kernel, dim3(nslab, td.L), dim3(1024), (size_t)nbins * 4, s, codes_t, td.N, lb, nbins,
                     bh, nslab);
  hipLaunchKernelGGL(part_scan_kernel, dim3(td.L), dim3(1024), 0, s, bh, nslab, nbins, pbase, ctrl);
  int rowbits = 1;
  while (((int64_t)1 << rowbits) < td.N) ++rowbits;
  if (lb + rowbits <= 32) {
    hipLaunchKernelGGL(part_scatter_kernel<true>, dim3(nslab, td.L), dim3(1024), part_scatter_lds(nbins), s, codes_t, td.N,
                       lb, rowbits, nbins, bh, nslab, pbase, (uint32_t*)entries);
    hipLaunchKernelGGL(part_buckets_kernel<true>, dim3(nbins, td.L), dim3(256), part_buckets_lds(lb), s,
                       (const uint32_t*)entries, pbase, nbins, lb, rowbits, td.nb, td.N, td.C, td.off, td.ids, worklist,
                       wl_cap, ctrl);
  } else {
    hipLaunchKernelGGL(part_scatter_kernel<false>, dim3(nslab, td.L), dim3(1024), part_scatter_lds(nbins), s, codes_t, td.N,
                       lb, rowbits, nbins, bh, nslab, pbase, entries);
    hipLaunchKernelGGL(part_buckets_kernel<false>, dim3(nbins, td.L), dim3(256), part_buckets_lds(lb), s,
                       (const uint2*)entries, pbase, nbins, lb, rowbits, td.nb, td.N, td.C, td.off, td.ids, worklist,
                       wl_cap, ctrl);
  }
  hipLaunchKernelGGL(big_buckets_kernel, dim3(2048), dim3(256), 0, s, td.off, td.ids, td.nb, td.N, td.C, policy,
                     r, prio_a, prio_b, worklist, wl_cap, ctrl);
  return hipGetLastError();
}

}  // namespace slide
