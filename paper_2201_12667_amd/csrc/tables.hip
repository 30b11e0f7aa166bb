// Hash-table build / rebuild (paper Algorithm 1 "hash weights to hash tables", rebuilt on a
// schedule, Section 3.1).  Layout: per table a CSR over the 2^bits codes -- off[t][code] is the
// start of the bucket inside ids[t][0..N).  A bucket's first min(size, C) ids are its kept members,
// ascending by id; which members are kept when size > C is decided by the smallest
// (priority, id) keys.
//
// Passes: (1) hash every row of W2 and take a ticket in its bucket's counter, (2) exclusive scan
// of the counters per table, (3) scatter ids to bucket start + ticket, (4) sort every bucket by id
// (tickets arrive in arbitrary order) and apply the capacity rule.
#include "slide_internal.h"

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

// Exclusive scan over the 256 threads of a workgroup; *total gets the sum.  sm: 8 words of LDS.
__device__ uint32_t block_excl_scan256(uint32_t v, uint32_t* sm, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_incl_scan(v);
  __syncthreads();
  if (lane == 63) sm[wave] = inc;
  __syncthreads();
  uint32_t base = 0;
  for (int w = 0; w < wave; ++w) base += sm[w];
  *total = sm[0] + sm[1] + sm[2] + sm[3];
  return base + inc - v;
}

__global__ __launch_bounds__(256) void seg_sum_kernel(const uint32_t* __restrict__ off, uint32_t nb,
                                                      uint32_t nseg, uint32_t* __restrict__ segsum) {
  __shared__ uint32_t sm[8];
  const uint32_t seg = blockIdx.x, t = blockIdx.y;
  const uint32_t* p = off + (size_t)t * (nb + 1);
  uint32_t acc = 0;
  for (int k = 0; k < kScanSeg / 256; ++k) {
    const uint32_t i = seg * kScanSeg + k * 256 + threadIdx.x;
    if (i < nb) acc += p[i];
  }
  uint32_t total;
  block_excl_scan256(acc, sm, &total);
  if (threadIdx.x == 0) segsum[(size_t)t * nseg + seg] = total;
}

__global__ __launch_bounds__(256) void seg_scan_kernel(uint32_t* segsum, uint32_t nseg, Ctrl* ctrl) {
  __shared__ uint32_t sm[8];
  uint32_t* p = segsum + (size_t)blockIdx.x * nseg;
  uint32_t carry = 0;
  for (uint32_t base = 0; base < nseg; base += 256) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t v = i < nseg ? p[i] : 0;
    uint32_t total;
    const uint32_t ex = block_excl_scan256(v, sm, &total);
    if (i < nseg) p[i] = carry + ex;
    carry += total;
    __syncthreads();
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) { ctrl->wl_count = 0; ctrl->overflowed = 0; }
}

__global__ __launch_bounds__(256) void seg_apply_kernel(uint32_t* off, uint32_t nb, uint32_t nseg,
                                                        const uint32_t* __restrict__ segsum, uint32_t N) {
  __shared__ uint32_t sm[8];
  constexpr int PER = kScanSeg / 256;
  const uint32_t seg = blockIdx.x, t = blockIdx.y;
  uint32_t* p = off + (size_t)t * (nb + 1);
  const uint32_t first = seg * kScanSeg + threadIdx.x * PER;
  uint32_t v[PER], sum = 0;
#pragma unroll
  for (int k = 0; k < PER; ++k) { v[k] = first + k < nb ? p[first + k] : 0; sum += v[k]; }
  uint32_t total;
  uint32_t run = block_excl_scan256(sum, sm, &total) + segsum[(size_t)t * nseg + seg];
#pragma unroll
  for (int k = 0; k < PER; ++k) { if (first + k < nb) p[first + k] = run; run += v[k]; }
  if (seg == 0 && threadIdx.x == 0) p[nb] = N;
}

__global__ __launch_bounds__(256) void scatter_ids_kernel(const uint32_t* __restrict__ codes_t,
                                                          const uint32_t* __restrict__ rank_t,
                                                          const uint32_t* __restrict__ off, int32_t* ids,
                                                          uint32_t nb, int64_t N) {
  const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const size_t t = blockIdx.y;
  if (j >= N) return;
  const uint32_t code = codes_t[t * N + j];
  ids[t * N + off[t * (nb + 1) + code] + rank_t[t * N + j]] = (int32_t)j;
}

// One thread per bucket: sorts small buckets in place, queues the others.
__global__ __launch_bounds__(256) void small_buckets_kernel(const uint32_t* __restrict__ off, int32_t* ids,
                                                            uint32_t nb, int lgnb, int64_t N, int L, int C,
                                                            uint64_t* worklist, uint32_t wl_cap, Ctrl* ctrl) {
  const uint64_t b = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  const uint64_t t = b >> lgnb;
  if (t >= (uint64_t)L) return;
  const uint32_t c = (uint32_t)(b & (nb - 1));
  const uint32_t o0 = off[t * (nb + 1) + c];
  const uint32_t s = off[t * (nb + 1) + c + 1] - o0;
  if (s > (uint32_t)C) atomicAdd(&ctrl->overflowed, 1u);
  if (s < 2) return;
  if (s <= (uint32_t)kSmallBucket && s <= (uint32_t)C) {
    int32_t* p = ids + t * N + o0;
    for (uint32_t a = 1; a < s; ++a) {
      const int32_t key = p[a];
      int q = (int)a - 1;
      while (q >= 0 && p[q] > key) { p[q + 1] = p[q]; --q; }
      p[q + 1] = key;
    }
  } else {
    const uint32_t slot = atomicAdd(&ctrl->wl_count, 1u);
    if (slot < wl_cap) worklist[slot] = (t << 32) | c;
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

hipError_t launch_build_tables(const HashDev& hd, const TablesDev& td, const float* W2,
                               uint32_t* codes_t, uint32_t* rank_t, uint32_t* segsum,
                               uint64_t* worklist, uint32_t wl_cap, Ctrl* ctrl, int policy,
                               uint32_t r, uint32_t prio_a, uint32_t prio_b, int tables_per_block,
                               hipStream_t s) {
  hipError_t e;
  const uint32_t nb = td.nb;
  const uint32_t nseg = (nb + kScanSeg - 1) / kScanSeg;
  int lgnb = 0;
  while ((1u << lgnb) < nb) ++lgnb;
  if ((e = launch_fill_u32(td.off, (size_t)td.L * (nb + 1), 0u, s)) != hipSuccess) return e;
  if ((e = launch_hash(hd, W2, td.N, codes_t, 1, td.N, td.off, rank_t, nb, tables_per_block, s)) != hipSuccess)
    return e;
  hipLaunchKernelGGL(seg_sum_kernel, dim3(nseg, td.L), dim3(256), 0, s, td.off, nb, nseg, segsum);
  hipLaunchKernelGGL(seg_scan_kernel, dim3(td.L), dim3(256), 0, s, segsum, nseg, ctrl);
  hipLaunchKernelGGL(seg_apply_kernel, dim3(nseg, td.L), dim3(256), 0, s, td.off, nb, nseg, segsum,
                     (uint32_t)td.N);
  if (td.N > 0)
    hipLaunchKernelGGL(scatter_ids_kernel, dim3((unsigned)ceil_div(td.N, 256), td.L), dim3(256), 0, s,
                       codes_t, rank_t, td.off, td.ids, nb, td.N);
  const uint64_t buckets = (uint64_t)td.L << lgnb;
  hipLaunchKernelGGL(small_buckets_kernel, dim3((unsigned)((buckets + 255) / 256)), dim3(256), 0, s, td.off,
                     td.ids, nb, lgnb, td.N, td.L, td.C, worklist, wl_cap, ctrl);
  hipLaunchKernelGGL(big_buckets_kernel, dim3(2048), dim3(256), 0, s, td.off, td.ids, nb, td.N, td.C, policy,
                     r, prio_a, prio_b, worklist, wl_cap, ctrl);
  return hipGetLastError();
}

}  // namespace slide
