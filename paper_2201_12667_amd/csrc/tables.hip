// Hash-table build / rebuild (paper Algorithm 1, the table-construction step before the loop, rebuilt on a
// schedule, Section 3.1).  Layout: per table a CSR over the 2^bits codes -- off[t][code] is the
// start of the bucket inside ids[t][0..N).  A bucket's first min(size, C) ids are its kept members,
// ascending by id; which members are kept when size > C is decided by the smallest
// (priority, id) keys.
//
// The build is a two-level counting sort with every counter in LDS (no global atomics on the
// tables): (1) hash every row of W2, codes stored table-major; (2) every slab of 16,384 rows of a
// table is grouped by the high bits of the code in LDS and written back in place, with the run
// boundaries per (slab, digit); (3) a scan over slabs gives the partition starts; (4) one workgroup per
// (table, partition) gathers the partition's runs from the slabs, counts the low bits in LDS, writes
// that partition's offsets, places the ids and sorts the small buckets in place; (5) buckets that are
// long or over capacity are queued and handled by one workgroup each.
#include "slide_internal.h"
#include "wave_ops.h"

namespace slide {

__global__ void fill_u32_kernel(uint32_t* p, size_t n, uint32_t v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t step = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += step) p[i] = v;
}

// Plain streaming copy: the yardstick the HBM counters and the achievable bandwidth are calibrated
// against.  Of the plain forms tried (grid-stride with one, four or eight 16-byte words per thread in
// flight, cached or streaming accesses, 2 K to 256 K workgroups) this one -- four words per thread in
// flight, loads and stores past the caches -- is the fastest on a 1 GiB buffer (6.3 TB/s against
// 5.4 for the one-word cached loop).
typedef float copy_v4f __attribute__((ext_vector_type(4)));
constexpr size_t kCopyChunk = 1024;       // 16-byte words a workgroup of 256 moves per step
__global__ __launch_bounds__(256) void copy_kernel(copy_v4f* __restrict__ dst, const copy_v4f* __restrict__ src, size_t n16) {
  size_t base = (size_t)blockIdx.x * kCopyChunk;
  const size_t step = (size_t)gridDim.x * kCopyChunk;
  for (; base + kCopyChunk <= n16; base += step) {
    copy_v4f v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + base + (size_t)u * 256 + threadIdx.x);
#pragma unroll
    for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + base + (size_t)u * 256 + threadIdx.x);
  }
  // (the last, partial chunk: only the workgroup whose turn it would have been gets here with base < n16)
  for (size_t i = base + threadIdx.x; i < n16; i += 256) dst[i] = src[i];
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  const size_t n16 = bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + kCopyChunk - 1) / kCopyChunk;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (copy_v4f*)dst, (const copy_v4f*)src, n16);
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
  return hipGetLastError();
}

constexpr int kSlabBits = 15;
constexpr int kSlab = 1 << kSlabBits;   // rows per slab of the grouping pass
constexpr int kRunBlock = 1024;         // slabs whose run boundaries a bucket workgroup holds in LDS at a time

// Exclusive scan over a workgroup of 1024 threads; sm: 17 words of LDS.
__device__ uint32_t block_excl_scan1024(uint32_t v, uint32_t* sm, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t inc = wave_incl_scan_add(v);
  __syncthreads();
  if (lane == 63) sm[wave] = inc;
  __syncthreads();
  uint32_t base = 0, tot = 0;
  for (int w = 0; w < 16; ++w) { const uint32_t x = sm[w]; if (w < wave) base += x; tot += x; }
  *total = tot;
  return base + inc - v;
}

// One workgroup per (slab, table): the slab's rows grouped by the high digit of their code, in place
// -- the grouped entries of slab s stay in entries[t][s*kSlab ..), so no table-wide histogram has to
// exist before this pass.  An entry is (low digit << kSlabBits) | row inside the slab (the reader
// knows the slab).  runs[t][s][d] = first entry of digit d inside the slab's stretch,
// runs[t][s][nbins] = rows of the slab.  The grouping happens in LDS and the slab is written out as
// one coalesced stretch.
__global__ __launch_bounds__(1024) void slab_group_kernel(const uint32_t* __restrict__ codes_t, int64_t N, int lb,
                                                          int nbins, uint32_t* __restrict__ runs, int nslab,
                                                          uint32_t* __restrict__ entries) {
  extern __shared__ uint32_t lds[];
  uint32_t* stage = lds;                           // [kSlab] entries grouped by digit
  uint32_t* cur = lds + kSlab;                     // [nbins] counters, then cursors
  uint32_t* sm = cur + nbins;                      // [20]
  const int slab = blockIdx.x, tid = threadIdx.x;
  const size_t t = blockIdx.y;
  for (int b = tid; b < nbins; b += 1024) cur[b] = 0;
  __syncthreads();
  const int64_t j0 = (int64_t)slab * kSlab;
  const int nvalid = (int)(N - j0 < kSlab ? N - j0 : kSlab);
  uint32_t code[kSlab / 1024];
#pragma unroll
  for (int k = 0; k < kSlab / 1024; ++k) {
    const int r = k * 1024 + tid;
    code[k] = r < nvalid ? codes_t[t * N + j0 + r] : 0u;
  }
#pragma unroll
  for (int k = 0; k < kSlab / 1024; ++k)
    if (k * 1024 + tid < nvalid) atomicAdd(&cur[code[k] >> lb], 1u);
  __syncthreads();
  uint32_t* rrow = runs + (t * nslab + slab) * (size_t)(nbins + 1);
  uint32_t carry = 0;
  for (int base = 0; base < nbins; base += 1024) {
    const int b = base + tid;
    const uint32_t v = b < nbins ? cur[b] : 0u;
    uint32_t total;
    const uint32_t ex = block_excl_scan1024(v, sm, &total);   // (its barriers separate the read of cur from the write)
    if (b < nbins) { cur[b] = carry + ex; rrow[b] = carry + ex; }
    carry += total;
  }
  if (tid == 0) rrow[nbins] = (uint32_t)nvalid;
  __syncthreads();
  const uint32_t lowmask = (1u << lb) - 1u;
#pragma unroll
  for (int k = 0; k < kSlab / 1024; ++k) {
    const int r = k * 1024 + tid;
    if (r < nvalid) stage[atomicAdd(&cur[code[k] >> lb], 1u)] = ((code[k] & lowmask) << kSlabBits) | (uint32_t)r;
  }
  __syncthreads();
  uint32_t* out = entries + t * N + j0;
  for (int k = tid; k < nvalid; k += 1024) out[k] = stage[k];
}

// One workgroup per table: pbase[t][d] = rows of the table whose digit is below d (the start of
// partition d in the table's id array), from the per-slab run boundaries.
__global__ __launch_bounds__(1024) void part_scan_kernel(const uint32_t* __restrict__ runs, int nslab, int nbins,
                                                         uint32_t* __restrict__ pbase, Ctrl* ctrl) {
  __shared__ uint32_t sm[20];
  const size_t t = blockIdx.x;
  const int tid = threadIdx.x;
  uint32_t carry = 0;
  for (int base = 0; base < nbins; base += 1024) {
    const int d = base + tid;
    uint32_t run = 0;
    if (d < nbins)
      for (int slab = 0; slab < nslab; ++slab) {
        const uint32_t* p = runs + (t * nslab + slab) * (size_t)(nbins + 1) + d;
        run += p[1] - p[0];
      }
    uint32_t total;
    const uint32_t ex = block_excl_scan1024(run, sm, &total);
    if (d < nbins) pbase[t * (nbins + 1) + d] = carry + ex;
    carry += total;
    __syncthreads();
  }
  if (tid == 0) pbase[t * (nbins + 1) + nbins] = carry;
  if (t == 0 && tid == 0) { ctrl->wl_count = 0; ctrl->wl_short = 0; ctrl->overflowed = 0; }
}

constexpr int kStageIds = 4096;    // most ids of a partition staged in LDS by part_buckets (larger partitions go through memory)
constexpr int kStageMin = 1024;    // the staging area is four mean partitions, within these two
constexpr int kRankMax = 64;       // staged buckets up to this size are sorted where they are staged
constexpr int kWaveSort = 64;      // queued buckets up to this size (within capacity) are sorted by one wave
static __host__ __device__ inline int med_cap(int stage) { return stage / 9 + 1; }   // staged buckets of more than eight ids
constexpr int kSlotBatch = 16;     // 64-entry pieces of runs a wave keeps in flight

// One workgroup per (pair of partitions d, d + 1; table t); partition d holds the buckets (d << lb) ..
// (d << lb) + 2^lb - 1 and its entries are the runs of digit d of every slab.  Per partition: counts the
// low digit, writes the partition's offsets, groups the ids by bucket -- in LDS when the partition fits,
// so that the table receives whole lines -- and sorts the small buckets; long and over-capacity buckets
// are queued.  A partition's work starts with two dependent round trips to memory (its run boundaries,
// then its entries) that take as long as all the rest: the workgroup makes them for both of its
// partitions at once, so the second partition's entries sit in registers when its turn comes.
__global__ __launch_bounds__(256) void part_buckets_kernel(const uint32_t* __restrict__ entries,
                                                           const uint32_t* __restrict__ runs, int nslab,
                                                           const uint32_t* __restrict__ pbase, int nbins, int lb,
                                                           uint32_t nb, int64_t N, int C,
                                                           uint32_t* __restrict__ off,
                                                           int32_t* ids, uint64_t* worklist, uint32_t wl_cap,
                                                           Ctrl* ctrl, int nsb /* min(nslab, kRunBlock) */,
                                                           int stage /* ids of a partition that fit the staging area */) {
  extern __shared__ uint32_t lds[];
  const int nlo = 1 << lb, tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nchunk = (nlo + 63) >> 6;    // 64 buckets per scan chunk
  uint32_t* cur = lds;                   // [nlo] counters, then bucket starts, then (after placing) bucket ends
  uint4* cur4 = reinterpret_cast<uint4*>(lds);
  const bool vec = (nlo & 1023) == 0;    // many buckets per partition: the passes over them take four per lane
  uint32_t* csum = cur + nlo;            // [nchunk] ids in the chunk, then in the chunks before it
  const int slot_cap = nsb + stage / 64;
  const int medcap = med_cap(stage);
  const int set_words = 2 * nsb + slot_cap;
  uint32_t* sets = csum + nchunk;        // per partition of the pair: [nsb] start of the slab's run inside the slab's
                                         // stretch, [nsb] its length, [slot_cap] 64-entry pieces of the runs: run | piece << 16
  const size_t t = blockIdx.y;
  int32_t* idl = (int32_t*)(sets + 2 * set_words);             // [stage] the partition's ids grouped by bucket
  uint32_t* nslots_p = (uint32_t*)(idl + stage);           // [2] pieces of each partition of the pair
  uint32_t* nmed_p = nslots_p + 2;                             // [2] staged buckets of 9 .. 16 ids / of 17 .. kRankMax
  uint32_t* medq = nmed_p + 2;                                 // [medcap] the former from the front, the latter from the back
  const uint32_t* tent = entries + t * N;
  const uint32_t* truns0 = runs + t * nslab * (size_t)(nbins + 1);
  auto ra_of = [&](int set) { return sets + set * set_words; };
  auto rn_of = [&](int set) { return sets + set * set_words + nsb; };
  auto slots_of = [&](int set) { return sets + set * set_words + 2 * nsb; };
  // wave-wide: the pieces of the runs of one set, in run order
  auto cut_pieces = [&](int set, int ns) {
    const uint32_t* rn = rn_of(set);
    uint32_t* slots = slots_of(set);
    uint32_t carry = 0;
    for (int q0 = 0; q0 < ns; q0 += 64) {
      const int q = q0 + lane;
      const uint32_t np = q < ns ? (rn[q] + 63u) >> 6 : 0u;
      const uint32_t inc = wave_incl_scan_add(np);
      uint32_t at = carry + inc - np;
      for (uint32_t j = 0; j < np; ++j, ++at)
        if (at < (uint32_t)slot_cap) slots[at] = (uint32_t)q | (j << 16);
      carry += (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
    }
    if (lane == 0) nslots_p[set] = carry;
  };
  // A partition's entries are visited twice (count, then place).  The slabs are taken in blocks of nsb:
  // prepare() fetches the run boundaries of a block together and cuts the runs into pieces of 64
  // entries; a wave takes a piece, a lane an entry, kSlotBatch pieces per wave in flight at once.
  auto prepare = [&](uint32_t d, int sb, int set) -> int {
    const int ns = min(nsb, nslab - sb);
    uint32_t *ra = ra_of(set), *rn = rn_of(set);
    __syncthreads();
    for (int q = tid; q < ns; q += 256) {
      const uint32_t* p = truns0 + (size_t)(sb + q) * (nbins + 1) + d;
      const uint32_t a = p[0];
      ra[q] = a; rn[q] = p[1] - a;
    }
    __syncthreads();
    if (wave == 0) cut_pieces(set, ns);
    __syncthreads();
    return ns;
  };
  // the same for both partitions of the pair at once (one block of slabs): one round of reads, two waves cutting
  auto prepare_pair = [&](uint32_t d, bool both) -> int {
    const int ns = nslab;
    __syncthreads();
    for (int q = tid; q < ns; q += 256) {
      const uint32_t* p = truns0 + (size_t)q * (nbins + 1) + d;
      const uint32_t a0 = p[0], a1 = p[1];
      ra_of(0)[q] = a0; rn_of(0)[q] = a1 - a0;
      if (both) { ra_of(1)[q] = a1; rn_of(1)[q] = p[2] - a1; }
    }
    __syncthreads();
    if (wave == 0 || (wave == 1 && both)) cut_pieces(wave, ns);
    __syncthreads();
    return ns;
  };
  auto load_batch = [&](int set, int sb, int base, int nslots, uint32_t (&x)[kSlotBatch]) {
    const uint32_t *ra = ra_of(set), *rn = rn_of(set), *slots = slots_of(set);
#pragma unroll
    for (int k = 0; k < kSlotBatch; ++k) {
      const int sl = base + 4 * k + wave;            // (wave-uniform)
      x[k] = 0xffffffffu;                            // (no entry has all bits set: at most 28 are used)
      if (sl < nslots) {
        const uint32_t info = slots[sl];
        const uint32_t q = info & 0xffffu, o = (info >> 16) * 64u + (uint32_t)lane;
        if (o < rn[q]) x[k] = tent[(size_t)((uint32_t)(sb + q) << kSlabBits) + ra[q] + o];
      }
    }
  };
  // f(global row, low digit) for the entries a wave holds in x (pieces base + 4k + wave of the set)
  auto visit_batch = [&](int set, int sb, int base, const uint32_t (&x)[kSlotBatch], auto&& f) {
    const uint32_t* slots = slots_of(set);
#pragma unroll
    for (int k = 0; k < kSlotBatch; ++k)
      if (x[k] != 0xffffffffu) {
        const uint32_t rowbase = (uint32_t)(sb + (int)(slots[base + 4 * k + wave] & 0xffffu)) << kSlabBits;
        f(rowbase + (x[k] & (uint32_t)(kSlab - 1)), x[k] >> kSlabBits);
      }
  };
  auto visit_block = [&](int set, int sb, int ns, auto&& f) {   // f(global row, low digit) for every entry of the block
    const int nslots = (int)nslots_p[set];
    if (nslots <= slot_cap) {
      for (int base = 0; base < nslots; base += 4 * kSlotBatch) {
        uint32_t x[kSlotBatch];
        load_batch(set, sb, base, nslots, x);
        visit_batch(set, sb, base, x, f);
      }
    } else {
      // more pieces than the slot table holds (a partition far too large to stage): a wave per run
      const uint32_t *ra = ra_of(set), *rn = rn_of(set);
      for (int q = wave; q < ns; q += 4) {
        const uint32_t a = ra[q], n = rn[q], rowbase = (uint32_t)(sb + q) << kSlabBits;
        for (uint32_t e = lane; e < n; e += 64) {
          const uint32_t x = tent[(size_t)rowbase + a + e];
          f(rowbase + (x & (uint32_t)(kSlab - 1)), x >> kSlabBits);
        }
      }
    }
  };
  const bool single = nslab <= nsb;
  // One partition.  cached: every entry of the partition sits in a register of some lane (x: at most
  // 4 * kSlotBatch pieces, fetched by the caller), and both visits use the registers.
  auto run_partition = [&](const uint32_t d, const int set, const bool cached, const uint32_t (&x0)[kSlotBatch], const int ns0) {
  if (vec) for (int q = tid; q < nlo / 4; q += 256) cur4[q] = make_uint4(0u, 0u, 0u, 0u);
  else for (int b = tid; b < nlo; b += 256) cur[b] = 0;
  if (tid < 2) nmed_p[tid] = 0;
  __syncthreads();
  const uint32_t s0 = pbase[t * (nbins + 1) + d], s1 = pbase[t * (nbins + 1) + d + 1];
  const bool staged = s1 - s0 <= (uint32_t)stage;
  auto visit = [&](auto&& f) {
    if (cached) {
      visit_batch(set, 0, 0, x0, f);
    } else if (single) {
      visit_block(set, 0, ns0, f);
    } else {
      for (int sb = 0; sb < nslab; sb += nsb) { const int ns = prepare(d, sb, set); visit_block(set, sb, ns, f); }
    }
    __syncthreads();
  };
  visit([&](uint32_t, uint32_t low) { atomicAdd(&cur[low], 1u); });
  // exclusive scan of the counters: every wave scans chunks of 64 lanes in registers, wave 0 the chunk
  // sums.  Many buckets per partition (vec): a lane holds four neighbouring counters, a chunk is 256.
  const int nch = vec ? nlo >> 8 : nchunk;
  if (vec) {
    for (int c = wave; c < nch; c += 4) {
      const uint4 v = cur4[c * 64 + lane];
      const uint32_t p1 = v.x, p2 = p1 + v.y, p3 = p2 + v.z, p4 = p3 + v.w;
      const uint32_t inc = wave_incl_scan_add(p4), base = inc - p4;
      cur4[c * 64 + lane] = make_uint4(base, base + p1, base + p2, base + p3);
      if (lane == 63) csum[c] = inc;
    }
  } else {
    for (int c = wave; c < nch; c += 4) {
      const int b = c * 64 + lane;
      const uint32_t v = b < nlo ? cur[b] : 0u;
      const uint32_t inc = wave_incl_scan_add(v);
      if (b < nlo) cur[b] = inc - v;
      if (lane == 63) csum[c] = inc;
    }
  }
  __syncthreads();
  if (wave == 0) {
    uint32_t carry = 0;
    for (int c0 = 0; c0 < nch; c0 += 64) {
      const int c = c0 + lane;
      const uint32_t v = c < nch ? csum[c] : 0u;
      const uint32_t inc = wave_incl_scan_add(v);
      if (c < nch) csum[c] = carry + inc - v;
      carry += (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
    }
  }
  __syncthreads();
  uint32_t* orow = off + t * (nb + 1) + ((size_t)d << lb);
  if (vec) {
    // (a table's offsets start at a multiple of nb + 1 words: word-aligned only)
    struct __attribute__((packed, aligned(4))) Words4 { uint32_t x, y, z, w; };
    for (int q = tid; q < nlo / 4; q += 256) {
      uint4 v = cur4[q];
      const uint32_t add = csum[q >> 6];
      v.x += add; v.y += add; v.z += add; v.w += add;
      cur4[q] = v;
      reinterpret_cast<Words4*>(orow)[q] = Words4{s0 + v.x, s0 + v.y, s0 + v.z, s0 + v.w};
    }
  } else {
    for (int b = tid; b < nlo; b += 256) {
      const uint32_t st = cur[b] + csum[b >> 6];
      cur[b] = st;
      orow[b] = s0 + st;
    }
  }
  if (d == (uint32_t)nbins - 1 && tid == 0) off[t * (nb + 1) + nb] = (uint32_t)N;
  int32_t* seg = ids + t * N + s0;
  int32_t* place = staged ? idl : seg;
  __syncthreads();
  visit([&](uint32_t row, uint32_t low) { place[atomicAdd(&cur[low], 1u)] = (int32_t)row; });
  // cur[b] is now the end of bucket b = the start of bucket b + 1
  uint32_t over = 0;
  auto enqueue = [&](int b, uint32_t sz) {           // short lists from the back of the worklist, long ones from the front
    const uint64_t item = ((uint64_t)t << 32) | ((d << lb) + (uint32_t)b);
    if (sz <= (uint32_t)kWaveSort && sz <= (uint32_t)C) {
      const uint32_t slot = atomicAdd(&ctrl->wl_short, 1u);
      if (slot < wl_cap) worklist[wl_cap - 1u - slot] = item;
    } else {
      const uint32_t slot = atomicAdd(&ctrl->wl_count, 1u);
      if (slot < wl_cap) worklist[slot] = item;
    }
  };
  if (staged) {
    // The ids sit in idl grouped by bucket, in arrival order, and are sorted where they are; the whole
    // partition then goes to the table in one coalesced copy (a store per bucket costs far more than
    // its bytes).  A thread takes a bucket.  Up to eight ids (nearly every bucket of a fresh layer) are
    // sorted in registers by a fixed network of comparators -- the same instructions in every lane,
    // whatever the bucket's size.  Longer buckets are noted for the pass below; those beyond kRankMax
    // or over capacity stay as they are and are queued.
    // bucket b = ids a .. a + sz - 1 (every lane of a wave calls it together: the network is wave-wide)
    auto bucket = [&](const int b, const uint32_t a, const uint32_t sz) {
      if (sz > (uint32_t)C) ++over;
      const bool big = sz > (uint32_t)kRankMax || sz > (uint32_t)C;
      if (big) {
        enqueue(b, sz);
      } else if (sz > 16u) {
        medq[medcap - 1 - atomicAdd(&nmed_p[1], 1u)] = (uint32_t)b;   // (lane groups / waves order these below:
      } else if (sz > 8u) {                                             //  at most stage / 9 of them exist)
        medq[atomicAdd(&nmed_p[0], 1u)] = (uint32_t)b;
      }
      const uint32_t n8 = (big || sz > 8u) ? 0u : sz;
      if (!__any(n8 > 1u)) return;                       // (sparse tables: nearly every bucket is empty or a single id)
      if (!__any(n8 > 2u)) {
        if (n8 > 1u) {
          const int32_t u0 = idl[a], u1 = idl[a + 1];
          idl[a] = min(u0, u1);
          idl[a + 1] = max(u0, u1);
        }
        return;
      }
      int32_t v[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = (uint32_t)i < n8 ? idl[a + i] : 0x7fffffff;
      if (__any(n8 > 4u)) {
#pragma unroll
        for (int i = 4; i < 8; ++i) v[i] = (uint32_t)i < n8 ? idl[a + i] : 0x7fffffff;
      } else {
#pragma unroll
        for (int i = 4; i < 8; ++i) v[i] = 0x7fffffff;
      }
#define SLIDE_CE(i, j) { const int32_t lo_ = min(v[i], v[j]), hi_ = max(v[i], v[j]); v[i] = lo_; v[j] = hi_; }
      SLIDE_CE(0, 1) SLIDE_CE(2, 3) SLIDE_CE(4, 5) SLIDE_CE(6, 7)         // odd-even merge sort of 8: 19 comparators
      SLIDE_CE(0, 2) SLIDE_CE(1, 3) SLIDE_CE(4, 6) SLIDE_CE(5, 7)
      SLIDE_CE(1, 2) SLIDE_CE(5, 6)
      SLIDE_CE(0, 4) SLIDE_CE(1, 5) SLIDE_CE(2, 6) SLIDE_CE(3, 7)
      SLIDE_CE(2, 4) SLIDE_CE(3, 5)
      SLIDE_CE(1, 2) SLIDE_CE(3, 4) SLIDE_CE(5, 6)
#undef SLIDE_CE
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if ((uint32_t)i < n8) idl[a + i] = v[i];
    };
    if (vec) {
      // a wave takes 256 neighbouring buckets, a lane four of them; nearly always, with so many
      // buckets, none of the 256 holds two ids and there is nothing to sort
      for (int b0 = wave * 256; b0 < nlo; b0 += 1024) {
        const int q = (b0 >> 2) + lane;
        const uint4 e = cur4[q];
        const uint32_t a = q ? cur[4 * q - 1] : 0u;
        const uint32_t most = max(max(e.x - a, e.y - e.x), max(e.z - e.y, e.w - e.z));
        if (__any(most > 1u)) {
          bucket(4 * q, a, e.x - a);
          bucket(4 * q + 1, e.x, e.y - e.x);
          bucket(4 * q + 2, e.y, e.z - e.y);
          bucket(4 * q + 3, e.z, e.w - e.z);
        }
      }
    } else {
      for (int b0 = 0; b0 < nlo; b0 += 256) {
        const int b = b0 + tid;
        const uint32_t a = (b && b < nlo) ? cur[b - 1] : 0u;
        bucket(b, a, b < nlo ? cur[b] - a : 0u);
      }
    }
    // Longer buckets (a trained layer has many): one thread sorting its bucket alone would hold up its
    // wave for the square of the bucket's length.  9 .. 16 ids: a row of 16 lanes each, an id per lane,
    // its place = the number of smaller ids in the row (register moves only).  17 .. kRankMax: a wave
    // each, a bitonic sort across the lanes.
    __syncthreads();
    const uint32_t nrow = nmed_p[0], nwav = nmed_p[1];
    for (uint32_t m0 = 0; m0 < nrow; m0 += 16) {
      const uint32_t m = m0 + (uint32_t)(tid >> 4);
      const int l16 = tid & 15;
      uint32_t a = 0, sz = 0;
      if (m < nrow) { const uint32_t b = medq[m]; a = b ? cur[b - 1] : 0u; sz = cur[b] - a; }
      const int32_t key = (uint32_t)l16 < sz ? idl[a + l16] : 0x7fffffff;
      const uint32_t rank = row_rank_i32(key);
      if ((uint32_t)l16 < sz) idl[a + rank] = key;
    }
    for (uint32_t m = wave; m < nwav; m += 4) {
      const uint32_t b = medq[medcap - 1 - m];
      const uint32_t a = b ? cur[b - 1] : 0u, sz = cur[b] - a;
      int32_t key = (uint32_t)lane < sz ? idl[a + lane] : 0x7fffffff;
#pragma unroll
      for (int k = 2; k <= 64; k <<= 1)
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
          const int32_t other = __shfl_xor(key, j);
          const bool up = (lane & k) == 0, lower = (lane & j) == 0;
          const int32_t mn = key < other ? key : other, mx = key < other ? other : key;
          key = (lower == up) ? mn : mx;
        }
      if ((uint32_t)lane < sz) idl[a + lane] = key;
    }
    __syncthreads();
    for (uint32_t p = tid; p < s1 - s0; p += 256) seg[p] = idl[p];
  } else {
    for (int b = tid; b < nlo; b += 256) {
      const uint32_t a = b ? cur[b - 1] : 0u, sz = cur[b] - a;
      if (sz > (uint32_t)C) ++over;
      if (sz < 2) continue;
      if (sz <= (uint32_t)kSmallBucket && sz <= (uint32_t)C) {
        int32_t* p = seg + a;                       // arrival order is arbitrary: restore ascending ids
        for (uint32_t i = 1; i < sz; ++i) {
          const int32_t key = p[i];
          int q = (int)i - 1;
          while (q >= 0 && p[q] > key) { p[q + 1] = p[q]; --q; }
          p[q + 1] = key;
        }
      } else {
        enqueue(b, sz);
      }
    }
  }
  if (over) atomicAdd(&ctrl->overflowed, over);
  __syncthreads();                                   // (the next partition of the pair reuses the counters and the staging)
  };
  const uint32_t dA = 2u * blockIdx.x, dB = dA + 1u;
  const bool both = dB < (uint32_t)nbins;
  uint32_t xA[kSlotBatch], xB[kSlotBatch];
  bool cachedA = false, cachedB = false;
  int ns0 = 0;
  if (single) {
    ns0 = prepare_pair(dA, both);
    const int nA = (int)nslots_p[0], nB = both ? (int)nslots_p[1] : 0;
    cachedA = nA <= 4 * kSlotBatch && nA <= slot_cap;
    cachedB = both && nB <= 4 * kSlotBatch && nB <= slot_cap;
    if (cachedA) load_batch(0, 0, 0, nA, xA);
    if (cachedB) load_batch(1, 0, 0, nB, xB);
  }
  run_partition(dA, 0, cachedA, xA, ns0);
  if (both) run_partition(dB, 1, cachedB, xB, ns0);
}

// One wave per queued bucket of at most 64 ids (within capacity): a bitonic sort across the lanes.
__global__ __launch_bounds__(256) void short_buckets_kernel(const uint32_t* __restrict__ off, int32_t* ids, uint32_t nb,
                                                            int64_t N, const uint64_t* __restrict__ worklist,
                                                            uint32_t wl_cap, const Ctrl* ctrl) {
  uint32_t n_items = ctrl->wl_short;
  if (n_items > wl_cap) n_items = wl_cap;
  const int lane = threadIdx.x & 63;
  const uint32_t wave = blockIdx.x * 4u + (threadIdx.x >> 6), nwaves = gridDim.x * 4u;
  for (uint32_t item = wave; item < n_items; item += nwaves) {
    const uint64_t w = worklist[wl_cap - 1u - item];
    const uint64_t t = w >> 32;
    const uint32_t c = (uint32_t)w;
    const uint32_t o0 = off[t * (nb + 1) + c];
    const uint32_t s = off[t * (nb + 1) + c + 1] - o0;          // <= 64
    int32_t* p = ids + t * N + o0;
    int32_t key = (uint32_t)lane < s ? p[lane] : 0x7fffffff;
#pragma unroll
    for (int k = 2; k <= 64; k <<= 1)
#pragma unroll
      for (int j = k >> 1; j > 0; j >>= 1) {
        const int32_t other = __shfl_xor(key, j);
        const bool up = (lane & k) == 0, lower = (lane & j) == 0;
        const int32_t mn = key < other ? key : other, mx = key < other ? other : key;
        key = (lower == up) ? mn : mx;
      }
    if ((uint32_t)lane < s) p[lane] = key;
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

constexpr int kSelStage = 4096;    // members of an over-capacity bucket staged in LDS while its survivors are chosen

// One workgroup per queued bucket.  size <= C: sort by id.  size > C: the survivors are the C members
// with the smallest (priority, id) keys.  The C-th smallest key is found digit by digit from the top
// (a 256-bin histogram of the candidates' next eight bits, a scan, the bin that holds rank C; the
// search ends as soon as the bins up to the chosen one hold exactly the wanted number, which with
// hashed priorities happens after two or three digits); then the members at or below it are gathered
// and put in id order.  A handful of barriers per bucket where a full sort of the members took eighty.
__global__ __launch_bounds__(256) void big_buckets_kernel(const uint32_t* __restrict__ off, int32_t* ids,
                                                          uint32_t nb, int64_t N, int C, int policy, uint32_t r,
                                                          uint32_t pa, uint32_t pb,
                                                          const uint64_t* __restrict__ worklist,
                                                          uint32_t wl_cap, const Ctrl* ctrl) {
  __shared__ uint64_t keys[kSortCap];
  __shared__ uint32_t sid[kSelStage];
  __shared__ uint32_t hist[256];
  __shared__ uint32_t pick[4];                 // chosen digit, rank left inside it, 1 when the search is over, survivors gathered
  uint32_t n_items = ctrl->wl_count;
  if (n_items > wl_cap) n_items = wl_cap;
  int capp = 1;
  while (capp < C) capp <<= 1;
  const int tid = threadIdx.x, lane = tid & 63;
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
      for (int i = tid; i < n2; i += 256) keys[i] = (uint32_t)i < s ? (uint64_t)(uint32_t)p[i] : ~0ull;
      __syncthreads();
      bitonic_sort_u64(keys, n2);
      for (uint32_t i = tid; i < s; i += 256) p[i] = (int32_t)(uint32_t)keys[i];
    } else {
      const bool in_lds = s <= (uint32_t)kSelStage;
      if (in_lds) for (uint32_t i = tid; i < s; i += 256) sid[i] = (uint32_t)p[i];
      hist[tid] = 0;
      if (tid == 0) pick[3] = 0;
      __syncthreads();
      auto member = [&](uint32_t i) { return in_lds ? sid[i] : (uint32_t)p[i]; };
      auto key_of = [&](uint32_t j) {
        const uint32_t pr = policy == SLIDE_KEEP_LOWEST_ID ? 0u : overflow_prio(j, (uint32_t)t, r, pa, pb);
        return ((uint64_t)pr << 32) | j;
      };
      uint64_t prefix = 0;                      // the digits chosen so far, in place
      uint32_t want = (uint32_t)C;              // rank of the wanted key among the candidates (1-based)
      int shift = policy == SLIDE_KEEP_LOWEST_ID ? 24 : 56;   // (without priorities the upper half of every key is zero)
      for (;; shift -= 8) {
        // candidates: the members whose digits above this one equal the chosen ones
        for (uint32_t i = tid; i < s; i += 256) {
          const uint64_t k = key_of(member(i));
          if (shift == 56 || (k >> (shift + 8)) == (prefix >> (shift + 8))) atomicAdd(&hist[(uint32_t)(k >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < 64) {                         // lane l: bins 4l .. 4l + 3
          const uint32_t c0 = hist[4 * lane], c1 = hist[4 * lane + 1], c2 = hist[4 * lane + 2], c3 = hist[4 * lane + 3];
          hist[4 * lane] = 0; hist[4 * lane + 1] = 0; hist[4 * lane + 2] = 0; hist[4 * lane + 3] = 0;
          const uint32_t tot = c0 + c1 + c2 + c3, incl = wave_incl_scan_add(tot), excl = incl - tot;
          if (excl < want && want <= incl) {    // (one lane: the candidates number at least `want`)
            uint32_t before = excl, digit = 4u * (uint32_t)lane, in_bin = c0;
            if (before + in_bin < want) { before += in_bin; ++digit; in_bin = c1; }
            if (before + in_bin < want) { before += in_bin; ++digit; in_bin = c2; }
            if (before + in_bin < want) { before += in_bin; ++digit; in_bin = c3; }
            pick[0] = digit;
            pick[1] = want - before;
            pick[2] = (before + in_bin == want || shift == 0) ? 1u : 0u;
          }
        }
        __syncthreads();
        prefix |= (uint64_t)pick[0] << shift;
        want = pick[1];
        const bool found = pick[2] != 0u;
        if (found || shift == 0) break;         // (uniform; at shift 0 a bin holds one key, so the search ends there at the latest)
      }
      // every key up to the chosen digit with all lower digits set survives: exactly C of them
      const uint64_t limit = prefix | (shift ? ((uint64_t)1 << shift) - 1u : 0u);
      uint32_t* surv = reinterpret_cast<uint32_t*>(keys);
      for (uint32_t i = tid; i < s; i += 256) {
        const uint32_t j = member(i);
        if (key_of(j) <= limit) {
          const uint32_t slot = atomicAdd(&pick[3], 1u);
          if (slot < (uint32_t)C) surv[slot] = j;
        }
      }
      __syncthreads();
      if (C <= 256) {
        // id order by counting: a survivor's place is the number of survivors with a smaller id
        if (tid < C) {
          const uint32_t mine = surv[tid];
          uint32_t place = 0;
          for (int q = 0; q < C; ++q) place += surv[q] < mine ? 1u : 0u;
          p[place] = (int32_t)mine;
        }
      } else {
        uint64_t mine[kSortCap / 512];            // capp <= 1024: at most 4 per thread
        for (int i = tid, q = 0; i < capp; i += 256, ++q) mine[q] = i < C ? (uint64_t)surv[i] : ~0ull;
        __syncthreads();
        for (int i = tid, q = 0; i < capp; i += 256, ++q) keys[i] = mine[q];
        __syncthreads();
        bitonic_sort_u64(keys, capp);
        for (int i = tid; i < C; i += 256) p[i] = (int32_t)(uint32_t)keys[i];
      }
    }
    __syncthreads();
  }
}

// Split of the code into partition digit (high hb bits) and in-partition digit (low lb bits).
void tables_split(int bits, int64_t N, int* hb, int* lb) {
  int want = 0;
  while (want < 11 && ((int64_t)2048 << want) < N) ++want;     // about 1024 to 2048 rows per partition
  int h = want < bits ? want : bits;
  if (bits - h > 13) h = bits - 13;                            // low digit counters must fit in LDS
  *hb = h;
  *lb = bits - h;
}

size_t tables_bh_words(int bits, int64_t N, int L) {      // run boundaries per (table, slab)
  int hb, lb;
  tables_split(bits, N, &hb, &lb);
  const int64_t nslab = (N + kSlab - 1) / kSlab;
  return (size_t)L * (size_t)(nslab > 0 ? nslab : 1) * (((size_t)1 << hb) + 1);
}

size_t tables_pbase_words(int bits, int64_t N, int L) {
  int hb, lb;
  tables_split(bits, N, &hb, &lb);
  return (size_t)L * (((size_t)1 << hb) + 1);
}

static int run_block(int nslab) { return nslab < kRunBlock ? nslab : kRunBlock; }
static size_t part_buckets_lds(int lb, int nsb, int stage) {
  const size_t nlo = (size_t)1 << lb;
  return (nlo + ((nlo + 63) >> 6) + 2 * (3 * (size_t)nsb + stage / 64) + stage + 4 + med_cap(stage)) * 4;
}
// The staging area of the bucket kernel: four mean partitions (a fresh layer's partitions stay within a
// few percent of the mean, a trained one's within a few times), so that tables with many buckets per
// partition, whose counters take most of the LDS, still fit another workgroup per compute unit.
static int stage_ids(int64_t N, int nbins) {
  const int64_t want = 4 * ((N + nbins - 1) / nbins);
  const int64_t s = want < kStageMin ? kStageMin : (want > kStageIds ? kStageIds : want);
  return (int)((s + 63) / 64 * 64);
}
static size_t slab_group_lds(int nbins) { return ((size_t)kSlab + (size_t)nbins + 20) * 4; }

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
  SLIDE_SET(part_buckets_kernel, part_buckets_lds(13, kRunBlock, kStageIds))
  SLIDE_SET(slab_group_kernel, slab_group_lds(2048))
#undef SLIDE_SET
  return hipSuccess;
}

hipError_t launch_build_tables(const HashDev& hd, const TablesDev& td, const float* W2, uint32_t* codes_t,
                               uint32_t* entries, uint32_t* bh, uint32_t* pbase, uint64_t* worklist,
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
  // (2) every slab grouped by the high digit in place, (3) partition starts, (4) buckets
  hipLaunchKernelGGL(slab_group_kernel, dim3(nslab, td.L), dim3(1024), slab_group_lds(nbins), s, codes_t, td.N, lb, nbins,
                     bh, nslab, entries);
  hipLaunchKernelGGL(part_scan_kernel, dim3(td.L), dim3(1024), 0, s, bh, nslab, nbins, pbase, ctrl);
  const int nsb = run_block(nslab);
  const int stage = stage_ids(td.N, nbins);
  hipLaunchKernelGGL(part_buckets_kernel, dim3((nbins + 1) / 2, td.L), dim3(256), part_buckets_lds(lb, nsb, stage), s, entries, bh,
                     nslab, pbase, nbins, lb, td.nb, td.N, td.C, td.off, td.ids, worklist, wl_cap, ctrl, nsb, stage);
  hipLaunchKernelGGL(short_buckets_kernel, dim3(2048), dim3(256), 0, s, td.off, td.ids, td.nb, td.N, worklist, wl_cap, ctrl);
  hipLaunchKernelGGL(big_buckets_kernel, dim3(2048), dim3(256), 0, s, td.off, td.ids, td.nb, td.N, td.C, policy,
                     r, prio_a, prio_b, worklist, wl_cap, ctrl);
  return hipGetLastError();
}

}  // namespace slide

