// Locality-sensitive hash codes of fp32 vectors (hidden activations when the tables are
// queried, rows of W2 when they are built; paper Sections 2.1, 3.1, 4.1).
//
// Mapping: one lane owns one vector; the workgroup stages a tile of vectors in LDS transposed
// ([coordinate][vector], odd row pitch), so for a given elementary hash every lane reads the
// same coordinate of its own vector: the coordinate tables are wave-uniform (scalar loads) and
// the LDS reads hit consecutive banks.  The waves of a workgroup take different tables; when a
// tile holds fewer than 64 vectors (long vectors), the lane groups of a wave take different tables
// too, and the workgroup has more waves to cover the LDS latency.
// For DWTA the tile holds order-preserving integer keys instead of floats (0 = entry absent: zero or
// NaN), so that a comparison is one unsigned compare and two selects.
#include "slide_internal.h"

namespace slide {

// Vectors per tile of the row-tile kernel: 64 (a wave per table) while two tiles fit a compute unit's LDS;
// beyond that 16, so that two workgroups still share a compute unit and one reads its tile while the
// other hashes (with 32 vectors of 1,024 coordinates a single workgroup filled the LDS and the unit
// idled through every tile read).
static int rows_per_tile(int H) { return H <= 512 ? 64 : 16; }
size_t hash_lds_bytes(int H) { return ((size_t)H + 1) * (rows_per_tile(H) + 1) * sizeof(float); }
int hash_tile_pitch(int H) { return rows_per_tile(H) + 1; }

// Key of a coordinate: 0 if it cannot win (zero of either sign, NaN), else an unsigned integer that
// orders like the float (equal floats <-> equal keys), at least 1.
__device__ __forceinline__ uint32_t dwta_key(float x) {
  const uint32_t u = __float_as_uint(x);
  const uint32_t k = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return (x != 0.0f && x == x) ? k : 0u;
}

// The row-tile kernel reads its coordinates from a second parameter table, offs: one 32-bit entry
// per coordinate = its byte offset in the transposed tile (coordinate * pitch * 4), so that an LDS
// address is one add (the 16-bit coordinate table would cost a mask, a multiply and a shift per
// element); SimHash entries carry the sign in bit 31, and a bit's entries are padded to a multiple
// of eight with pointers to a row of zeros behind the tile (adding +0 changes no sum).
//
// Winner position of elementary hash e for the vector whose keys start at byte address col0 of the
// tile; -1 when the bin has no entry.  Strictly greater wins, so ties keep the lowest position.
// Eight keys of the lane's vector at the (wave-uniform) byte offsets o[0..8) of the tile, whose vector
// of lane l starts 4*l bytes into every coordinate's row: the read that adds the lane number to a scalar
// base address, so that no lane spends an instruction on the address (a wait state between the write of
// the base register and the read is required on this family).  tile_base: LDS address of the tile.
__device__ __forceinline__ void read8_lane_rows(uint32_t (&k)[8], const uint32_t* __restrict__ o, uint32_t tile_base) {
  asm volatile(
      "s_add_u32 m0, %16, %8\n\ts_nop 0\n\tds_read_addtid_b32 %0\n\t"
      "s_add_u32 m0, %16, %9\n\ts_nop 0\n\tds_read_addtid_b32 %1\n\t"
      "s_add_u32 m0, %16, %10\n\ts_nop 0\n\tds_read_addtid_b32 %2\n\t"
      "s_add_u32 m0, %16, %11\n\ts_nop 0\n\tds_read_addtid_b32 %3\n\t"
      "s_add_u32 m0, %16, %12\n\ts_nop 0\n\tds_read_addtid_b32 %4\n\t"
      "s_add_u32 m0, %16, %13\n\ts_nop 0\n\tds_read_addtid_b32 %5\n\t"
      "s_add_u32 m0, %16, %14\n\ts_nop 0\n\tds_read_addtid_b32 %6\n\t"
      "s_add_u32 m0, %16, %15\n\ts_nop 0\n\tds_read_addtid_b32 %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(k[0]), "=&v"(k[1]), "=&v"(k[2]), "=&v"(k[3]), "=&v"(k[4]), "=&v"(k[5]), "=&v"(k[6]), "=&v"(k[7])
      : "s"(o[0]), "s"(o[1]), "s"(o[2]), "s"(o[3]), "s"(o[4]), "s"(o[5]), "s"(o[6]), "s"(o[7]), "s"(tile_base)
      : "m0", "scc", "memory");
}

// The same for two bins at once (sixteen reads in flight before the wait).
__device__ __forceinline__ void read16_lane_rows(uint32_t (&a)[8], uint32_t (&b)[8], const uint32_t* __restrict__ oa,
                                                 const uint32_t* __restrict__ ob, uint32_t tile_base) {
  asm volatile(
      "s_add_u32 m0, %16, %8\n\ts_nop 0\n\tds_read_addtid_b32 %0\n\t"
      "s_add_u32 m0, %16, %9\n\ts_nop 0\n\tds_read_addtid_b32 %1\n\t"
      "s_add_u32 m0, %16, %10\n\ts_nop 0\n\tds_read_addtid_b32 %2\n\t"
      "s_add_u32 m0, %16, %11\n\ts_nop 0\n\tds_read_addtid_b32 %3\n\t"
      "s_add_u32 m0, %16, %12\n\ts_nop 0\n\tds_read_addtid_b32 %4\n\t"
      "s_add_u32 m0, %16, %13\n\ts_nop 0\n\tds_read_addtid_b32 %5\n\t"
      "s_add_u32 m0, %16, %14\n\ts_nop 0\n\tds_read_addtid_b32 %6\n\t"
      "s_add_u32 m0, %16, %15\n\ts_nop 0\n\tds_read_addtid_b32 %7"
      : "=&v"(a[0]), "=&v"(a[1]), "=&v"(a[2]), "=&v"(a[3]), "=&v"(a[4]), "=&v"(a[5]), "=&v"(a[6]), "=&v"(a[7])
      : "s"(oa[0]), "s"(oa[1]), "s"(oa[2]), "s"(oa[3]), "s"(oa[4]), "s"(oa[5]), "s"(oa[6]), "s"(oa[7]), "s"(tile_base)
      : "m0", "scc", "memory");
  asm volatile(
      "s_add_u32 m0, %16, %8\n\ts_nop 0\n\tds_read_addtid_b32 %0\n\t"
      "s_add_u32 m0, %16, %9\n\ts_nop 0\n\tds_read_addtid_b32 %1\n\t"
      "s_add_u32 m0, %16, %10\n\ts_nop 0\n\tds_read_addtid_b32 %2\n\t"
      "s_add_u32 m0, %16, %11\n\ts_nop 0\n\tds_read_addtid_b32 %3\n\t"
      "s_add_u32 m0, %16, %12\n\ts_nop 0\n\tds_read_addtid_b32 %4\n\t"
      "s_add_u32 m0, %16, %13\n\ts_nop 0\n\tds_read_addtid_b32 %5\n\t"
      "s_add_u32 m0, %16, %14\n\ts_nop 0\n\tds_read_addtid_b32 %6\n\t"
      "s_add_u32 m0, %16, %15\n\ts_nop 0\n\tds_read_addtid_b32 %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(b[0]), "=&v"(b[1]), "=&v"(b[2]), "=&v"(b[3]), "=&v"(b[4]), "=&v"(b[5]), "=&v"(b[6]), "=&v"(b[7])
      : "s"(ob[0]), "s"(ob[1]), "s"(ob[2]), "s"(ob[3]), "s"(ob[4]), "s"(ob[5]), "s"(ob[6]), "s"(ob[7]), "s"(tile_base)
      : "m0", "scc", "memory");
  // (the first eight registers are filled only once the wait above has passed: nothing may read them earlier)
  asm volatile("" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]));
}

// Winner position among the M keys of a bin, and the winning key (0: the bin has no entry).
template <int M>
__device__ __forceinline__ uint32_t dwta_winner(const uint32_t (&k)[M], uint32_t& best) {
  best = k[0];                                       // the largest key first (three-operand maxima) ...
#pragma unroll
  for (int p = 1; p < M; ++p) best = max(best, k[p]);
  bool eq[M];                                        // ... then the lowest position that holds it
#pragma unroll
  for (int p = 0; p < M; ++p) eq[p] = k[p] == best;
  uint32_t best_p = M - 1;
#pragma unroll
  for (int p = M - 2; p >= 0; --p) best_p = eq[p] ? (uint32_t)p : best_p;
  return best_p;
}

template <int M, bool UNI>
__device__ __forceinline__ int dwta_raw(const char* col0, const uint32_t* __restrict__ offs, int e, uint32_t tile_base = 0) {
  const uint32_t* o = offs + (size_t)(UNI ? __builtin_amdgcn_readfirstlane(e) : e) * M;
  uint32_t k[M];
  if constexpr (M == 8 && UNI) {
    read8_lane_rows(k, o, tile_base);
  } else {
#pragma unroll
    for (int p = 0; p < M; ++p) k[p] = *(const uint32_t*)(col0 + o[p]);
  }
  uint32_t best = k[0];                              // the largest key first (three-operand maxima) ...
#pragma unroll
  for (int p = 1; p < M; ++p) best = max(best, k[p]);
  bool eq[M];                                        // ... then the lowest position that holds it
#pragma unroll
  for (int p = 0; p < M; ++p) eq[p] = k[p] == best;
  int best_p = M - 1;
#pragma unroll
  for (int p = M - 2; p >= 0; --p) best_p = eq[p] ? p : best_p;
  return best == 0u ? -1 : best_p;
}

template <int M, bool UNI>
__device__ __forceinline__ uint32_t dwta_code(const HashDev& hd, const uint32_t* __restrict__ offs, const char* col0,
                                              int pitch_bytes, int t, int& rowstate, uint32_t tile_base) {
  // Empty bin: borrow the winner of another elementary hash (rare, per lane).
  auto borrow = [&](int e) -> int {
    if (rowstate < 0) {
      rowstate = 0;
      for (int c = 0; c < hd.H; ++c) if (*(const uint32_t*)(col0 + (size_t)c * pitch_bytes) != 0u) { rowstate = 1; break; }
    }
    if (rowstate == 1)
      for (uint32_t tr = 1; tr <= 100; ++tr) {
        const uint32_t u = hd.dens_a * (uint32_t)(e + 1) + hd.dens_b * tr;
        const int e2 = (int)((u >> 8) % (uint32_t)hd.NH);
        const int r2 = dwta_raw<M, false>(col0, offs, e2);
        if (r2 >= 0) return r2;
      }
    return 0;
  };
  uint32_t code = 0;
  const int e0 = UNI ? __builtin_amdgcn_readfirstlane(t * hd.K) : t * hd.K;   // uniform over the lanes of a table
  int k = 0;
  for (; k + 1 < hd.K; k += 2) {                     // two independent argmax chains in flight
    if constexpr (M == 8 && UNI) {
      const uint32_t* o = offs + (size_t)(e0 + k) * 8;
      uint32_t ka[8], kb[8], ba, bb;
      read16_lane_rows(ka, kb, o, o + 8, tile_base);
      uint32_t v0 = dwta_winner<8>(ka, ba), v1 = dwta_winner<8>(kb, bb);
      if (__any(min(ba, bb) == 0u)) {                // (an empty bin in some lane: rare)
        if (ba == 0u) v0 = (uint32_t)borrow(e0 + k);
        if (bb == 0u) v1 = (uint32_t)borrow(e0 + k + 1);
      }
      code |= (v0 << (k * hd.lgm)) | (v1 << ((k + 1) * hd.lgm));
    } else {
      int v0 = dwta_raw<M, UNI>(col0, offs, e0 + k, tile_base);
      int v1 = dwta_raw<M, UNI>(col0, offs, e0 + k + 1, tile_base);
      if (v0 < 0) v0 = borrow(e0 + k);
      if (v1 < 0) v1 = borrow(e0 + k + 1);
      code |= ((uint32_t)v0 << (k * hd.lgm)) | ((uint32_t)v1 << ((k + 1) * hd.lgm));
    }
  }
  if (k < hd.K) {
    int v0 = dwta_raw<M, UNI>(col0, offs, e0 + k, tile_base);
    if (v0 < 0) v0 = borrow(e0 + k);
    code |= (uint32_t)v0 << (k * hd.lgm);
  }
  return code;
}

template <bool UNI>
__device__ __forceinline__ uint32_t simhash_code(const HashDev& hd, const uint32_t* __restrict__ offs, const char* col0,
                                                 int t) {
  uint32_t code = 0;
  for (int k = 0; k < hd.K; ++k) {
    const int e = UNI ? __builtin_amdgcn_readfirstlane(t * hd.K + k) : t * hd.K + k;
    const uint32_t* __restrict__ o = offs + (size_t)e * hd.So;        // So is a multiple of 8
    float acc = 0.0f;
    for (int q = 0; q < hd.So; q += 8) {             // sequential sum: a - x is a + (-x) bit for bit
      uint32_t w[8], x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) w[j] = o[q + j];
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = *(const uint32_t*)(col0 + (w[j] & 0x7fffffffu));
#pragma unroll
      for (int j = 0; j < 8; ++j) acc += __uint_as_float(x[j] ^ (w[j] & 0x80000000u));
    }
    code |= (acc > 0.0f ? 1u : 0u) << k;
  }
  return code;
}

// MODE 0: SimHash; 2,4,8,16: DWTA with that bin size.  UNI: a tile holds 64 vectors, so a wave works
// on one table at a time and reads its coordinates through scalar loads.
// rowlist == nullptr: vectors 0 .. rows-1 of V.  Otherwise the vectors rowlist[0 .. *nrows_dev) of V
// (the grid covers rows; tiles past the device-side count leave at once; a count equal to rows means
// all of them, and the list is not read).
template <int MODE, bool UNI>
__global__ __launch_bounds__(1024) void hash_rows_kernel(HashDev hd, const uint32_t* __restrict__ offs,
                                                        const float* __restrict__ V,
                                                        int64_t rows, int RPT, uint32_t* __restrict__ codes,
                                                        int64_t row_stride, int64_t tab_stride,
                                                        const int32_t* __restrict__ rowlist,
                                                        const uint32_t* __restrict__ nrows_dev, int tpb) {
  extern __shared__ float tile[];                    // [H + 1][RPT + 1]; the last row is zero
  __shared__ int64_t rid[64];                        // vector held by tile column r, -1 = none
  const int stride = RPT + 1, H = hd.H;
  const int64_t row0 = (int64_t)blockIdx.x * RPT;
  if (rowlist) {
    const int64_t listed = (int64_t)*nrows_dev;
    if (listed == rows) rowlist = nullptr;           // every vector: in place, without the list
    rows = listed;
  }
  if (row0 >= rows) return;
  if ((int)threadIdx.x < RPT) {
    const int64_t q = row0 + threadIdx.x;
    rid[threadIdx.x] = q < rows ? (rowlist ? (int64_t)rowlist[q] : q) : -1;
  }
  if ((int)threadIdx.x < stride) tile[H * stride + threadIdx.x] = 0.0f;
  __syncthreads();
  // coalesced reads, eight per thread in flight (a tile of long vectors is tens of elements per thread,
  // and one at a time would be as many round trips to memory); conflict-free stores
  constexpr int kTileBatch = 8;
  const int total = RPT * H;
  for (int base = 0; base < total; base += kTileBatch * (int)blockDim.x) {
    float x[kTileBatch];
    int at[kTileBatch];
#pragma unroll
    for (int u = 0; u < kTileBatch; ++u) {
      const int idx = base + u * (int)blockDim.x + (int)threadIdx.x;
      x[u] = 0.0f;
      at[u] = -1;
      if (idx < total) {
        const int r = idx / H, c = idx - r * H;
        const int64_t row = rid[r];
        at[u] = c * stride + r;
        if (row >= 0) x[u] = V[row * H + c];
      }
    }
#pragma unroll
    for (int u = 0; u < kTileBatch; ++u)
      if (at[u] >= 0) tile[at[u]] = MODE == 0 ? x[u] : __uint_as_float(dwta_key(x[u]));
  }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
  const int tps = 64 / RPT;                          // tables per wave and step (RPT is 16, 32 or 64)
  const int r = lane & (RPT - 1), sub = lane / RPT;
  const int64_t row = rid[r];
  const char* col0 = (const char*)(tile + r);
  const uint32_t tile_base = (uint32_t)(uintptr_t)tile;   // (the low half of a generic LDS address is the LDS address)
  const int t_end = min((int)(blockIdx.y + 1) * tpb, hd.L);
  int rowstate = -1;
  for (int t0 = blockIdx.y * tpb + wave * tps; t0 < t_end; t0 += nw * tps) {
    const int t = t0 + sub;
    if (t >= t_end) continue;
    uint32_t code;
    if (MODE == 0) code = simhash_code<UNI>(hd, offs, col0, t);
    else code = dwta_code<(MODE == 0 ? 2 : MODE), UNI>(hd, offs, col0, stride * 4, t, rowstate, tile_base);
    if (row >= 0) codes[row * row_stride + (int64_t)t * tab_stride] = code;
  }
}

template <int MODE>
static hipError_t launch_mode(const HashDev& hd, const float* V, int64_t rows, uint32_t* codes,
                              int64_t row_stride, int64_t tab_stride, const int32_t* rowlist,
                              const uint32_t* nrows_dev, int tpb, hipStream_t s) {
  const int RPT = rows_per_tile(hd.H);
  dim3 grid((unsigned)ceil_div(rows, RPT), (unsigned)ceil_div(hd.L, tpb));
  if (RPT == 64)
    hipLaunchKernelGGL((hash_rows_kernel<MODE, true>), grid, dim3(1024), hash_lds_bytes(hd.H), s, hd, hd.offs, V, rows,
                       RPT, codes, row_stride, tab_stride, rowlist, nrows_dev, tpb);
  else
    hipLaunchKernelGGL((hash_rows_kernel<MODE, false>), grid, dim3(1024), hash_lds_bytes(hd.H), s, hd, hd.offs, V, rows,
                       RPT, codes, row_stride, tab_stride, rowlist, nrows_dev, tpb);
  return hipGetLastError();
}

hipError_t launch_hash(const HashDev& hd, const float* V, int64_t rows, uint32_t* codes,
                       int64_t row_stride, int64_t tab_stride, const int32_t* rowlist,
                       const uint32_t* nrows_dev, int tables_per_block, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const int tpb = tables_per_block < 1 ? 1 : tables_per_block;
  if (hd.kind == SLIDE_HASH_SIMHASH)
    return launch_mode<0>(hd, V, rows, codes, row_stride, tab_stride, rowlist, nrows_dev, tpb, s);
  switch (hd.m) {
    case 2: return launch_mode<2>(hd, V, rows, codes, row_stride, tab_stride, rowlist, nrows_dev, tpb, s);
    case 4: return launch_mode<4>(hd, V, rows, codes, row_stride, tab_stride, rowlist, nrows_dev, tpb, s);
    case 8: return launch_mode<8>(hd, V, rows, codes, row_stride, tab_stride, rowlist, nrows_dev, tpb, s);
    case 16: return launch_mode<16>(hd, V, rows, codes, row_stride, tab_stride, rowlist, nrows_dev, tpb, s);
  }
  return hipErrorInvalidValue;
}

hipError_t hash_setup_attributes(int H) {
  const int bytes = (int)hash_lds_bytes(H);
  hipError_t e;
#define SLIDE_SET(K) \
  e = hipFuncSetAttribute((const void*)&K, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); \
  if (e != hipSuccess) return e;
  SLIDE_SET((hash_rows_kernel<0, true>))
  SLIDE_SET((hash_rows_kernel<2, true>))
  SLIDE_SET((hash_rows_kernel<4, true>))
  SLIDE_SET((hash_rows_kernel<8, true>))
  SLIDE_SET((hash_rows_kernel<16, true>))
  SLIDE_SET((hash_rows_kernel<0, false>))
  SLIDE_SET((hash_rows_kernel<2, false>))
  SLIDE_SET((hash_rows_kernel<4, false>))
  SLIDE_SET((hash_rows_kernel<8, false>))
  SLIDE_SET((hash_rows_kernel<16, false>))
#undef SLIDE_SET
  return hipSuccess;
}

}  // namespace slide
