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

static int rows_per_tile(int H) { return H <= 512 ? 64 : (H <= 1024 ? 32 : 16); }
size_t hash_lds_bytes(int H) { return (size_t)H * (rows_per_tile(H) + 1) * sizeof(float); }

// Key of a coordinate: 0 if it cannot win (zero of either sign, NaN), else an unsigned integer that
// orders like the float (equal floats <-> equal keys), at least 1.
__device__ __forceinline__ uint32_t dwta_key(float x) {
  const uint32_t u = __float_as_uint(x);
  const uint32_t k = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return (x != 0.0f && x == x) ? k : 0u;
}

// Winner position of elementary hash e for the vector whose keys start at col0 (pitch `stride`);
// -1 when the bin has no entry.  Strictly greater wins, so ties keep the lowest position.
template <int M>
__device__ __forceinline__ int dwta_raw(const uint32_t* col0, int stride, const uint32_t* __restrict__ words, int e) {
  int best_p = -1;
  uint32_t best = 0u;
#pragma unroll
  for (int p2 = 0; p2 < M / 2; ++p2) {
    const uint32_t w = words[(size_t)e * (M / 2) + p2];
    const uint32_t k0 = col0[(w & 0xffffu) * stride];
    const uint32_t k1 = col0[(w >> 16) * stride];
    if (k0 > best) { best_p = 2 * p2; best = k0; }
    if (k1 > best) { best_p = 2 * p2 + 1; best = k1; }
  }
  return best_p;
}

template <int M>
__device__ uint32_t dwta_code(const HashDev& hd, const uint32_t* col0, int stride, int t, int& rowstate) {
  uint32_t code = 0;
  for (int k = 0; k < hd.K; ++k) {
    const int e = t * hd.K + k;                      // uniform over the lanes of a table
    int val = dwta_raw<M>(col0, stride, hd.words, e);
    if (val < 0) {                                   // empty bin: borrow (rare, per lane)
      if (rowstate < 0) {
        rowstate = 0;
        for (int c = 0; c < hd.H; ++c) if (col0[c * stride] != 0u) { rowstate = 1; break; }
      }
      val = 0;
      if (rowstate == 1) {
        for (uint32_t tr = 1; tr <= 100; ++tr) {
          const uint32_t u = hd.dens_a * (uint32_t)(e + 1) + hd.dens_b * tr;
          const int e2 = (int)((u >> 8) % (uint32_t)hd.NH);
          const int r2 = dwta_raw<M>(col0, stride, hd.words, e2);
          if (r2 >= 0) { val = r2; break; }
        }
      }
    }
    code |= (uint32_t)val << (k * hd.lgm);
  }
  return code;
}

__device__ uint32_t simhash_code(const HashDev& hd, const float* col0, int stride, int t) {
  uint32_t code = 0;
  const int half = hd.Spad / 2;
  for (int k = 0; k < hd.K; ++k) {
    const int e = t * hd.K + k;
    const uint32_t* __restrict__ sw = hd.words + (size_t)e * half;
    float acc = 0.0f;
    for (int s2 = 0; s2 < half; ++s2) {
      const uint32_t w = sw[s2];
      const float x0 = col0[(w & 0x7fffu) * stride];
      acc = (w & 0x8000u) ? acc - x0 : acc + x0;
      if (2 * s2 + 1 < hd.S) {
        const float x1 = col0[((w >> 16) & 0x7fffu) * stride];
        acc = (w & 0x80000000u) ? acc - x1 : acc + x1;
      }
    }
    code |= (acc > 0.0f ? 1u : 0u) << k;
  }
  return code;
}

// MODE 0: SimHash; 2,4,8,16: DWTA with that bin size.
template <int MODE, int THREADS>
__global__ __launch_bounds__(THREADS) void hash_rows_kernel(HashDev hd, const float* __restrict__ V,
                                                        int64_t rows, int RPT, uint32_t* __restrict__ codes,
                                                        int64_t row_stride, int64_t tab_stride,
                                                        uint32_t* hist, uint32_t* __restrict__ rank,
                                                        uint32_t nbp1, int tpb) {
  extern __shared__ float tile[];                    // [H][RPT + 1]
  const int stride = RPT + 1, H = hd.H;
  const int64_t row0 = (int64_t)blockIdx.x * RPT;
  for (int idx = threadIdx.x; idx < RPT * H; idx += blockDim.x) {   // coalesced read, conflict-free store
    const int r = idx / H, c = idx - r * H;
    const float x = (row0 + r < rows) ? V[(row0 + r) * H + c] : 0.0f;
    tile[c * stride + r] = MODE == 0 ? x : __uint_as_float(dwta_key(x));
  }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), nw = blockDim.x >> 6;
  const int tps = 64 / RPT;                          // tables per wave and step (RPT is 16, 32 or 64)
  const int r = lane & (RPT - 1), sub = lane / RPT;
  const bool active = row0 + r < rows;
  const float* col0 = tile + r;
  const int t_end = min((int)(blockIdx.y + 1) * tpb, hd.L);
  int rowstate = -1;
  for (int t0 = blockIdx.y * tpb + wave * tps; t0 < t_end; t0 += nw * tps) {
    const int t = t0 + sub;
    if (t >= t_end) continue;
    uint32_t code;
    if (MODE == 0) code = simhash_code(hd, col0, stride, t);
    else code = dwta_code<(MODE == 0 ? 2 : MODE)>(hd, (const uint32_t*)col0, stride, t, rowstate);
    if (active) {
      const int64_t row = row0 + r;
      codes[row * row_stride + (int64_t)t * tab_stride] = code;
      if (hist) {
        const uint32_t pos = atomicAdd(&hist[(size_t)t * nbp1 + code], 1u);
        rank[(size_t)t * rows + row] = pos;
      }
    }
  }
}

template <int MODE>
static hipError_t launch_mode(const HashDev& hd, const float* V, int64_t rows, uint32_t* codes,
                              int64_t row_stride, int64_t tab_stride, uint32_t* hist, uint32_t* rank,
                              uint32_t nb, int tpb, hipStream_t s) {
  const int RPT = rows_per_tile(hd.H);
  dim3 grid((unsigned)ceil_div(rows, RPT), (unsigned)ceil_div(hd.L, tpb));
  if (RPT == 64)
    hipLaunchKernelGGL((hash_rows_kernel<MODE, 256>), grid, dim3(256), hash_lds_bytes(hd.H), s, hd, V, rows, RPT, codes,
                       row_stride, tab_stride, hist, rank, nb + 1, tpb);
  else
    hipLaunchKernelGGL((hash_rows_kernel<MODE, 1024>), grid, dim3(1024), hash_lds_bytes(hd.H), s, hd, V, rows, RPT,
                       codes, row_stride, tab_stride, hist, rank, nb + 1, tpb);
  return hipGetLastError();
}

hipError_t launch_hash(const HashDev& hd, const float* V, int64_t rows, uint32_t* codes,
                       int64_t row_stride, int64_t tab_stride, uint32_t* hist, uint32_t* rank,
                       uint32_t nb, int tables_per_block, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const int tpb = tables_per_block < 1 ? 1 : tables_per_block;
  if (hd.kind == SLIDE_HASH_SIMHASH)
    return launch_mode<0>(hd, V, rows, codes, row_stride, tab_stride, hist, rank, nb, tpb, s);
  switch (hd.m) {
    case 2: return launch_mode<2>(hd, V, rows, codes, row_stride, tab_stride, hist, rank, nb, tpb, s);
    case 4: return launch_mode<4>(hd, V, rows, codes, row_stride, tab_stride, hist, rank, nb, tpb, s);
    case 8: return launch_mode<8>(hd, V, rows, codes, row_stride, tab_stride, hist, rank, nb, tpb, s);
    case 16: return launch_mode<16>(hd, V, rows, codes, row_stride, tab_stride, hist, rank, nb, tpb, s);
  }
  return hipErrorInvalidValue;
}

hipError_t hash_setup_attributes(int H) {
  const int bytes = (int)hash_lds_bytes(H);
  hipError_t e;
#define SLIDE_SET(K) \
  e = hipFuncSetAttribute((const void*)&K, hipFuncAttributeMaxDynamicSharedMemorySize, bytes); \
  if (e != hipSuccess) return e;
  SLIDE_SET((hash_rows_kernel<0, 256>))
  SLIDE_SET((hash_rows_kernel<2, 256>))
  SLIDE_SET((hash_rows_kernel<4, 256>))
  SLIDE_SET((hash_rows_kernel<8, 256>))
  SLIDE_SET((hash_rows_kernel<16, 256>))
  SLIDE_SET((hash_rows_kernel<0, 1024>))
  SLIDE_SET((hash_rows_kernel<2, 1024>))
  SLIDE_SET((hash_rows_kernel<4, 1024>))
  SLIDE_SET((hash_rows_kernel<8, 1024>))
  SLIDE_SET((hash_rows_kernel<16, 1024>))
#undef SLIDE_SET
  return hipSuccess;
}

}  // namespace slide
