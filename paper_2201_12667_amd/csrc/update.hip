// Sparse backpropagation into the parameters fused with row-sparse Adam (paper Algorithm 1:
// gradients reach only the active neurons, then the optimizer step after the batch; Section 3.5: every
// weight and bias carries a momentum and a velocity value; constants of Section 4.1).
//
// rowgrad_adam: each touched row is read once (w, m, v), its gradient is formed in registers from
// the row's pair list -- g = sum_i coef_i * V[sample_i][:], samples ascending, so the sum order is
// fixed -- and w, m, v are written back once: 6 row transfers per touched row, no gradient buffer
// and no atomics.  V is the hidden activations (output layer) or their gradient (input layer),
// small enough to stay cache resident.  Rows that are not listed are never touched.
#include "slide_internal.h"
#include "wave_ops.h"

#include <algorithm>

namespace slide {

typedef float slide_v4f __attribute__((ext_vector_type(4)));
// Moment rows are touched once per step and by nothing else: streamed past the caches.
__device__ __forceinline__ float4 load_stream(const float* p) {
  const slide_v4f v = __builtin_nontemporal_load((const slide_v4f*)p);
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(float* p, const float4& x) {
  slide_v4f v; v.x = x.x; v.y = x.y; v.z = x.z; v.w = x.w;
  __builtin_nontemporal_store(v, (slide_v4f*)p);
}

constexpr int kUpdateThreads = 256;

// One element of the Adam update.  The square root and the reciprocal are the hardware's one-ulp
// instructions rather than the correctly rounded library sequences (about 25 instructions per element
// otherwise, which the row kernels feel once the rows come from cache): the step
// lr * mhat / (sqrt(vhat) + eps) is off by a few units in its last place, i.e. by about 1e-7 of a
// quantity that is itself at most lr.  (A denormal vhat may be taken as zero by the square root; eps
// dominates the denominator long before that.)
__device__ __forceinline__ void adam1(float& w, float& m, float& v, float g, const AdamDev& a) {
  m = a.beta1 * m + a.omb1 * g;
  v = a.beta2 * v + a.omb2 * g * g;
  w = w - (a.lr * (m * a.inv_bc1)) * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(v * a.inv_bc2) + a.eps);
}

// Gradient of one row from its pair list, pairs first, first + stride, ... (this lane group's share).
// Every load is unconditional (lanes past the end of their list read pair 0 of the list, sample 0,
// and select zero afterwards), so that all of a step's loads are in flight together.  FULL: the
// lane groups cover the vector exactly (H == LPR*CH*4), no column test.
template <int LPR, int CH, int UNR, bool FULL>
__device__ __forceinline__ void row_gradient(int H, int sub, const PairsDev& pd, const float* __restrict__ coef,
                                             const float* __restrict__ V, uint32_t st, int cn, int first,
                                             int stride, float4 (&g)[CH], float& gb) {
  for (int q = first; __any(q < cn); q += UNR * stride) {
    float d[UNR];
    float4 hv[UNR][CH];
#pragma unroll
    for (int a = 0; a < UNR; ++a) {
      const bool ok = q + a * stride < cn;
      const int2 pr = pd.pairs[st + (ok ? q + a * stride : 0)];
      const int si = ok ? pr.x : 0;
      const float dv = coef[ok ? pr.y : 0];
      d[a] = ok ? dv : 0.f;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int col = (c * LPR + sub) * 4;
        const bool cok = FULL || col < H;
        const float4 x = *(const float4*)(V + (size_t)si * H + (cok ? col : 0));
        hv[a][c] = cok ? x : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int a = 0; a < UNR; ++a) {
      gb += d[a];
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        g[c].x += d[a] * hv[a][c].x; g[c].y += d[a] * hv[a][c].y;
        g[c].z += d[a] * hv[a][c].z; g[c].w += d[a] * hv[a][c].w;
      }
    }
  }
}

// Work item = RPW consecutive row slots of one tile (RPW = 64/LPR rows per wave, LPR lanes per row,
// CH float4 per lane).  Rows with more than kLongRow pairs are skipped here and taken afterwards,
// with more lanes on the pair list: by a whole wave each when a row needs only part of a wave (its
// RPW lane groups accumulate interleaved shares of the list, added in a fixed butterfly order), by
// a whole workgroup each when a row fills a wave (the waves accumulate interleaved shares, added in
// wave order through LDS).
template <int LPR, int CH, int UNR, bool FULL>
__device__ void rowgrad_adam(int H, const RowUpdate& ru, const AdamDev& ad, int block, int nblocks) {
  const PairsDev& pd = ru.pd;
  const float* __restrict__ coef = ru.coef;
  const float* __restrict__ V = ru.V;
  float* __restrict__ W = ru.W;
  float* __restrict__ M = ru.M;
  float* __restrict__ Vv = ru.Vv;
  float* __restrict__ bias = ru.bias;
  float* __restrict__ mbias = ru.mbias;
  float* __restrict__ vbias = ru.vbias;
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane % LPR, grp = lane / LPR;
  const int wave_global = block * 4 + (threadIdx.x >> 6), nwaves = nblocks * 4;
  const int cpt = ((int)*pd.max_nu + RPW - 1) / RPW;       // items per tile that can hold rows
  const int nitems = pd.ntiles * cpt;
  for (int item = wave_global; item < nitems; item += nwaves) {
    // chunk-major order: the non-empty items (low chunk numbers of every tile) are contiguous, so
    // consecutive waves all get work
    const int ch = item / pd.ntiles, t = item - ch * pd.ntiles;
    const int nu = pd.tile_nu[t];
    if (ch * RPW >= nu) continue;
    const int r = ch * RPW + grp;
    const int slot = t * pd.rows_per_tile + r;
    const int4 meta = r < nu ? pd.umeta[slot] : make_int4(0, 0, 0, 0);
    int cn = meta.z;
    const bool valid = r < nu && cn <= kLongRow;
    if (!valid) cn = 0;
    const int j = valid ? meta.x : 0;
    const size_t ro = (size_t)j * H;
    const uint32_t st = (uint32_t)meta.y;
    // the gradient first (few registers live, so that many waves fit and cover its chain of
    // dependent reads: header -> pairs -> coefficients and vectors), then the row itself
    float4 g[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    float gb = 0.f;
    row_gradient<LPR, CH, UNR, FULL>(H, sub, pd, coef, V, st, cn, 0, 1, g, gb);
    if (!valid) continue;
    asm volatile("" ::: "memory");                       // keep the row's loads behind the gradient loop
    float4 w[CH], m[CH], v[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      if (FULL || col < H) {
        w[c] = *(const float4*)(W + ro + col);
        m[c] = load_stream(M + ro + col);
        v[c] = load_stream(Vv + ro + col);
      }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      if (FULL || col < H) {
        adam1(w[c].x, m[c].x, v[c].x, g[c].x, ad); adam1(w[c].y, m[c].y, v[c].y, g[c].y, ad);
        adam1(w[c].z, m[c].z, v[c].z, g[c].z, ad); adam1(w[c].w, m[c].w, v[c].w, g[c].w, ad);
        *(float4*)(W + ro + col) = w[c];
        store_stream(M + ro + col, m[c]);
        store_stream(Vv + ro + col, v[c]);
      }
    }
    if (bias && sub == 0) {
      float bw = bias[j], bm = mbias[j], bv = vbias[j];
      adam1(bw, bm, bv, gb, ad);
      bias[j] = bw; mbias[j] = bm; vbias[j] = bv;
    }
  }
  const int nlong = min((int)*pd.nlong, pd.long_cap);
  if constexpr (RPW == 1) {
    constexpr int NW = kUpdateThreads / 64;              // waves of the workgroup
    __shared__ float4 part[NW - 1][CH][64];
    __shared__ float partb[NW - 1];
    const int wv = threadIdx.x >> 6;
    for (int l = block; l < nlong; l += nblocks) {       // (the same trip count for every wave of the workgroup)
      const int slot = pd.longlist[l];
      const int4 meta = pd.umeta[slot];
      const int j = meta.x, cn = meta.z;
      const size_t ro = (size_t)j * H;
      const uint32_t st = (uint32_t)meta.y;
      float4 g[CH];
#pragma unroll
      for (int c = 0; c < CH; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
      float gb = 0.f;
      row_gradient<LPR, CH, 2 * UNR, FULL>(H, sub, pd, coef, V, st, cn, wv, NW, g, gb);
      if (wv > 0) {
#pragma unroll
        for (int c = 0; c < CH; ++c) part[wv - 1][c][lane] = g[c];
        if (lane == 0) partb[wv - 1] = gb;
      }
      __syncthreads();
      if (wv == 0) {
        float4 w[CH], m[CH], v[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const int col = (c * LPR + sub) * 4;
          if (FULL || col < H) {
            w[c] = *(const float4*)(W + ro + col);
            m[c] = load_stream(M + ro + col);
            v[c] = load_stream(Vv + ro + col);
          }
        }
        for (int k = 0; k < NW - 1; ++k) {
          gb += partb[k];
#pragma unroll
          for (int c = 0; c < CH; ++c) {
            const float4 p = part[k][c][lane];
            g[c].x += p.x; g[c].y += p.y; g[c].z += p.z; g[c].w += p.w;
          }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const int col = (c * LPR + sub) * 4;
          if (FULL || col < H) {
            adam1(w[c].x, m[c].x, v[c].x, g[c].x, ad); adam1(w[c].y, m[c].y, v[c].y, g[c].y, ad);
            adam1(w[c].z, m[c].z, v[c].z, g[c].z, ad); adam1(w[c].w, m[c].w, v[c].w, g[c].w, ad);
            *(float4*)(W + ro + col) = w[c];
            store_stream(M + ro + col, m[c]);
            store_stream(Vv + ro + col, v[c]);
          }
        }
        if (bias && sub == 0) {
          float bw = bias[j], bm = mbias[j], bv = vbias[j];
          adam1(bw, bm, bv, gb, ad);
          bias[j] = bw; mbias[j] = bm; vbias[j] = bv;
        }
      }
      __syncthreads();
    }
    return;
  }
  for (int l = wave_global; l < nlong; l += nwaves) {
    const int slot = pd.longlist[l];
    const int4 meta = pd.umeta[slot];
    const int j = meta.x, cn = meta.z;
    const size_t ro = (size_t)j * H;
    const uint32_t st = (uint32_t)meta.y;
    float4 g[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    float gb = 0.f;
    row_gradient<LPR, CH, UNR, FULL>(H, sub, pd, coef, V, st, cn, grp, RPW, g, gb);
#pragma unroll
    for (int d = LPR; d < 64; d <<= 1) {
      gb += __shfl_xor(gb, d);
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        g[c].x += __shfl_xor(g[c].x, d); g[c].y += __shfl_xor(g[c].y, d);
        g[c].z += __shfl_xor(g[c].z, d); g[c].w += __shfl_xor(g[c].w, d);
      }
    }
    if (grp != 0) continue;
    float4 w[CH], m[CH], v[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      if (FULL || col < H) {
        w[c] = *(const float4*)(W + ro + col);
        m[c] = load_stream(M + ro + col);
        v[c] = load_stream(Vv + ro + col);
      }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      if (FULL || col < H) {
        adam1(w[c].x, m[c].x, v[c].x, g[c].x, ad); adam1(w[c].y, m[c].y, v[c].y, g[c].y, ad);
        adam1(w[c].z, m[c].z, v[c].z, g[c].z, ad); adam1(w[c].w, m[c].w, v[c].w, g[c].w, ad);
        *(float4*)(W + ro + col) = w[c];
        store_stream(M + ro + col, m[c]);
        store_stream(Vv + ro + col, v[c]);
      }
    }
    if (bias && sub == 0) {
      float bw = bias[j], bm = mbias[j], bv = vbias[j];
      adam1(bw, bm, bv, gb, ad);
      bias[j] = bw; mbias[j] = bm; vbias[j] = bv;
    }
  }
}

// Block 0: loss = mean_i loss_i (fixed-shape reduction) and the step statistics.  With b1: every
// block takes 32 columns of gb1[u] = sum_i dh[i][u]; 8 partial sums per column over interleaved
// samples, added in a fixed order, then Adam on the dense hidden bias.
__device__ void finish_role(int H, const FinishArgs& f, const AdamDev& ad, int block) {
  const int B = f.B;
  const float* __restrict__ loss_i = f.loss_i;
  float* __restrict__ d_loss = f.d_loss;
  const float* __restrict__ dh = f.dh;
  float* __restrict__ b1 = f.b1;
  float* __restrict__ mb1 = f.mb1;
  float* __restrict__ vb1 = f.vb1;
  Ctrl* ctrl = f.ctrl;
  const int32_t* __restrict__ tile_nu2 = f.tile_nu2;
  const int32_t* __restrict__ tile_nu1 = f.tile_nu1;
  const int ntiles2 = f.ntiles2, ntiles1 = f.ntiles1;
  __shared__ float red[256];
  __shared__ unsigned long long ured[4][256];
  const int tid = threadIdx.x;
  const bool act = tid < 256;             // (workgroups may be larger: the first 256 threads do the work)
  if (block == 0) {
    float acc = 0.f;
    unsigned long long u2 = 0, u1 = 0, pairs = 0, cand = 0;
    if (act) {
      for (int i = tid; i < B; i += 256) acc += loss_i[i];
      for (int t = tid; t < ntiles2; t += 256) u2 += (unsigned long long)tile_nu2[t];
      for (int t = tid; t < ntiles1; t += 256) u1 += (unsigned long long)tile_nu1[t];
      for (int i = tid; i < B; i += 256) { pairs += (unsigned long long)f.cnt[i]; cand += (unsigned long long)f.ncand[i]; }
      red[tid] = acc; ured[0][tid] = u2; ured[1][tid] = u1; ured[2][tid] = pairs; ured[3][tid] = cand;
    }
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
      if (tid < d) {
        red[tid] += red[tid + d];
        for (int q = 0; q < 4; ++q) ured[q][tid] += ured[q][tid + d];
      }
      __syncthreads();
    }
    if (tid == 0) {
      if (d_loss) *d_loss = red[0] / (float)B;
      ctrl->u2 = ured[0][0]; ctrl->u1 = ured[1][0];
      ctrl->total_pairs = (uint32_t)ured[2][0];
      ctrl->candidates_lo = (uint32_t)ured[3][0];
      ctrl->candidates_hi = (uint32_t)(ured[3][0] >> 32);
      ctrl->sum_pairs += ctrl->total_pairs;
      ctrl->sum_u2 += ured[0][0];
      ctrl->sum_u1 += ured[1][0];
      ctrl->sum_candidates += ((unsigned long long)ctrl->candidates_hi << 32) | ctrl->candidates_lo;
      ctrl->sum_steps += 1;
    }
    __syncthreads();
  }
  if (!b1) return;
  const int col = tid & 31, part = tid >> 5;
  const int u = block * 32 + col;
  float g = 0.f;
  if (act && u < H)
    for (int i = part; i < B; i += 8) g += dh[(size_t)i * H + u];
  if (act) red[tid] = g;
  __syncthreads();
  if (part == 0 && u < H) {
    float s = red[col];
    for (int k = 1; k < 8; ++k) s += red[k * 32 + col];
    float w = b1[u], m = mb1[u], v = vb1[u];
    adam1(w, m, v, s, ad);
    b1[u] = w; mb1[u] = m; vb1[u] = v;
  }
}


template <int LPR, int CH, int UNR>
__global__ __launch_bounds__(kUpdateThreads) void update_kernel(int H, RowUpdate out, RowUpdate in, FinishArgs fin, AdamDev ad) {
  int blk = blockIdx.x;
  if (blk < fin.nblocks) { finish_role(H, fin, ad, blk); return; }
  blk -= fin.nblocks;
  // every other workgroup takes its share of both row lists (their sizes are known on the device only)
  if (H == LPR * CH * 4) {                               // the lane groups cover the vector exactly
    if (in.nblocks) rowgrad_adam<LPR, CH, UNR, true>(H, in, ad, blk, out.nblocks);
    rowgrad_adam<LPR, CH, UNR, true>(H, out, ad, blk, out.nblocks);
  } else {
    if (in.nblocks) rowgrad_adam<LPR, CH, UNR, false>(H, in, ad, blk, out.nblocks);
    rowgrad_adam<LPR, CH, UNR, false>(H, out, ad, blk, out.nblocks);
  }
}

template <int LPR, int CH, int UNR>
static hipError_t launch_up(int H, const RowUpdate& out, const RowUpdate& in, const FinishArgs& fin,
                            const AdamDev& ad, hipStream_t s) {
  hipLaunchKernelGGL((update_kernel<LPR, CH, UNR>), dim3(fin.nblocks + out.nblocks), dim3(kUpdateThreads), 0, s, H,
                     out, in, fin, ad);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// The same update for batches whose samples share most rows (saturated buckets: a touched row is
// listed by many samples, and the list lengths have a heavy tail).  Then a pair -- one (row, sample)
// incidence -- costs one read of the sample's vector, and reading it from the cache hierarchy is
// what bounds the plain kernel; and lane groups that each walk their own list spend most steps waiting
// for the longest of them.  Here a workgroup first copies a slice of CW columns of all B sample vectors
// into LDS (B*CW floats) and then walks the row lists for that slice only, a WAVE per row: lane l owns
// columns l*CPL .. of the slice, the list entries and coefficients are fetched 64 at a time (a lane
// each) and handed round as wave-uniform values, so a pair costs one LDS read and no step is shared
// with another row.  The slices of a row are independent (gradient, moments and weights are per
// column), so H/CW workgroups update a row together, each its own columns; the one with the first
// columns also takes the bias.  Sums run over ascending samples as in the plain kernel.
// ---------------------------------------------------------------------------------------------
constexpr int kSlicedThreads = 1024;
constexpr int kSlicedGroup = 1;          // rows a wave takes through each memory round trip
constexpr int kSlicedPad = 4;            // floats between the LDS rows of two samples (spreads them over the banks)
constexpr size_t kSlicedStatic = 10240;  // LDS the launch's other role (finish_role) declares statically

// Sum of a float over the wave in a fixed order (butterfly), returned in every lane.
__device__ __forceinline__ float wave_sum_f32(float v) {
  v += dpp_f32<kDppQuadSwap1>(v);
  v += dpp_f32<kDppQuadSwap2>(v);
  v += dpp_f32<kDppRowHalfMirror>(v);
  v += dpp_f32<kDppRowMirror>(v);
  v += __shfl_xor(v, 16);
  v += __shfl_xor(v, 32);
  return v;
}

template <int CPL> struct LaneCols { typedef float type; };
template <> struct LaneCols<2> { typedef float2 type; };

typedef float slide_v2f __attribute__((ext_vector_type(2)));
template <int CPL>
__device__ __forceinline__ typename LaneCols<CPL>::type load_cols_stream(const float* p) {
  if constexpr (CPL == 2) { const slide_v2f v = __builtin_nontemporal_load((const slide_v2f*)p); return make_float2(v.x, v.y); }
  else return __builtin_nontemporal_load(p);
}
template <int CPL>
__device__ __forceinline__ void store_cols_stream(float* p, const typename LaneCols<CPL>::type& x) {
  if constexpr (CPL == 2) { slide_v2f v; v.x = x.x; v.y = x.y; __builtin_nontemporal_store(v, (slide_v2f*)p); }
  else __builtin_nontemporal_store(x, p);
}

template <int CPL>
__device__ __forceinline__ void fma_cols(typename LaneCols<CPL>::type& g, float d, const typename LaneCols<CPL>::type& x) {
  if constexpr (CPL == 2) { g.x += d * x.x; g.y += d * x.y; } else { g += d * x; }
}

// The rows of one matrix, columns [c0, c0 + 64*CPL): share `part` of `nparts` of the rows.
// The workgroup fills its compute unit alone (the LDS slice), so nothing but the wave itself can hide
// the chain header -> list entries -> coefficients: the headers are fetched three rows ahead, the
// first 64 list entries two ahead, their coefficients one ahead.
template <int CPL, int R, bool LDSV>
__device__ void rowgrad_adam_sliced(int H, int c0, const RowUpdate& ru, const AdamDev& ad, const float* ldsV,
                                    const uint32_t* tpre, uint32_t* cursor, int part, int nparts) {
  typedef typename LaneCols<CPL>::type cols_t;
  constexpr int PITCH = 64 * CPL + kSlicedPad;
  const PairsDev& pd = ru.pd;
  const float* __restrict__ coef = ru.coef;
  const int lane = threadIdx.x & 63;
  constexpr int WPB = kSlicedThreads / 64;
  const int wave_global = __builtin_amdgcn_readfirstlane(part * WPB + (threadIdx.x >> 6)), nwaves = nparts * WPB;
  const int col = c0 + lane * CPL;
  const bool col_ok = col < H;                             // (H is a multiple of 4, so a lane's columns go together)
  const bool bias_lane_any = c0 == 0 && ru.bias != nullptr;   // (uniform) this workgroup also updates the biases
  const bool bias_lane = bias_lane_any && lane == 0;
  const float* lds_mine = ldsV + lane * CPL;
  // The touched rows sit in per-tile slot ranges (tile t: slots t*rows_per_tile .. + tile_nu[t]).  With
  // the running sum of tile_nu in LDS (tpre, when the tiles are few enough) the workgroup owns a
  // contiguous stretch of the touched rows and its waves draw rows from it one at a time through an LDS
  // counter (the lists' lengths have a heavy tail: a fixed share per wave leaves most waves waiting for
  // the few with the long lists); a row's slot is found by stepping through the sums.  Otherwise a wave
  // visits the slots r * ntiles + t (the tiles' r-th rows side by side) and skips the empty ones.
  const bool dense = tpre != nullptr;
  int count = 0x7fffffff, tc = 0;
  uint32_t hi = 0;
  if (dense) {
    const uint32_t U = tpre[pd.ntiles];
    const uint32_t lo = (uint32_t)((uint64_t)U * (uint32_t)part / (uint32_t)nparts);
    hi = (uint32_t)((uint64_t)U * (uint32_t)(part + 1) / (uint32_t)nparts);
    int a = 0, b = pd.ntiles;                              // last tile whose sum is <= lo
    while (b - a > 1) { const int mid = (a + b) >> 1; if (tpre[mid] <= lo) a = mid; else b = mid; }
    tc = a;
  } else {
    const int nrows = pd.ntiles * (int)*pd.max_nu;
    count = wave_global < nrows ? (nrows - wave_global + nwaves - 1) / nwaves : 0;
  }
  // header of the k-th row of this wave: (row, first list entry, entries, -); entries = 0: an empty slot,
  // entries < 0: no more rows.  (Called once per k, ascending, so the tile cursor only moves forward.)
  auto header = [&](int k) -> int4 {
    if (k >= count) return make_int4(0, 0, -1, 0);
    int slot;
    if (dense) {
      uint32_t g = 0;
      if (lane == 0) g = atomicAdd(cursor, 1u);
      g = (uint32_t)__builtin_amdgcn_readfirstlane((int)g);
      if (g >= hi) { count = k; return make_int4(0, 0, -1, 0); }   // (the counter only grows: later draws fail too)
      while (g >= tpre[tc + 1]) ++tc;
      slot = tc * pd.rows_per_tile + (int)(g - tpre[tc]);
    } else {
      const int idx = wave_global + k * nwaves;
      const int r = idx / pd.ntiles, t = idx - r * pd.ntiles;
      if (r >= pd.tile_nu[t]) return make_int4(0, 0, 0, 0);
      slot = t * pd.rows_per_tile + r;
    }
    return pd.umeta[slot];                                 // (not looked at before its turn comes: see below)
  };
  auto entry = [&](const int4& m, int q0) -> int2 {        // this lane's entry of the batch that starts at q0
    const int q = q0 + lane;
    return pd.pairs[(uint32_t)m.y + (q < m.z ? q : 0)];
  };
  auto coefficient = [&](const int4& m, int q0, int2& e) -> float {   // its coefficient; lanes past the end: sample 0, 0
    const bool ok = q0 + lane < m.z;
    const float dv = coef[ok ? e.y : 0];
    if (!ok) e.x = 0;
    return ok ? dv : 0.f;
  };
  // Software pipeline over the wave's rows, R rows at a time.  Vector loads and stores share one in-order
  // counter on this target, and once both kinds are outstanding a wait for any load waits for
  // everything, so the loop has one point per group of R rows where it waits (its top), and everything
  // outstanding there was issued a whole group of LDS arithmetic earlier: group g's headers were requested
  // during group g-3, its first 64 list entries during g-2, their coefficients and the rows' old w, m, v
  // during g-1; group g's results are stored during g+1.  (With short lists a row's arithmetic is far
  // shorter than a memory round trip: R rows share each round trip.)
  auto scalar = [](const int4& m) {
    return make_int4(__builtin_amdgcn_readfirstlane(m.x), __builtin_amdgcn_readfirstlane(m.y),
                     __builtin_amdgcn_readfirstlane(m.z), 0);
  };
  auto row_offset = [&](const int4& m) -> size_t { return (size_t)m.x * H + col; };
  int4 m0[R], m1[R], m2[R];
  int2 e0[R], e1[R];
  float d0[R];
  cols_t w0[R], mo0[R], v0[R];                             // old values of the group's rows (requested a group earlier)
  float b0w[R], b0m[R], b0v[R];
  cols_t ws[R], ms[R], vs[R];                              // results of the previous group, not stored yet
  float bsw[R], bsm[R], bsv[R];
  size_t ro_s[R];
  int j_s[R];                                              // row they belong to (-1: nothing pending)
#pragma unroll
  for (int r = 0; r < R; ++r) m0[r] = header(r);
#pragma unroll
  for (int r = 0; r < R; ++r) m1[r] = header(R + r);
#pragma unroll
  for (int r = 0; r < R; ++r) m2[r] = header(2 * R + r);
#pragma unroll
  for (int r = 0; r < R; ++r) { e0[r] = entry(m0[r], 0); e1[r] = entry(m1[r], 0); }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    d0[r] = coefficient(m0[r], 0, e0[r]);
    b0w[r] = 0.f; b0m[r] = 0.f; b0v[r] = 0.f; bsw[r] = 0.f; bsm[r] = 0.f; bsv[r] = 0.f;
    ro_s[r] = 0; j_s[r] = -1;
    if (col_ok && m0[r].z > 0) { const size_t ro = row_offset(m0[r]); w0[r] = *(const cols_t*)(ru.W + ro); mo0[r] = load_cols_stream<CPL>(ru.M + ro); v0[r] = load_cols_stream<CPL>(ru.Vv + ro); }
    if (bias_lane && m0[r].z > 0) { b0w[r] = ru.bias[m0[r].x]; b0m[r] = ru.mbias[m0[r].x]; b0v[r] = ru.vbias[m0[r].x]; }
  }
  for (int g = 0;; ++g) {
    int4 cur[R];
#pragma unroll
    for (int r = 0; r < R; ++r) cur[r] = scalar(m0[r]);    // ---- the one waiting point of this group
    if (cur[0].z < 0) break;                               // (no more rows: they are handed out in order; uniform)
    int2 ecur[R];
    float dcur[R], bcw[R], bcm[R], bcv[R];
    cols_t wc[R], mc[R], vc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) { ecur[r] = e0[r]; dcur[r] = d0[r]; wc[r] = w0[r]; mc[r] = mo0[r]; vc[r] = v0[r]; bcw[r] = b0w[r]; bcm[r] = b0m[r]; bcv[r] = b0v[r]; }
    // ---- requests for the groups to come, and the previous group's stores
    int4 m3[R];
    int2 e2[R];
    float d1[R];
#pragma unroll
    for (int r = 0; r < R; ++r) m3[r] = header((g + 3) * R + r);
#pragma unroll
    for (int r = 0; r < R; ++r) e2[r] = entry(m2[r], 0);
#pragma unroll
    for (int r = 0; r < R; ++r) {
      d1[r] = coefficient(m1[r], 0, e1[r]);
      if (col_ok && m1[r].z > 0) { const size_t ro = row_offset(m1[r]); w0[r] = *(const cols_t*)(ru.W + ro); mo0[r] = load_cols_stream<CPL>(ru.M + ro); v0[r] = load_cols_stream<CPL>(ru.Vv + ro); }
      if (bias_lane && m1[r].z > 0) { b0w[r] = ru.bias[m1[r].x]; b0m[r] = ru.mbias[m1[r].x]; b0v[r] = ru.vbias[m1[r].x]; }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
      if (j_s[r] >= 0) {
        if (col_ok) { *(cols_t*)(ru.W + ro_s[r]) = ws[r]; store_cols_stream<CPL>(ru.M + ro_s[r], ms[r]); store_cols_stream<CPL>(ru.Vv + ro_s[r], vs[r]); }
        if (bias_lane) { ru.bias[j_s[r]] = bsw[r]; ru.mbias[j_s[r]] = bsm[r]; ru.vbias[j_s[r]] = bsv[r]; }
        j_s[r] = -1;
      }
    // ---- the group's rows: gradient from LDS, Adam in registers
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int cn = cur[r].z;
      if (cn <= 0) continue;
      cols_t gsum;
      if constexpr (CPL == 2) gsum = make_float2(0.f, 0.f); else gsum = 0.f;
      float gb = 0.f;
      int2 e = ecur[r];
      float d = dcur[r];
      for (int q0 = 0; q0 < cn; q0 += 64) {
        int2 en = e;
        const bool more = q0 + 64 < cn;                    // (uniform; rows this long wait in place)
        if (more) en = entry(cur[r], q0 + 64);
        const int n = min(64, cn - q0);
        for (int a0 = 0; a0 < n; a0 += 8) {                // lanes past the end hold (sample 0, 0.0)
          cols_t x[8];
          float dd[8];
#pragma unroll
          for (int a = 0; a < 8; ++a) {
            const int si = __builtin_amdgcn_readlane(e.x, a0 + a);
            dd[a] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(d), a0 + a));
            if constexpr (LDSV) x[a] = *(const cols_t*)(lds_mine + (size_t)si * PITCH);
            else if (col_ok) x[a] = *(const cols_t*)(ru.V + (size_t)si * H + col);     // (few pairs: from the caches)
            else { if constexpr (CPL == 2) x[a] = make_float2(0.f, 0.f); else x[a] = 0.f; }
          }
#pragma unroll
          for (int a = 0; a < 8; ++a) fma_cols<CPL>(gsum, dd[a], x[a]);
        }
        if (bias_lane_any) gb += wave_sum_f32(d);          // (lanes past the end hold 0; fixed order)
        if (more) { e = en; d = coefficient(cur[r], q0 + 64, e); }
      }
      ws[r] = wc[r]; ms[r] = mc[r]; vs[r] = vc[r];
      if constexpr (CPL == 2) { adam1(ws[r].x, ms[r].x, vs[r].x, gsum.x, ad); adam1(ws[r].y, ms[r].y, vs[r].y, gsum.y, ad); }
      else adam1(ws[r], ms[r], vs[r], gsum, ad);
      bsw[r] = bcw[r]; bsm[r] = bcm[r]; bsv[r] = bcv[r];
      adam1(bsw[r], bsm[r], bsv[r], gb, ad);
      ro_s[r] = (size_t)cur[r].x * H + col;
      j_s[r] = cur[r].x;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) { m0[r] = m1[r]; m1[r] = m2[r]; m2[r] = m3[r]; e0[r] = e1[r]; e1[r] = e2[r]; d0[r] = d1[r]; }
  }
#pragma unroll
  for (int r = 0; r < R; ++r)
    if (j_s[r] >= 0) {
      if (col_ok) { *(cols_t*)(ru.W + ro_s[r]) = ws[r]; store_cols_stream<CPL>(ru.M + ro_s[r], ms[r]); store_cols_stream<CPL>(ru.Vv + ro_s[r], vs[r]); }
      if (bias_lane) { ru.bias[j_s[r]] = bsw[r]; ru.mbias[j_s[r]] = bsm[r]; ru.vbias[j_s[r]] = bsv[r]; }
    }
}

template <int CPL>
__global__ __launch_bounds__(kSlicedThreads) void update_sliced_kernel(int H, int B, RowUpdate out, RowUpdate in,
                                                                       FinishArgs fin, AdamDev ad, int nslices,
                                                                       int parts, int tile_words) {
  extern __shared__ float ldsV[];                          // [B][64*CPL + kSlicedPad], then [tile_words] tile sums
  constexpr int CW = 64 * CPL, PITCH = CW + kSlicedPad;
  uint32_t* tsum = (uint32_t*)(ldsV + (size_t)B * PITCH);
  __shared__ uint32_t wsum[kSlicedThreads / 64];
  __shared__ uint32_t row_cursor[2];                       // next touched row of this workgroup's stretch (input / output layer)
  int blk = blockIdx.x;
  if (blk < fin.nblocks) { finish_role(H, fin, ad, blk); return; }
  blk -= fin.nblocks;
  // neighbours in launch order take the slices of the same share of the rows: they read the same
  // lists and coefficients at about the same time
  const int slice = blk % nslices, part = blk / nslices;
  const int c0 = slice * CW;
  // The batch's vectors for the output layer's rows (the slice): the input layer's rows are few, their
  // vectors (the hidden gradient) are read from the caches, and the waves go from the one list to the
  // other without meeting.
  for (int idx = threadIdx.x; idx < B * (CW / 4); idx += kSlicedThreads) {
    const int i = idx / (CW / 4), q = idx - i * (CW / 4);
    const int col = c0 + q * 4;
    const float4 x = col < H ? *(const float4*)(out.V + (size_t)i * H + col) : make_float4(0.f, 0.f, 0.f, 0.f);
    *(float4*)(ldsV + (size_t)i * PITCH + q * 4) = x;
  }
  // running sum of the touched rows per tile (sums[t] = rows in tiles before t), when it fits
  auto tile_sums = [&](const RowUpdate& ru, uint32_t* sums, uint32_t* cursor) {
    const int nt = ru.pd.ntiles;
    uint32_t carry = 0;
    for (int base = 0; base < nt; base += kSlicedThreads) {   // (uniform trip count)
      const int t = base + (int)threadIdx.x;
      const uint32_t v = t < nt ? (uint32_t)ru.pd.tile_nu[t] : 0u;
      const uint32_t inc = wave_incl_scan_add(v);
      __syncthreads();
      if ((threadIdx.x & 63) == 63) wsum[threadIdx.x >> 6] = inc;
      __syncthreads();
      uint32_t before = 0, total = 0;
      for (int w = 0; w < kSlicedThreads / 64; ++w) { const uint32_t x = wsum[w]; if (w < (int)(threadIdx.x >> 6)) before += x; total += x; }
      if (t < nt) sums[t] = carry + before + inc - v;
      carry += total;
    }
    if (threadIdx.x == 0) {
      sums[nt] = carry;
      *cursor = (uint32_t)((uint64_t)carry * (uint32_t)part / (uint32_t)parts);
    }
  };
  const bool dense_in = in.W && in.pd.ntiles + 1 <= tile_words;
  uint32_t* tsum_out = tsum + (dense_in ? in.pd.ntiles + 1 : 0);
  const bool dense_out = out.pd.ntiles + 1 <= tile_words - (int)(tsum_out - tsum);
  if (dense_in) tile_sums(in, tsum, &row_cursor[0]);
  if (dense_out) tile_sums(out, tsum_out, &row_cursor[1]);
  __syncthreads();
  if (in.W) rowgrad_adam_sliced<CPL, kSlicedGroup, false>(H, c0, in, ad, ldsV, dense_in ? tsum : nullptr, &row_cursor[0], part, parts);
  rowgrad_adam_sliced<CPL, kSlicedGroup, true>(H, c0, out, ad, ldsV, dense_out ? tsum_out : nullptr, &row_cursor[1], part, parts);
}

// Columns per slice for a batch of B vectors of length H (0: the sliced kernel does not apply).
static int sliced_width(int B, int H, size_t lds_limit) {
  for (int cw = 128; cw >= 64; cw >>= 1) {
    if (cw > 64 && cw / 2 >= H) continue;                  // a narrower slice still covers the vector
    if ((size_t)B * (cw + kSlicedPad) * 4 + kSlicedStatic <= lds_limit) return cw;
  }
  return 0;
}

bool update_sliced_applies(int B, int H, size_t lds_limit) { return sliced_width(B, H, lds_limit) != 0; }

hipError_t update_setup_attributes(size_t lds_limit) {
  if (lds_limit <= kSlicedStatic) return hipErrorInvalidValue;
  const int dyn = (int)(lds_limit - kSlicedStatic);
  hipError_t e = hipFuncSetAttribute((const void*)update_sliced_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
  if (e == hipSuccess) e = hipFuncSetAttribute((const void*)update_sliced_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, dyn);
  return e;
}

hipError_t launch_update_sliced(int H, int B, const RowUpdate& out_, const RowUpdate& in_, const FinishArgs& fin_,
                                const AdamDev& ad, size_t lds_limit, int num_cus, hipStream_t s) {
  RowUpdate out = out_, in = in_;
  FinishArgs fin = fin_;
  fin.nblocks = fin.b1 ? ceil_div(H, 32) : 1;
  const int cw = sliced_width(B, H, lds_limit);
  if (!cw) return hipErrorInvalidValue;
  const int nslices = ceil_div(H, cw);
  // one workgroup per compute unit, the short-lived ones of the other role included
  const int parts = (num_cus - fin.nblocks) / nslices > 0 ? (num_cus - fin.nblocks) / nslices : 1;
  // what the slice leaves of the LDS holds the running sums of touched rows per tile (if the tiles fit)
  const size_t slice_bytes = (size_t)B * (cw + kSlicedPad) * 4;
  const int tile_words = (int)std::min<size_t>((lds_limit - kSlicedStatic - slice_bytes) / 4, 8192);
  const size_t lds = slice_bytes + (size_t)tile_words * 4;
  const dim3 grid(fin.nblocks + nslices * parts), block(kSlicedThreads);
  if (cw == 128) hipLaunchKernelGGL((update_sliced_kernel<2>), grid, block, lds, s, H, B, out, in, fin, ad, nslices, parts, tile_words);
  else hipLaunchKernelGGL((update_sliced_kernel<1>), grid, block, lds, s, H, B, out, in, fin, ad, nslices, parts, tile_words);
  return hipGetLastError();
}

hipError_t launch_update(int H, const RowUpdate& out_, const RowUpdate& in_, const FinishArgs& fin_,
                         const AdamDev& ad, int num_cus, hipStream_t s) {
  RowUpdate out = out_, in = in_;
  FinishArgs fin = fin_;
  out.nblocks = 8 * num_cus;          // twice what the device holds at four waves per SIMD: the tail stays short
  in.nblocks = in.W ? 1 : 0;          // present / absent
  fin.nblocks = fin.b1 ? ceil_div(H, 32) : 1;
#define SLIDE_UP(L_, C_, U_) return launch_up<L_, C_, U_>(H, out, in, fin, ad, s)
  if (H <= 32) SLIDE_UP(8, 1, 4);
  if (H <= 64) SLIDE_UP(8, 2, 4);
  if (H <= 128) SLIDE_UP(8, 4, 2);
  if (H <= 256) SLIDE_UP(16, 4, 2);
  if (H <= 512) SLIDE_UP(32, 4, 2);
  if (H <= 1024) SLIDE_UP(64, 4, 2);
  SLIDE_UP(64, 8, 2);
#undef SLIDE_UP
}

}  // namespace slide
