// Sparse backpropagation into the parameters fused with row-sparse Adam (paper Algorithm 1:
// gradients reach only the active neurons, then "update weights with Adam"; Section 3.5: every
// weight and bias carries a momentum and a velocity value; constants of Section 4.1).
//
// rowgrad_adam: each touched row is read once (w, m, v), its gradient is formed in registers from
// the row's pair list -- g = sum_i coef_i * V[sample_i][:], samples ascending, so the sum order is
// fixed -- and w, m, v are written back once: 6 row transfers per touched row, no gradient buffer
// and no atomics.  V is the hidden activations (output layer) or their gradient (input layer),
// small enough to stay cache resident.  Rows that are not listed are never touched.
#include "slide_internal.h"

namespace slide {

constexpr int kUpdateThreads = 256;
constexpr int kUpdateBlocksOut = 2048;

__device__ __forceinline__ void adam1(float& w, float& m, float& v, float g, const AdamDev& a) {
  m = a.beta1 * m + a.omb1 * g;
  v = a.beta2 * v + a.omb2 * g * g;
  w = w - a.lr * (m * a.inv_bc1) / (sqrtf(v * a.inv_bc2) + a.eps);
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
        m[c] = *(const float4*)(M + ro + col);
        v[c] = *(const float4*)(Vv + ro + col);
      }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      if (FULL || col < H) {
        adam1(w[c].x, m[c].x, v[c].x, g[c].x, ad); adam1(w[c].y, m[c].y, v[c].y, g[c].y, ad);
        adam1(w[c].z, m[c].z, v[c].z, g[c].z, ad); adam1(w[c].w, m[c].w, v[c].w, g[c].w, ad);
        *(float4*)(W + ro + col) = w[c];
        *(float4*)(M + ro + col) = m[c];
        *(float4*)(Vv + ro + col) = v[c];
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
            m[c] = *(const float4*)(M + ro + col);
            v[c] = *(const float4*)(Vv + ro + col);
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
            *(float4*)(M + ro + col) = m[c];
            *(float4*)(Vv + ro + col) = v[c];
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
        m[c] = *(const float4*)(M + ro + col);
        v[c] = *(const float4*)(Vv + ro + col);
      }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      if (FULL || col < H) {
        adam1(w[c].x, m[c].x, v[c].x, g[c].x, ad); adam1(w[c].y, m[c].y, v[c].y, g[c].y, ad);
        adam1(w[c].z, m[c].z, v[c].z, g[c].z, ad); adam1(w[c].w, m[c].w, v[c].w, g[c].w, ad);
        *(float4*)(W + ro + col) = w[c];
        *(float4*)(M + ro + col) = m[c];
        *(float4*)(Vv + ro + col) = v[c];
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
  if (block == 0) {
    float acc = 0.f;
    for (int i = tid; i < B; i += 256) acc += loss_i[i];
    unsigned long long u2 = 0, u1 = 0, pairs = 0, cand = 0;
    for (int t = tid; t < ntiles2; t += 256) u2 += (unsigned long long)tile_nu2[t];
    for (int t = tid; t < ntiles1; t += 256) u1 += (unsigned long long)tile_nu1[t];
    for (int i = tid; i < B; i += 256) { pairs += (unsigned long long)f.cnt[i]; cand += (unsigned long long)f.ncand[i]; }
    red[tid] = acc; ured[0][tid] = u2; ured[1][tid] = u1; ured[2][tid] = pairs; ured[3][tid] = cand;
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
  if (u < H)
    for (int i = part; i < B; i += 8) g += dh[(size_t)i * H + u];
  red[tid] = g;
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

hipError_t launch_update(int H, const RowUpdate& out_, const RowUpdate& in_, const FinishArgs& fin_,
                         const AdamDev& ad, hipStream_t s) {
  RowUpdate out = out_, in = in_;
  FinishArgs fin = fin_;
  out.nblocks = kUpdateBlocksOut;
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
