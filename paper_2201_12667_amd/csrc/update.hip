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

__device__ __forceinline__ void adam1(float& w, float& m, float& v, float g, const AdamDev& a) {
  m = a.beta1 * m + a.omb1 * g;
  v = a.beta2 * v + a.omb2 * g * g;
  w = w - a.lr * (m * a.inv_bc1) / (sqrtf(v * a.inv_bc2) + a.eps);
}

// Gradient of one row from its pair list, pairs first, first + stride, ... (this lane group's share).
template <int LPR, int CH, int UNR>
__device__ __forceinline__ void row_gradient(int H, int sub, const PairsDev& pd, const float* __restrict__ coef,
                                             const float* __restrict__ V, uint32_t st, int cn, int first,
                                             int stride, float4 (&g)[CH], float& gb) {
  for (int q = first; __any(q < cn); q += UNR * stride) {
    float d[UNR];
    float4 hv[UNR][CH];
#pragma unroll
    for (int a = 0; a < UNR; ++a) {
      const bool ok = q + a * stride < cn;
      const int2 pr = ok ? pd.pairs[st + q + a * stride] : make_int2(0, 0);
      const int si = pr.x;
      d[a] = ok ? coef[pr.y] : 0.f;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int col = (c * LPR + sub) * 4;
        hv[a][c] = (ok && col < H) ? *(const float4*)(V + (size_t)si * H + col) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
#pragma unroll
    for (int a = 0; a < UNR; ++a) {
      if (q + a * stride < cn) {
        gb += d[a];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          g[c].x += d[a] * hv[a][c].x; g[c].y += d[a] * hv[a][c].y;
          g[c].z += d[a] * hv[a][c].z; g[c].w += d[a] * hv[a][c].w;
        }
      }
    }
  }
}

// Work item = RPW consecutive row slots of one tile (RPW = 64/LPR rows per wave, LPR lanes per row,
// CH float4 per lane).  Rows with more than kLongRow pairs are skipped here and taken afterwards by
// a whole wave each: its RPW lane groups accumulate interleaved shares of the pair list and the
// shares are added in a fixed butterfly order.
template <int LPR, int CH, int UNR, bool OUTPUT_LAYER>
__global__ __launch_bounds__(256) void rowgrad_adam_kernel(int H, PairsDev pd, const float* __restrict__ coef,
                                                           const float* __restrict__ V, float* __restrict__ W,
                                                           float* __restrict__ M, float* __restrict__ Vv,
                                                           float* __restrict__ bias, float* __restrict__ mbias,
                                                           float* __restrict__ vbias, AdamDev ad) {
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane % LPR, grp = lane / LPR;
  const int wave_global = blockIdx.x * 4 + (threadIdx.x >> 6), nwaves = gridDim.x * 4;
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
    const bool valid = r < nu && (RPW == 1 || cn <= kLongRow);
    if (!valid) cn = 0;
    const int j = valid ? meta.x : 0;
    const size_t ro = (size_t)j * H;
    const uint32_t st = (uint32_t)meta.y;
    float4 w[CH], m[CH], v[CH], g[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (valid && col < H) {
        w[c] = *(const float4*)(W + ro + col);
        m[c] = *(const float4*)(M + ro + col);
        v[c] = *(const float4*)(Vv + ro + col);
      }
    }
    float gb = 0.f;
    row_gradient<LPR, CH, UNR>(H, sub, pd, coef, V, st, cn, 0, 1, g, gb);
    if (!valid) continue;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      if (col < H) {
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
  if (RPW == 1) return;
  const int nlong = min((int)*pd.nlong, pd.long_cap);
  for (int l = wave_global; l < nlong; l += nwaves) {
    const int slot = pd.longlist[l];
    const int4 meta = pd.umeta[slot];
    const int j = meta.x, cn = meta.z;
    const size_t ro = (size_t)j * H;
    const uint32_t st = (uint32_t)meta.y;
    float4 w[CH], m[CH], v[CH], g[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      g[c] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (grp == 0 && col < H) {
        w[c] = *(const float4*)(W + ro + col);
        m[c] = *(const float4*)(M + ro + col);
        v[c] = *(const float4*)(Vv + ro + col);
      }
    }
    float gb = 0.f;
    row_gradient<LPR, CH, UNR>(H, sub, pd, coef, V, st, cn, grp, RPW, g, gb);
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
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      if (col < H) {
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

template <int LPR, int CH, int UNR = (CH <= 4 ? 4 : 2)>
static hipError_t launch_rg(int H, const PairsDev& pd, const float* coef, const float* V, float* W, float* M,
                            float* Vv, float* bias, float* mbias, float* vbias, const AdamDev& ad, hipStream_t s) {
  // OUTPUT_LAYER only gives the two uses distinct kernel names in profiles (bias present = output layer)
  if (bias)
    hipLaunchKernelGGL((rowgrad_adam_kernel<LPR, CH, UNR, true>), dim3(2048), dim3(256), 0, s, H, pd, coef, V, W, M,
                       Vv, bias, mbias, vbias, ad);
  else
    hipLaunchKernelGGL((rowgrad_adam_kernel<LPR, CH, UNR, false>), dim3(2048), dim3(256), 0, s, H, pd, coef, V, W, M,
                       Vv, bias, mbias, vbias, ad);
  return hipGetLastError();
}

hipError_t launch_rowgrad_adam(int H, const PairsDev& pd, const float* coef, const float* V, float* W, float* M,
                               float* Vv, float* bias, float* mbias, float* vbias, const AdamDev& ad,
                               hipStream_t s) {
#define SLIDE_RG(L_, C_) return launch_rg<L_, C_>(H, pd, coef, V, W, M, Vv, bias, mbias, vbias, ad, s)
  if (H <= 32) SLIDE_RG(8, 1);
  if (H <= 64) SLIDE_RG(8, 2);
  if (H <= 128) {
    return launch_rg<8, 4, 2>(H, pd, coef, V, W, M, Vv, bias, mbias, vbias, ad, s);
  }
  if (H <= 256) SLIDE_RG(16, 4);
  if (H <= 512) SLIDE_RG(32, 4);
  if (H <= 1024) SLIDE_RG(64, 4);
  SLIDE_RG(64, 8);
#undef SLIDE_RG
}

// Block 0: loss = mean_i loss_i (fixed-shape reduction) and the step statistics.  With b1: every
// block takes 32 columns of gb1[u] = sum_i dh[i][u]; 8 partial sums per column over interleaved
// samples, added in a fixed order, then Adam on the dense hidden bias.
__global__ __launch_bounds__(256) void finish_kernel(int B, int H, const float* __restrict__ loss_i,
                                                     float* __restrict__ d_loss, const float* __restrict__ dh,
                                                     float* __restrict__ b1, float* __restrict__ mb1,
                                                     float* __restrict__ vb1, AdamDev ad, Ctrl* ctrl,
                                                     const int32_t* __restrict__ tile_nu2, int ntiles2,
                                                     const int32_t* __restrict__ tile_nu1, int ntiles1) {
  __shared__ float red[256];
  __shared__ uint32_t ured[2][256];
  const int tid = threadIdx.x;
  if (blockIdx.x == 0) {
    float acc = 0.f;
    for (int i = tid; i < B; i += 256) acc += loss_i[i];
    uint32_t u2 = 0, u1 = 0;
    for (int t = tid; t < ntiles2; t += 256) u2 += (uint32_t)tile_nu2[t];
    for (int t = tid; t < ntiles1; t += 256) u1 += (uint32_t)tile_nu1[t];
    red[tid] = acc; ured[0][tid] = u2; ured[1][tid] = u1;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
      if (tid < d) { red[tid] += red[tid + d]; ured[0][tid] += ured[0][tid + d]; ured[1][tid] += ured[1][tid + d]; }
      __syncthreads();
    }
    if (tid == 0) {
      if (d_loss) *d_loss = red[0] / (float)B;
      ctrl->u2 = ured[0][0]; ctrl->u1 = ured[1][0];
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
  const int u = blockIdx.x * 32 + col;
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

hipError_t launch_finish(int B, int H, const float* loss_i, float* d_loss, const float* dh, float* b1,
                         float* mb1, float* vb1, const AdamDev& ad, Ctrl* ctrl, const int32_t* tile_nu2,
                         int ntiles2, const int32_t* tile_nu1, int ntiles1, hipStream_t s) {
  const int blocks = b1 ? ceil_div(H, 32) : 1;
  hipLaunchKernelGGL(finish_kernel, dim3(blocks), dim3(256), 0, s, B, H, loss_i, d_loss, dh, b1, mb1, vb1, ad,
                     ctrl, tile_nu2, ntiles2, tile_nu1, ntiles1);
  return hipGetLastError();
}

}  // namespace slide
