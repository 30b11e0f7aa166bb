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

template <int LPR, int CH>
__global__ __launch_bounds__(256) void rowgrad_adam_kernel(int H, PairsDev pd, const float* __restrict__ coef,
                                                           const float* __restrict__ V, float* __restrict__ W,
                                                           float* __restrict__ M, float* __restrict__ Vv,
                                                           float* __restrict__ bias, float* __restrict__ mbias,
                                                           float* __restrict__ vbias, AdamDev ad) {
  constexpr int RPW = 64 / LPR;
  constexpr int UNR = CH <= 4 ? 4 : 2;
  const int lane = threadIdx.x & 63, sub = lane % LPR, grp = lane / LPR;
  const uint32_t U = *pd.ucount;
  const uint32_t step = gridDim.x * 4 * RPW;
  for (uint32_t base = (blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW; base < U; base += step) {
    const uint32_t r = base + grp;
    const bool valid = r < U;
    const size_t ro = valid ? (size_t)pd.urow[r] * H : 0;
    const uint32_t st = valid ? pd.ustart[r] : 0u;
    const int cn = valid ? pd.ucnt[r] : 0;
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
    for (int q = 0; __any(q < cn); q += UNR) {
      float d[UNR];
      float4 hv[UNR][CH];
#pragma unroll
      for (int a = 0; a < UNR; ++a) {
        const bool ok = q + a < cn;
        const int si = ok ? pd.psample[st + q + a] : 0;
        d[a] = ok ? coef[pd.psrc[st + q + a]] : 0.f;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const int col = (c * LPR + sub) * 4;
          hv[a][c] = (ok && col < H) ? *(const float4*)(V + (size_t)si * H + col) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
#pragma unroll
      for (int a = 0; a < UNR; ++a) {
        if (q + a < cn) {
          gb += d[a];
#pragma unroll
          for (int c = 0; c < CH; ++c) {
            g[c].x += d[a] * hv[a][c].x; g[c].y += d[a] * hv[a][c].y;
            g[c].z += d[a] * hv[a][c].z; g[c].w += d[a] * hv[a][c].w;
          }
        }
      }
    }
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
      const int j = pd.urow[r];
      float bw = bias[j], bm = mbias[j], bv = vbias[j];
      adam1(bw, bm, bv, gb, ad);
      bias[j] = bw; mbias[j] = bm; vbias[j] = bv;
    }
  }
}

template <int LPR, int CH>
static hipError_t launch_rg(int H, const PairsDev& pd, const float* coef, const float* V, float* W, float* M,
                            float* Vv, float* bias, float* mbias, float* vbias, const AdamDev& ad, hipStream_t s) {
  hipLaunchKernelGGL((rowgrad_adam_kernel<LPR, CH>), dim3(2048), dim3(256), 0, s, H, pd, coef, V, W, M, Vv, bias,
                     mbias, vbias, ad);
  return hipGetLastError();
}

hipError_t launch_rowgrad_adam(int H, const PairsDev& pd, const float* coef, const float* V, float* W, float* M,
                               float* Vv, float* bias, float* mbias, float* vbias, const AdamDev& ad,
                               hipStream_t s) {
#define SLIDE_RG(L_, C_) return launch_rg<L_, C_>(H, pd, coef, V, W, M, Vv, bias, mbias, vbias, ad, s)
  if (H <= 32) SLIDE_RG(8, 1);
  if (H <= 64) SLIDE_RG(8, 2);
  if (H <= 128) SLIDE_RG(8, 4);
  if (H <= 256) SLIDE_RG(16, 4);
  if (H <= 512) SLIDE_RG(32, 4);
  if (H <= 1024) SLIDE_RG(64, 4);
  SLIDE_RG(64, 8);
#undef SLIDE_RG
}

// loss = mean_i loss_i (fixed-shape reduction); with b1: gb1[u] = sum_i dh[i][u] in sample order
// and Adam on the dense hidden bias.
__global__ __launch_bounds__(256) void finish_kernel(int B, int H, const float* __restrict__ loss_i,
                                                     float* __restrict__ d_loss, const float* __restrict__ dh,
                                                     float* __restrict__ b1, float* __restrict__ mb1,
                                                     float* __restrict__ vb1, AdamDev ad, Ctrl* ctrl) {
  __shared__ float red[256];
  const int tid = threadIdx.x;
  if (blockIdx.x == 0 && tid == 0) {          // statistics: totals over the steps
    ctrl->sum_pairs += ctrl->total_pairs;
    ctrl->sum_u2 += ctrl->u2;
    ctrl->sum_u1 += ctrl->u1;
    ctrl->sum_candidates += ((unsigned long long)ctrl->candidates_hi << 32) | ctrl->candidates_lo;
    ctrl->sum_steps += 1;
  }
  if (blockIdx.x == 0 && d_loss) {
    float acc = 0.f;
    for (int i = tid; i < B; i += 256) acc += loss_i[i];
    red[tid] = acc;
    __syncthreads();
    for (int d = 128; d > 0; d >>= 1) {
      if (tid < d) red[tid] += red[tid + d];
      __syncthreads();
    }
    if (tid == 0) *d_loss = red[0] / (float)B;
  }
  if (!b1) return;
  const int u = blockIdx.x * 256 + tid;
  if (u >= H) return;
  float g = 0.f;
  for (int i = 0; i < B; ++i) g += dh[(size_t)i * H + u];
  float w = b1[u], m = mb1[u], v = vb1[u];
  adam1(w, m, v, g, ad);
  b1[u] = w; mb1[u] = m; vb1[u] = v;
}

hipError_t launch_finish(int B, int H, const float* loss_i, float* d_loss, const float* dh, float* b1,
                         float* mb1, float* vb1, const AdamDev& ad, Ctrl* ctrl, hipStream_t s) {
  hipLaunchKernelGGL(finish_kernel, dim3(ceil_div(H, 256)), dim3(256), 0, s, B, H, loss_i, d_loss, dh, b1, mb1,
                     vb1, ad, ctrl);
  return hipGetLastError();
}

}  // namespace slide
