// Inference over all output neurons: scores z[i][j] = b2[j] + W2[j,:].h_i for every neuron j, and
// the k best per sample.  This is the dense evaluation the paper compares the hashed retrieval
// against (Section 2.1: the tables are meant to return the neurons with the highest activations;
// Section 4: accuracy is measured on full predictions).  Unlike the training path it is a dense
// contraction: a register-tiled fp32 kernel (fp32 so that the scores agree with a double-precision
// evaluation to 1e-4; half-precision matrix instructions would not), run over the neurons in
// chunks whose scores stay in a modest scratch buffer, with a streaming top-k per sample.
#include "slide_internal.h"

namespace slide {

constexpr int kBM = 64;    // samples per workgroup tile
constexpr int kBN = 128;   // neurons per workgroup tile
constexpr int kBK = 16;    // contraction step

// zc[i][j - j0] = b2[j] + sum_k W2[j][k] * h[i][k] for j0 <= j < j0 + nc.  256 threads, each 4
// samples x 8 neurons; both operand tiles go through LDS transposed ([k][row], padded).
__global__ __launch_bounds__(256) void dense_scores_kernel(int B, int64_t N, int H, const float* __restrict__ h,
                                                           const float* __restrict__ W2,
                                                           const float* __restrict__ b2, int64_t j0, int nc,
                                                           float* __restrict__ zc) {
  __shared__ float As[kBK][kBM + 4];
  __shared__ float Bs[kBK][kBN + 4];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int i0 = blockIdx.y * kBM;
  const int64_t n0 = j0 + (int64_t)blockIdx.x * kBN;
  float acc[4][8];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 8; ++b) acc[a][b] = 0.f;
  const int lr = tid >> 2, lc = (tid & 3) * 4;          // loader: row within the tile, first of four k
  for (int k0 = 0; k0 < H; k0 += kBK) {
    const bool kok = k0 + lc < H;                        // H is a multiple of 4
    const float4 av = (kok && i0 + lr < B) ? *(const float4*)(h + (size_t)(i0 + lr) * H + k0 + lc)
                                           : make_float4(0.f, 0.f, 0.f, 0.f);
    As[lc][lr] = av.x; As[lc + 1][lr] = av.y; As[lc + 2][lr] = av.z; As[lc + 3][lr] = av.w;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const int r = lr + 64 * q;
      const float4 bv = (kok && n0 + r < j0 + nc) ? *(const float4*)(W2 + (size_t)(n0 + r) * H + k0 + lc)
                                                  : make_float4(0.f, 0.f, 0.f, 0.f);
      Bs[lc][r] = bv.x; Bs[lc + 1][r] = bv.y; Bs[lc + 2][r] = bv.z; Bs[lc + 3][r] = bv.w;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kBK; ++k) {
      const float4 a = *(const float4*)&As[k][ty * 4];
      const float4 b0 = *(const float4*)&Bs[k][tx * 8], b1 = *(const float4*)&Bs[k][tx * 8 + 4];
      const float av4[4] = {a.x, a.y, a.z, a.w};
      const float bv8[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
#pragma unroll
      for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[p][q] = fmaf(av4[p], bv8[q], acc[p][q]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int i = i0 + ty * 4 + p;
    if (i >= B) continue;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int64_t n = n0 + tx * 8 + q;
      if (n < j0 + nc) zc[(size_t)i * nc + (size_t)(n - j0)] = acc[p][q] + b2[n];
    }
  }
}

// Sort key of (score, id): ascending keys = descending scores, ties to the lower id.
__device__ __forceinline__ uint64_t topk_key(float score, uint32_t id) {
  const uint32_t u = __float_as_uint(score);
  const uint32_t asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);   // orders like the float
  return ((uint64_t)(~asc) << 32) | id;
}
__device__ __forceinline__ float topk_score(uint64_t key) {
  const uint32_t asc = ~(uint32_t)(key >> 32);
  return __uint_as_float((asc & 0x80000000u) ? (asc & 0x7fffffffu) : ~asc);
}

constexpr int kTopkBuf = 2048;     // candidate keys held in LDS by the streaming top-k

__device__ void bitonic_sort_keys(uint64_t* keys, int n) {
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

// One workgroup per sample: folds the scores of one chunk of neurons into the sample's running list
// of the topk best keys (best[i][0..64), ascending; ~0 = empty).  Only scores that beat the current
// topk-th key are collected; when the LDS buffer fills it is sorted and cut back to topk, which
// raises the bar.  The last chunk also decodes the list into the caller's arrays.
__global__ __launch_bounds__(256) void topk_merge_kernel(int nc, int64_t j0, const float* __restrict__ zc, int topk,
                                                         uint64_t* __restrict__ best, int first, int last,
                                                         int32_t* __restrict__ out_ids,
                                                         float* __restrict__ out_scores) {
  __shared__ uint64_t keys[kTopkBuf];
  __shared__ uint32_t cnt;
  const int i = blockIdx.x, tid = threadIdx.x;
  uint64_t* mine = best + (size_t)i * 64;
  for (int q = tid; q < kTopkBuf; q += 256) keys[q] = (q < topk && !first) ? mine[q] : ~0ull;
  if (tid == 0) cnt = (uint32_t)topk;
  __syncthreads();
  uint64_t bar = keys[topk - 1];
  const float* row = zc + (size_t)i * nc;
  for (int base = 0; base < nc; base += 256) {
    const int q = base + tid;
    if (q < nc) {
      const uint64_t key = topk_key(row[q], (uint32_t)(j0 + q));
      if (key < bar) keys[atomicAdd(&cnt, 1u)] = key;   // at most 256 more per round: the buffer has room
    }
    __syncthreads();
    if (cnt > (uint32_t)(kTopkBuf - 256)) {              // (uniform: cnt is read after the barrier)
      __syncthreads();
      bitonic_sort_keys(keys, kTopkBuf);
      for (int p = topk + tid; p < kTopkBuf; p += 256) keys[p] = ~0ull;
      if (tid == 0) cnt = (uint32_t)topk;
      __syncthreads();
      bar = keys[topk - 1];
    }
  }
  __syncthreads();
  bitonic_sort_keys(keys, kTopkBuf);
  for (int q = tid; q < topk; q += 256) {
    const uint64_t key = keys[q];
    mine[q] = key;
    if (last) {
      const bool empty = key == ~0ull;
      out_ids[(size_t)i * topk + q] = empty ? -1 : (int32_t)(uint32_t)key;
      out_scores[(size_t)i * topk + q] = empty ? -INFINITY : topk_score(key);
    }
  }
}

int64_t dense_chunk_neurons(int64_t N, int Bmax) {
  int64_t nc = ((int64_t)64 << 20) / ((int64_t)Bmax * 4);     // about 64 MiB of scores
  nc = nc / kBN * kBN;
  if (nc < kBN) nc = kBN;
  const int64_t npad = (N + kBN - 1) / kBN * kBN;
  return nc < npad ? nc : npad;
}

hipError_t launch_dense_topk(int B, int64_t N, int H, const float* h, const float* W2, const float* b2, int topk,
                             float* zc, int64_t chunk, uint64_t* best, int32_t* out_ids, float* out_scores,
                             hipStream_t s) {
  for (int64_t j0 = 0; j0 < N; j0 += chunk) {
    const int nc = (int)(N - j0 < chunk ? N - j0 : chunk);
    hipLaunchKernelGGL(dense_scores_kernel, dim3((unsigned)ceil_div(nc, kBN), (unsigned)ceil_div(B, kBM)), dim3(256), 0,
                       s, B, N, H, h, W2, b2, j0, nc, zc);
    hipLaunchKernelGGL(topk_merge_kernel, dim3(B), dim3(256), 0, s, nc, j0, zc, topk, best, j0 == 0 ? 1 : 0,
                       j0 + chunk >= N ? 1 : 0, out_ids, out_scores);
  }
  return hipGetLastError();
}

}  // namespace slide
