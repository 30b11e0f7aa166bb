// Inference over all output neurons: scores z[i][j] = b2[j] + W2[j,:].h_i for every neuron j, and
// the k best per sample.  This is the dense evaluation the paper compares the hashed retrieval
// against (Section 2.1: the tables are meant to return the neurons with the highest activations;
// Section 4: accuracy is measured on full predictions).  Unlike the training path it is a dense
// contraction: an fp32 matrix-core kernel (fp32 so that the scores agree with a double-precision
// evaluation to 1e-4; half-precision matrix instructions would not), run over the neurons in
// chunks, with a running list of the k best per sample.  From the second chunk on the scoring
// kernel itself compares every score with the sample's current k-th best and hands only the ones
// that beat it to the merge (a few per sample and chunk once the list has settled); the scores
// also go to a scratch buffer, which the merge reads only for the first chunk or when a sample's
// candidate buffer overflowed.
#include "slide_internal.h"

namespace slide {

constexpr int kBN = 128;   // neurons per workgroup tile of the scoring kernel (chunks are multiples of it)
constexpr int kTopkBuf = 2048;     // keys held in LDS by the top-k merge
constexpr int kCand = kTopkBuf - 64; // candidate keys per sample and chunk handed over by the scoring kernel

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


typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kNB = 128;       // neurons per workgroup tile: 32 per wave
constexpr int kKB = 32;        // contraction block: 16 matrix instructions of depth 2
constexpr int kHP = kKB + 4;   // LDS pitch of a staged row of h (16-byte reads without bank conflicts)
constexpr int kLocalCand = 2048; // candidates a workgroup gathers in LDS before handing them over
constexpr int kCntPitch = 16;  // words between the candidate counters of two samples (one line each)

// zc[i][j - j0] = b2[j] + sum_k h[i][k] * W2[j][k] for j0 <= j < j0 + nc, on the fp32 matrix cores
// (32x32x2: one value of each operand per lane and step, 16 accumulators per lane and 32x32 block).
// Rows of the product are samples, columns neurons.  A wave owns 32 neurons and all (up to 256) samples
// of the tile: its W2 values come straight from memory (lane l: row l%32, the 16 consecutive k of
// half l/32, so the two lanes of a row read one 128-byte line per block), the h values from an LDS
// tile staged per block of 32 k (double-buffered, one barrier per block).  Step c of a block
// contracts k = c and k = 16 + c: any pairing works as long as both operands use it.
// Epilogue: bias, the score to zc, and -- from the second chunk on -- every score that beats the
// sample's current topk-th key goes to the sample's candidate buffer.
// NIB: row blocks of 32 samples per tile (1, 2, 4 or 8; rows past the batch are zeros).
template <int NIB>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 4))) void dense_scores_kernel(int B, int64_t N, int H, const float* __restrict__ h,
                                                           const float* __restrict__ W2,
                                                           const float* __restrict__ b2, int64_t j0, int nc,
                                                           float* __restrict__ zc, int topk,
                                                           const uint64_t* __restrict__ best,
                                                           uint64_t* __restrict__ cand, uint32_t* ccnt) {
  constexpr int MB = NIB * 32;                                   // samples per tile
  __shared__ __attribute__((aligned(16))) float hs[2][(MB * kHP * 4 < kLocalCand * 12 ? kLocalCand * 3 : MB * kHP)];
  __shared__ uint64_t bars[MB];
  __shared__ __attribute__((aligned(16))) float thr[MB];                                      // score of the bar: a cheap first test
  __shared__ uint32_t lcnt;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 31, half = lane >> 5;
  const int i0 = blockIdx.y * MB;
  const int rows = min(B - i0, MB);
  const int64_t n0 = j0 + (int64_t)blockIdx.x * kNB + wave * 32;
  const int64_t nend = j0 + nc;
  const int64_t jrow = min(n0 + col, N - 1);                     // clamped: columns past the end are not stored
  const float* wrow = W2 + (size_t)jrow * H + 16 * half;
  if (tid < MB) {
    const uint64_t bar = (best && tid < rows) ? best[(size_t)(i0 + tid) * 64 + topk - 1] : 0ull;
    bars[tid] = bar;
    thr[tid] = bar == ~0ull ? -INFINITY : topk_score(bar);       // (list not full yet: everything is a candidate)
  }

  f32x16 acc[NIB];
#pragma unroll
  for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[ib][r] = 0.f;

  // staging of h: 256 threads x NIB float4 cover MB rows x 32 k
  const int srow = tid >> 3, sk = (tid & 7) * 4;
  float4 hreg[NIB], wreg[4];
  auto load_block = [&](int k0) {
#pragma unroll
    for (int q = 0; q < NIB; ++q) {
      const int r = srow + 32 * q;
      hreg[q] = (r < rows && k0 + sk < H) ? *(const float4*)(h + (size_t)(i0 + r) * H + k0 + sk)
                                           : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int wq = 0; wq < 4; ++wq)
      wreg[wq] = (k0 + 16 * half + 4 * wq < H) ? *(const float4*)(wrow + k0 + 4 * wq) : make_float4(0.f, 0.f, 0.f, 0.f);
  };
  auto store_block = [&](int buf) {
#pragma unroll
    for (int q = 0; q < NIB; ++q) *(float4*)&hs[buf][(srow + 32 * q) * kHP + sk] = hreg[q];
  };

  load_block(0);
  store_block(0);
  __syncthreads();
  const int nkb = (H + kKB - 1) / kKB;
  for (int kb = 0; kb < nkb; ++kb) {
    const int cur = kb & 1;
    float4 w[4] = {wreg[0], wreg[1], wreg[2], wreg[3]};
    if (kb + 1 < nkb) load_block((kb + 1) * kKB);                // in flight while this block is contracted
    const float* hb = &hs[cur][col * kHP + 16 * half];
#pragma unroll
    for (int wq = 0; wq < 4; ++wq) {
      float4 a[NIB];
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) a[ib] = *(const float4*)(hb + ib * 32 * kHP + 4 * wq);
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) acc[ib] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ib].x, w[wq].x, acc[ib], 0, 0, 0);
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) acc[ib] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ib].y, w[wq].y, acc[ib], 0, 0, 0);
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) acc[ib] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ib].z, w[wq].z, acc[ib], 0, 0, 0);
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) acc[ib] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[ib].w, w[wq].w, acc[ib], 0, 0, 0);
    }
    if (kb + 1 < nkb) store_block(cur ^ 1);                      // the other buffer was last read before the previous barrier
    __syncthreads();
  }

  // lane holds column `col`, rows 8*(r/4) + 4*half + r%4 of each 32x32 block.  Two passes, so that the
  // 128 score stores of a lane are issued back to back with no memory operation of another kind between
  // them: first the scores that beat their sample's bar are gathered in LDS (over the h tiles, which are
  // no longer read), then everything is stored.  The gathered candidates are handed to the samples'
  // global buffers afterwards, one entry per thread, so that the round trips of the counter updates overlap.
  uint64_t* lkey = (uint64_t*)&hs[0][0];
  uint32_t* lsmp = (uint32_t*)(lkey + kLocalCand);
  if (tid == 0) lcnt = 0;
  __syncthreads();
  const int64_t n = n0 + col;
  const bool live = n < nend;
  const float bias = live ? b2[n] : 0.f;
  if (best != nullptr) {
    {
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int il0 = ib * 32 + 8 * g + 4 * half;            // four consecutive samples
          const float4 t4 = *(const float4*)&thr[il0];
          const float t[4] = {t4.x, t4.y, t4.z, t4.w};
          float z[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) z[e] = acc[ib][4 * g + e] + bias;
          if (live && (!(z[0] < t[0]) | !(z[1] < t[1]) | !(z[2] < t[2]) | !(z[3] < t[3]))) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (!(z[e] < t[e]) && il0 + e < rows) {              // rare: now the exact test, ties by id
                const uint64_t key = topk_key(z[e], (uint32_t)n);
                if (key < bars[il0 + e]) {
                  const uint32_t pos = atomicAdd(&lcnt, 1u);
                  if (pos < (uint32_t)kLocalCand) { lkey[pos] = key; lsmp[pos] = (uint32_t)(il0 + e); }
                }
              }
          }
        }
      }
    }
  }
  if (live) {
    const bool whole = rows == MB;
    float* zcol = zc + (size_t)(i0 + 4 * half) * nc + (size_t)(n - j0);
    if (whole) {
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
        for (int r = 0; r < 16; ++r) zcol[(size_t)(ib * 32 + 8 * (r >> 2) + (r & 3)) * nc] = acc[ib][r] + bias;
    } else {
#pragma unroll
      for (int ib = 0; ib < NIB; ++ib)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rl = ib * 32 + 8 * (r >> 2) + (r & 3);
          if (rl + 4 * half < rows) zcol[(size_t)rl * nc] = acc[ib][r] + bias;
        }
    }
  }
  __syncthreads();
  const uint32_t nl = lcnt;
  if (nl > (uint32_t)kLocalCand) {
    // more candidates than the LDS holds: every sample of the tile is told to stream this chunk's scores
    if (tid < rows) atomicAdd(&ccnt[(size_t)(i0 + tid) * kCntPitch], (uint32_t)kCand + 1u);
    return;
  }
  for (uint32_t e = tid; e < nl; e += 256) {
    const int i = i0 + (int)lsmp[e];
    const uint32_t pos = atomicAdd(&ccnt[(size_t)i * kCntPitch], 1u);
    if (pos < (uint32_t)kCand) cand[(size_t)i * kCand + pos] = lkey[e];
  }
}

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

// One workgroup per sample: folds one chunk of neurons into the sample's running list of the topk
// best keys (best[i][0..64), ascending; ~0 = empty).  Normally the chunk arrives as the candidate keys
// the scoring kernel collected; for the first chunk, or when more than kCand scores beat the bar, it
// streams the chunk's scores instead: only scores that beat the current topk-th key are collected,
// and when the LDS buffer fills it is sorted and cut back to topk, which raises the bar.  The last
// chunk also decodes the list into the caller's arrays.
__global__ __launch_bounds__(256) void topk_merge_kernel(int nc, int64_t j0, const float* __restrict__ zc, int topk,
                                                         uint64_t* __restrict__ best, int first, int last,
                                                         const uint64_t* __restrict__ cand, uint32_t* ccnt,
                                                         int32_t* __restrict__ out_ids,
                                                         float* __restrict__ out_scores) {
  __shared__ uint64_t keys[kTopkBuf];
  __shared__ uint32_t cnt;
  const int i = blockIdx.x, tid = threadIdx.x;
  uint64_t* mine = best + (size_t)i * 64;
  const uint32_t ncand = first ? 0u : ccnt[(size_t)i * kCntPitch];
  const bool stream = first || ncand > (uint32_t)kCand;
  __syncthreads();
  if (tid == 0) ccnt[(size_t)i * kCntPitch] = 0;
  if (!stream && ncand == 0 && !last) return;          // nothing beat the bar: the list stands
  int nsort = kTopkBuf;
  if (!stream) {
    nsort = 128;                                        // power of two holding the list and the candidates
    while (nsort < 64 + (int)ncand) nsort <<= 1;
    const uint64_t* cv = cand + (size_t)i * kCand;
    for (int q = tid; q < nsort; q += 256)
      keys[q] = q < topk ? mine[q] : (q >= 64 && q < 64 + (int)ncand ? cv[q - 64] : ~0ull);
    __syncthreads();
  } else {
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
    nsort = 128;                                        // the collected keys sit at the front, ~0 behind them
    while (nsort < (int)cnt) nsort <<= 1;
  }
  bitonic_sort_keys(keys, nsort);
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

size_t dense_cand_keys() { return (size_t)kCand; }
size_t dense_counter_words() { return (size_t)kCntPitch; }

int64_t dense_chunk_neurons(int64_t N, int Bmax) {
  int64_t nc = ((int64_t)256 << 20) / ((int64_t)Bmax * 4);    // about 256 MiB of scores
  nc = nc / kBN * kBN;
  if (nc < kBN) nc = kBN;
  const int64_t npad = (N + kBN - 1) / kBN * kBN;
  return nc < npad ? nc : npad;
}

hipError_t launch_dense_topk(int B, int64_t N, int H, const float* h, const float* W2, const float* b2, int topk,
                             float* zc, int64_t chunk, uint64_t* best, uint64_t* cand, uint32_t* ccnt,
                             int32_t* out_ids, float* out_scores, hipStream_t s) {
  hipError_t e = launch_fill_u32(ccnt, (size_t)B * kCntPitch, 0u, s);
  if (e != hipSuccess) return e;
  // The first chunk is what the merge can stream without an intermediate sort.  Later chunks grow with
  // the number of neurons already seen -- in random order about topk * chunk / seen scores of a chunk
  // beat a list settled on the neurons before it, kept near 512 of the kCand a sample can hand over --
  // up to the scratch buffer's size.
  const int64_t grow = topk <= 32 ? 16 : 512 / topk;
  const int64_t first_nc = (kTopkBuf - 256 - 64) / kBN * kBN;
  int64_t nc = chunk < first_nc ? chunk : first_nc;
  for (int64_t j0 = 0; j0 < N; j0 += nc, nc = (j0 * grow < chunk ? j0 * grow / kBN * kBN : chunk)) {
    if (nc > N - j0) nc = N - j0;
    const int first = j0 == 0 ? 1 : 0, last = j0 + nc >= N ? 1 : 0;
    const uint64_t* bars = first ? (const uint64_t*)nullptr : best;
    const unsigned gx = (unsigned)ceil_div(nc, kNB);
#define SLIDE_SCORES(NIB) \
    hipLaunchKernelGGL((dense_scores_kernel<NIB>), dim3(gx, (unsigned)ceil_div(B, NIB * 32)), dim3(256), 0, s, B, N, H, h, \
                       W2, b2, j0, (int)nc, zc, topk, bars, cand, ccnt)
    if (B <= 32) SLIDE_SCORES(1); else if (B <= 64) SLIDE_SCORES(2); else if (B <= 128) SLIDE_SCORES(4); else SLIDE_SCORES(8);
#undef SLIDE_SCORES
    hipLaunchKernelGGL(topk_merge_kernel, dim3(B), dim3(256), 0, s, (int)nc, j0, zc, topk, best, first, last, cand, ccnt,
                       out_ids, out_scores);
  }
  return hipGetLastError();
}

}  // namespace slide
