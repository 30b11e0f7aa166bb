// Float half of the forward pass: sparse-input hidden layer, logits + softmax over the active set
// only, the gradient with respect to the hidden activations, and top-k for inference
// (paper Section 2.1: activations are computed for the retrieved neurons only; Section 3.6: the
// first layer is fed by index/value arrays, the second by the first layer's activations).
#include "slide_internal.h"
#include "spmm.h"
#include "transpose.h"

#include <algorithm>

namespace slide {

// The hidden layer as a launch of its own (prediction over all neurons; the training step runs it
// inside the lookup workgroups).
__global__ __launch_bounds__(64) void spmm_relu_kernel(SpmmArgs a, Ctrl* ctrl) {
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
    ctrl->p1 = 0; ctrl->nlong1 = 0; ctrl->max_nu1 = 0;
    for (int r = 0; r < kPairRegions; ++r) ctrl->p1r[r] = 0;
  }
  spmm_sample(a, blockIdx.x, gridDim.x, blockIdx.y, threadIdx.x, nullptr, ctrl);
}

hipError_t launch_spmm_relu(int B, const SpmmArgs& a, Ctrl* ctrl, hipStream_t s) {
  hipLaunchKernelGGL(spmm_relu_kernel, dim3(B, ceil_div(a.H, 128)), dim3(64), 0, s, a, ctrl);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Forward over the active set, one pass over the gathered rows of W2.
// Work item = up to kChunk consecutive active neurons of one sample, handled by one wave.  A row
// is read by LPR lanes (float4 each, CH of them per lane), so 64/LPR rows are in flight per wave.
// For each row: logit z = w.h + b (stored), and a running soft-max state (max M, sum s of
// exp(z - M), acc = sum of exp(z - M) * w) that is rescaled when the maximum moves.  acc/s is the
// probability-weighted sum of the rows, which is all the hidden-layer gradient needs, so the rows
// are not read a second time.  Partial states are merged per sample by combine_kernel.
// The same launch builds the row lists of the two weight matrices (tile workgroups behind the logit
// workers): they depend on the lookup only, like the logits, and are latency-bound where the logit
// workers are bandwidth-bound.
// ---------------------------------------------------------------------------------------------
constexpr int kForwardThreads = 512;

template <int LPR, int CH, bool FULL>
__device__ __forceinline__ void forward_items(const ActiveDev& ad, int H, const float* __restrict__ h, const float* __restrict__ W2,
                              const float* __restrict__ b2, float* __restrict__ z, float* __restrict__ partials,
                              const Ctrl* __restrict__ ctrl, int block, int nblocks) {
  constexpr int RPW = 64 / LPR;
  const int lane = threadIdx.x & 63, sub = lane % LPR, grp = lane / LPR;
  constexpr int WPB = kForwardThreads / 64;
  // Work item (i, c) = chunk c (kChunk active neurons) of sample i, enumerated as c * B + i: items that are
  // neighbours in this order cover about the same stretch of neuron ids (the ids of a sample ascend),
  // so when samples share rows (saturated buckets) a row is fetched once and then found in L2.  With
  // many chunks per sample every XCD (workgroup k runs on XCD k % 8, each with its own L2) also takes
  // its own eighth of the chunk indices, a contiguous one, so that the stretches it works on at the
  // same time are neighbours and a row is fetched by one XCD only.  (That workgroup k runs on die
  // k % nxcd is how this device family hands out workgroups; slide_init sets nxcd = 1, which turns the
  // split off, when it does not recognise the device.)
  const int B = ad.B;
  const int maxnch = (int)ctrl->max_nch[ad.par];
  const int nx = ad.nxcd;
  const bool affine = nx > 1 && maxnch >= 8 * nx && nblocks % nx == 0;   // (otherwise the dies would get unequal shares)
  const int xcd = block % nx;
  const int c_lo = affine ? xcd * maxnch / nx : 0, c_hi = affine ? (xcd + 1) * maxnch / nx : maxnch;
  const int lwave = (affine ? (block / nx) : block) * WPB + (threadIdx.x >> 6);
  const int lwaves = (affine ? (nblocks / nx) : nblocks) * WPB;
  const int T = (c_hi - c_lo) * B;
  const int PS = H + 4;
  for (int t = lwave; t < T; t += lwaves) {
    const int i = t % B, ch = c_lo + t / B;
    const int done = ch * kChunk, cnt = ad.cnt[i];
    if (done >= cnt) continue;
    const int item = ad.chunk_ptr[i] + ch;             // slot of the partial result
    const int first = ad.as_base[i] + done;
    const int n = min(kChunk, cnt - done);
    float4 hv[CH], acc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) {
      const int col = (c * LPR + sub) * 4;
      hv[c] = (FULL || col < H) ? *(const float4*)(h + (size_t)i * H + col) : make_float4(0.f, 0.f, 0.f, 0.f);
      acc[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    // the item's ids and their biases in one coalesced read each (lane l: neuron l of the item), handed to
    // the row groups step by step: a step then waits for its rows only, not for an id first
    const int my_j = ad.as_ids[first + (lane < n ? lane : 0)];
    const float my_b = b2[my_j];
    float M = -INFINITY, s = 0.f;
    for (int q0 = 0; q0 < n; q0 += RPW) {
      const int q = q0 + grp;
      const bool valid = q < n;
      const int slot = first + (valid ? q : 0);
      const int j = __shfl(my_j, valid ? q : 0);
      const float bj = __shfl(my_b, valid ? q : 0);
      const float* wr = W2 + (size_t)j * H;
      float4 row[CH];
      float dot = 0.f;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int col = (c * LPR + sub) * 4;
        row[c] = (FULL || col < H) ? *(const float4*)(wr + col) : make_float4(0.f, 0.f, 0.f, 0.f);
        dot += row[c].x * hv[c].x + row[c].y * hv[c].y + row[c].z * hv[c].z + row[c].w * hv[c].w;
      }
      dot = group_sum<LPR>(dot);
      const float zz = dot + bj;
      if (valid) {
        if (sub == 0) z[slot] = zz;
        const float Mn = fmaxf(M, zz);
        const float sc = __expf(M - Mn), e = __expf(zz - Mn);
        s = s * sc + e;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          acc[c].x = acc[c].x * sc + e * row[c].x;
          acc[c].y = acc[c].y * sc + e * row[c].y;
          acc[c].z = acc[c].z * sc + e * row[c].z;
          acc[c].w = acc[c].w * sc + e * row[c].w;
        }
        M = Mn;
      }
    }
#pragma unroll
    for (int d = LPR; d < 64; d <<= 1) {               // merge the row groups of the wave
      const float Mo = __shfl_xor(M, d), so = __shfl_xor(s, d);
      const float Mn = fmaxf(M, Mo);
      const float a = M == -INFINITY ? 0.f : __expf(M - Mn);
      const float b = Mo == -INFINITY ? 0.f : __expf(Mo - Mn);
      s = s * a + so * b;
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        acc[c].x = acc[c].x * a + __shfl_xor(acc[c].x, d) * b;
        acc[c].y = acc[c].y * a + __shfl_xor(acc[c].y, d) * b;
        acc[c].z = acc[c].z * a + __shfl_xor(acc[c].z, d) * b;
        acc[c].w = acc[c].w * a + __shfl_xor(acc[c].w, d) * b;
      }
      M = Mn;
    }
    if (grp == 0) {
      float* pp = partials + (size_t)item * PS;
      if (sub == 0) { pp[0] = M; pp[1] = s; }
#pragma unroll
      for (int c = 0; c < CH; ++c) {
        const int col = (c * LPR + sub) * 4;
        if (FULL || col < H) *(float4*)(pp + 4 + col) = acc[c];
      }
    }
  }
}

template <int LPR, int CH>
__global__ __launch_bounds__(kForwardThreads) void forward_kernel(ActiveDev ad, int H, const float* __restrict__ h,
                                                                  const float* __restrict__ W2,
                                                                  const float* __restrict__ b2, float* __restrict__ z,
                                                                  float* __restrict__ partials,
                                                                  const Ctrl* __restrict__ ctrl, TransposeArgs t1,
                                                                  TransposeArgs t2, int nworkers) {
  extern __shared__ uint32_t dyn_lds[];
  // Workgroups start in index order and the machine holds a few hundred at a time.  The logit
  // workers go first (they are what the memory system is busy with); the tiles fill in behind them
  // as workers without an item leave, the feature tiles (fewer, and with a global counter on their
  // critical path) before the active-set tiles.
  const int k = blockIdx.x;
  if (k < nworkers) {
    // With several items per wave the workers would hold every slot of the machine until the end and
    // the tiles would run after them: then the last workers leave at once and make room.
    const int items = (int)ctrl->max_nch[ad.par] * ad.B;   // (upper bound: samples differ in length)
    // (more of them when the tiles are many for the amount of logit work)
    const int ntiles = t1.ntiles + t2.ntiles;
    const int workers = (ntiles == 0 || items <= 2 * nworkers * (kForwardThreads / 64)) ? nworkers
                        : (items < 20 * ntiles ? nworkers * 2 / 3 : nworkers * 5 / 6);
    if (k >= workers) return;
    if (H == LPR * CH * 4) forward_items<LPR, CH, true>(ad, H, h, W2, b2, z, partials, ctrl, k, workers);
    else forward_items<LPR, CH, false>(ad, H, h, W2, b2, z, partials, ctrl, k, workers);
  }
  else {
    if (k >= nworkers + t1.ntiles) transpose_tile<false, false>(t2, k - nworkers - t1.ntiles, dyn_lds);
    else transpose_tile<true, false>(t1, k - nworkers, dyn_lds);
  }
}

template <int LPR, int CH>
static hipError_t launch_fwd(const ActiveDev& ad, int H, const float* h, const float* W2, const float* b2, float* z,
                             float* partials, const Ctrl* ctrl, const TransposeArgs& t1, const TransposeArgs& t2,
                             int nworkers, hipStream_t s) {
  size_t lds = 0;
  if (t1.ntiles) lds = transpose_lds(t1.TW, t1.Bpad);
  if (t2.ntiles) lds = std::max(lds, transpose_lds(t2.TW, t2.Bpad));
  if (t1.grouped) return hipErrorInvalidValue;           // (grouped feature tiles ride in the combine launch)
  if (t2.ntiles + t1.ntiles + nworkers == 0) return hipSuccess;
  hipLaunchKernelGGL((forward_kernel<LPR, CH>), dim3(t2.ntiles + t1.ntiles + nworkers), dim3(kForwardThreads),
                     lds, s, ad, H, h, W2, b2, z, partials, ctrl, t1, t2, nworkers);
  return hipGetLastError();
}

template <int LPR, int CH>
static hipError_t fwd_attr(int lim) {
  return hipFuncSetAttribute((const void*)forward_kernel<LPR, CH>, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
}

static hipError_t combine_setup_attributes(int lim);

hipError_t forward_setup_attributes(size_t lds_limit) {
  const int lim = (int)std::min<size_t>(lds_limit, 72 * 1024);
  hipError_t e = fwd_attr<8, 1>(lim);
  if (e == hipSuccess) e = fwd_attr<8, 2>(lim);
  if (e == hipSuccess) e = fwd_attr<8, 4>(lim);
  if (e == hipSuccess) e = fwd_attr<16, 4>(lim);
  if (e == hipSuccess) e = fwd_attr<32, 4>(lim);
  if (e == hipSuccess) e = fwd_attr<64, 4>(lim);
  if (e == hipSuccess) e = fwd_attr<64, 8>(lim);
  if (e == hipSuccess) e = combine_setup_attributes(lim);
  return e;
}

hipError_t launch_forward(const ActiveDev& ad, int H, const float* h, const float* W2, const float* b2, float* z,
                          float* partials, const Ctrl* ctrl, const TransposeArgs& t1, const TransposeArgs& t2,
                          bool logits, int num_cus, hipStream_t s) {
  // three logit workgroups of 16 waves per compute unit (768 on the 256 of an MI355X)
  const int nworkers = logits ? 3 * num_cus : 0;
#define SLIDE_FWD(L_, C_) return launch_fwd<L_, C_>(ad, H, h, W2, b2, z, partials, ctrl, t1, t2, nworkers, s)
  if (H <= 32) SLIDE_FWD(8, 1);
  if (H <= 64) SLIDE_FWD(8, 2);
  if (H <= 128) SLIDE_FWD(8, 4);
  if (H <= 256) SLIDE_FWD(16, 4);
  if (H <= 512) SLIDE_FWD(32, 4);
  if (H <= 1024) SLIDE_FWD(64, 4);
  SLIDE_FWD(64, 8);
#undef SLIDE_FWD
}

// ---------------------------------------------------------------------------------------------
// One workgroup per sample: merges the forward partials into the soft-max normaliser, then
//   delta_ij = (p_ij - y_ij) / B,  loss_i = -sum_{j in Y_i} log(p_ij) / |Y_i|,
//   dh_i = [h_i > 0] * (sum_j p_ij w_j - mean_{j in Y_i} w_j) / B
// (the first sum is acc/s from the forward pass; the label rows are read here, in label order).
// A sample without labels contributes nothing.
// ---------------------------------------------------------------------------------------------
constexpr int kCombineThreads = 512;

struct CombineArgs {
  const float *h, *z, *partials, *W2;
  const int32_t *y_indptr, *ylist;
  float *delta, *dh, *dh_copy, *loss_i, *msum;
};

__device__ __forceinline__ void combine_sample(const ActiveDev& ad, int H, const CombineArgs& ca, int sample) {
  const float* __restrict__ h = ca.h;
  const float* __restrict__ z = ca.z;
  const float* __restrict__ partials = ca.partials;
  const float* __restrict__ W2 = ca.W2;
  const int32_t* __restrict__ y_indptr = ca.y_indptr;
  const int32_t* __restrict__ ylist = ca.ylist;
  float* __restrict__ delta = ca.delta;
  float* __restrict__ dh = ca.dh;
  float* __restrict__ dh_copy = ca.dh_copy;
  float* __restrict__ loss_i = ca.loss_i;
  float* __restrict__ msum = ca.msum;
  constexpr int kMaxCh = 1024, kMaxLab = 256;            // LDS-staged chunk scales / label rows; more fall back to global reads
  __shared__ float red[kCombineThreads / 64];
  __shared__ float scale[kMaxCh];                        // exp(M_c - M) per forward work item of the sample
  __shared__ int ylab[kMaxLab];                          // neuron of each label entry, -1 = not counted
  __shared__ int yslot[kMaxLab];                         // its slot in the sample-major arrays, -1 = not counted
  __shared__ float ms[2];
  const int i = sample, tid = threadIdx.x, lane = tid & 63;
  const int c0 = ad.chunk_ptr[i], nch = (ad.cnt[i] + kChunk - 1) / kChunk;
  const int first = ad.as_base[i], n = ad.cnt[i];
  const int ny = ad.ny[i];
  const int PS = H + 4;
  const float* pmine = partials + (size_t)c0 * PS;
  const float invB = 1.0f / (float)ad.B;
  const int y0 = min(max(y_indptr[i], 0), ad.num_labels);               // (clamped like the lookup does)
  const int nlab = min(max(y_indptr[i + 1], y0), ad.num_labels) - y0;
  // label rows: both lookups for all labels at once (a chain of dependent reads per label otherwise)
  for (int q = tid; q < min(nlab, kMaxLab); q += kCombineThreads) {
    const int slot = ylist[y0 + q];
    yslot[q] = slot;
    ylab[q] = slot >= 0 ? ad.as_ids[slot] : -1;
  }
  // soft-max normaliser from the partial states: wave 0, one lane per work item, fixed butterfly order
  if (tid < 64) {
    float Mi = -INFINITY;
    for (int c = lane; c < nch; c += 64) Mi = fmaxf(Mi, pmine[(size_t)c * PS]);
    for (int d = 32; d > 0; d >>= 1) Mi = fmaxf(Mi, __shfl_xor(Mi, d));
    float s = 0.f;
    for (int c = lane; c < nch; c += 64) {
      const float* pp = pmine + (size_t)c * PS;
      const float sc = __expf(pp[0] - Mi);
      if (c < kMaxCh) scale[c] = sc;
      s += pp[1] * sc;
    }
    for (int d = 32; d > 0; d >>= 1) s += __shfl_xor(s, d);
    if (lane == 0) { ms[0] = Mi; ms[1] = s; msum[2 * i] = Mi; msum[2 * i + 1] = s; }
  }
  __syncthreads();
  const float Mi = ms[0], s = ms[1];
  const bool live = n > 0 && ny > 0;
  // Hidden gradient: column u sums the chunks' partial sums (scaled) and subtracts the label rows.  A
  // column's chain of reads is what this costs, so when the workgroup has several threads per column
  // each takes a stretch of the chunks (eight reads in flight) and the stretches are added in order.
  const int nsub = H <= kCombineThreads ? kCombineThreads / H : 1;
  if (nsub > 1) {
    __shared__ float part[kCombineThreads];              // [nsub][H] sums of the stretches
    __shared__ float ysum[kCombineThreads];              // [H] sum of the label rows
    const int u = tid % H, sub = tid / H;
    if (sub < nsub) {
      float acc = 0.f, accy = 0.f;
      if (live && h[(size_t)i * H + u] > 0.f) {
        const float* pu = pmine + 4 + u;
        const int nchl = min(nch, kMaxCh), per = (nchl + nsub - 1) / nsub;
        const int ce = min(nchl, (sub + 1) * per);
        int c = sub * per;
        for (; c + 8 <= ce; c += 8) {
          float a[8];
#pragma unroll
          for (int k = 0; k < 8; ++k) a[k] = pu[(size_t)(c + k) * PS];
#pragma unroll
          for (int k = 0; k < 8; ++k) acc += a[k] * scale[c + k];
        }
        for (; c < ce; ++c) acc += pu[(size_t)c * PS] * scale[c];
        if (sub == nsub - 1) {
          for (c = kMaxCh; c < nch; ++c) acc += pu[(size_t)c * PS] * __expf(pu[(size_t)c * PS - 4 - u] - Mi);
          for (int q = 0; q < nlab; ++q) {
            int j;
            if (q < kMaxLab) j = ylab[q];
            else { const int slot = ylist[y0 + q]; j = slot >= 0 ? ad.as_ids[slot] : -1; }
            if (j >= 0) accy += W2[(size_t)j * H + u];
          }
          ysum[u] = accy;
        }
      }
      part[tid] = acc;
    }
    __syncthreads();
    if (tid < H) {
      float g = 0.f;
      if (live && h[(size_t)i * H + tid] > 0.f) {
        float acc = 0.f;
        for (int k = 0; k < nsub; ++k) acc += part[k * H + tid];
        g = (acc / s - ysum[tid] / (float)ny) * invB;
      }
      dh[(size_t)i * H + tid] = g;
      if (dh_copy) dh_copy[(size_t)i * H + tid] = g;
    }
  } else
  for (int u = tid; u < H; u += kCombineThreads) {
    float g = 0.f;
    if (live && h[(size_t)i * H + u] > 0.f) {
      float acc = 0.f;
      const float* pu = pmine + 4 + u;
      int c = 0;
      for (; c + 4 <= min(nch, kMaxCh); c += 4) {         // four reads in flight, added in chunk order
        const float a0 = pu[(size_t)c * PS], a1 = pu[(size_t)(c + 1) * PS], a2 = pu[(size_t)(c + 2) * PS],
                    a3 = pu[(size_t)(c + 3) * PS];
        acc += a0 * scale[c]; acc += a1 * scale[c + 1]; acc += a2 * scale[c + 2]; acc += a3 * scale[c + 3];
      }
      for (; c < nch; ++c) acc += pu[(size_t)c * PS] * (c < kMaxCh ? scale[c] : __expf(pu[(size_t)c * PS - 4 - u] - Mi));
      float accy = 0.f;
      for (int q = 0; q < nlab; ++q) {
        int j;
        if (q < kMaxLab) j = ylab[q];
        else { const int slot = ylist[y0 + q]; j = slot >= 0 ? ad.as_ids[slot] : -1; }
        if (j >= 0) accy += W2[(size_t)j * H + u];
      }
      g = (acc / s - accy / (float)ny) * invB;
    }
    dh[(size_t)i * H + u] = g;
    if (dh_copy) dh_copy[(size_t)i * H + u] = g;
  }
  float lacc = 0.f;
  const float logs = live ? __logf(s) : 0.f;
  const float yv = ny > 0 ? 1.0f / (float)ny : 0.f;
  // A slot holds a label iff a counted label entry names it.  Few entries (the usual case): every
  // slot is compared with them.  Many: the labels' slots are rewritten in a second pass.
  constexpr int kFewLabels = 16;
  const bool few = nlab <= kFewLabels;
  for (int q0 = tid; q0 < n; q0 += 4 * kCombineThreads) {  // four logits per thread in flight
    float zz[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int q = q0 + k * kCombineThreads;
      zz[k] = (live && q < n) ? z[first + q] : 0.f;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int q = q0 + k * kCombineThreads, slot = first + q;
      if (q >= n) continue;
      float d = 0.f;
      if (live) {
        bool lab = false;
        if (few) for (int y = 0; y < nlab; ++y) lab |= yslot[y] == slot;
        d = (__expf(zz[k] - Mi) / s - (lab ? yv : 0.f)) * invB;
        if (lab) lacc -= yv * (zz[k] - Mi - logs);
      }
      delta[slot] = d;
    }
  }
  if (!few) {
    __syncthreads();                                     // (orders the first pass's writes before these)
    for (int q = tid; q < nlab; q += kCombineThreads) {
      const int slot = q < kMaxLab ? yslot[q] : ylist[y0 + q];
      if (slot < 0 || !live) continue;
      const float zz = z[slot];
      delta[slot] = (__expf(zz - Mi) / s - yv) * invB;
      lacc -= yv * (zz - Mi - logs);
    }
  }
  for (int d = 32; d > 0; d >>= 1) lacc += __shfl_xor(lacc, d);
  if ((tid & 63) == 0) red[tid >> 6] = lacc;
  __syncthreads();
  if (tid == 0) {                     // fixed order
    float t = 0.f;
    for (int w = 0; w < kCombineThreads / 64; ++w) t += red[w];
    loss_i[i] = t;
  }
}

// The samples' workgroups; behind them, optionally, the row-list tiles (t1: features, t2: active sets):
// the lists depend on the lookup only and are not needed before the update launch, and when they are many
// (batches whose samples share most rows) they are best kept out of the logit workers' way.
__global__ __launch_bounds__(kCombineThreads, 6) void combine_kernel(ActiveDev ad, int H, CombineArgs ca, TransposeArgs t1,
                                                                  TransposeArgs t2) {
  extern __shared__ uint32_t dyn_lds[];
  const int k = blockIdx.x;
  const int r1 = transpose_roles(t1, kCombineThreads);
  if (k < ad.B) combine_sample(ad, H, ca, k);
  else if (k >= ad.B + r1) transpose_tile<false, true>(t2, k - ad.B - r1, dyn_lds);
  else feature_tile_role(t1, k - ad.B, dyn_lds);
}

static hipError_t combine_setup_attributes(int lim) {
  return hipFuncSetAttribute((const void*)combine_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
}

hipError_t launch_combine(const ActiveDev& ad, int H, const float* h, const float* z, const float* partials,
                          const float* W2, const int32_t* y_indptr, const int32_t* ylist, float* delta,
                          float* dh, float* dh_copy, float* loss_i, float* msum, const TransposeArgs& t1,
                          const TransposeArgs& t2, hipStream_t s) {
  static_assert(kCombineThreads == kForwardThreads, "the tiles are written for one workgroup size");
  CombineArgs ca{h, z, partials, W2, y_indptr, ylist, delta, dh, dh_copy, loss_i, msum};
  size_t lds = 0;
  if (t1.ntiles) lds = transpose_lds(t1.TW, t1.Bpad);
  if (t2.ntiles) lds = std::max(lds, transpose_lds(t2.TW, t2.Bpad));
  hipLaunchKernelGGL(combine_kernel, dim3(ad.B + transpose_roles(t1, kCombineThreads) + t2.ntiles), dim3(kCombineThreads), lds, s, ad, H,
                     ca, t1, t2);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Top-k of the logits of each sample's active set: k rounds of "largest score strictly after the
// previous pick" in the order (score descending, id ascending).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void topk_kernel(ActiveDev ad, const float* __restrict__ z, int topk,
                                                   int32_t* __restrict__ out_ids, float* __restrict__ out_scores) {
  __shared__ float rz[4];
  __shared__ int rj[4];
  const int i = blockIdx.x, tid = threadIdx.x;
  const int first = ad.as_base[i], n = ad.cnt[i];
  float pz = INFINITY;
  int pj = -1;
  for (int k = 0; k < topk; ++k) {
    float bz = -INFINITY;
    int bj = -1;
    for (int q = tid; q < n; q += 256) {
      const float zz = z[first + q];
      const int j = ad.as_ids[first + q];
      const bool after = zz < pz || (zz == pz && j > pj);
      if (after && (bj < 0 || zz > bz || (zz == bz && j < bj))) { bz = zz; bj = j; }
    }
    for (int d = 32; d > 0; d >>= 1) {
      const float oz = __shfl_xor(bz, d);
      const int oj = __shfl_xor(bj, d);
      if (oj >= 0 && (bj < 0 || oz > bz || (oz == bz && oj < bj))) { bz = oz; bj = oj; }
    }
    __syncthreads();
    if ((tid & 63) == 0) { rz[tid >> 6] = bz; rj[tid >> 6] = bj; }
    __syncthreads();
    bz = rz[0]; bj = rj[0];
    for (int w = 1; w < 4; ++w)
      if (rj[w] >= 0 && (bj < 0 || rz[w] > bz || (rz[w] == bz && rj[w] < bj))) { bz = rz[w]; bj = rj[w]; }
    if (tid == 0) {
      out_ids[(size_t)i * topk + k] = bj;
      out_scores[(size_t)i * topk + k] = bj >= 0 ? bz : -INFINITY;
    }
    if (bj < 0) { pz = -INFINITY; pj = 0x7fffffff; } else { pz = bz; pj = bj; }
  }
}

hipError_t launch_topk(const ActiveDev& ad, const float* z, int topk, int32_t* out_ids, float* out_scores,
                       hipStream_t s) {
  hipLaunchKernelGGL(topk_kernel, dim3(ad.B), dim3(256), 0, s, ad, z, topk, out_ids, out_scores);
  return hipGetLastError();
}

}  // namespace slide
