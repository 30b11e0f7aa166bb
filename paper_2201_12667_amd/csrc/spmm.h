// Sparse-input hidden layer of one sample (paper Section 3.6: the first layer is fed by index /
// value arrays), as a device function so that it can run as a kernel of its own or inside the
// lookup workgroup of the sample.
#pragma once
#include "slide_internal.h"

namespace slide {

// ---------------------------------------------------------------------------------------------
// The same hidden layer by a whole workgroup, for a caller that can lend `stage_words` words of LDS.
// When one wave owns the sample the layer costs a chain of dependent row fetches (sixteen in flight
// at a time); here the indices and values of up to `cap` features are read once into LDS, every
// thread fetches its share of their W1 rows at once into LDS, and then one thread per column runs
// the multiply-adds over the staged rows in storage order: the same arithmetic, bit for bit (a
// feature index outside [0, D) contributes 0 * 0, which leaves every sum as it is).  The feature
// segments per tile and the data flags are derived from the staged indices exactly as spmm_sample
// derives them.  Needs H <= blockDim.x.  Every thread of the workgroup must call; ends with the
// result in hvec (LDS) and in a.h, after a barrier.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int spmm_stage_rows(int stage_words, int H, int nthr) {
  const int cap = (stage_words - 2) / (H + 2);           // a row, its feature index and its value; two carries
  return cap > nthr ? nthr : cap;
}

__device__ __forceinline__ void spmm_sample_staged(const SpmmArgs& a, int i, int B, float* stage, int stage_words,
                                                   float* hvec, Ctrl* ctrl) {
  const int64_t D = a.D;
  const int H = a.H, H4 = H >> 2, rows_per_tile = a.rows_per_tile;
  const int tid = threadIdx.x, nthr = blockDim.x;
  const float* __restrict__ W1 = a.W1;
  int2* __restrict__ xse = a.xse;
  const int cap = spmm_stage_rows(stage_words, H, nthr);
  int* sk = (int*)(stage + (size_t)cap * H);             // [cap] feature of the staged row, -1: left out
  float* sv = (float*)(sk + cap);                        // [cap] its value (0 when left out)
  int* carry = (int*)(sv + cap);                         // [0] entry before the batch, [1] last valid feature before it
  const int p0 = max(a.x_indptr[i], 0), p1 = min(a.x_indptr[i + 1], a.nnz_total);
  float acc = tid < H ? a.b1[tid] : 0.f;
  uint32_t flags = 0;
  if (tid == 0) { carry[0] = -1; carry[1] = -1; }
  for (int pb = p0; pb < p1; pb += cap) {
    const int cnt = min(cap, p1 - pb);
    int kk = -1;
    if (tid < cnt) {
      const int k = a.x_indices[pb + tid];
      const float v = a.x_values[pb + tid];
      const bool bad = k < 0 || k >= D;
      if (bad) flags |= SLIDE_FLAG_BAD_FEATURE;
      kk = bad ? -1 : k;
      sk[tid] = kk;
      sv[tid] = bad ? 0.f : v;
    }
    __syncthreads();
    const int total = cnt * H4;
    for (int idx0 = 0; idx0 < total; idx0 += 4 * nthr) {  // four row pieces per thread in flight
      float4 w[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = idx0 + u * nthr + tid;
        const int k = idx < total ? sk[idx / H4] : -1;
        w[u] = k >= 0 ? *(const float4*)(W1 + (size_t)k * H + 4 * (idx % H4)) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = idx0 + u * nthr + tid;
        if (idx < total) ((float4*)stage)[idx] = w[u];
      }
    }
    if (kk >= 0) {
      // order: against the last valid feature before this one
      int q = tid - 1;
      while (q >= 0 && sk[q] < 0) --q;
      const int prev = q >= 0 ? sk[q] : carry[1];
      if (kk <= prev) flags |= SLIDE_FLAG_UNSORTED;
      // segment ends: a feature whose predecessor lies in another tile starts its own tile's segment
      // and ends the predecessor's
      if (xse) {
        const int before = tid > 0 ? sk[tid - 1] : carry[0];
        const int tile = kk / rows_per_tile, tb = before >= 0 ? before / rows_per_tile : -1;
        if (tb != tile) {
          xse[(size_t)tile * B + i].x = pb + tid;
          if (tb >= 0) xse[(size_t)tb * B + i].y = pb + tid;
        }
        if (pb + tid == p1 - 1) xse[(size_t)tile * B + i].y = p1;
      }
    }
    __syncthreads();
    if (tid < H) {
#pragma unroll 8
      for (int q = 0; q < cnt; ++q) acc = fmaf(sv[q], stage[(size_t)q * H + tid], acc);
    }
    if (tid == 0 && pb + cap < p1) {                     // carries for the next batch
      int q = cnt - 1;
      while (q >= 0 && sk[q] < 0) --q;
      if (q >= 0) carry[1] = sk[q];
      carry[0] = sk[cnt - 1];
    }
    __syncthreads();
  }
  if (tid < H) {
    const float r = acc > 0.f ? acc : 0.f;
    a.h[(size_t)i * H + tid] = r;
    hvec[tid] = r;
  }
  if (flags) atomicOr(&ctrl->status, flags);
  __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// h[i][:] = max(0, b1 + sum_k x_ik * W1[k][:]), one fused multiply-add per stored feature, in
// storage order (so any other fp32 implementation using the same order gets the same bits).
// One wave per (sample, 128 columns); each lane owns two columns and reads a float2 per W1 row.
// The first column block also records, per tile of rows_per_tile features, where the sample's
// features of the tile start and end in the CSR arrays (the row lists of the W1 update are built
// from these segments; a.xse == nullptr: not recorded).  hvec (optional, LDS): a second copy of the
// result for the caller.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void spmm_sample(const SpmmArgs& a, int i, int B, int cb, int lane, float* hvec,
                                            Ctrl* ctrl) {
  const int64_t D = a.D;
  const int H = a.H, nnz_total = a.nnz_total, rows_per_tile = a.rows_per_tile;
  const int32_t* __restrict__ x_indptr = a.x_indptr;
  const int32_t* __restrict__ x_indices = a.x_indices;
  const float* __restrict__ x_values = a.x_values;
  const float* __restrict__ W1 = a.W1;
  const float* __restrict__ b1 = a.b1;
  float* __restrict__ h = a.h;
  int2* __restrict__ xse = a.xse;
  const int c0 = (cb * 64 + lane) * 2;
  const bool col_ok = c0 < H;
  int p0 = x_indptr[i], p1 = x_indptr[i + 1];
  p0 = max(p0, 0);
  p1 = min(p1, nnz_total);
  float2 acc = col_ok ? *(const float2*)(b1 + c0) : make_float2(0.f, 0.f);
  int prev = -1, last = -1;                              // last: feature of the pair before this batch of 64
  uint32_t flags = 0;
  constexpr int UN = 16;
  for (int pb = p0; pb < p1; pb += 64) {
    // one coalesced read of the next 64 (index, value) pairs; lane q holds pair pb + q
    const int mine = pb + lane < p1 ? x_indices[pb + lane] : -1;
    const float myv = pb + lane < p1 ? x_values[pb + lane] : 0.f;
    const bool bad = pb + lane < p1 && (mine < 0 || mine >= D);
    if (__any(bad)) flags |= SLIDE_FLAG_BAD_FEATURE;
    const int kk = bad ? -1 : mine;
    if (cb == 0 && xse) {         // segment ends: a feature whose predecessor lies in another tile
      int before = __shfl_up(kk, 1);      // starts its own tile's segment and ends the predecessor's
      if (lane == 0) before = last;
      last = __shfl(kk, 63);
      if (kk >= 0) {
        const int tile = kk / rows_per_tile, tb = before >= 0 ? before / rows_per_tile : -1;
        if (tb != tile) {
          xse[(size_t)tile * B + i].x = pb + lane;
          if (tb >= 0) xse[(size_t)tb * B + i].y = pb + lane;
        }
        if (pb + lane == p1 - 1) xse[(size_t)tile * B + i].y = p1;
      }
    }
    const int cnt = min(64, p1 - pb);
    for (int q0 = 0; q0 < cnt; q0 += UN) {
      int k[UN];
      float v[UN];
      float2 w[UN];
#pragma unroll
      for (int q = 0; q < UN; ++q) {                       // broadcast pair q0 + q to the whole wave
        k[q] = __shfl(kk, q0 + q);
        v[q] = __shfl(myv, q0 + q);
      }
#pragma unroll
      for (int q = 0; q < UN; ++q)
        w[q] = (q0 + q < cnt && k[q] >= 0 && col_ok) ? *(const float2*)(W1 + (size_t)k[q] * H + c0)
                                                    : make_float2(0.f, 0.f);
#pragma unroll
      for (int q = 0; q < UN; ++q) {
        if (q0 + q >= cnt || k[q] < 0) continue;
        if (k[q] <= prev) flags |= SLIDE_FLAG_UNSORTED;
        prev = k[q];
        acc.x = fmaf(v[q], w[q].x, acc.x);
        acc.y = fmaf(v[q], w[q].y, acc.y);
      }
    }
  }
  const float2 r = make_float2(acc.x > 0.f ? acc.x : 0.f, acc.y > 0.f ? acc.y : 0.f);
  if (col_ok) {
    *(float2*)(h + (size_t)i * H + c0) = r;
    if (hvec) { hvec[c0] = r.x; hvec[c0 + 1] = r.y; }
  }
  if (flags && lane == 0 && cb == 0) atomicOr(&ctrl->status, flags);
}

}  // namespace slide
