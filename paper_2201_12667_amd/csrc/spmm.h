// Sparse-input hidden layer of one sample (paper Section 3.6: the first layer is fed by index /
// value arrays), as a device function so that it can run as a kernel of its own or inside the
// lookup workgroup of the sample.
#pragma once
#include "slide_internal.h"

namespace slide {

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
