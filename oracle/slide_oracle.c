/*
 * slide_oracle.c -- plain, slow, step-by-step CPU implementation of one SLIDE
 * training step (sparse-input hidden layer, LSH of the hidden activations,
 * bucket lookup + union with the labels, softmax over the active set, sparse
 * backpropagation, row-sparse Adam, hash-table rebuild).
 *
 * THIS IS TEST INFRASTRUCTURE.  It exists to check the HIP library and to be
 * timed beside it; nothing in the product path may call it.  It shares no code
 * with the HIP library.
 *
 * The method is an approximate (LSH-sampled) training step, so this file takes
 * the algorithm's steps in the order of the paper's Algorithm 1 (retrieve
 * active neurons -> feed forward -> compute errors -> backpropagate -> Adam ->
 * rebuild tables), with the SLIDE phases of Section 2.1 (tables indexed by the
 * weight vectors, queried with the layer input; only retrieved neurons get
 * activations and gradients) and the layer interface of Section 3.6 (a first
 * layer fed by sparse index/value arrays, a second fed by the first layer's
 * activations).  Hyper-parameter names K (hash functions per table) and L
 * (tables) follow Section 4.1.  The paper names DWTA and sparse random
 * projections without defining them; the definitions used here are spelled out
 * at each function.
 *
 * Precision: weights and Adam state are stored in fp32.  Everything that
 * decides an integer (hidden activations feeding the hash codes, the hash
 * codes themselves) is computed in fp32 in one fixed order so that another
 * fp32 implementation can reproduce it bit for bit.  Logits, softmax, loss,
 * gradients and the Adam arithmetic are computed in fp64.
 *
 * Every function is pinned by tests/test_oracle_*.py; none is "parity unpinned"
 * except the multi-step loss trajectory (no published curve exists for it).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_SIMHASH 0
#define ORC_DWTA 1

typedef struct {
  int32_t kind;              /* ORC_SIMHASH or ORC_DWTA                                  */
  int32_t H, K, L;           /* vector length, hash functions per table, tables           */
  int32_t m;                 /* DWTA bin size (power of two)                              */
  int32_t S;                 /* SimHash: coordinates per projection                       */
  const int32_t* dwta_perm;  /* [ceil(K*L / (H/m))][H] permutations of 0..H-1             */
  const int32_t* srp_idx;    /* [K*L][S] ascending coordinates                            */
  const int8_t* srp_sign;    /* [K*L][S] +1 / -1                                          */
  uint32_t dens_a, dens_b;   /* odd multipliers of the densification probe                */
} orc_hash;

static int ilog2(int x) { int b = 0; while ((1 << b) < x) ++b; return b; }

/* ------------------------------------------------------------------------------------
 * Hidden layer (Section 3.6, feed-forward of the first kind: sparse index/value arrays).
 *   h[i][u] = max(0, b1[u] + sum_k x_ik * W1[k][u])
 * fp32, one fused multiply-add per non-zero, non-zeros taken in storage order
 * (ascending feature index).  W1 is [D][H] row-major.
 * ------------------------------------------------------------------------------------ */
int orc_hidden_forward(int32_t B, int64_t D, int32_t H, const int32_t* indptr,
                       const int32_t* idx, const float* val, const float* W1,
                       const float* b1, float* h) {
  for (int32_t i = 0; i < B; ++i)
    for (int32_t p = indptr[i]; p < indptr[i + 1]; ++p)
      if (idx[p] < 0 || idx[p] >= D) return -1;
#pragma omp parallel for schedule(static)
  for (int32_t i = 0; i < B; ++i) {
    for (int32_t u = 0; u < H; ++u) {
      float acc = b1[u];
      for (int32_t p = indptr[i]; p < indptr[i + 1]; ++p)
        acc = fmaf(val[p], W1[(int64_t)idx[p] * H + u], acc);
      h[(int64_t)i * H + u] = acc > 0.0f ? acc : 0.0f;
    }
  }
  return 0;
}

/* ------------------------------------------------------------------------------------
 * Elementary hashes and table codes of a vector v in R^H (Section 4.1 names the two
 * families; the same functions hash rows of W2 when tables are built and hidden
 * activations when they are queried, Section 3.1).
 *
 * SimHash / sparse random projection, bit e: acc = 0; for s = 0..S-1 in order
 *   acc = acc + v[idx[e][s]]  (sign +1)   or   acc - v[idx[e][s]]  (sign -1)
 * in fp32; bit = (acc > 0).  code_t = sum_k bit[t*K+k] << k.
 *
 * DWTA, elementary hash e = q*P + b (P = H/m bins per permutation q):
 *   the bin holds coordinates perm[q][b*m + p], p = 0..m-1; raw[e] = position p of the
 *   largest value among the bin's non-zero, non-NaN entries (strictly larger wins, so
 *   ties keep the lowest p); a bin with no such entry is empty (raw = -1).
 *   Densification of an empty e: for t = 1..100,
 *     u = dens_a*(e+1) + dens_b*t  (mod 2^32);  e2 = (u >> 8) mod NH;
 *   the first e2 whose raw bin is non-empty lends its value; none -> 0.
 *   code_t = sum_k val[t*K+k] << (k*log2 m).
 * ------------------------------------------------------------------------------------ */
static void hash_one(const orc_hash* hc, const float* v, int* raw, uint32_t* codes) {
  const int NH = hc->K * hc->L;
  if (hc->kind == ORC_SIMHASH) {
    for (int e = 0; e < NH; ++e) {
      float acc = 0.0f;
      for (int s = 0; s < hc->S; ++s) {
        float x = v[hc->srp_idx[(int64_t)e * hc->S + s]];
        if (hc->srp_sign[(int64_t)e * hc->S + s] > 0) acc = acc + x; else acc = acc - x;
      }
      raw[e] = acc > 0.0f ? 1 : 0;
    }
    for (int t = 0; t < hc->L; ++t) {
      uint32_t c = 0;
      for (int k = 0; k < hc->K; ++k) c |= (uint32_t)raw[t * hc->K + k] << k;
      codes[t] = c;
    }
    return;
  }
  const int m = hc->m, P = hc->H / m, lg = ilog2(m);
  for (int e = 0; e < NH; ++e) {
    const int q = e / P, b = e % P;
    const int32_t* coord = hc->dwta_perm + (int64_t)q * hc->H + (int64_t)b * m;
    int best_p = -1;
    float best = 0.0f;
    for (int p = 0; p < m; ++p) {
      float x = v[coord[p]];
      if (x != 0.0f && !isnan(x) && (best_p < 0 || x > best)) { best_p = p; best = x; }
    }
    raw[e] = best_p;
  }
  for (int t = 0; t < hc->L; ++t) {
    uint32_t c = 0;
    for (int k = 0; k < hc->K; ++k) {
      const int e = t * hc->K + k;
      int val = raw[e];
      if (val < 0) {
        val = 0;
        for (uint32_t tr = 1; tr <= 100; ++tr) {
          uint32_t u = hc->dens_a * (uint32_t)(e + 1) + hc->dens_b * tr;
          int e2 = (int)((u >> 8) % (uint32_t)NH);
          if (raw[e2] >= 0) { val = raw[e2]; break; }
        }
      }
      c |= (uint32_t)val << (k * lg);
    }
    codes[t] = c;
  }
}

int orc_hash_codes(const orc_hash* hc, const float* V, int64_t rows, uint32_t* codes) {
  const int NH = hc->K * hc->L;
  if (hc->kind == ORC_DWTA && (hc->H % hc->m != 0 || (1 << ilog2(hc->m)) != hc->m)) return -1;
#pragma omp parallel
  {
    int* raw = (int*)malloc(sizeof(int) * (size_t)NH);
#pragma omp for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
      hash_one(hc, V + r * hc->H, raw, codes + r * hc->L);
    free(raw);
  }
  return 0;
}

/* ------------------------------------------------------------------------------------
 * Hash tables (Section 2.1 phase 1 and Algorithm 1, the table-construction step before the
 * loop; rebuilt on a schedule, Section 3.1).  For table t and code c the bucket is the set
 * of neurons j with code_t(W2[j,:]) = c, stored ascending by id.  A bucket keeps at most
 * C members: the C smallest keys, key = j (policy 0) or key = (prio(j,t,r), j) (policy 1)
 * with   u = prio_a*(j+1) + prio_b*(t*65537 + r + 1); u ^= u >> 15; u *= prio_a; u ^= u >> 13
 * (mod 2^32), r = number of rebuilds so far.  Kept members are then stored ascending by id.
 * ------------------------------------------------------------------------------------ */
typedef struct {
  int32_t L, C;
  int64_t N;
  int64_t* cnt;       /* [L] kept entries per table                   */
  uint32_t** kcode;   /* [L][cnt] codes, ascending                    */
  int32_t** kid;      /* [L][cnt] ids, ascending inside equal codes   */
  int64_t overflowed; /* buckets that had more than C members         */
} orc_tables;

static int cmp_u64(const void* a, const void* b) {
  uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}
static int cmp_i32(const void* a, const void* b) {
  int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
  return x < y ? -1 : (x > y ? 1 : 0);
}

static uint32_t prio(uint32_t j, uint32_t t, uint32_t r, uint32_t pa, uint32_t pb) {
  uint32_t u = pa * (j + 1u) + pb * (t * 65537u + r + 1u);
  u ^= u >> 15; u *= pa; u ^= u >> 13;
  return u;
}

void orc_tables_free(orc_tables* T) {
  if (!T) return;
  for (int t = 0; t < T->L; ++t) { free(T->kcode[t]); free(T->kid[t]); }
  free(T->kcode); free(T->kid); free(T->cnt); free(T);
}

/* codes: [N][L] as produced by orc_hash_codes on the rows of W2. */
orc_tables* orc_tables_build(const uint32_t* codes, int64_t N, int32_t L, int32_t C,
                             int32_t policy, uint32_t r, uint32_t prio_a, uint32_t prio_b) {
  orc_tables* T = (orc_tables*)calloc(1, sizeof(orc_tables));
  T->L = L; T->C = C; T->N = N;
  T->cnt = (int64_t*)calloc((size_t)L, sizeof(int64_t));
  T->kcode = (uint32_t**)calloc((size_t)L, sizeof(uint32_t*));
  T->kid = (int32_t**)calloc((size_t)L, sizeof(int32_t*));
  int64_t over = 0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : over)
  for (int32_t t = 0; t < L; ++t) {
    uint64_t* key = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(N > 0 ? N : 1));
    for (int64_t j = 0; j < N; ++j) key[j] = ((uint64_t)codes[j * L + t] << 32) | (uint64_t)j;
    qsort(key, (size_t)N, sizeof(uint64_t), cmp_u64); /* by code, then by id */
    uint32_t* kc = (uint32_t*)malloc(sizeof(uint32_t) * (size_t)(N > 0 ? N : 1));
    int32_t* ki = (int32_t*)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    int64_t out = 0, a = 0;
    while (a < N) {
      int64_t b = a;
      const uint32_t c = (uint32_t)(key[a] >> 32);
      while (b < N && (uint32_t)(key[b] >> 32) == c) ++b;
      const int64_t s = b - a;
      if (s <= C) {
        for (int64_t q = a; q < b; ++q) { kc[out] = c; ki[out] = (int32_t)(key[q] & 0xffffffffu); ++out; }
      } else {
        ++over;
        uint64_t* pk = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)s);
        for (int64_t q = a; q < b; ++q) {
          uint32_t j = (uint32_t)(key[q] & 0xffffffffu);
          uint32_t pr = policy == 0 ? 0u : prio(j, (uint32_t)t, r, prio_a, prio_b);
          pk[q - a] = ((uint64_t)pr << 32) | j;
        }
        qsort(pk, (size_t)s, sizeof(uint64_t), cmp_u64); /* by (priority, id) */
        int32_t* keep = (int32_t*)malloc(sizeof(int32_t) * (size_t)C);
        for (int q = 0; q < C; ++q) keep[q] = (int32_t)(pk[q] & 0xffffffffu);
        qsort(keep, (size_t)C, sizeof(int32_t), cmp_i32);
        for (int q = 0; q < C; ++q) { kc[out] = c; ki[out] = keep[q]; ++out; }
        free(keep); free(pk);
      }
      a = b;
    }
    T->cnt[t] = out;
    T->kcode[t] = kc; T->kid[t] = ki;
    free(key);
  }
  T->overflowed = over;
  return T;
}

int64_t orc_tables_overflowed(const orc_tables* T) { return T->overflowed; }
int64_t orc_tables_entries(const orc_tables* T, int32_t t) { return T->cnt[t]; }

/* Copies bucket (t, code) into out (capacity cap); returns its size. */
int32_t orc_tables_bucket(const orc_tables* T, int32_t t, uint32_t code, int32_t* out, int32_t cap) {
  const uint32_t* kc = T->kcode[t];
  int64_t lo = 0, hi = T->cnt[t];
  while (lo < hi) { int64_t mid = (lo + hi) / 2; if (kc[mid] < code) lo = mid + 1; else hi = mid; }
  int32_t n = 0;
  while (lo < T->cnt[t] && kc[lo] == code) { if (n < cap) out[n] = T->kid[t][lo]; ++n; ++lo; }
  return n;
}

/* Order-sensitive fingerprint of the whole table set (schedule tests). */
uint64_t orc_tables_fingerprint(const orc_tables* T) {
  uint64_t f = 1469598103934665603ull;
  for (int t = 0; t < T->L; ++t)
    for (int64_t q = 0; q < T->cnt[t]; ++q) {
      f = (f ^ T->kcode[t][q]) * 1099511628211ull;
      f = (f ^ (uint32_t)T->kid[t][q]) * 1099511628211ull;
    }
  return f;
}

/* ------------------------------------------------------------------------------------
 * Active sets (Algorithm 1, the retrieval step of the loop body; Figure 1: the union of the
 * neurons retrieved from every table).  AS_i = sorted(set(union_t bucket_t(code_t(h_i))) + set(Y_i));
 * is_label marks the members of Y_i.  With include_labels = 0 (prediction) Y_i is left out.
 * A label entry outside [0, N) names no neuron of this layer: it is left out of Y_i (as if it were
 * not in the batch) and counted in *n_bad_labels.
 * Pass as_ids = NULL to obtain only as_ptr (sizes); as_ptr has B+1 entries.
 * ------------------------------------------------------------------------------------ */
int orc_active_sets(const orc_tables* T, const uint32_t* codes /*[B][L]*/, int32_t B,
                    const int32_t* y_indptr, const int32_t* y_idx, int32_t include_labels,
                    int64_t* as_ptr, int32_t* as_ids, uint8_t* is_label, int64_t* n_candidates,
                    int64_t* n_bad_labels) {
  int64_t cand_total = 0, bad = 0;
  const int fill = as_ids != NULL;
  if (!fill) as_ptr[0] = 0;
  for (int32_t i = 0; i < B; ++i) {
    const int32_t nl = include_labels ? y_indptr[i + 1] - y_indptr[i] : 0;
    int32_t* buf = (int32_t*)malloc(sizeof(int32_t) * ((size_t)T->L * (size_t)T->C + (size_t)nl + 1));
    int64_t n = 0;
    for (int32_t t = 0; t < T->L; ++t)
      n += orc_tables_bucket(T, t, codes[(int64_t)i * T->L + t], buf + n, T->C);
    cand_total += n;
    for (int32_t q = 0; q < nl; ++q) {
      int32_t y = y_idx[y_indptr[i] + q];
      if (y < 0 || y >= T->N) { ++bad; continue; }
      buf[n++] = y;
    }
    qsort(buf, (size_t)n, sizeof(int32_t), cmp_i32);
    int64_t u = 0;
    for (int64_t q = 0; q < n; ++q) if (q == 0 || buf[q] != buf[q - 1]) buf[u++] = buf[q];
    if (!fill) {
      as_ptr[i + 1] = as_ptr[i] + u;
    } else {
      if (as_ptr[i + 1] - as_ptr[i] != u) { free(buf); return -2; }
      memcpy(as_ids + as_ptr[i], buf, sizeof(int32_t) * (size_t)u);
      memset(is_label + as_ptr[i], 0, (size_t)u);
      for (int32_t q = 0; q < nl; ++q) {
        int32_t y = y_idx[y_indptr[i] + q];
        if (y < 0 || y >= T->N) continue;
        int64_t lo = 0, hi = u;
        while (lo < hi) { int64_t mid = (lo + hi) / 2; if (buf[mid] < y) lo = mid + 1; else hi = mid; }
        is_label[as_ptr[i] + lo] = 1;
      }
    }
    free(buf);
  }
  if (n_candidates) *n_candidates = cand_total;
  if (n_bad_labels) *n_bad_labels = bad;
  return 0;
}

/* ------------------------------------------------------------------------------------
 * Output layer on the active set (Section 2.1: activations of retrieved neurons only,
 * all others are exactly zero / untouched; Algorithm 1, the error computation).
 *   z_ij = b2[j] + sum_u W2[j][u]*h[i][u]                  j in AS_i
 *   p_ij = softmax over AS_i only
 *   y_ij = 1/|Y_i| for labels (distinct), 0 otherwise
 *   loss_i = -sum_{j in Y_i} y_ij * log p_ij
 *   delta_ij = (p_ij - y_ij) / B          (gradient of the batch-mean loss w.r.t. z_ij)
 *   dh[i][u] = (h[i][u] > 0) ? sum_j delta_ij * W2[j][u] : 0
 * A sample with no label contributes nothing: delta = 0, loss_i = 0 (its p is still returned).
 * All arithmetic in fp64 on the fp32 inputs.
 * ------------------------------------------------------------------------------------ */
int orc_output_forward_backward(int32_t B, int32_t H, const float* h, const int64_t* as_ptr,
                                const int32_t* as_ids, const uint8_t* is_label,
                                const float* W2, const float* b2, double* z, double* p,
                                double* delta, double* loss_i, double* dh) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int32_t i = 0; i < B; ++i) {
    const int64_t a = as_ptr[i], b = as_ptr[i + 1];
    const float* hi = h + (int64_t)i * H;
    double* dhi = dh + (int64_t)i * H;
    for (int32_t u = 0; u < H; ++u) dhi[u] = 0.0;
    loss_i[i] = 0.0;
    if (b == a) continue;
    double zmax = -INFINITY;
    int64_t ny = 0;
    for (int64_t q = a; q < b; ++q) {
      const float* w = W2 + (int64_t)as_ids[q] * H;
      double acc = (double)b2[as_ids[q]];
      for (int32_t u = 0; u < H; ++u) acc += (double)w[u] * (double)hi[u];
      z[q] = acc;
      if (acc > zmax) zmax = acc;
      ny += is_label[q] ? 1 : 0;
    }
    double s = 0.0;
    for (int64_t q = a; q < b; ++q) s += exp(z[q] - zmax);
    for (int64_t q = a; q < b; ++q) p[q] = exp(z[q] - zmax) / s;
    for (int64_t q = a; q < b; ++q) {
      if (ny == 0) { delta[q] = 0.0; continue; }
      const double y = is_label[q] ? 1.0 / (double)ny : 0.0;
      if (is_label[q]) loss_i[i] -= y * (z[q] - zmax - log(s));
      delta[q] = (p[q] - y) / (double)B;
    }
    for (int64_t q = a; q < b; ++q) {
      const float* w = W2 + (int64_t)as_ids[q] * H;
      for (int32_t u = 0; u < H; ++u) dhi[u] += delta[q] * (double)w[u];
    }
    for (int32_t u = 0; u < H; ++u) if (!(hi[u] > 0.0f)) dhi[u] = 0.0;
  }
  return 0;
}

static int64_t find_i32(const int32_t* a, int64_t n, int32_t x) {
  int64_t lo = 0, hi = n;
  while (lo < hi) { int64_t mid = (lo + hi) / 2; if (a[mid] < x) lo = mid + 1; else hi = mid; }
  return (lo < n && a[lo] == x) ? lo : -1;
}

/* Sparse backpropagation into the output layer's parameters (Algorithm 1, backward):
 *   gW2[j][u] = sum_{i: j in AS_i} delta_ij * h[i][u],   gb2[j] = sum_i delta_ij
 * for the U distinct touched neurons uniq[0..U) (ascending); sums run in sample order. */
int orc_output_grads(int32_t B, int32_t H, const float* h, const int64_t* as_ptr,
                     const int32_t* as_ids, const double* delta, int64_t U, const int32_t* uniq,
                     double* gW2 /*[U][H]*/, double* gb2 /*[U]*/) {
  memset(gW2, 0, sizeof(double) * (size_t)U * (size_t)H);
  memset(gb2, 0, sizeof(double) * (size_t)U);
  for (int32_t i = 0; i < B; ++i)
    for (int64_t q = as_ptr[i]; q < as_ptr[i + 1]; ++q) {
      const int64_t r = find_i32(uniq, U, as_ids[q]);
      if (r < 0) return -1;
      gb2[r] += delta[q];
      for (int32_t u = 0; u < H; ++u) gW2[r * H + u] += delta[q] * (double)h[(int64_t)i * H + u];
    }
  return 0;
}

/* Backpropagation into the hidden layer's parameters:
 *   gW1[k][u] = sum_{i: x_ik != stored} x_ik * dh[i][u],   gb1[u] = sum_i dh[i][u]
 * for the U1 distinct features present in the batch, uniq1 ascending. */
int orc_hidden_grads(int32_t B, int32_t H, const int32_t* indptr, const int32_t* idx,
                     const float* val, const double* dh, int64_t U1, const int32_t* uniq1,
                     double* gW1 /*[U1][H]*/, double* gb1 /*[H]*/) {
  memset(gW1, 0, sizeof(double) * (size_t)U1 * (size_t)H);
  memset(gb1, 0, sizeof(double) * (size_t)H);
  for (int32_t i = 0; i < B; ++i) {
    for (int32_t u = 0; u < H; ++u) gb1[u] += dh[(int64_t)i * H + u];
    for (int32_t p = indptr[i]; p < indptr[i + 1]; ++p) {
      const int64_t r = find_i32(uniq1, U1, idx[p]);
      if (r < 0) return -1;
      for (int32_t u = 0; u < H; ++u) gW1[r * H + u] += (double)val[p] * dh[(int64_t)i * H + u];
    }
  }
  return 0;
}

/* ------------------------------------------------------------------------------------
 * Row-sparse Adam (Algorithm 1, the optimizer step after the batch; Section 3.5: every weight and
 * bias carries a momentum and a velocity value; constants of Section 4.1).  Only the
 * listed rows change; t is the global 1-based step:
 *   m = b1*m + (1-b1)*g;  v = b2*v + (1-b2)*g*g;
 *   w = w - lr * (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
 * fp64 arithmetic, fp32 storage.  rowlen = H for a matrix, 1 for a bias vector.
 * ------------------------------------------------------------------------------------ */
int orc_adam_rows(float* W, float* M, float* V, int32_t rowlen, int64_t U, const int32_t* ids,
                  const double* g /*[U][rowlen]*/, double lr, double beta1, double beta2,
                  double eps, int64_t t) {
  const double bc1 = 1.0 - pow(beta1, (double)t), bc2 = 1.0 - pow(beta2, (double)t);
  for (int64_t r = 0; r < U; ++r) {
    const int64_t base = (int64_t)ids[r] * rowlen;
    for (int32_t u = 0; u < rowlen; ++u) {
      const double gg = g[r * rowlen + u];
      const double m = beta1 * (double)M[base + u] + (1.0 - beta1) * gg;
      const double v = beta2 * (double)V[base + u] + (1.0 - beta2) * gg * gg;
      const double w = (double)W[base + u] - lr * (m / bc1) / (sqrt(v / bc2) + eps);
      M[base + u] = (float)m; V[base + u] = (float)v; W[base + u] = (float)w;
    }
  }
  return 0;
}

int orc_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
