// Host side of the C ABI: validation, workspace layout, kernel sequencing on the caller's stream.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "slide_internal.h"

using namespace slide;

// Scratch memory of slide_predict_static, the one entry point that uses no caller-supplied workspace:
// a fixed array in the library's device image (every GPU the library runs on holds its own copy until
// the process ends).  Host code never uses the array's name as an address: each device's address is
// looked up once, in slide_init, with that device current, and kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = (size_t)SLIDE_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_last_error;

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];      // per device: address of `scratch` on that device
std::mutex g_scratch_mu;

// Address of the static scratch array on the current device (looked up on first use per device).
hipError_t static_scratch_of_current_device(int* dev_out, void** ptr_out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *dev_out = dev;
  *ptr_out = g_scratch_ptr[dev];
  return hipSuccess;
}

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Entries of the byte-offset copy of the hash parameters (see hash_offsets).
static size_t hash_offset_count(const slide_config* c) {
  if (c->hash_kind == SLIDE_HASH_DWTA) return (size_t)c->K * c->L * c->dwta_bin;
  return (size_t)c->K * c->L * simhash_offset_stride(c->srp_nnz);
}

struct Layout {
  // derived sizes
  int Bmax, Bpad, H, L, K, C, TW, TWF, NWpad, NT, NT2, NT1, DWpad, bits, PS;
  int64_t dense_chunk;   // neurons per chunk of the dense prediction pass
  int64_t N, D, Amax, max_chunks, U2max, U1max, P1max, long2, long1;
  uint32_t nb, wl_cap;
  size_t hash_words;
  // workspace offsets
  size_t ctrl, hashw, hashoff, xse, zc, best, cand, ccnt, h, dh, codes, act, rankT, cnt, ny, ncand, as_base, chunk_ptr, tile_nu2, tile_nu1, longlist2, longlist1, as_ids,
      ylist, z, delta, partials, msum, loss_i, umeta2, pairs2, umeta1, pairs1, codes_t, entries, bh, pbase, worklist, touched, touched_rows, ws_total;
  // tables offsets
  size_t t_off, t_ids, tables_total;
};

int ilog2_exact(int x) {
  int b = 0;
  while ((1 << b) < x) ++b;
  return (1 << b) == x ? b : -1;
}

#define FAIL(code, ...)                                  \
  do {                                                   \
    char buf_[512];                                      \
    snprintf(buf_, sizeof(buf_), __VA_ARGS__);           \
    err = buf_;                                          \
    return code;                                         \
  } while (0)

int make_layout(const slide_config* c, Layout* lo, std::string& err) {
  if (!c) FAIL(SLIDE_EINVAL, "config is NULL");
  if (c->struct_size != sizeof(slide_config) || c->abi_version != SLIDE_ABI_VERSION)
    FAIL(SLIDE_EINVAL, "slide_config size/version mismatch (got %u/%u, want %zu/%u)", c->struct_size,
         c->abi_version, sizeof(slide_config), SLIDE_ABI_VERSION);
  if (c->hidden_dim < 4 || c->hidden_dim > 2048 || c->hidden_dim % 4) FAIL(SLIDE_EINVAL, "hidden_dim must be a multiple of 4 in [4, 2048]");
  if (c->num_classes < 1 || c->num_classes > (int64_t)1 << 30) FAIL(SLIDE_EINVAL, "num_classes out of range");
  if (c->input_dim < 0 || c->input_dim > (int64_t)1 << 30) FAIL(SLIDE_EINVAL, "input_dim out of range");
  if (c->max_batch < 1 || c->max_batch > 2048) FAIL(SLIDE_EINVAL, "max_batch must be in [1, 2048]");
  if (c->K < 1 || c->L < 1 || c->L > 65535) FAIL(SLIDE_EINVAL, "K and L must be positive (L <= 65535)");
  if (c->bucket_cap < 1 || c->bucket_cap > 1024) FAIL(SLIDE_EINVAL, "bucket_cap must be in [1, 1024]");
  if (c->max_labels_per_batch < 0 || c->max_nnz_per_batch < 0) FAIL(SLIDE_EINVAL, "negative batch capacity");
  if (c->input_dim > 0 && c->max_nnz_per_batch < 1) FAIL(SLIDE_EINVAL, "max_nnz_per_batch must be positive in sparse-input mode");
  if (c->overflow_policy != SLIDE_KEEP_LOWEST_ID && c->overflow_policy != SLIDE_KEEP_PRIORITY) FAIL(SLIDE_EINVAL, "unknown overflow_policy");
  if (c->rebuild_every < 0) FAIL(SLIDE_EINVAL, "rebuild_every must be >= 0");
  if (!(c->lr > 0) || !(c->beta1 >= 0 && c->beta1 < 1) || !(c->beta2 >= 0 && c->beta2 < 1) || !(c->eps > 0))
    FAIL(SLIDE_EINVAL, "Adam constants out of range");
  lo->H = c->hidden_dim; lo->L = c->L; lo->K = c->K; lo->C = c->bucket_cap; lo->N = c->num_classes; lo->D = c->input_dim;
  if (c->hash_kind == SLIDE_HASH_DWTA) {
    const int lg = ilog2_exact(c->dwta_bin);
    if (lg < 1 || lg > 4) FAIL(SLIDE_EINVAL, "dwta_bin must be 2, 4, 8 or 16");
    if (c->hidden_dim % c->dwta_bin) FAIL(SLIDE_EINVAL, "hidden_dim must be a multiple of dwta_bin");
    lo->bits = c->K * lg;
    lo->hash_words = (size_t)c->K * c->L * (c->dwta_bin / 2);
  } else if (c->hash_kind == SLIDE_HASH_SIMHASH) {
    if (c->srp_nnz < 1 || c->srp_nnz > c->hidden_dim) FAIL(SLIDE_EINVAL, "srp_nnz must be in [1, hidden_dim]");
    lo->bits = c->K;
    lo->hash_words = (size_t)c->K * c->L * ((c->srp_nnz + 1) / 2);
  } else {
    FAIL(SLIDE_EINVAL, "unknown hash_kind");
  }
  if (lo->bits > 24) FAIL(SLIDE_EINVAL, "hash code wider than 24 bits");
  lo->nb = 1u << lo->bits;
  lo->Bmax = c->max_batch;
  lo->Bpad = (c->max_batch + 63) & ~63;
  int tw = 32;
  while (tw > 4 && tw * lo->Bpad > 8192) tw >>= 1;
  lo->TW = tw;
  lo->TWF = tw;
  lo->NWpad = (int)(((lo->N + 31) / 32 + 31) / 32 * 32);
  lo->NT = lo->NWpad / tw;
  lo->NT2 = lo->NWpad / tw;
  lo->DWpad = (int)(((lo->D + 31) / 32 + 31) / 32 * 32);
  lo->NT1 = lo->DWpad / lo->TWF;
  if (c->sample_budget < 0) FAIL(SLIDE_EINVAL, "sample_budget must be >= 0");
  if (c->incremental_rebuild != 0 && c->incremental_rebuild != 1) FAIL(SLIDE_EINVAL, "incremental_rebuild must be 0 or 1");
  if (c->row_major_mode < SLIDE_ROWS_AUTO || c->row_major_mode > SLIDE_ROWS_ALWAYS) FAIL(SLIDE_EINVAL, "unknown row_major_mode");
  const int64_t per_sample = std::min<int64_t>(std::max<int64_t>((int64_t)c->L * c->bucket_cap, c->sample_budget), lo->N);
  lo->PS = (int)per_sample;
  lo->Amax = (int64_t)c->max_batch * per_sample + c->max_labels_per_batch;
  if (lo->Amax >= ((int64_t)1 << 31) - 64) FAIL(SLIDE_EINVAL, "max_batch * L * bucket_cap does not fit 31 bits");
  if ((int64_t)c->L * lo->N >= ((int64_t)1 << 32)) FAIL(SLIDE_EINVAL, "L * num_classes does not fit 32 bits");
  lo->max_chunks = lo->Amax / kChunk + c->max_batch + 1;
  {
    // the lookup kernel keeps, besides a segment of the per-sample bitmap, 2L + H + NT words and K*L bytes
    // in LDS: that has to leave room for a segment worth sweeping
    const size_t fixed = lookup_fixed_lds(c->L, c->hidden_dim, lo->NT, c->K * c->L);
    if (fixed + (size_t)kLookupMinSegment * 4 > kDeviceLdsBytes)
      FAIL(SLIDE_EINVAL, "L, K*L, hidden_dim and num_classes / tile need %zu bytes of LDS in the lookup kernel; "
                         "%zu are available", fixed + (size_t)kLookupMinSegment * 4, kDeviceLdsBytes);
  }
  lo->U2max = (int64_t)lo->NWpad * 32;
  lo->P1max = c->max_nnz_per_batch;
  if (lo->P1max * kPairRegions + (int64_t)lo->NT1 * 64 >= ((int64_t)1 << 31)) FAIL(SLIDE_EINVAL, "max_nnz_per_batch too large");
  lo->U1max = (int64_t)lo->DWpad * 32;
  lo->long2 = lo->Amax / kLongRow + 1;
  lo->long1 = lo->P1max / kLongRow + 1;
  const int small = std::min(kSmallBucket, c->bucket_cap);
  const uint64_t wl = (uint64_t)c->L * (uint64_t)(lo->N / (small + 1) + 1);
  lo->wl_cap = (uint32_t)std::min<uint64_t>(wl, 0xfffffff0u);

  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  const size_t B = lo->Bmax, H = lo->H, A = (size_t)lo->Amax;
  lo->ctrl = take(sizeof(Ctrl));
  lo->hashw = take(lo->hash_words * 4);
  lo->hashoff = take(hash_offset_count(c) * 4);
  lo->xse = take(lo->D ? B * lo->NT1 * 8 : 0);
  lo->dense_chunk = dense_chunk_neurons(lo->N, lo->Bmax);
  lo->zc = take(B * (size_t)lo->dense_chunk * 4);
  lo->best = take(B * 64 * 8);
  lo->cand = take(B * dense_cand_keys() * 8); lo->ccnt = take(B * dense_counter_words() * 4);
  lo->h = take(lo->D ? B * H * 4 : 0);
  lo->dh = take(B * H * 4);
  lo->codes = take(B * lo->L * 4);
  lo->act = take(B * lo->NWpad * 4);
  lo->rankT = take(B * (lo->NT + 1) * 4);
  lo->cnt = take(B * 4); lo->ny = take(B * 4); lo->ncand = take(B * 4);
  lo->as_base = take(B * 4); lo->chunk_ptr = take((B + 1) * 4);
  lo->tile_nu2 = take((size_t)lo->NT2 * 4); lo->tile_nu1 = take((size_t)lo->NT1 * 4 + 4);
  lo->longlist2 = take((size_t)lo->long2 * 4); lo->longlist1 = take((size_t)lo->long1 * 4);
  lo->as_ids = take(A * 4); lo->ylist = take((size_t)c->max_labels_per_batch * 4 + 4);
  lo->z = take(A * 4); lo->delta = take(A * 4);
  lo->partials = take((size_t)lo->max_chunks * (H + 4) * 4);
  lo->msum = take(B * 8); lo->loss_i = take(B * 4);
  lo->umeta2 = take((size_t)lo->U2max * 16); lo->pairs2 = take(A * 8);
  lo->umeta1 = take((size_t)lo->U1max * 16); lo->pairs1 = take(((size_t)lo->P1max * kPairRegions + (size_t)lo->NT1 * 64) * 8);
  lo->codes_t = take((size_t)lo->L * lo->N * 4); lo->entries = take((size_t)lo->L * lo->N * 4);
  lo->bh = take(tables_bh_words(lo->bits, lo->N, lo->L) * 4);
  lo->pbase = take(tables_pbase_words(lo->bits, lo->N, lo->L) * 4);
  lo->worklist = take((size_t)lo->wl_cap * 8);
  lo->touched = lo->touched_rows = 0;
  if (c->incremental_rebuild) {
    lo->touched = take(((size_t)lo->N + 3) / 4 * 4);
    lo->touched_rows = take((size_t)lo->N * 4);
  }
  lo->ws_total = o;
  o = 0;
  lo->t_off = take((size_t)lo->L * (lo->nb + 1) * 4);
  lo->t_ids = take((size_t)lo->L * lo->N * 4);
  lo->tables_total = o;
  return SLIDE_OK;
}

}  // namespace

struct slide_ctx {
  slide_config cfg;
  slide_buffers buf;
  Layout lo;
  HashDev hd;
  TablesDev td;
  uint32_t prio_a, prio_b;
  size_t lds_limit;
  int num_cus = 256;             // compute units of the device (persistent launches are sized by it)
  int nxcd = 1;                  // accelerator dies (workgroup k of a launch runs on die k % nxcd); 1 = unknown
  int device = -1;               // device that was current at slide_init
  char* static_scratch = nullptr;   // this device's copy of the static scratch array
  int64_t t = 0, r = 0;
  bool built = false;
  bool ever_built = false;       // a build has happened (later ones count as rebuilds)
  bool codes_current = false;    // codes_t holds the codes of W2 under the current hash functions, up to the marked rows
  int last_B = 0;
  int last_labels = 0;           // label entries of the last forward pass (0: prediction)
  uint64_t calls = 0;            // forward passes launched (selects the set of per-call device accumulators)
  const float* last_h = nullptr;
  float* last_dh = nullptr;
  std::string err;
  // per-stage HIP-event timing (slide_profile)
  struct ProfRec { int stage; hipEvent_t a, b; };
  uint32_t prof_mask = 0;
  std::vector<ProfRec> prof_live;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> prof_pool;
  double prof_ms[SLIDE_NUM_STAGES] = {};
  int64_t prof_n[SLIDE_NUM_STAGES] = {};
  char* ws() const { return (char*)buf.workspace; }
  template <typename T> T* at(size_t off) const { return (T*)(ws() + off); }
  Ctrl* ctrl() const { return at<Ctrl>(lo.ctrl); }
};

namespace {

int set_err(slide_ctx* ctx, int code, const char* fmt, ...) {
  char b[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(b, sizeof(b), fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = b; else g_last_error = b;
  return code;
}

#define HIPCHK(ctx, expr)                                                                         \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return set_err(ctx, SLIDE_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

// Runs one stage; with profiling enabled for it, brackets the launch with a pair of events on the
// same stream.
template <typename F>
hipError_t stage(slide_ctx* ctx, int id, hipStream_t s, F&& launch) {
  if (!(ctx->prof_mask & (1u << id))) return launch();
  std::pair<hipEvent_t, hipEvent_t> ev;
  if (!ctx->prof_pool.empty()) {
    ev = ctx->prof_pool.back();
    ctx->prof_pool.pop_back();
  } else {
    hipError_t e = hipEventCreate(&ev.first);
    if (e == hipSuccess) e = hipEventCreate(&ev.second);
    if (e != hipSuccess) return e;
  }
  hipError_t e = hipEventRecord(ev.first, s);
  if (e == hipSuccess) e = launch();
  if (e == hipSuccess) e = hipEventRecord(ev.second, s);
  ctx->prof_live.push_back({id, ev.first, ev.second});
  return e;
}

SpmmArgs make_spmm(slide_ctx* ctx, const slide_batch* b) {
  const Layout& lo = ctx->lo;
  SpmmArgs a{};
  a.D = lo.D; a.H = lo.H; a.nnz_total = b->nnz; a.rows_per_tile = lo.TWF * 32;
  a.x_indptr = b->x_indptr; a.x_indices = b->x_indices; a.x_values = b->x_values;
  a.W1 = ctx->buf.W1; a.b1 = ctx->buf.b1;
  a.h = ctx->at<float>(lo.h); a.xse = ctx->at<int2>(lo.xse);
  return a;
}

ActiveDev make_active(const slide_ctx* c, int B) {
  ActiveDev ad;
  const Layout& lo = c->lo;
  ad.B = B; ad.L = lo.L; ad.C = lo.C; ad.TW = lo.TW; ad.N = lo.N; ad.NWpad = lo.NWpad; ad.NT = lo.NT;
  ad.act = c->at<uint32_t>(lo.act); ad.rankT = c->at<uint32_t>(lo.rankT);
  ad.cnt = c->at<int32_t>(lo.cnt); ad.ny = c->at<int32_t>(lo.ny);
  ad.PS = lo.PS; ad.num_labels = 0;
  ad.budget = 0; ad.fill = 0; ad.sample_seed = c->cfg.sample_seed; ad.step = 0;
  ad.par = 0; ad.nxcd = c->nxcd; ad.write_act = 0;
  ad.as_base = c->at<int32_t>(lo.as_base); ad.chunk_ptr = c->at<int32_t>(lo.chunk_ptr);
  ad.as_ids = c->at<int32_t>(lo.as_ids); ad.ylist = c->at<int32_t>(lo.ylist);
  return ad;
}

int check_batch(slide_ctx* ctx, const slide_batch* b, bool need_labels) {
  const slide_config& c = ctx->cfg;
  if (!b) return set_err(ctx, SLIDE_EINVAL, "batch is NULL");
  if (b->batch < 1 || b->batch > c.max_batch) return set_err(ctx, SLIDE_EINVAL, "batch size %d outside [1, max_batch=%d]", b->batch, c.max_batch);
  if (c.input_dim > 0) {
    if (!b->x_indptr || (b->nnz > 0 && (!b->x_indices || !b->x_values))) return set_err(ctx, SLIDE_EINVAL, "sparse-input mode needs x_indptr/x_indices/x_values");
    if (b->nnz < 0 || b->nnz > c.max_nnz_per_batch) return set_err(ctx, SLIDE_ENOMEM, "batch nnz %d exceeds max_nnz_per_batch %d", b->nnz, c.max_nnz_per_batch);
  } else if (!b->hidden) {
    return set_err(ctx, SLIDE_EINVAL, "dense-hidden mode needs batch->hidden");
  }
  if (need_labels) {
    if (!b->y_indptr || (b->num_labels > 0 && !b->y_indices)) return set_err(ctx, SLIDE_EINVAL, "training needs y_indptr/y_indices");
    if (b->num_labels < 0 || b->num_labels > c.max_labels_per_batch) return set_err(ctx, SLIDE_ENOMEM, "batch labels %d exceed max_labels_per_batch %d", b->num_labels, c.max_labels_per_batch);
  }
  return SLIDE_OK;
}

// Whether this call's float kernels walk the incidences row-major (see slide_config::row_major_mode).
// Automatic rule: the tables return about L * min(C, N / 2^bits) neurons per sample; when the batch's
// total is several times the layer, a touched row belongs to several samples.
bool row_major(const slide_ctx* ctx, int batch) {
  const slide_config& c = ctx->cfg;
  if (c.row_major_mode == SLIDE_ROWS_NEVER) return false;
  if (c.row_major_mode == SLIDE_ROWS_ALWAYS) return true;
  const int64_t per_bucket = std::max<int64_t>(1, ctx->lo.N >> ctx->lo.bits);
  const int64_t est = (int64_t)batch * c.L * std::min<int64_t>(c.bucket_cap, per_bucket);
  return est >= 4 * ctx->lo.N;
}

// Hidden activations, hash codes + active sets, and the logits pass; t1 and t2 (training only) are
// the row-list constructions for the features and the active sets that ride in the logits launch (the
// bit-matrix pointers of t2 are filled in here).
int forward_common(slide_ctx* ctx, const slide_batch* b, bool with_labels, hipStream_t s, ActiveDev* ad_out,
                   const TransposeArgs& t1, TransposeArgs t2, bool write_act) {
  const Layout& lo = ctx->lo;
  const int B = b->batch;
  const float* h = b->hidden;
  SpmmArgs sp{};
  if (lo.D > 0) {
    sp = make_spmm(ctx, b);
    h = sp.h;
    // One lookup workgroup per sample holds a compute unit (its bitmap fills the LDS): while the batch
    // fits the machine in one round the hidden layer rides in it; a larger batch would pay the hidden
    // layer's latency once per round, so it gets its own, fully parallel launch.
    if (B > ctx->num_cus) {
      HIPCHK(ctx, stage(ctx, SLIDE_STAGE_HIDDEN, s, [&] { return launch_spmm_relu(B, sp, ctx->ctrl(), s); }));
      sp = SpmmArgs{};
    }
  }
  ctx->last_h = h;
  ctx->last_B = B;
  ctx->last_labels = with_labels ? b->num_labels : 0;
  uint32_t* codes = ctx->at<uint32_t>(lo.codes);
  ActiveDev ad = make_active(ctx, B);
  ad.num_labels = with_labels ? b->num_labels : 0;
  ad.par = (int)(ctx->calls++ & 1);
  ad.nxcd = ctx->nxcd;
  ad.write_act = write_act ? 1 : 0;                    // (row lists from the bitmaps: see slide_train_step)
  if (with_labels) { ad.budget = ctx->cfg.sample_budget; ad.fill = ctx->cfg.sample_fill; ad.step = (uint32_t)(ctx->t + 1); }
  int32_t* ncand = ctx->at<int32_t>(lo.ncand);
  HIPCHK(ctx, stage(ctx, SLIDE_STAGE_LOOKUP, s, [&] {
    return launch_lookup_union(ad, ctx->hd, h, sp, ctx->td, codes, b->y_indptr, b->y_indices, with_labels ? 1 : 0,
                               ncand, ctx->ctrl(), ctx->lds_limit, s); }));
  t2.ids = ad.as_ids; t2.rankT = ad.rankT; t2.as_base = ad.as_base;
  HIPCHK(ctx, stage(ctx, SLIDE_STAGE_FORWARD, s, [&] {
    return launch_forward(ad, lo.H, h, ctx->buf.W2, ctx->buf.b2, ctx->at<float>(lo.z),
                          ctx->at<float>(lo.partials), ctx->ctrl(), t1, t2, true, ctx->num_cus, s); }));
  *ad_out = ad;
  return SLIDE_OK;
}

// scheduled: the build is the training step's own, so the rows marked by the steps since the last
// build are the only ones whose weights (hence codes) can differ from what codes_t holds.
int do_build(slide_ctx* ctx, hipStream_t s, bool scheduled) {
  const Layout& lo = ctx->lo;
  const bool inc = ctx->cfg.incremental_rebuild != 0;
  const bool only_touched = inc && scheduled && ctx->codes_current;
  HIPCHK(ctx, stage(ctx, SLIDE_STAGE_REBUILD, s, [&] {
    return launch_build_tables(ctx->hd, ctx->td, ctx->buf.W2, ctx->at<uint32_t>(lo.codes_t),
                               ctx->at<uint32_t>(lo.entries), ctx->at<uint32_t>(lo.bh), ctx->at<uint32_t>(lo.pbase),
                               ctx->at<uint64_t>(lo.worklist), lo.wl_cap, ctx->ctrl(), ctx->cfg.overflow_policy,
                               (uint32_t)ctx->r, ctx->prio_a, ctx->prio_b,
                               inc ? ctx->at<uint8_t>(lo.touched) : nullptr,
                               inc ? ctx->at<int32_t>(lo.touched_rows) : nullptr, only_touched, s); }));
  ctx->codes_current = true;
  return SLIDE_OK;
}

}  // namespace

extern "C" {

int slide_query_memory(const slide_config* cfg, slide_mem_req* out) {
  Layout lo;
  std::string err;
  if (!out) { g_last_error = "out is NULL"; return SLIDE_EINVAL; }
  const int rc = make_layout(cfg, &lo, err);
  if (rc != SLIDE_OK) { g_last_error = err; return rc; }
  out->tables_bytes = lo.tables_total;
  out->workspace_bytes = lo.ws_total;
  return SLIDE_OK;
}

// The packed coordinate words as byte offsets into the LDS tile of the row-tile hash kernel.  A
// SimHash bit owns simhash_offset_stride(S) entries; the ones past S point at the row of zeros.
static std::vector<uint32_t> hash_offsets(const slide_config* cfg, const std::vector<uint32_t>& words) {
  const uint32_t pitch = (uint32_t)hash_tile_pitch(cfg->hidden_dim) * 4u;
  std::vector<uint32_t> offs(hash_offset_count(cfg));
  if (cfg->hash_kind == SLIDE_HASH_DWTA) {
    for (size_t w = 0; w < words.size(); ++w) {
      offs[2 * w] = (words[w] & 0xffffu) * pitch;
      offs[2 * w + 1] = (words[w] >> 16) * pitch;
    }
  } else {
    const int S = cfg->srp_nnz, half = (S + 1) / 2, So = simhash_offset_stride(S);
    const uint32_t zero_cell = (uint32_t)cfg->hidden_dim * pitch;
    const size_t NH = (size_t)cfg->K * cfg->L;
    for (size_t e = 0; e < NH; ++e)
      for (int q = 0; q < So; ++q) {
        const uint32_t v = q < S ? (words[e * half + q / 2] >> (16 * (q & 1))) & 0xffffu : 0u;
        offs[e * So + q] = q < S ? (((v & 0x7fffu) * pitch) | ((v & 0x8000u) << 16)) : zero_cell;
      }
  }
  return offs;
}

// Hash-function parameters -> packed 16-bit coordinate words (validated).
static int pack_hash_params(const slide_config* cfg, const Layout& lo, const slide_hash_params* hp,
                            std::vector<uint32_t>& words) {
  const int H = cfg->hidden_dim, NH = cfg->K * cfg->L;
  words.assign(lo.hash_words, 0u);
  if (cfg->hash_kind == SLIDE_HASH_DWTA) {
    if (!hp->dwta_perm) return set_err(nullptr, SLIDE_EINVAL, "dwta_perm is NULL");
    const int m = cfg->dwta_bin, P = H / m;
    std::vector<uint8_t> seen(H);
    const int NP = (NH + P - 1) / P;
    for (int q = 0; q < NP; ++q) {
      std::fill(seen.begin(), seen.end(), 0);
      for (int c = 0; c < H; ++c) {
        const int v = hp->dwta_perm[(size_t)q * H + c];
        if (v < 0 || v >= H || seen[v]) return set_err(nullptr, SLIDE_EINVAL, "dwta_perm row %d is not a permutation of 0..H-1", q);
        seen[v] = 1;
      }
    }
    for (int e = 0; e < NH; ++e) {
      const int q = e / P, b = e % P;
      for (int p = 0; p < m; ++p) {
        const uint32_t c = (uint32_t)hp->dwta_perm[(size_t)q * H + (size_t)b * m + p];
        words[(size_t)e * (m / 2) + p / 2] |= c << (16 * (p & 1));
      }
    }
  } else {
    if (!hp->srp_idx || !hp->srp_sign) return set_err(nullptr, SLIDE_EINVAL, "srp_idx / srp_sign is NULL");
    const int S = cfg->srp_nnz, half = (S + 1) / 2;
    for (int e = 0; e < NH; ++e)
      for (int s = 0; s < S; ++s) {
        const int c = hp->srp_idx[(size_t)e * S + s];
        const int sg = hp->srp_sign[(size_t)e * S + s];
        if (c < 0 || c >= H || (sg != 1 && sg != -1)) return set_err(nullptr, SLIDE_EINVAL, "bad sparse-projection entry (bit %d, position %d)", e, s);
        const uint32_t v = (uint32_t)c | (sg < 0 ? 0x8000u : 0u);
        words[(size_t)e * half + s / 2] |= v << (16 * (s & 1));
      }
  }
  if (!(hp->dens_a & 1u) || !(hp->dens_b & 1u) || !(hp->prio_a & 1u) || !(hp->prio_b & 1u))
    return set_err(nullptr, SLIDE_EINVAL, "dens_a, dens_b, prio_a, prio_b must be odd");

  return SLIDE_OK;
}

int slide_init(const slide_config* cfg, const slide_buffers* buf, const slide_hash_params* hp, slide_ctx** out) {
  if (!out) return set_err(nullptr, SLIDE_EINVAL, "out is NULL");
  *out = nullptr;
  Layout lo;
  std::string err;
  int rc = make_layout(cfg, &lo, err);
  if (rc != SLIDE_OK) { g_last_error = err; return rc; }
  if (!buf || !hp) return set_err(nullptr, SLIDE_EINVAL, "buffers / hash params are NULL");
  if (!buf->W2 || !buf->b2 || !buf->mW2 || !buf->vW2 || !buf->mb2 || !buf->vb2)
    return set_err(nullptr, SLIDE_EINVAL, "output-layer parameter / Adam-state pointer is NULL");
  if (cfg->input_dim > 0 && (!buf->W1 || !buf->b1 || !buf->mW1 || !buf->vW1 || !buf->mb1 || !buf->vb1))
    return set_err(nullptr, SLIDE_EINVAL, "hidden-layer parameter / Adam-state pointer is NULL");
  const void* al[] = {buf->W1, buf->W2, buf->mW1, buf->vW1, buf->mW2, buf->vW2, buf->b1, buf->workspace, buf->tables};
  for (const void* p : al)
    if (((uintptr_t)p) & 15) return set_err(nullptr, SLIDE_EINVAL, "device buffers must be 16-byte aligned");
  if (!buf->tables || buf->tables_bytes < lo.tables_total)
    return set_err(nullptr, SLIDE_ENOMEM, "tables buffer too small: %zu < %zu", buf->tables_bytes, lo.tables_total);
  if (!buf->workspace || buf->workspace_bytes < lo.ws_total)
    return set_err(nullptr, SLIDE_ENOMEM, "workspace too small: %zu < %zu", buf->workspace_bytes, lo.ws_total);

  std::vector<uint32_t> words;
  if ((rc = pack_hash_params(cfg, lo, hp, words)) != SLIDE_OK) return rc;
  const int H = cfg->hidden_dim, NH = cfg->K * cfg->L;

  slide_ctx* ctx = new slide_ctx();
  ctx->cfg = *cfg; ctx->buf = *buf; ctx->lo = lo;
  ctx->prio_a = hp->prio_a; ctx->prio_b = hp->prio_b;
  const char* what = "hipMemset(ctrl)";
  hipError_t e = hipMemset(ctx->ws() + lo.ctrl, 0, sizeof(Ctrl));
  if (e == hipSuccess && lo.D) { what = "hipMemset(feature segments)"; e = hipMemset(ctx->ws() + lo.xse, 0, (size_t)lo.Bmax * lo.NT1 * 8); }
  if (e == hipSuccess && !words.empty()) { what = "hipMemcpy(hash parameters)"; e = hipMemcpy(ctx->ws() + lo.hashw, words.data(), words.size() * 4, hipMemcpyHostToDevice); }
  if (e == hipSuccess && !words.empty()) {
    const std::vector<uint32_t> offs = hash_offsets(cfg, words);
    what = "hipMemcpy(hash offsets)";
    e = hipMemcpy(ctx->ws() + lo.hashoff, offs.data(), offs.size() * 4, hipMemcpyHostToDevice);
  }
  if (e == hipSuccess) { what = "hipFuncSetAttribute(hash kernels)"; e = hash_setup_attributes(H); }
  if (e == hipSuccess) { what = "hipFuncSetAttribute(active-set kernels)"; e = active_setup_attributes(&ctx->lds_limit); }
  if (e == hipSuccess) { what = "hipFuncSetAttribute(table kernels)"; e = tables_setup_attributes(); }
  if (e == hipSuccess) { what = "hipFuncSetAttribute(forward kernels)"; e = forward_setup_attributes(ctx->lds_limit); }
  if (e == hipSuccess) { what = "hipFuncSetAttribute(update kernels)"; e = update_setup_attributes(ctx->lds_limit); }
  if (e == hipSuccess) {
    what = "hipDeviceGetAttribute(compute units)";
    int dev = 0, cus = 0;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess && cus > 0) ctx->num_cus = cus;
    hipDeviceProp_t prop;
    if (e == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) {
      // gfx942 / gfx950 parts are built from dies of 32 active compute units (MI355X: 8 x 32)
      const std::string arch = prop.gcnArchName;
      if ((arch.rfind("gfx950", 0) == 0 || arch.rfind("gfx942", 0) == 0) && cus % 32 == 0) ctx->nxcd = cus / 32;
    }
  }
  if (e == hipSuccess) {
    what = "hipGetSymbolAddress(static scratch)";
    void* p = nullptr;
    e = static_scratch_of_current_device(&ctx->device, &p);
    ctx->static_scratch = (char*)p;
  }
  if (e == hipSuccess) { what = "hipDeviceSynchronize"; e = hipDeviceSynchronize(); }
  if (e != hipSuccess) {
    set_err(nullptr, SLIDE_EHIP, "slide_init: %s failed: %s", what, hipGetErrorString(e));
    slide_destroy(ctx);
    return SLIDE_EHIP;
  }
  if (cfg->sample_budget > 0 && !lookup_bitmap_fits(lo.NWpad, lo.NT, lo.L, H, NH, ctx->lds_limit)) {
    set_err(nullptr, SLIDE_EINVAL, "sample_budget needs the per-sample bitmap in LDS: num_classes is too large");
    slide_destroy(ctx);
    return SLIDE_EINVAL;
  }
  if (lookup_fixed_lds(lo.L, H, lo.NT, NH) + (size_t)kLookupMinSegment * 4 > ctx->lds_limit) {
    set_err(nullptr, SLIDE_EINVAL, "the lookup kernel needs more LDS than the device offers (%zu bytes)", ctx->lds_limit);
    slide_destroy(ctx);
    return SLIDE_EINVAL;
  }
  if (hash_lds_bytes(H) + 1024 > ctx->lds_limit) {
    set_err(nullptr, SLIDE_EINVAL, "hidden_dim %d needs %zu bytes of LDS, device offers %zu", H, hash_lds_bytes(H), ctx->lds_limit);
    slide_destroy(ctx);
    return SLIDE_EINVAL;
  }
  HashDev& hd = ctx->hd;
  hd.kind = cfg->hash_kind; hd.H = H; hd.K = cfg->K; hd.L = cfg->L; hd.NH = NH;
  hd.m = cfg->dwta_bin; hd.lgm = cfg->hash_kind == SLIDE_HASH_DWTA ? ilog2_exact(cfg->dwta_bin) : 0;
  hd.S = cfg->srp_nnz; hd.Spad = (cfg->srp_nnz + 1) / 2 * 2; hd.So = simhash_offset_stride(cfg->srp_nnz);
  hd.words = ctx->at<uint32_t>(lo.hashw);
  hd.offs = ctx->at<uint32_t>(lo.hashoff);
  hd.dens_a = hp->dens_a; hd.dens_b = hp->dens_b;
  TablesDev& td = ctx->td;
  td.off = (uint32_t*)((char*)buf->tables + lo.t_off);
  td.ids = (int32_t*)((char*)buf->tables + lo.t_ids);
  td.nb = lo.nb; td.N = lo.N; td.L = lo.L; td.C = lo.C;
  *out = ctx;
  return SLIDE_OK;
}

int slide_build_tables(slide_ctx* ctx, void* hip_stream) {
  if (!ctx) return SLIDE_EINVAL;
  // the rebuild count enters the overflow priorities: the build runs with the count it will have, and the
  // count is kept only if the build was enqueued
  const int64_t r_before = ctx->r;
  if (ctx->ever_built) ctx->r += 1;
  const int rc = do_build(ctx, (hipStream_t)hip_stream, false);
  if (rc == SLIDE_OK) { ctx->built = true; ctx->ever_built = true; }
  else ctx->r = r_before;
  return rc;
}

int slide_set_hash_params(slide_ctx* ctx, const slide_hash_params* hp, void* hip_stream) {
  if (!ctx) return SLIDE_EINVAL;
  if (!hp) return set_err(ctx, SLIDE_EINVAL, "hash params are NULL");
  std::vector<uint32_t> words;
  const int rc = pack_hash_params(&ctx->cfg, ctx->lo, hp, words);
  if (rc != SLIDE_OK) { ctx->err = g_last_error; return rc; }
  HIPCHK(ctx, hipStreamSynchronize((hipStream_t)hip_stream));   // nothing in flight may still read the old functions
  if (!words.empty()) {
    const std::vector<uint32_t> offs = hash_offsets(&ctx->cfg, words);
    HIPCHK(ctx, hipMemcpy(ctx->ws() + ctx->lo.hashw, words.data(), words.size() * 4, hipMemcpyHostToDevice));
    HIPCHK(ctx, hipMemcpy(ctx->ws() + ctx->lo.hashoff, offs.data(), offs.size() * 4, hipMemcpyHostToDevice));
  }
  ctx->hd.dens_a = hp->dens_a; ctx->hd.dens_b = hp->dens_b;
  ctx->codes_current = false;
  ctx->prio_a = hp->prio_a; ctx->prio_b = hp->prio_b;
  ctx->built = false;                                           // the tables belong to the old functions
  return SLIDE_OK;
}

int slide_train_step(slide_ctx* ctx, const slide_batch* b, float* d_loss, void* hip_stream) {
  if (!ctx) return SLIDE_EINVAL;
  if (!ctx->built) return set_err(ctx, SLIDE_ESTATE, "slide_build_tables must run before slide_train_step");
  if (!d_loss) return set_err(ctx, SLIDE_EINVAL, "d_loss is NULL");
  int rc = check_batch(ctx, b, true);
  if (rc != SLIDE_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  const Layout& lo = ctx->lo;
  const slide_config& c = ctx->cfg;
  PairsDev p2, p1;
  p2.rows_per_tile = lo.TW * 32; p2.ntiles = lo.NT2; p2.tile_nu = ctx->at<int32_t>(lo.tile_nu2);
  p2.umeta = ctx->at<int4>(lo.umeta2); p2.pairs = ctx->at<int2>(lo.pairs2);
  p2.pcount = nullptr; p2.region_pairs = 0; p2.region0 = 0; p2.longlist = ctx->at<int32_t>(lo.longlist2); p2.nlong = &ctx->ctrl()->nlong2;
  p2.long_cap = (int)lo.long2; p2.max_nu = &ctx->ctrl()->max_nu2;
  p1.rows_per_tile = lo.TWF * 32; p1.ntiles = lo.NT1; p1.tile_nu = ctx->at<int32_t>(lo.tile_nu1);
  p1.umeta = ctx->at<int4>(lo.umeta1); p1.pairs = ctx->at<int2>(lo.pairs1);
  p1.pcount = ctx->ctrl()->p1r; p1.region_pairs = (uint32_t)lo.P1max; p1.region0 = 0; p1.longlist = ctx->at<int32_t>(lo.longlist1); p1.nlong = &ctx->ctrl()->nlong1;
  p1.long_cap = (int)lo.long1; p1.max_nu = &ctx->ctrl()->max_nu1;
  const int Bpad = (b->batch + 63) & ~63;
  TransposeArgs t2{}, t1{};
  t2.B = b->batch; t2.Bpad = Bpad; t2.TW = lo.TW; t2.ntiles = lo.NT2; t2.pd = p2;
  t2.touched = c.incremental_rebuild ? ctx->at<uint8_t>(lo.touched) : nullptr;
  if (lo.D > 0) {
    t1.B = b->batch; t1.Bpad = Bpad; t1.TW = lo.TWF; t1.ntiles = lo.NT1; t1.pd = p1;
    t1.ids = b->x_indices; t1.xse = ctx->at<int2>(lo.xse); t1.x_nnz = b->nnz;
    t1.grouped = (int64_t)b->nnz <= 16 * (int64_t)lo.NT1 ? 1 : 0;   // (a handful of features per tile on average)
    if (t1.grouped) { p1.region0 = (uint32_t)lo.NT1 * 64u; t1.pd = p1; }
  }
  ActiveDev ad;
  const bool rows_mode = row_major(ctx, b->batch);
  // Where the row lists are built.  Usually behind the logit workers of the forward launch.  When the
  // samples share most rows the logit workers keep the machine busy for long and the lists are many:
  // they then ride in the combine launch (they are not needed before the update).  The feature tiles of
  // a very wide input layer, taken a wave each, ride there too.
  const bool t1_late = rows_mode || t1.grouped, t2_late = rows_mode;
  if ((rc = forward_common(ctx, b, true, s, &ad, t1_late ? TransposeArgs{} : t1, t2_late ? TransposeArgs{} : t2,
                           rows_mode)) != SLIDE_OK) return rc;
  t2.ids = ad.as_ids; t2.rankT = ad.rankT; t2.as_base = ad.as_base;   // (for the lists that ride in the combine launch)
  // With many ids per sample and tile the lists are built from the samples' bitmaps (one coalesced read per
  // sample and tile) instead of chains of reads of the id lists.
  if (rows_mode) t2.act = ad.act;
  float* dh = ctx->at<float>(lo.dh);
  float* delta = ctx->at<float>(lo.delta);
  HIPCHK(ctx, stage(ctx, SLIDE_STAGE_COMBINE, s, [&] {
    return launch_combine(ad, lo.H, ctx->last_h, ctx->at<float>(lo.z), ctx->at<float>(lo.partials), ctx->buf.W2,
                          b->y_indptr, ad.ylist, delta, dh, b->dhidden_out, ctx->at<float>(lo.loss_i),
                          ctx->at<float>(lo.msum), t1_late ? t1 : TransposeArgs{}, t2_late ? t2 : TransposeArgs{}, s); }));
  ctx->last_dh = dh;
  const int64_t t = ctx->t + 1;
  AdamDev a;
  a.beta1 = (float)c.beta1; a.omb1 = (float)(1.0 - c.beta1);
  a.beta2 = (float)c.beta2; a.omb2 = (float)(1.0 - c.beta2);
  a.lr = (float)c.lr; a.eps = (float)c.eps;
  a.inv_bc1 = (float)(1.0 / (1.0 - std::pow(c.beta1, (double)t)));
  a.inv_bc2 = (float)(1.0 / (1.0 - std::pow(c.beta2, (double)t)));
  RowUpdate out{}, in{};
  out.pd = p2; out.coef = delta; out.V = ctx->last_h;
  out.W = ctx->buf.W2; out.M = ctx->buf.mW2; out.Vv = ctx->buf.vW2;
  out.bias = ctx->buf.b2; out.mbias = ctx->buf.mb2; out.vbias = ctx->buf.vb2;
  FinishArgs fin{};
  fin.B = b->batch; fin.loss_i = ctx->at<float>(lo.loss_i); fin.d_loss = d_loss; fin.dh = dh; fin.ctrl = ctx->ctrl();
  fin.tile_nu2 = p2.tile_nu; fin.ntiles2 = p2.ntiles; fin.cnt = ad.cnt; fin.ncand = ctx->at<int32_t>(lo.ncand);
  if (lo.D > 0) {
    in.pd = p1; in.coef = b->x_values; in.V = dh;
    in.W = ctx->buf.W1; in.M = ctx->buf.mW1; in.Vv = ctx->buf.vW1;
    fin.b1 = ctx->buf.b1; fin.mb1 = ctx->buf.mb1; fin.vb1 = ctx->buf.vb1;
    fin.tile_nu1 = p1.tile_nu; fin.ntiles1 = p1.ntiles;
  }
  const bool rows = rows_mode && update_sliced_applies(b->batch, lo.H, ctx->lds_limit);
  HIPCHK(ctx, stage(ctx, SLIDE_STAGE_UPDATE, s, [&] {
    return rows ? launch_update_sliced(lo.H, b->batch, out, in, fin, a, ctx->lds_limit, ctx->num_cus, s)
                : launch_update(lo.H, out, in, fin, a, ctx->num_cus, s); }));
  ctx->t = t;
  if (c.rebuild_every > 0 && t % c.rebuild_every == 0) {
    ctx->r += 1;
    if ((rc = do_build(ctx, s, true)) != SLIDE_OK) { ctx->r -= 1; return rc; }
  }
  return SLIDE_OK;
}

int slide_predict(slide_ctx* ctx, const slide_batch* b, int mode, int topk, int32_t* d_out_ids,
                  float* d_out_scores, void* hip_stream) {
  if (!ctx) return SLIDE_EINVAL;
  if (!ctx->built) return set_err(ctx, SLIDE_ESTATE, "slide_build_tables must run before slide_predict");
  if (topk < 1 || topk > 64 || !d_out_ids || !d_out_scores) return set_err(ctx, SLIDE_EINVAL, "topk must be in [1, 64] and outputs non-NULL");
  if (mode != 0 && mode != 1) return set_err(ctx, SLIDE_EINVAL, "mode must be 0 (retrieved neurons) or 1 (all neurons)");
  int rc = check_batch(ctx, b, false);
  if (rc != SLIDE_OK) return rc;
  hipStream_t s = (hipStream_t)hip_stream;
  if (mode == 1) {
    const Layout& lo = ctx->lo;
    const float* h = b->hidden;
    if (lo.D > 0) {
      const SpmmArgs sp = make_spmm(ctx, b);
      HIPCHK(ctx, stage(ctx, SLIDE_STAGE_HIDDEN, s, [&] { return launch_spmm_relu(b->batch, sp, ctx->ctrl(), s); }));
      HIPCHK(ctx, launch_fill_u32(ctx->at<uint32_t>(lo.xse), (size_t)b->batch * lo.NT1 * 2, 0u, s));
      h = sp.h;
    }
    ctx->last_h = h;
    ctx->last_B = b->batch;
    ctx->last_labels = 0;
    ctx->last_dh = nullptr;
    HIPCHK(ctx, launch_dense_topk(b->batch, lo.N, lo.H, h, ctx->buf.W2, ctx->buf.b2, topk, ctx->at<float>(lo.zc),
                                  lo.dense_chunk, ctx->at<uint64_t>(lo.best), ctx->at<uint64_t>(lo.cand),
                                  ctx->at<uint32_t>(lo.ccnt), d_out_ids, d_out_scores, s));
    return SLIDE_OK;
  }
  ActiveDev ad;
  if ((rc = forward_common(ctx, b, false, s, &ad, TransposeArgs{}, TransposeArgs{}, false)) != SLIDE_OK) return rc;
  if (ctx->lo.D > 0)   // the feature segments are only consumed by training: clear them again
    HIPCHK(ctx, launch_fill_u32(ctx->at<uint32_t>(ctx->lo.xse), (size_t)b->batch * ctx->lo.NT1 * 2, 0u, s));
  HIPCHK(ctx, launch_topk(ad, ctx->at<float>(ctx->lo.z), topk, d_out_ids, d_out_scores, s));
  ctx->last_dh = nullptr;
  return SLIDE_OK;
}

int slide_predict_static(slide_ctx* ctx, const slide_batch* b, int topk, int32_t* d_out_ids, float* d_out_scores,
                         void* hip_stream) {
  if (!ctx) return SLIDE_EINVAL;
  if (topk < 1 || topk > 64 || !d_out_ids || !d_out_scores) return set_err(ctx, SLIDE_EINVAL, "topk must be in [1, 64] and outputs non-NULL");
  int rc = check_batch(ctx, b, false);
  if (rc != SLIDE_OK) return rc;
  if (b->batch > SLIDE_STATIC_MAX_BATCH)
    return set_err(ctx, SLIDE_ENOMEM, "batch %d exceeds the static scratch's maximum of %d samples", b->batch, SLIDE_STATIC_MAX_BATCH);
  int dev = -1;
  HIPCHK(ctx, hipGetDevice(&dev));
  if (dev != ctx->device || !ctx->static_scratch)
    return set_err(ctx, SLIDE_ESTATE, "the current device (%d) is not the one this context was created on (%d)", dev, ctx->device);
  hipStream_t s = (hipStream_t)hip_stream;
  const Layout& lo = ctx->lo;
  // the scratch array, carved up for the largest case (SLIDE_STATIC_MAX_BATCH samples, hidden_dim 2048);
  // what is left holds the scores of one chunk of neurons
  const size_t B = (size_t)b->batch, Bmax = SLIDE_STATIC_MAX_BATCH;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return ctx->static_scratch + at; };
  float* hbuf = (float*)take(Bmax * 2048 * 4);
  uint64_t* best = (uint64_t*)take(Bmax * 64 * 8);
  uint64_t* cand = (uint64_t*)take(Bmax * dense_cand_keys() * 8);
  uint32_t* ccnt = (uint32_t*)take(Bmax * dense_counter_words() * 4);
  float* zc = (float*)take(0);
  if (o + B * 128 * 4 > kStaticScratchBytes) return set_err(ctx, SLIDE_ENOMEM, "static scratch too small");
  int64_t chunk = (int64_t)((kStaticScratchBytes - o) / (B * 4)) / 128 * 128;
  const int64_t npad = (lo.N + 127) / 128 * 128;
  if (chunk > npad) chunk = npad;
  const float* h = b->hidden;
  if (lo.D > 0) {
    SpmmArgs sp = make_spmm(ctx, b);
    sp.h = hbuf;
    sp.xse = nullptr;                                   // (no training step follows on these activations)
    HIPCHK(ctx, launch_spmm_relu(b->batch, sp, ctx->ctrl(), s));
    h = hbuf;
  }
  ctx->last_h = h;
  ctx->last_B = b->batch;
  ctx->last_labels = 0;
  ctx->last_dh = nullptr;
  HIPCHK(ctx, launch_dense_topk(b->batch, lo.N, lo.H, h, ctx->buf.W2, ctx->buf.b2, topk, zc, chunk, best, cand, ccnt,
                                d_out_ids, d_out_scores, s));
  return SLIDE_OK;
}

int slide_status(slide_ctx* ctx, void* hip_stream, uint32_t* flags) {
  if (!ctx) return SLIDE_EINVAL;
  HIPCHK(ctx, hipStreamSynchronize((hipStream_t)hip_stream));
  uint32_t st = 0;
  HIPCHK(ctx, hipMemcpy(&st, &ctx->ctrl()->status, 4, hipMemcpyDeviceToHost));
  if (flags) *flags = st;
  if (st) {
    HIPCHK(ctx, hipMemset(&ctx->ctrl()->status, 0, 4));
    return set_err(ctx, SLIDE_EDATA, "device flagged bad batch data (flags 0x%x)", st);
  }
  return SLIDE_OK;
}

int slide_get_stats(slide_ctx* ctx, void* hip_stream, slide_stats* out) {
  if (!ctx || !out) return SLIDE_EINVAL;
  HIPCHK(ctx, hipStreamSynchronize((hipStream_t)hip_stream));
  Ctrl c;
  HIPCHK(ctx, hipMemcpy(&c, ctx->ctrl(), sizeof(Ctrl), hipMemcpyDeviceToHost));
  out->active_pairs = c.total_pairs;
  out->unique_out_rows = c.u2;
  out->unique_in_rows = c.u1;
  out->candidates = ((int64_t)c.candidates_hi << 32) | c.candidates_lo;
  out->overflowed_buckets = c.overflowed;
  out->rehashed_rows = c.rehashed;
  out->steps = ctx->t;
  out->rebuilds = ctx->r;
  out->sum_active_pairs = (int64_t)c.sum_pairs;
  out->sum_unique_out_rows = (int64_t)c.sum_u2;
  out->sum_unique_in_rows = (int64_t)c.sum_u1;
  out->sum_candidates = (int64_t)c.sum_candidates;
  out->sum_steps = (int64_t)c.sum_steps;
  return SLIDE_OK;
}

int slide_reset_stats(slide_ctx* ctx, void* hip_stream) {
  if (!ctx) return SLIDE_EINVAL;
  HIPCHK(ctx, hipStreamSynchronize((hipStream_t)hip_stream));
  HIPCHK(ctx, hipMemset(&ctx->ctrl()->sum_pairs, 0, 5 * sizeof(unsigned long long)));
  return SLIDE_OK;
}

int slide_profile(slide_ctx* ctx, uint32_t stage_mask) {
  if (!ctx) return SLIDE_EINVAL;
  ctx->prof_mask = stage_mask & ((1u << SLIDE_NUM_STAGES) - 1u);
  return SLIDE_OK;
}

int slide_profile_read(slide_ctx* ctx, void* hip_stream, double* ms_sum, int64_t* launches) {
  if (!ctx || !ms_sum || !launches) return SLIDE_EINVAL;
  HIPCHK(ctx, hipStreamSynchronize((hipStream_t)hip_stream));
  for (auto& r : ctx->prof_live) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) { ctx->prof_ms[r.stage] += ms; ctx->prof_n[r.stage] += 1; }
    ctx->prof_pool.emplace_back(r.a, r.b);
  }
  ctx->prof_live.clear();
  for (int i = 0; i < SLIDE_NUM_STAGES; ++i) {
    ms_sum[i] = ctx->prof_ms[i]; launches[i] = ctx->prof_n[i];
    ctx->prof_ms[i] = 0; ctx->prof_n[i] = 0;
  }
  return SLIDE_OK;
}

int slide_destroy(slide_ctx* ctx) {
  if (!ctx) return SLIDE_OK;
  for (auto& r : ctx->prof_live) ctx->prof_pool.emplace_back(r.a, r.b);
  for (auto& e : ctx->prof_pool) { (void)hipEventDestroy(e.first); (void)hipEventDestroy(e.second); }
  delete ctx;
  return SLIDE_OK;
}

const char* slide_last_error(const slide_ctx* ctx) { return ctx ? ctx->err.c_str() : g_last_error.c_str(); }

int slide_debug_copy(void* d_dst, const void* d_src, size_t bytes, void* hip_stream) {
  if (!d_dst || !d_src || (bytes & 15) || (((uintptr_t)d_dst | (uintptr_t)d_src) & 15)) return SLIDE_EINVAL;
  return launch_copy(d_dst, d_src, bytes, (hipStream_t)hip_stream) == hipSuccess ? SLIDE_OK : SLIDE_EHIP;
}

int slide_debug_hash(slide_ctx* ctx, const float* d_vectors, int64_t rows, uint32_t* d_codes, void* hip_stream) {
  if (!ctx || !d_vectors || !d_codes || rows < 0) return SLIDE_EINVAL;
  HIPCHK(ctx, launch_hash(ctx->hd, d_vectors, rows, d_codes, ctx->lo.L, 1, nullptr, nullptr, 4,
                          (hipStream_t)hip_stream));
  return SLIDE_OK;
}

int slide_debug_get_bucket(slide_ctx* ctx, int table, uint32_t code, int32_t* h_ids, int cap, int* h_count) {
  if (!ctx || !h_count) return SLIDE_EINVAL;
  if (!ctx->built) return set_err(ctx, SLIDE_ESTATE, "tables not built");
  if (table < 0 || table >= ctx->lo.L || code >= ctx->lo.nb) return set_err(ctx, SLIDE_EINVAL, "table / code out of range");
  HIPCHK(ctx, hipDeviceSynchronize());
  uint32_t o[2];
  HIPCHK(ctx, hipMemcpy(o, ctx->td.off + (size_t)table * (ctx->lo.nb + 1) + code, 8, hipMemcpyDeviceToHost));
  const int n = (int)std::min<uint32_t>(o[1] - o[0], (uint32_t)ctx->lo.C);
  *h_count = n;
  const int m = std::min(n, cap);
  if (m > 0 && h_ids)
    HIPCHK(ctx, hipMemcpy(h_ids, ctx->td.ids + (size_t)table * ctx->lo.N + o[0], (size_t)m * 4, hipMemcpyDeviceToHost));
  return SLIDE_OK;
}

int slide_debug_get_active(slide_ctx* ctx, int64_t* h_as_ptr, int32_t* h_as_ids, uint8_t* h_is_label,
                           float* h_logits, float* h_delta, int64_t capacity) {
  if (!ctx || !h_as_ptr) return SLIDE_EINVAL;
  if (ctx->last_B < 1) return set_err(ctx, SLIDE_ESTATE, "no step has run yet");
  HIPCHK(ctx, hipDeviceSynchronize());
  const int B = ctx->last_B;
  std::vector<int32_t> base(B), cnt(B);
  HIPCHK(ctx, hipMemcpy(base.data(), ctx->at<int32_t>(ctx->lo.as_base), (size_t)B * 4, hipMemcpyDeviceToHost));
  HIPCHK(ctx, hipMemcpy(cnt.data(), ctx->at<int32_t>(ctx->lo.cnt), (size_t)B * 4, hipMemcpyDeviceToHost));
  h_as_ptr[0] = 0;
  for (int i = 0; i < B; ++i) h_as_ptr[i + 1] = h_as_ptr[i] + cnt[i];
  const int64_t A = h_as_ptr[B];
  if (A > capacity) return set_err(ctx, SLIDE_ENOMEM, "capacity %lld < active pairs %lld", (long long)capacity, (long long)A);
  // the device keeps each sample's slice at its own base; the caller gets them back to back
  for (int i = 0; i < B; ++i) {
    const size_t n = (size_t)cnt[i], src = (size_t)base[i], dst = (size_t)h_as_ptr[i];
    if (!n) continue;
    if (h_as_ids) HIPCHK(ctx, hipMemcpy(h_as_ids + dst, ctx->at<int32_t>(ctx->lo.as_ids) + src, n * 4, hipMemcpyDeviceToHost));
    if (h_logits) HIPCHK(ctx, hipMemcpy(h_logits + dst, ctx->at<float>(ctx->lo.z) + src, n * 4, hipMemcpyDeviceToHost));
    if (h_delta) HIPCHK(ctx, hipMemcpy(h_delta + dst, ctx->at<float>(ctx->lo.delta) + src, n * 4, hipMemcpyDeviceToHost));
  }
  if (h_is_label) {
    // the device keeps the label flags as the slot of every counted label entry
    std::fill(h_is_label, h_is_label + A, (uint8_t)0);
    std::vector<int32_t> slots((size_t)ctx->last_labels);
    if (!slots.empty())
      HIPCHK(ctx, hipMemcpy(slots.data(), ctx->at<int32_t>(ctx->lo.ylist), slots.size() * 4, hipMemcpyDeviceToHost));
    for (const int32_t slot : slots) {
      if (slot < 0) continue;
      const int i = (int)(std::upper_bound(base.begin(), base.end(), slot) - base.begin()) - 1;   // bases ascend
      if (i >= 0 && slot - base[i] < cnt[i]) h_is_label[h_as_ptr[i] + (slot - base[i])] = 1;
    }
  }
  return SLIDE_OK;
}

int slide_debug_get_hidden(slide_ctx* ctx, float* h_hidden, float* h_dhidden) {
  if (!ctx) return SLIDE_EINVAL;
  if (ctx->last_B < 1 || !ctx->last_h) return set_err(ctx, SLIDE_ESTATE, "no step has run yet");
  HIPCHK(ctx, hipDeviceSynchronize());
  const size_t n = (size_t)ctx->last_B * ctx->lo.H * 4;
  if (h_hidden) HIPCHK(ctx, hipMemcpy(h_hidden, ctx->last_h, n, hipMemcpyDeviceToHost));
  if (h_dhidden) {
    if (!ctx->last_dh) return set_err(ctx, SLIDE_ESTATE, "the last call was not a training step");
    HIPCHK(ctx, hipMemcpy(h_dhidden, ctx->last_dh, n, hipMemcpyDeviceToHost));
  }
  return SLIDE_OK;
}

}  // extern "C"
