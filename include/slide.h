/*
 * slide.h -- C ABI of the MI355X (gfx950) SLIDE training-step library.
 *
 * One GPU holds a two-layer network: a hidden layer fed by sparse index/value arrays and
 * a wide output layer whose neurons are sampled per input by locality-sensitive hashing
 * (the SLIDE algorithm of the paper's Section 2.1, trained as in its Algorithm 1; K hash
 * functions per table and L tables as in Section 4.1; DWTA or sparse random projections).
 * The GPU may hold the whole output layer or one node's shard of it (Section 3.1: a node
 * owns a slice of the neurons and the hash tables built over exactly that slice).
 *
 * Conventions
 *   - All `d_` / "device" pointers are HIP device pointers on the current device; all others
 *     are host pointers.  The library allocates no device memory: the caller owns parameters,
 *     Adam state, tables, workspace, batches and outputs, and the library borrows them until
 *     slide_destroy.  Sizes come from slide_query_memory.
 *   - Every call that takes `hip_stream` (a hipStream_t passed as void*) enqueues its kernels
 *     on that stream and returns without synchronising, unless stated otherwise.
 *   - Return value: SLIDE_OK (0) or a negative slide_error.  Errors found on the host are
 *     returned at once and leave device state untouched.  Errors found on the device (a feature
 *     index or label out of range, unsorted feature indices) never fault, a sticky flag is set, and
 *     slide_status reports it.  A label outside the layer is left out of its sample's label set
 *     (the step is the one the batch without that entry would give).  A feature index outside the
 *     input layer is left out of the forward pass; with that flag, or with unsorted / repeated feature
 *     indices in a sample, the step's update of W1 and b1 is UNSPECIFIED (entries next to the
 *     offending one may be missing from the gradient): treat the step as lost for the hidden layer.
 *   - Matrices are row-major fp32: W1 [input_dim][hidden_dim] (one row per input feature),
 *     W2 [num_classes][hidden_dim] (one row per output neuron).  Ids are int32.
 */
#ifndef SLIDE_H_
#define SLIDE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SLIDE_ABI_VERSION 4u

typedef struct slide_ctx slide_ctx; /* opaque, host side */

enum slide_error {
  SLIDE_OK = 0,
  SLIDE_EINVAL = -1,    /* bad argument or configuration                         */
  SLIDE_ENOMEM = -2,    /* a caller-supplied buffer is too small                 */
  SLIDE_EHIP = -3,      /* a HIP runtime call failed                             */
  SLIDE_ESTATE = -4,    /* call order (e.g. training before slide_build_tables)  */
  SLIDE_EDATA = -5      /* device-detected bad batch data (see slide_status)     */
};

enum slide_hash_kind { SLIDE_HASH_SIMHASH = 0, SLIDE_HASH_DWTA = 1 };

/* Which members of an over-full bucket survive (both store survivors ascending by id). */
enum slide_overflow_policy { SLIDE_KEEP_LOWEST_ID = 0, SLIDE_KEEP_PRIORITY = 1 };

enum slide_row_major_mode { SLIDE_ROWS_AUTO = 0, SLIDE_ROWS_NEVER = 1, SLIDE_ROWS_ALWAYS = 2 };

/* Bits of the sticky device status word returned (negated into SLIDE_EDATA) by slide_status. */
#define SLIDE_FLAG_BAD_FEATURE 1u   /* x_indices entry outside [0, input_dim): left out of the forward pass; */
                                    /* the step's W1 / b1 update is unspecified                              */
#define SLIDE_FLAG_UNSORTED 2u      /* x_indices of a sample not strictly ascending: the step's W1 / b1      */
                                    /* update is unspecified                                                 */
#define SLIDE_FLAG_BAD_LABEL 4u     /* y_indices entry outside [0, num_classes): left out of the label set   */

typedef struct {
  uint32_t struct_size;      /* sizeof(slide_config)                                            */
  uint32_t abi_version;      /* SLIDE_ABI_VERSION                                               */
  int64_t input_dim;         /* D; 0 = dense-hidden mode: the batch carries hidden[B][H]         */
  int64_t num_classes;       /* N, output neurons held by this GPU                               */
  int32_t hidden_dim;        /* H, multiple of 4, <= 2048                                        */
  int32_t max_batch;         /* largest batch any call will pass, <= 2048                        */
  int32_t max_nnz_per_batch; /* largest total number of stored features in a batch              */
  int32_t max_labels_per_batch; /* largest total number of label entries in a batch             */
  int32_t hash_kind;         /* slide_hash_kind                                                  */
  int32_t K;                 /* hash functions per table (Section 4.1)                           */
  int32_t L;                 /* tables (Section 4.1)                                             */
  int32_t dwta_bin;          /* m: DWTA bin size, 2, 4, 8 or 16; code width = K*log2(m) bits     */
  int32_t srp_nnz;           /* S: coordinates per sparse random projection; code width K bits   */
  int32_t bucket_cap;        /* C: a bucket returns at most C neurons, <= 1024                   */
  int32_t overflow_policy;   /* slide_overflow_policy                                            */
  int32_t rebuild_every;     /* R: rebuild the tables after every R-th step; 0 = never           */
  double lr, beta1, beta2, eps; /* Adam (Section 4.1: 1e-4, 0.9, 0.999, 1e-8)                    */
  /* Sampling budget of training steps (Section 3.7); 0 = none.  At most sample_budget retrieved
   * neurons per sample enter the active set (labels are always added and do not count): a uniform
   * random subset when the tables return more; when they return fewer and sample_fill != 0, uniformly
   * drawn neurons make up the difference.  Random numbers come from a counter-based generator keyed by
   * (sample_seed, step number, sample index), so a step is reproducible.  Needs the per-sample bitmap
   * in LDS (num_classes up to about 1.2 million).  slide_predict ignores the budget. */
  int32_t sample_budget;
  int32_t sample_fill;
  uint32_t sample_seed;
  /* 1: a rebuild scheduled by rebuild_every hashes only the rows of W2 that the training steps since the
   * last build have updated (Section 3.1: the tables are updated locally) and keeps the codes of the
   * others (when more than three quarters of the rows were updated it hashes them all, which is then
   * cheaper); the tables come out exactly as from a full rebuild.  The library then assumes that nobody
   * else writes W2 between builds: after changing W2 yourself, call slide_build_tables, which always
   * hashes every row.  Costs 5 bytes per output neuron of workspace. */
  int32_t incremental_rebuild;
  /* How the float kernels walk the (sample, neuron) incidences of a batch.  Sample-major work (a sample's
   * active neurons, rows gathered per incidence) suits batches whose samples share few rows; when every
   * bucket is over capacity each sample retrieves L*C neurons and a touched row belongs to many samples:
   * then the rows are streamed once and the batch's vectors are kept in LDS instead.  The results agree
   * to rounding; integers are identical.  SLIDE_ROWS_AUTO decides per call from the configuration
   * (batch * L * min(C, N / 2^bits) against N). */
  int32_t row_major_mode;      /* slide_row_major_mode */
} slide_config;

typedef struct {
  size_t tables_bytes;       /* hash tables (persist between calls)                              */
  size_t workspace_bytes;    /* per-step scratch + hash-function parameters                      */
} slide_mem_req;

/* Device buffers, all caller-owned.  W1/b1 and their state are ignored in dense-hidden mode.
 * m* and v* are Adam's momentum and velocity (Section 3.5), same shapes as the parameters. */
typedef struct {
  float *W1, *b1, *W2, *b2;
  float *mW1, *vW1, *mb1, *vb1, *mW2, *vW2, *mb2, *vb2;
  void* tables;      size_t tables_bytes;
  void* workspace;   size_t workspace_bytes;
} slide_buffers;

/* Hash-function parameters, HOST pointers, copied at slide_init.
 *   DWTA:    dwta_perm [ceil(K*L / (H/m))][H] int32, each row a permutation of 0..H-1; elementary
 *            hash e = q*(H/m) + b reads coordinates dwta_perm[q][b*m .. b*m+m).
 *   SimHash: srp_idx [K*L][S] int32 ascending coordinates, srp_sign [K*L][S] int8 (+1 / -1).
 * dens_a/dens_b: odd multipliers of the DWTA densification probe; prio_a/prio_b: odd multipliers
 * of the overflow priority hash. */
typedef struct {
  const int32_t* dwta_perm;
  const int32_t* srp_idx;
  const int8_t* srp_sign;
  uint32_t dens_a, dens_b, prio_a, prio_b;
} slide_hash_params;

/* One batch, device pointers.  Features are CSR with strictly ascending indices per sample
 * (Section 3.6: arrays of indices, values and labels); labels are CSR, duplicates allowed.
 * nnz = x_indptr[batch], num_labels = y_indptr[batch] (host copies of the totals). */
typedef struct {
  int32_t batch;
  int32_t nnz;
  int32_t num_labels;
  const int32_t* x_indptr;   /* [batch+1]           (sparse-input mode)   */
  const int32_t* x_indices;  /* [nnz]                                     */
  const float* x_values;     /* [nnz]                                     */
  const float* hidden;       /* [batch][H]          (dense-hidden mode)   */
  const int32_t* y_indptr;   /* [batch+1]; may be NULL for slide_predict  */
  const int32_t* y_indices;  /* [num_labels]                              */
  float* dhidden_out;        /* optional [batch][H]: gradient w.r.t. the hidden activations */
} slide_batch;

/* Counters of the last step / build, read back by slide_get_stats. */
typedef struct {
  int64_t active_pairs;      /* A = sum_i |AS_i|                                   */
  int64_t unique_out_rows;   /* U = touched rows of W2                              */
  int64_t unique_in_rows;    /* U1 = touched rows of W1                             */
  int64_t candidates;        /* bucket entries read before deduplication            */
  int64_t overflowed_buckets;/* buckets that held more than C neurons at last build */
  int64_t steps;             /* t, training steps done                              */
  int64_t rebuilds;          /* r, rebuilds done after the first build              */
  int64_t rehashed_rows;     /* rows of W2 hashed by the last build                 */
  /* totals over the training steps since the last slide_reset_stats */
  int64_t sum_active_pairs, sum_unique_out_rows, sum_unique_in_rows, sum_candidates, sum_steps;
} slide_stats;

/* Sizes of the tables and workspace buffers for this configuration (host only; no passage of the
 * paper: the caller owns all device memory, and this says how much of it the hashing parameters of
 * Section 4.1 and the batch limits imply).  Also rejects configurations the kernels cannot run. */
int slide_query_memory(const slide_config* cfg, slide_mem_req* out);

/* Validates the configuration and buffers, copies the hash-function parameters into the
 * workspace (synchronous), and returns a context.  Parameters must already be initialised
 * (Algorithm 1, the initialisation step: random weights); the library has no random number
 * generator.  Adam state is used as given (normally zero). */
int slide_init(const slide_config* cfg, const slide_buffers* buf, const slide_hash_params* hp,
               slide_ctx** out);

/* Algorithm 1, the table-construction step before the loop (Section 2.1 phase 1): hashes every
 * row of the current W2 into L tables.  The first call is the initial build;
 * later explicit calls count as rebuilds. */
int slide_build_tables(slide_ctx* ctx, void* hip_stream);

/* Replaces the hash functions (Algorithm 1's rebuild step renews the functions together with the
 * tables; the library draws no random numbers, so the caller supplies the new functions).
 * Synchronises the stream, uploads the parameters, and marks the tables stale: slide_build_tables
 * must run before the next slide_train_step / slide_predict; it counts as a rebuild.  Same
 * validation and ownership as in slide_init (host arrays, copied). */
int slide_set_hash_params(slide_ctx* ctx, const slide_hash_params* params, void* hip_stream);

/* One training step on one batch, Algorithm 1's loop body: retrieve active neurons (hash the
 * hidden activations, read one bucket per table, union with the labels), feed forward over the
 * active set only, softmax errors, sparse backpropagation, Adam on the touched rows only, then
 * a table rebuild if the step count is a multiple of rebuild_every.  Writes the batch-mean loss
 * to d_loss (device, one float). */
int slide_train_step(slide_ctx* ctx, const slide_batch* batch, float* d_loss, void* hip_stream);

/* Inference (Section 2.1: the tables are queried with the layer input and only the retrieved
 * neurons are scored; Section 4 reports accuracy on full predictions): scores of the neurons
 * retrieved by the hash tables (mode 0, labels not used) or of all N neurons (mode 1); the topk largest per sample go to d_out_ids / d_out_scores
 * ([batch][topk], device), ties to the lower id, missing entries id -1 / score -inf. topk <= 64. */
int slide_predict(slide_ctx* ctx, const slide_batch* batch, int mode, int topk,
                  int32_t* d_out_ids, float* d_out_scores, void* hip_stream);

/* For callers that cannot allocate device memory or hand over a workspace at the call (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): slide_predict with mode 1 (scores
 * of all N neurons, the topk best per sample), with every intermediate -- the hidden activations in
 * sparse-input mode, one chunk of scores, the running best lists, the candidate buffers and their
 * counters -- in a fixed array of SLIDE_STATIC_SCRATCH_MIB MiB inside the library's device image instead
 * of the context's workspace.  Same arguments, results and ordering rules as slide_predict; calls no
 * hipMalloc / hipFree or other allocating routine.
 * Limits: batch <= SLIDE_STATIC_MAX_BATCH (SLIDE_ENOMEM beyond); the context's device must be current
 * (SLIDE_ESTATE otherwise).  Every call on a GPU shares that GPU's array, whatever the context or
 * stream: calls that overlap on one GPU race; calls on one stream are ordered and safe.  The array
 * keeps the previous call's contents; the call clears what it needs cleared itself. */
#define SLIDE_STATIC_MAX_BATCH 64
#define SLIDE_STATIC_SCRATCH_MIB 16
int slide_predict_static(slide_ctx* ctx, const slide_batch* batch, int topk, int32_t* d_out_ids,
                         float* d_out_scores, void* hip_stream);

/* Synchronises the stream; returns SLIDE_OK, SLIDE_EHIP, or SLIDE_EDATA with the flag bits in
 * *flags (may be NULL).  The flags are then cleared.  (Housekeeping, no passage of the paper: this is
 * how the device-side checks of the batch arrays of Section 3.6 reach the caller.) */
int slide_status(slide_ctx* ctx, void* hip_stream, uint32_t* flags);

/* Synchronises the stream and copies the counters (measurement aid; the sparsity the paper's argument
 * rests on -- active neurons per sample, Sections 1 and 2.1 -- is read off these). */
int slide_get_stats(slide_ctx* ctx, void* hip_stream, slide_stats* out);

/* Launches of a step, in order, for slide_profile. */
enum slide_stage {
  SLIDE_STAGE_HIDDEN = 0,   /* sparse-input hidden layer as a launch of its own (batches above 256,   */
                            /* slide_predict mode 1)                                                   */
  SLIDE_STAGE_LOOKUP = 1,   /* hidden layer of the sample (sparse-input mode), hash codes, bucket     */
                            /* reads, union, sorted id lists, forward work items                      */
  SLIDE_STAGE_FORWARD = 2,  /* logits + running soft-max over the gathered rows; the same launch turns */
                            /* the batch's features and active sets into per-row sample lists         */
  SLIDE_STAGE_COMBINE = 3,  /* normaliser, errors, loss, hidden gradient                               */
  SLIDE_STAGE_UPDATE = 4,   /* gradient + Adam on the touched rows of W2, b2, W1; b1; loss mean        */
  SLIDE_STAGE_REBUILD = 5,  /* table build / rebuild (all its kernels)                                */
  SLIDE_NUM_STAGES = 6
};

/* Measurement aid: for every stage whose bit (1 << slide_stage) is set in stage_mask, later calls
 * bracket that stage's launches with a pair of HIP events on the call's stream.  0 turns it off.
 * slide_profile_read synchronises the stream, adds up the elapsed milliseconds and the number of
 * launches per stage since the last read into ms_sum / launches (SLIDE_NUM_STAGES entries each,
 * host), and resets them. */
int slide_profile(slide_ctx* ctx, uint32_t stage_mask);
int slide_profile_read(slide_ctx* ctx, void* hip_stream, double* ms_sum, int64_t* launches);

/* Synchronises the stream and zeroes the running totals of slide_stats. */
int slide_reset_stats(slide_ctx* ctx, void* hip_stream);

int slide_destroy(slide_ctx* ctx);

/* Message of the last error on this context (ctx == NULL: last slide_init / query failure). */
const char* slide_last_error(const slide_ctx* ctx);

/* ---- read-backs for staged verification (synchronous; not part of the hot path) ---------- */

/* Measurement aid: a plain device-to-device copy kernel (four 16-byte words per thread in flight,
 * streaming loads and stores: the fastest plain copy found on this device), the yardstick against
 * which hardware counters and achieved bandwidth are calibrated.  Enqueued on the stream; pointers
 * and bytes must be multiples of 16. */
int slide_debug_copy(void* d_dst, const void* d_src, size_t bytes, void* hip_stream);
/* Table codes of `rows` device vectors of length H with the context's hash functions. */
int slide_debug_hash(slide_ctx* ctx, const float* d_vectors, int64_t rows,
                     uint32_t* d_codes /*[rows][L]*/, void* hip_stream);
/* Contents of bucket (table, code): up to `cap` ids into h_ids, its size into *h_count. */
int slide_debug_get_bucket(slide_ctx* ctx, int table, uint32_t code, int32_t* h_ids, int cap,
                           int* h_count);
/* Active sets of the last step/predict: h_as_ptr [batch+1]; the other arrays (each may be NULL)
 * hold `capacity` entries; returns SLIDE_ENOMEM if capacity < as_ptr[batch]. */
int slide_debug_get_active(slide_ctx* ctx, int64_t* h_as_ptr, int32_t* h_as_ids,
                           uint8_t* h_is_label, float* h_logits, float* h_delta, int64_t capacity);
/* Hidden activations and their gradient of the last step, [batch][H] each (may be NULL). */
int slide_debug_get_hidden(slide_ctx* ctx, float* h_hidden, float* h_dhidden);

#ifdef __cplusplus
}
#endif
#endif /* SLIDE_H_ */
