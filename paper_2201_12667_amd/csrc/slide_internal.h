// Internal declarations shared by the HIP translation units of the SLIDE step library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "slide.h"

namespace slide {

constexpr int kWave = 64;
constexpr int kChunk = 64;         // active pairs per forward work item
constexpr int kSmallBucket = 8;    // buckets up to this size are sorted by one thread
constexpr int kSortCap = 2048;     // keys held in LDS by the big-bucket sorter
constexpr int kLongRow = 32;       // rows touched by more samples than this are reduced by a whole wave
constexpr int kPairRegions = 32;   // the input layer's pair space is handed out from this many counters (tile % regions)

// Device-side counters, one block at the start of the workspace.
struct Ctrl {
  uint32_t status;        // sticky SLIDE_FLAG_* bits
  uint32_t u2, wl_short;  // touched rows of W2 (statistics) / short-bucket worklist length (filled from the back)
  uint32_t u1, p1;        // touched rows of W1 (statistics) / pair space handed out for the input layer
  uint32_t wl_count;      // big-bucket worklist length
  uint32_t overflowed;    // buckets with more than C members at the last build
  uint32_t total_pairs;   // A
  uint32_t rehashed;      // rows of W2 hashed by the last build
  uint32_t candidates_lo, candidates_hi;
  uint32_t nlong2, nlong1; // long rows queued by the two transpositions
  uint32_t max_nu2, max_nu1; // most touched rows in any tile
  uint32_t pad[1];
  // Pair space of the input layer's row lists: region r (tiles with tile % kPairRegions == r) is handed
  // out from p1r[r].  (Updates of one word from every workgroup of a launch queue up behind each other
  // for tens of nanoseconds apiece, so per-launch counters that many workgroups bump are spread out.)
  uint32_t p1r[kPairRegions];
  // forward work items (chunks of kChunk active neurons): room for their partial results is handed out
  // by the lookup workgroups; a call uses counter (call number & 1) and clears the other
  uint32_t chunk_alloc[2];
  // running totals since the last slide_reset_stats (updated once per training step)
  unsigned long long sum_pairs, sum_u2, sum_u1, sum_candidates, sum_steps;
  uint32_t pad2[16];
  uint32_t max_nch[2];    // most work items of any sample, same parity scheme (a cache line of its own)
  uint32_t pad3[14];
};

// Hash functions as the kernels read them.
struct HashDev {
  int kind, H, K, L, NH;
  int m, lgm;             // DWTA bin size and its log2
  int S, Spad, So;        // SimHash coordinates per bit, padded to even; entries per bit in offs
  const uint32_t* words;  // DWTA: NH*m/2 words of two u16 coordinates; SimHash: NH*Spad/2 words of
                          // two u16 (bit 15 = subtract)
  const uint32_t* offs;   // the same coordinates as byte offsets into the row-tile kernel's LDS tile, one
                          // entry each (SimHash: bit 31 = subtract; padding entries point at a zero cell)
  uint32_t dens_a, dens_b;
};

struct AdamDev {
  float beta1, omb1, beta2, omb2, lr, inv_bc1, inv_bc2, eps;
};

inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// ---- hash.hip -------------------------------------------------------------------------
// codes[r*row_stride + t*tab_stride] for r < rows, t < L.  With hist != nullptr also
// pos = atomicAdd(&hist[t*(nb+1) + code], 1) and rank[t*rows + r] = pos.
// codes[row * row_stride + t * tab_stride] for the vectors 0 .. rows-1 of V, or, with a row list, for the
// vectors rowlist[0 .. *nrows_dev) (count on the device, at most rows).
hipError_t launch_hash(const HashDev& hd, const float* V, int64_t rows, uint32_t* codes,
                       int64_t row_stride, int64_t tab_stride, const int32_t* rowlist,
                       const uint32_t* nrows_dev, int tables_per_block, hipStream_t s);
hipError_t hash_setup_attributes(int H);
size_t hash_lds_bytes(int H);
int hash_tile_pitch(int H);
inline int simhash_offset_stride(int S) { return (S + 7) / 8 * 8; }       // words between consecutive coordinates in the row-tile kernel's LDS tile

// ---- tables.hip -----------------------------------------------------------------------
struct TablesDev {
  uint32_t* off;          // [L][nb+1]
  int32_t* ids;           // [L][N]
  uint32_t nb;
  int64_t N;
  int L, C;
};
hipError_t launch_build_tables(const HashDev& hd, const TablesDev& td, const float* W2, uint32_t* codes_t,
                               uint32_t* entries, uint32_t* bh, uint32_t* pbase, uint64_t* worklist,
                               uint32_t wl_cap, Ctrl* ctrl, int policy, uint32_t r, uint32_t prio_a,
                               uint32_t prio_b, uint8_t* touched, int32_t* touched_rows, bool only_touched,
                               hipStream_t s);
size_t tables_bh_words(int bits, int64_t N, int L);      // per-slab run boundaries
size_t tables_pbase_words(int bits, int64_t N, int L);   // partition starts
hipError_t tables_setup_attributes();

// ---- active.hip -----------------------------------------------------------------------
struct ActiveDev {
  int B, L, C, TW;                 // TW: bitmap words per rank tile (power of two <= 32)
  int64_t N;
  int NWpad, NT;                   // bitmap words per sample (multiple of TW), tiles per sample
  int PS;                          // slots reserved per sample for candidates: min(L*C, N)
  int num_labels;                  // label entries in the batch
  int par;                         // which work-item counter this call uses
  int nxcd;                        // accelerator dies whose workgroups alternate in launch order (1: unknown)
  int budget, fill;                // sampling budget of this call (0 = none) and its fill option
  uint32_t sample_seed, step;      // keys of the counter-based generator: seed, number of the step being run
  uint32_t* act;                   // [NT][B][TW] the samples' bitmaps, tile-major: written when a bitmap exceeds the LDS
  int write_act;                   // ... or when the row lists are to be built from the bitmaps (!= 0)
  uint32_t* rankT;                 // [NT+1][B] active neurons of the sample below the tile (last row: |AS_i|)
  int32_t* cnt;                    // [B] |AS_i|
  int32_t* ny;                     // [B] distinct labels
  int32_t* chunk_ptr;              // [B] where the partial results of the sample's work items start
  int32_t* as_base;                // [B] first slot of sample i = i*PS + (label entries before sample i)
  int32_t* as_ids;                 // [slots] ascending ids of sample i at as_base[i] .. +cnt[i]
  int32_t* ylist;                  // [labels] slot of each label entry, -1 for invalid / repeated ones
};
// Row lists: for every touched row the ascending samples that touch it.  Row slots are grouped by tile:
// tile t owns slots [t*rows_per_tile, t*rows_per_tile + tile_nu[t]).
struct PairsDev {
  int rows_per_tile, ntiles;
  int32_t* tile_nu; // [ntiles] touched rows in the tile
  int4* umeta;      // [slots] (row id, first pair, pairs, 0)
  int2* pairs;      // [pairs] (sample, index into the coefficient array)
  uint32_t* pcount; // pair space counters, kPairRegions of them (input layer only)
  uint32_t region_pairs; // pair slots per region
  uint32_t region0;      // pair slots ahead of the regions (64 per tile when a wave takes a tile: no counter)
  int32_t* longlist; // [long_cap] slots of rows with more than kLongRow pairs
  uint32_t* nlong;
  int long_cap;
  uint32_t* max_nu; // largest tile_nu (bounds the work items of the row kernel)
};

struct TransposeArgs {
  int B, Bpad, TW, ntiles;       // a tile is TW*32 rows; ntiles = 0: nothing to do
  int grouped;                   // features only: a wave per tile, a workgroup per group of tiles (tiles that hold
                                 // a handful of the batch's features each)
  const int32_t* ids;            // ascending id list per sample (active-set ids / CSR feature indices)
  const uint32_t* rankT;         // [ntiles+1][B] (active sets only) ids of the sample below the tile
  const int32_t* as_base;        // [B]           (active sets only) first slot of the sample
  const uint32_t* act;           // [ntiles][B][TW] (active sets only, optional) the samples' bitmaps: read instead of ids
  int2* xse;                     // [ntiles][B]   (features only) positions [start, end) of the sample's
                                 // features inside the tile; (0, 0) = none
  int x_nnz;                     // features only: entries in the batch's CSR arrays
  uint8_t* touched;              // optional [rows]: set to 1 for every row that gets a header
  PairsDev pd;
};

// Sparse-input hidden layer: CSR batch, parameters, outputs (W1 == nullptr: absent).
struct SpmmArgs {
  int64_t D;
  int H, nnz_total, rows_per_tile;
  const int32_t *x_indptr, *x_indices;
  const float *x_values, *W1, *b1;
  float* h;                      // [B][H] activations (output)
  int2* xse;                     // [tiles][B] feature segments per tile (output)
};

constexpr int kLookupMinSegment = 1024;   // bitmap words the lookup kernel must be able to hold at a time
constexpr size_t kDeviceLdsBytes = 160 * 1024;   // LDS of a gfx950 compute unit (the only target)
// LDS the lookup kernel needs besides its bitmap segment.
size_t lookup_fixed_lds(int L, int H, int NT, int NH);
hipError_t active_setup_attributes(size_t* lds_limit_out);
bool lookup_bitmap_fits(int NWpad, int NT, int L, int H, int NH, size_t lds_limit);
// sp.W1 != nullptr: the workgroup of a sample first computes the sample's hidden activations (h is
// then sp.h, written here); else h holds them already.
hipError_t launch_lookup_union(const ActiveDev& ad, const HashDev& hd, const float* h, const SpmmArgs& sp,
                               const TablesDev& td, uint32_t* codes, const int32_t* y_indptr,
                               const int32_t* y_indices, int include_labels, int32_t* ncand, Ctrl* ctrl,
                               size_t lds_limit, hipStream_t s);


// ---- output.hip -----------------------------------------------------------------------
hipError_t launch_spmm_relu(int B, const SpmmArgs& a, Ctrl* ctrl, hipStream_t s);
// Logits over the active sets (logits = true: three worker workgroups per compute unit); the same
// launch builds the two sets of row lists (t1: features, t2: active sets; ntiles = 0 leaves one out).
hipError_t launch_forward(const ActiveDev& ad, int H, const float* h, const float* W2, const float* b2, float* z,
                          float* partials, const Ctrl* ctrl, const TransposeArgs& t1, const TransposeArgs& t2,
                          bool logits, int num_cus, hipStream_t s);
hipError_t forward_setup_attributes(size_t lds_limit);
hipError_t launch_combine(const ActiveDev& ad, int H, const float* h, const float* z, const float* partials,
                          const float* W2, const int32_t* y_indptr, const int32_t* ylist, float* delta,
                          float* dh, float* dh_copy, float* loss_i, float* msum, const TransposeArgs& t1,
                          const TransposeArgs& t2, hipStream_t s);
hipError_t launch_topk(const ActiveDev& ad, const float* z, int topk, int32_t* out_ids,
                       float* out_scores, hipStream_t s);

// ---- predict.hip ----------------------------------------------------------------------
// Scores over all N neurons in chunks of `chunk` neurons (zc: [B][chunk] scratch) and the topk best
// per sample (best: [B][64] scratch keys).
int64_t dense_chunk_neurons(int64_t N, int Bmax);
hipError_t launch_dense_topk(int B, int64_t N, int H, const float* h, const float* W2, const float* b2, int topk,
                             float* zc, int64_t chunk, uint64_t* best, uint64_t* cand, uint32_t* ccnt,
                             int32_t* out_ids, float* out_scores, hipStream_t s);
size_t dense_cand_keys();     // candidate keys per sample (cand is [B][dense_cand_keys()])
size_t dense_counter_words(); // words per sample in ccnt

// ---- update.hip -----------------------------------------------------------------------
// Rows of one weight matrix to update: for every listed row r, g = sum over its pairs of
// coef[src] * V[sample][:], then Adam on W[r][:] (and on bias[r] with the sum of the coefficients
// when bias != nullptr).
struct RowUpdate {
  PairsDev pd;
  const float* coef;
  const float* V;
  float *W, *M, *Vv, *bias, *mbias, *vbias;
  int nblocks;                   // workgroups given to this matrix; 0 = absent
};
struct FinishArgs {
  int B;
  const float* loss_i;
  float* d_loss;
  const float* dh;
  float *b1, *mb1, *vb1;         // nullptr in dense-hidden mode
  Ctrl* ctrl;
  const int32_t* tile_nu2; int ntiles2;
  const int32_t* tile_nu1; int ntiles1;
  const int32_t* cnt;            // [B] |AS_i|
  const int32_t* ncand;          // [B] bucket entries read for sample i
  int nblocks;
};
// One launch, three roles by workgroup index: loss mean + hidden bias + statistics, the rows of W1,
// the rows of W2 (+ b2).
hipError_t launch_update(int H, const RowUpdate& out, const RowUpdate& in, const FinishArgs& fin, const AdamDev& ad,
                         int num_cus, hipStream_t s);
// The same launch for batches whose samples share most rows: sample vectors staged in LDS by column
// slices (see update.hip).  update_sliced_applies: whether a batch of B vectors of length H fits.
bool update_sliced_applies(int B, int H, size_t lds_limit);
hipError_t update_setup_attributes(size_t lds_limit);
hipError_t launch_update_sliced(int H, int B, const RowUpdate& out, const RowUpdate& in, const FinishArgs& fin,
                                const AdamDev& ad, size_t lds_limit, int num_cus, hipStream_t s);
hipError_t launch_fill_u32(uint32_t* p, size_t n, uint32_t v, hipStream_t s);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);

}  // namespace slide
