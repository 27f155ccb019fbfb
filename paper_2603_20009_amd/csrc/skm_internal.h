// Internal declarations shared by the HIP translation units of libskm.
// Nothing here is part of the public ABI (see include/skm.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace skm {

constexpr int kBlockDims = 64;  // Section 3.2: trailing dimensions are explored 64 at a time
constexpr int kMaxBlocks = 256; // (16384 - 16) / 64 rounded up
constexpr int kSegPoints = 512; // points per partial-sum segment of the centroid update

// One surviving (point, centroid) pair produced by the first pruning test
// (Algorithm 1, the `likely(distances[i,j] > theta(d', tau))` line inverted).
struct __attribute__((aligned(16))) Pair {
  int32_t i;   // point index (global row)
  int32_t j;   // centroid index in bits 0..23, first trailing block still to be added in bits 24..31
  float p;     // partial squared distance on the dimensions seen so far
  float tau;   // the point's pruning threshold for this step
};

// Error reporting shared by the translation units that hold entry points: records the text skm_last_error() returns
// on this thread and gives back the code (SKM_ENOMEM for an out-of-memory HIP error, SKM_EHIP for any other).
int report_error(int rc, const char *what);
int report_hip_error(hipError_t e, const char *where);

// ---- order-preserving float <-> uint32 map (for packed 64-bit atomic min) ----
__host__ __device__ inline uint32_t f2ord(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__host__ __device__ inline float ord2f(uint32_t u) {
  u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
  return __builtin_bit_cast(float, u);
}
__host__ __device__ inline uint64_t pack_key(float v, int32_t idx) {
  return ((uint64_t)f2ord(v) << 32) | (uint32_t)idx;
}

// ---------------------------------------------------------------- GEMM family
// C-shaped work: scores s(i, j) = sum_k A[i][k] * B[j][k] for an M x K row-major A and an
// N x K row-major B (both K-contiguous), on fp32 MFMA, with one of three fused epilogues.
struct GemmOperands {
  const float *A;
  int64_t lda;
  int32_t M;
  const float *B;
  int64_t ldb;
  int32_t N;
  int32_t K;
  int32_t panel_cols = 16;  // column tiles per panel of the tile walk (set by the launcher)
  // Device words holding the bit pattern of an upper bound of |A| and of |B| (see launch_absmax).  With both
  // set (and 16-byte aligned operands, K >= 32) the product runs in the split-fp16 form described below.
  const unsigned int *a_absmax = nullptr;
  const unsigned int *b_absmax = nullptr;
  // Optional workspace of N * (K + 32) words, 16-byte aligned: with it (and the bounds above, K a multiple of 32) a
  // tall product splits B into fp16 pairs there first and runs on 256 x 256 tiles.
  uint32_t *b_split = nullptr;
};

// Split-fp16 arithmetic.  A matrix whose largest magnitude is m is scaled by the power of two that brings m
// into [2^14, 2^15); a scaled value v is staged as hi = fp16(v) and lo = fp16(v - hi), which keeps 22
// significant bits of v (and an absolute error below 2^-40 m for values too small for that), and a product
// is taken as hi*hi' + hi*lo' + lo*hi' on v_mfma_f32_32x32x16_f16 with fp32 accumulation.  The dropped
// lo*lo' term is 2^-22 of the product.  Scaling by powers of two is exact, so the result is that of an fp32
// GEMM whose inputs were rounded to 22 bits.
__device__ inline float split_scale(unsigned int absmax_bits) {   // 2^(14 - floor(log2 m)), clamped to normal floats
  int e = 268 - (int)(absmax_bits >> 23);
  e = e < 1 ? 1 : (e > 253 ? 253 : e);
  return __builtin_bit_cast(float, (unsigned int)e << 23);
}
__device__ inline float split_unscale(unsigned int absmax_bits) {  // exactly 1 / split_scale
  int e = 268 - (int)(absmax_bits >> 23);
  e = e < 1 ? 1 : (e > 253 ? 253 : e);
  return __builtin_bit_cast(float, (unsigned int)(254 - e) << 23);
}
// *out = max(*out, bit pattern of max |A[i][j]|) over rows x cols; *out must hold 0 (or an earlier bound) before.
// max_blocks > 0 limits the grid (a pass that shares the device with other work should not take every wavefront slot).
hipError_t launch_absmax(const float *A, int64_t lda, int64_t rows, int32_t cols, unsigned int *out, hipStream_t st,
                         int max_blocks = 0);

// C[i][j] = alpha * s(i,j) + beta * C[i][j] for j < N; columns N <= j < Nstore are written as 0.
// If c_absmax is given, max |C| is folded into *c_absmax (as launch_absmax does).
hipError_t gemm_store(const GemmOperands &g, float *C, int64_t ldc, int32_t Nstore, float alpha, float beta,
                      hipStream_t st, unsigned int *c_absmax = nullptr);

// best[i] = min(best[i], pack_key(ynorm[j] - 2 s(i,j), j)) over all j: the row argmin of the squared
// distance up to the per-row constant ||x_i||^2 (Algorithm 1, iteration 1).
hipError_t gemm_argmin(const GemmOperands &g, const float *ynorm, unsigned long long *best, hipStream_t st);

// Launch choices of the GEMM family that tests force (process-wide; nothing here changes what is computed):
// tile256 -1 = by shape, 0 = never the 256 x 256 form, 1 = whenever the operands allow it; panel_cols > 0 = width of
// the tile walk's panels; max_tiles > 0 = tiles per launch (tall problems are cut into bands of row tiles).
void gemm_debug_config(int tile256, int panel_cols, int64_t max_tiles);

// Device scalars of one assignment step.  Every workgroup adds to the replica (blockIdx & (kStatReplicas-1))
// so that same-address atomics do not serialise; the host sums the replicas.
enum { SC_COMPLETED = 0, SC_CHANGED = 1, SC_SURVIVORS = 2, SC_DENSE_DIMS = 3, SC_DENSE_PB = 4, SC_GATHER_PB = 5,
       SC_GATHER_PAIRS = 6, SC_SCREEN_DIMS = 7, SC_LISTED_TILES = 8, SC_ENTER = 9, SC_COUNT = 9 + kMaxBlocks };
constexpr int kStatReplicas = 32;
// The hand-over list is split in kSubLists equal parts, one per XCD (workgroup id mod 8), each with its own
// fill counter (counters are kSubListStride words apart).
constexpr int kSubLists = 8;
constexpr int kSubListStride = 16;

// Progressive-pruning GEMM (Algorithm 1, iterations >= 2): a 128 x 128 tile is multiplied densely over
// d', d'+64, d'+128, ... dimensions; after each step the pairs whose partial distance exceeds
// theta(t, tau_i) die; the tile stops when nothing is alive, hands its pairs to the gather kernel when
// at most emit_max are alive, and offers finished distances below tau_i to best[] at t = d.
// Rows are local to the chunk: global row = row_base + i; tau/prev/best are indexed by global row.
// Split-fp16 copy of a matrix in the byte order of the progressive kernel's LDS tiles (launch_split_rows): row stride
// ds + 32 words; dims 16 g .. 16 g + 15 of a row are the 16 words at 16 (g + 1): 8 words of hi halves, 8 of lo halves
// of the values scaled by split_scale(*absmax); the 16 words before and after the row's data are zero.
// out_hi (optional): the hi halves once more as a plane of their own (row stride ds / 2 + 16 words: 8 zero words, the
// row two dimensions a word, 8 zero words), which the low-precision first filter reads.
hipError_t launch_split_rows(const float *A, int64_t lda, int64_t rows, int32_t ds, const unsigned int *absmax,
                             uint32_t *out, hipStream_t st, uint32_t *out_hi = nullptr);

struct ProgArgs {
  const uint32_t *A;       // split-fp16 copy of the rotated points of the chunk (launch_split_rows)
  int64_t lda;             // ds + 32 words
  int32_t M;
  const uint32_t *B;       // split-fp16 copy of the rotated centroids
  int64_t ldb;
  int32_t N;
  const unsigned int *a_absmax, *b_absmax;   // the bounds the copies were scaled by
  int32_t ds, d, dprime, nb;
  const float *ratio;      // [nb + 1] theta ratio at checkpoint m (t_m = min(d, d' + 64 m)); device array
  const float *tau;        // [n]
  const int32_t *prev;     // [n] incumbent (never a challenger)
  int64_t row_base;
  const float *xnp;        // [ds / 16][xn_stride] ||x_i[0 : 16 (p + 1))||^2, indexed like tau (row_base + tile row)
  int64_t xn_stride;
  const float *ynp;        // [nb + 1][N] ||y_c[0 : t_m)||^2
  Pair *pairs;             // kSubLists parts of sub_capacity slots each
  unsigned int *pair_count;   // [kSubLists * kSubListStride] fill counters of the parts
  unsigned int *tile_counter; // [8 * kSubListStride] next tile of every XCD's range; zero before the launch
  unsigned int sub_capacity;
  unsigned int *overflow;
  unsigned int emit_max;   // a tile with at most this many alive pairs is handed over
  unsigned long long *best;       // [n] packed (distance, centroid)
  unsigned long long *scal;       // [kStatReplicas][SC_COUNT] step scalars (SC_SURVIVORS, SC_COMPLETED, SC_DENSE_*, SC_ENTER..)
  int32_t block_stats;            // also count pairs entering every trailing block (SC_ENTER + m)
  // Listed columns (after launch_screen; all NULL otherwise): tile t is row tile tile_rt[t] against the 128 centroids
  // col_list[128 t ..] (ascending ids, -1 = none); *ntiles tiles in all.
  const int32_t *tile_rt = nullptr, *col_list = nullptr, *ntiles = nullptr;
};
hipError_t launch_progressive(const ProgArgs &g, hipStream_t st);

// Low-precision first filter (screen.hip): one fp16 product on the first d' dimensions and the first test
// theta(d', tau) widened by the error bound of the dropped halves; then, per row tile of 128 points, the centroids
// that some point of the tile may still pass, as an ascending id list padded with -1 to a multiple of 128.
// Outputs: cnt[row tiles], first[row tiles] (first tile of 128 listed columns of every row tile), *ntiles,
// col_list[128 * ntiles], tile_rt[ntiles]; capacity needed: one tile per (row tile, column tile) of the full problem.
struct ScreenLaunch {
  const uint32_t *A; int64_t lda; int32_t M;
  const uint32_t *B; int64_t ldb; int32_t N;
  const unsigned int *a_absmax, *b_absmax;
  int32_t ds, dprime;
  float ratio0;              // theta(d', tau) / tau
  const float *tau;          // [n], indexed by row_base + row
  int64_t row_base;
  const float *xn;           // [n] ||x_i[0 : d')||^2, indexed like tau
  const float *yn;           // [N] ||y_j[0 : d')||^2
  float *arow, *ycol;        // scratch: [M] and [N] (the test's per-point and per-centroid terms)
  uint32_t *colmask;         // scratch: [row tiles][4 * column tiles]
  int32_t *cnt, *first, *ntiles, *col_list, *tile_rt;   // (ntiles: two words, the second is scratch)
  unsigned int *tile_counter;   // (unused)
  unsigned long long *scal;     // step scalars (SC_SCREEN_DIMS)
  // Exact mode (iteration 1: dprime = ds, xn / yn the full norms, tau and ratio0 unused, no column lists): for every
  // point the centroids that can be its nearest are appended to `pairs` (partial distance 0, first block 0, no
  // threshold) for the gather kernel, which finishes their exact distances.  rowmin: [n] words of 0xffffffff before
  // the first launch of the step, indexed by row_base + row.
  int exact = 0;
  unsigned int *rowmin = nullptr;
  Pair *pairs = nullptr;
  unsigned int *pair_count = nullptr;
  unsigned int sub_capacity = 0;
  unsigned int *overflow = nullptr;
};
hipError_t launch_screen(const ScreenLaunch &a, hipStream_t st);
int64_t progressive_tiles(int64_t rows, int32_t k);
int32_t progressive_tile_pairs();
int32_t progressive_tile_cols();

// ---------------------------------------------------------------- pruning
struct PruneArgs {
  const Pair *pairs;           // kSubLists parts of sub_capacity slots each
  const unsigned int *count;   // [kSubLists * kSubListStride] fill counters
  unsigned int sub_capacity;
  const float *Xr;       // rotated points, row stride ldx, zero padded to ds columns
  int64_t ldx;
  int64_t n;             // number of points (entries naming a point beyond it are skipped)
  const float *Ypdx;     // [nb][k][64] trailing centroid dimensions, block-major (PDX-style)
  int32_t k;
  int32_t dprime;
  int32_t ds;            // padded row length (multiple of 16)
  int32_t nb;            // trailing blocks
  const float *ratio;    // [nb + 1] theta ratio at checkpoint m, t_m = min(d, d' + 64 m) (device array)
  unsigned long long *best;        // [n] packed (distance, centroid)
  unsigned long long *scal;        // [kStatReplicas][SC_COUNT]: SC_COMPLETED, SC_GATHER_*, and SC_ENTER + m when block_stats
  int32_t block_stats;
};
hipError_t launch_prune(const PruneArgs &a, hipStream_t st);

// ---------------------------------------------------------------- streaming kernels
// tau_i = ||x_i - y_{a_i}||^2 over all dims, best_i = pack(tau_i, a_i)
// (Algorithm 1, "Initial pruning threshold").  Either output may be NULL.
// With xnp ([ds / 16][n], ds a multiple of 16) the same pass writes the table of prefix norms
// xnp[p][i] = ||x_i[0 : 16 (p + 1))||^2 that the progressive kernel reads at its checkpoints; with xs also the
// split-fp16 copy of the points (the layout of launch_split_rows, scaled by the bound *x_absmax).
// Regrouping (order, xr_out, label_out: all or none): output slot p of every array above takes point order[p] (a
// permutation of 0 .. n - 1); the row of that point is copied to xr_out[p] (row stride ds) and its label to
// label_out[p].  `assign` is still indexed by point.
// xh (optional, with xs): also the plane of hi halves of launch_split_rows' out_hi.
hipError_t launch_tau_init(const float *Xr, int64_t ldx, int64_t n, int32_t ds, const float *Y, int64_t ldy,
                           const int32_t *assign, float *tau, unsigned long long *best, hipStream_t st,
                           float *xnp = nullptr, uint32_t *xs = nullptr, const unsigned int *x_absmax = nullptr,
                           const int32_t *order = nullptr, float *xr_out = nullptr, int32_t *label_out = nullptr,
                           uint32_t *xh = nullptr);
// dst[idx[p]] = src[p] for 4-byte items
hipError_t launch_scatter_by_index(const void *src, const int32_t *idx, int64_t n, void *dst, hipStream_t st);
// order_out = order_in (points grouped by cluster, segment c = [off[c], off[c+1])) with every segment stably sorted by
// the signs of the first four dimensions of its points.  key_scratch: n bytes.
hipError_t launch_suborder(const float *Xr, int64_t ldx, int64_t n, int32_t k, const int32_t *off, const int32_t *order_in,
                           unsigned char *key_scratch, int32_t *order_out, hipStream_t st);
// keys hold a point id in their low 32 bits (packed (distance, point) keys; ~0 = none): every id becomes the position
// p with perm[p] = id.  inv_scratch: n ints.
hipError_t launch_remap_key_ids(unsigned long long *keys, int64_t m, const int32_t *perm, int64_t n, int32_t *inv_scratch,
                                hipStream_t st);

// ynorm[c] = ||Y[c][0:dn)||^2 and (if Ypdx) the block-major copy of the dims from dprime on.
// ynp (optional, [nb + 1][k]): prefix norms of the centroids at the same checkpoints.
hipError_t launch_prep_centroids(const float *Y, int64_t ldy, int32_t k, int32_t ds, int32_t dn, float *ynorm,
                                 int32_t dprime, int32_t nb, float *Ypdx, hipStream_t st, float *ynp = nullptr);

// every non-zero row of A scaled to unit Euclidean length, in place (cols, lda multiples of 4; A 16-byte aligned)
hipError_t launch_normalize_rows(float *A, int64_t lda, int64_t rows, int32_t cols, hipStream_t st);

hipError_t launch_fill_u64(unsigned long long *p, int64_t n, unsigned long long v, hipStream_t st);
hipError_t launch_fill_u32(unsigned int *p, int64_t n, unsigned int v, hipStream_t st);

// Unpack best -> assign/dist, count cluster sizes (cnt[k], optional), changed assignments, per-block objective partials.
// *unset is set to 1 if some point still holds the "no centroid yet" key (an internal error).
hipError_t launch_finalize_assign(const unsigned long long *best, const int32_t *prev, int64_t n, int32_t *assign,
                                  float *dist, int32_t *cnt, int32_t k, double *obj_partial,
                                  unsigned long long *changed, unsigned int *unset, hipStream_t st);
int64_t finalize_blocks(int64_t n);
hipError_t launch_sum_partials(const double *part, int64_t m, double *out, hipStream_t st);
hipError_t launch_histogram(const int32_t *assign, int64_t n, int32_t *cnt, hipStream_t st);
hipError_t launch_check_labels(const int32_t *a, int64_t n, int32_t k, unsigned int *bad, hipStream_t st);

// Centroid update (Section 3.2) as a segmented reduction.
struct UpdateWs {
  int32_t *cnt;        // [k]   cluster sizes (input)
  int32_t *off;        // [k+1] exclusive scan of cnt
  int32_t *cursor;     // [k]
  int32_t *segoff;     // [k+1] exclusive scan of ceil(cnt / kSegPoints)
  int32_t *order;      // [n]   point ids grouped by cluster
  double *partial;     // [max_segments][ds]
  int64_t max_segments;
};
int64_t update_max_segments(int64_t n, int32_t k);
// The grouping half of launch_update alone: cnt[k] sizes, off[k+1] starts, order[n] point ids grouped by label (cursor[k]
// and segoff[k+1] are scratch).
hipError_t launch_group_order(const int32_t *labels, int64_t n, int32_t k, int32_t *cnt, int32_t *off, int32_t *cursor,
                              int32_t *segoff, int32_t *order, hipStream_t st);
// largest cluster whose members launch_update leaves sorted by index in w.order (larger ones: any order)
int32_t update_sort_cap();
// S (optional, [k][ds] fp64) receives the sum of every cluster; y_absmax (optional) the bit pattern of max |Y| of
// the new centroids (the launcher clears it first).  With `accumulate` the sums of these n points are added to S
// instead (one batch of a larger update); Y may then be NULL, and launch_means_from_sums finishes the update.
hipError_t launch_update(const float *Xr, int64_t ldx, int64_t n, int32_t ds, const int32_t *assign, int32_t k,
                         const UpdateWs &w, float *Y, int64_t ldy, hipStream_t st, double *S = nullptr,
                         unsigned int *y_absmax = nullptr, int accumulate = 0);
hipError_t launch_means_from_sums(const double *S, const int32_t *cnt, int32_t k, int32_t ds, float *Y, int64_t ldy,
                                  unsigned int *y_absmax, hipStream_t st);

// Workspace of the incremental update: room for 2 * (points that changed label) entries.
struct IncUpdateWs {
  int32_t *ent_id;     // [capacity] point id, or ~id for a point that left the cluster
  int32_t *ent_lab;    // [capacity] cluster of the entry
  int32_t *order;      // [capacity]
  int32_t *cnt, *off, *cursor, *segoff;   // [k], [k+1], [k], [k+1]
  unsigned int *counter;
  double *partial;     // [max_segments][ds]
  int64_t capacity, max_segments;
};
// Centroids from the cluster sums S of the previous update and the points whose label changed since
// (Section 3.2, the same means computed from the difference).
hipError_t launch_update_incremental(const float *Xr, int64_t ldx, int64_t n, int32_t ds, const int32_t *assign,
                                     const int32_t *prev, int64_t changed, int32_t k, const UpdateWs &w,
                                     const IncUpdateWs &inc, double *S, float *Y, int64_t ldy, hipStream_t st,
                                     unsigned int *y_absmax = nullptr);

// Empty-cluster splits: pairs_dev = (empty, donor) pairs grouped into chains (splits that share a cluster, in the
// host's order); chain_first_dev[c] .. chain_first_dev[c + 1] are the splits of chain c.  One workgroup per chain.
hipError_t launch_split(float *Y, int64_t ldy, int32_t d, const int32_t *pairs_dev, const int32_t *chain_first_dev,
                        int32_t nchains, float eps, hipStream_t st);
hipError_t launch_gather_rows(const float *src, int64_t lds, int32_t d, const int64_t *idx_dev, int32_t k, float *dst,
                              int64_t ldd, int32_t dpad, hipStream_t st);
hipError_t launch_pad_copy(const float *src, int64_t lds, int64_t n, int32_t d, float *dst, int64_t ldd, int32_t dpad,
                           int32_t transpose, hipStream_t st);

// ---------------------------------------------------------------- rotation matrix
// Haar-distributed orthogonal d x d matrix (fp32) from (d, seed); workspaces in doubles:
// Qwork d*d + 2, Cwork max(4*32*d, ceil(d/128)*1024), Wwork 8*32*d, Lwork 32*32.
hipError_t launch_make_rotation(int32_t d, uint64_t seed, double *Qwork, double *Cwork, double *Wwork, double *Lwork,
                                float *R_out, hipStream_t st);

// ---------------------------------------------------------------- ETR helpers
// Key lists hold (order-preserving distance bits << 32 | index), ascending; ~0 marks an empty slot.
// For each row q of S (nq x m scores q . x_c, row stride lds): merge the K smallest of
// colnorm[col_base + c] - 2 S[q][c] into the running list top[q][0..K).
hipError_t launch_topk_merge(const float *S, int64_t lds, int32_t nq, int32_t m, int64_t col_base,
                             const float *colnorm, int32_t K, unsigned long long *top, hipStream_t st);
// Recall numerator/denominator: per query, the nprobe centroids of smallest ynorm[c] - 2 S[q][c] are
// probed; a ground-truth neighbour counts as found iff its cluster (assign[id]) is probed.
hipError_t launch_recall_scores(const float *S, int64_t lds, int32_t nq, int32_t k, const float *ynorm, int32_t nprobe,
                                const unsigned long long *gt_keys, int32_t K, const int32_t *assign,
                                unsigned long long *hits, unsigned long long *total, hipStream_t st);
hipError_t launch_row_norms(const float *X, int64_t ldx, int64_t n, int32_t d, float *out, hipStream_t st);
hipError_t launch_keys_to_index(const unsigned long long *keys, int64_t n, int64_t *idx, hipStream_t st);
hipError_t launch_index_to_keys(const int64_t *idx, int64_t n, unsigned long long *keys, hipStream_t st);
constexpr int kMaxProbe = 8192;

}  // namespace skm
