/*
 * skm.h -- C ABI of libskm: the SuperKMeans k-means iteration on one AMD
 * MI355X (gfx950).  Citations are to the SuperKMeans paper (arxiv 2603.20009).
 *
 * Conventions for every entry point
 *   - Array arguments are DEVICE pointers (hipMalloc'd memory, e.g. the
 *     storage of a torch tensor), dense row-major, fp32 / int32 / int64 as
 *     declared, unless the comment says "host".  The params / trace structs
 *     themselves live in host memory.
 *   - The caller owns every buffer it passes.  The library allocates and
 *     frees its own workspace inside the call, unless the caller lends it one
 *     (params->workspace, see skm_workspace_bytes).
 *   - Work is enqueued on `params->stream` (a hipStream_t, NULL = the default
 *     stream) and the call returns after that stream has been synchronised,
 *     so outputs are complete on return.
 *   - Return value: 0 on success, a negative SKM_E* code otherwise.  An
 *     argument error (SKM_EINVAL, or SKM_ENOMEM for a workspace that is too
 *     small) is found before any work is enqueued and leaves the outputs
 *     untouched; after any other error their contents are unspecified.  No
 *     exception crosses this boundary.
 *   - Thread-compatible, not thread-safe: concurrent calls must use distinct
 *     streams and distinct buffers.
 *   - Limits: 16 <= d <= 16384, 1 <= k <= 2^24, n < 2^31; a fit needs k <= n
 *     (an assignment step may have more centroids than points).
 */
#ifndef SKM_H_
#define SKM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SKM_OK 0
#define SKM_EINVAL (-1)    /* null pointer, bad shape, k > n, d out of range ... */
#define SKM_ENOMEM (-2)    /* workspace allocation failed */
#define SKM_EHIP (-3)      /* a HIP call failed; see skm_last_error() */
#define SKM_EINTERNAL (-4) /* an internal invariant was violated */
#define SKM_EOVERFLOW (-5) /* the list that carries pairs from the dense tiles to the gather kernel overflowed
                              (cannot happen with the capacities the library derives from pair_budget; reported
                              instead of a wrong result if it ever does) */

#define SKM_MAX_BLOCKS 32 /* counters kept for at most this many trailing blocks */

/* One row per assignment step (Algorithm 1: iteration 1, iterations 2..n, and
 * the final assignment pass of Section 3.3 when it is requested). */
typedef struct skm_trace_row {
  double objective;    /* sum over points of the squared distance found by this step */
  double prune_frac;   /* share of (point, centroid != incumbent) pairs cut by the first
                          test theta(d', tau) (Section 4.8); 0 for iteration 1 */
  double recall;       /* ETR recall measured with this step's assignment; -1 if ETR is off */
  int64_t survivors;   /* pairs that passed the first test */
  int64_t completed;   /* pairs whose distance was finished over all d dimensions */
  int64_t changed;     /* points whose assignment changed in this step */
  int64_t nempty;      /* empty clusters found by the update that followed */
  int64_t dense_dims;  /* dimensions multiplied on the matrix cores, summed over the 128 x 128 tiles of the step
                          (x 2*128*128 = executed MFMA flop of the progressive kernel) */
  int64_t dense_pair_blocks; /* (pair, trailing block) steps of alive pairs that were done inside dense tiles
                                (the rest of the steps went through the gather kernel) */
  int64_t gather_pair_blocks; /* (pair, trailing block) steps done by the gather kernel: each reads 256 bytes of the
                                 point's row and 256 bytes of the centroid's block */
  int64_t gather_pairs; /* pairs handed from the dense tiles to the gather kernel (16-byte list entries) */
  int64_t screen_dims; /* dimensions multiplied by the low-precision first filter (one fp16 product), summed over
                          its 128 x 128 tiles; 0 when the step ran without it */
  int64_t listed_tiles; /* tiles of 128 listed centroids that the exact kernel then processed (0 without the filter:
                           the exact kernel then takes every (row tile, column tile) pair) */
  int32_t dprime;      /* d' used by this step (d for iteration 1) */
  int32_t nblocks;     /* trailing 64-dim blocks (the last may be shorter) */
  int64_t enter[SKM_MAX_BLOCKS]; /* pairs that entered trailing block m (only when
                                    params.block_stats != 0, else zeros) */
  float ms_tau;        /* stage times from HIP events on the call's stream */
  float ms_gemm;
  float ms_prune;
  float ms_update;
  float ms_etr;
  float ms_step;       /* whole step including the update */
} skm_trace_row;

typedef struct skm_trace {
  int32_t capacity;    /* in : rows available in `row` (iters + 1 is enough) */
  int32_t rows;        /* out: rows written */
  int32_t iters_run;   /* out: update steps performed */
  int32_t inc_updates; /* out: update steps done incrementally (from the points that changed cluster only) */
  float ms_rotate;     /* out: the X~ = X R GEMM alone (events around its launch) */
  float ms_init;       /* out: everything before iteration 1: workspace, R, rotation, initial centroids, ETR set-up */
  float ms_etr_gt;     /* out: ETR ground truth (0 when supplied or ETR off) */
  float ms_unrotate;   /* out: Y = Y~ R^T */
  float ms_total;      /* out: whole call, device time (HIP events on the call's stream) */
  float ms_host_total; /* out: whole call on the host clock, entry to return (skm_fit_ex, skm_assign_ex) */
  float ms_host_alloc; /* out: of that, getting the workspace (0 with params->workspace) */
  float ms_host_free;  /* out: of that, releasing it */
  skm_trace_row *row;  /* host array, caller-allocated */
} skm_trace;

/* Hyper-parameters.  Fill with skm_params_default() first. */
typedef struct skm_params {
  float dprime_frac;     /* 0.125 : d' = floor(d * frac), kept a multiple of 16 (Algorithm 1) */
  float eps0;            /* 2.1   : ADSampling's epsilon_0 in theta(t, tau) = tau * min(1, (t/d)(1 + eps0/sqrt(t))^2);
                                    +inf leaves only the exact bound p_t > tau (then the result is exact Lloyd) */
  int32_t adjust_dprime; /* 1     : Section 4.8 controller on/off */
  float adj_lo;          /* 0.95 */
  float adj_hi;          /* 0.97 */
  float adj_step;        /* 0.20 */
  float split_eps;       /* 2^-10 : relative perturbation of a split centroid (Section 3.2) */
  int32_t final_assign;  /* 1     : run the final two-phase assignment pass (Section 3.3) */
  int32_t block_stats;   /* 0     : count pairs entering every trailing block (slower) */
  int32_t rotate;        /* 1     : 0 = treat the input as already rotated (R = I) */
  const float *R;        /* NULL  : device d x d rotation to use instead of generating one from the seed */
  const int64_t *init_idx; /* NULL: host array of k row indices to use as initial centroids */
  /* Early Termination by Recall (Section 3.3) */
  int32_t etr;           /* 0 */
  int32_t nq;            /* 1000 : number of queries */
  int32_t topk;          /* 10   : K of recall@K */
  float probe_frac;      /* 0.01 : probed share of the centroids */
  float etr_tol;         /* 0.005 */
  int32_t etr_patience;  /* 2 */
  const float *queries;  /* NULL : device nq x d; NULL = sample nq rows of X with the seed */
  const int64_t *gt;     /* NULL : device nq x topk exact neighbours; NULL = computed by the call */
  /* plumbing */
  void *stream;          /* hipStream_t, NULL = default stream */
  skm_trace *trace;      /* NULL or host struct to fill */
  int64_t pair_budget;   /* 0 = default (2^29): capacity, in (point, centroid) pairs, of the list that carries pairs
                            from the dense tiles to the gather kernel; points are processed in chunks of rows
                            sized so that the list cannot overflow */
  float dense_frac;      /* 0.0125 : a 128 x 128 tile keeps multiplying densely, 64 dimensions at a time, while more
                            than this share of its pairs is alive; below it the alive pairs are finished one by
                            one by the gather kernel.  1 = hand over right after the first test (the paper's
                            split), 0 = dense tiles only.  Execution strategy only: the tests applied to a
                            pair, and so the result, do not depend on it */
  float sample_frac;     /* 0    : in (0, 1): run Algorithm 1 on a uniform sample of round(frac * n) rows (at least k),
                            then assign every point to the final centroids with the two-phase step (Section 4.4) */
  int32_t angular;       /* 0    : 1 = angular metric (Section 2, "Determining Assignments"): the rotated points are scaled
                            to unit length and every centroid is scaled back to unit length after each update, so
                            the nearest centroid by L2 is the one of smallest angle; centroids_out are unit vectors and
                            dist_out is 2 - 2 cos.  skm_fit_ex only (not with ETR, sample_frac, the hierarchical fit
                            or skm_assign_ex: SKM_EINVAL) */
  int32_t full_update;   /* 0    : 1 = recompute every cluster sum from all points in every update.  By default, once at most
                            one point in eight changes its cluster, the fp64 sums of the previous update are
                            corrected by the rows that joined and left (the same means up to fp64 rounding) */
  void *workspace;       /* NULL : device memory, 256-byte aligned, of at least skm_workspace_bytes(n, d, k, params)
                            bytes (skm_hier_workspace_bytes for the hierarchical fit) that skm_fit_ex (also with
                            sample_frac), skm_assign_ex and skm_fit_hierarchical use instead of allocating their own.
                            With it the call makes no device allocation at all; a workspace that is too small is
                            refused with SKM_ENOMEM before any work is enqueued (the hierarchical fit runs its fine
                            phase with as many concurrent fits, at most eight, as the workspace holds; one that cannot
                            hold the largest fine fit is refused at that point).  Contents are undefined afterwards.
                            skm_fit_host ignores it */
  int64_t workspace_bytes; /* 0  : size of `workspace` */
  float conv_tol;        /* 0    : > 0 = also stop (Section 3.3, the second termination condition) after an iteration
                            t >= 2 in which at most this share of the points changed its cluster */
  int32_t screen;        /* 0    : low-precision first filter (Section 4.14, closing remark): before the exact tile
                            kernel, one fp16 product on the first d' dimensions and the first test theta(d', tau)
                            widened by the rounding bound find, per tile of 128 points, the centroids that can still
                            pass; the exact kernel (three products, exact tests and counters) then runs on those
                            only.  In iteration 1, where nothing prunes, the same one-product multiply over all
                            dimensions lists for every point the centroids that can be its nearest (those within the
                            rounding bound of the row's smallest approximate distance), and only those get their exact
                            distance.  0 = in pruned steps that follow a step which cut at least half of the pairs at the
                            first test, and in iteration 1 from 2048 centroids on; 1 = in every step; -1 = never.
                            Execution strategy only: a pair the filter drops is dropped by the exact arithmetic too */
  int32_t tau_group;     /* 0    : centroids after which a point's threshold tau is refreshed inside a step.  0 (= k):
                            tau keeps its initial value for the whole step, the only form this library runs (the
                            result is then independent of the order in which tiles are processed); any other value
                            but k is refused with SKM_EINVAL */
} skm_params;

void skm_params_default(skm_params *p);

/* Device bytes that skm_fit_ex (and skm_assign_ex) of this shape and these parameters take as workspace: what the
 * call allocates itself when params->workspace is NULL, and what a caller-owned workspace must hold.  params may be
 * NULL (defaults).  Returns a negative SKM_E* code for an invalid shape. */
int64_t skm_workspace_bytes(int64_t n, int32_t d, int32_t k, const skm_params *params);
/* The same for skm_fit_hierarchical: the rotated rows, the centroids and membership arrays, and below them the largest
 * of the meso fit, the final assignment and the worst case of the fine phase (one meso-cluster holding nearly every row
 * and cluster: with balanced meso-clusters eight concurrent fine fits need a fraction of that). */
int64_t skm_hier_workspace_bytes(int64_t n, int32_t d, int32_t k, const skm_params *params);

/*
 * skm_fit -- Algorithm 1 with default parameters.
 *   X             device n x d fp32, the points (original space)
 *   iters         number of k-means iterations (assignment + update), >= 1
 *   seed          drives the rotation, the initial centroids, splits, ETR sampling
 *   centroids_out device k x d fp32: the centroids in the ORIGINAL space
 *                 (Algorithm 1, last line), i.e. the means under the last in-loop
 *                 assignment
 *   assign_out    device n int32 or NULL: the final assignment (Section 3.3:
 *                 one more two-phase assignment against the final centroids)
 */
int skm_fit(const float *X, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed,
            float *centroids_out, int32_t *assign_out);

/* Same with explicit parameters; dist_out (device n fp32 or NULL) receives the
 * squared distance of every point to its assigned centroid.  With
 * params->final_assign == 0, assign_out / dist_out are those of the last
 * in-loop assignment step. */
int skm_fit_ex(const float *X, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed,
               const skm_params *params, float *centroids_out, int32_t *assign_out, float *dist_out);

/*
 * skm_fit_host -- Algorithm 1 on points that stay in HOST memory (Section 7.1:
 *   the points pass through the device in batches; copies and kernels overlap).
 *   For data larger than the device memory.  Every pass over the data (an
 *   iteration, or the final assignment) copies the rows to the device in batches
 *   of batch_rows rows through two buffers, rotates the batch there, assigns it,
 *   and adds its cluster sums (fp64) to those of the pass; the means are taken
 *   when the pass is complete.  The result is that of skm_fit_ex with
 *   params->full_update = 1, up to the rounding of sums taken in another order.
 *   X_host          HOST n x d fp32.  Page-locked memory (hipHostMalloc) lets the
 *                   copies run beside the kernels; pageable memory works, each
 *                   copy then holds the calling thread until it is done.
 *   batch_rows      rows per batch, rounded up to a multiple of 128; 0 = 131072.
 *                   Device memory in use: about 3 * batch_rows * d * 4 bytes for the
 *                   batches plus 8 (12 with dist_out_host) bytes per point.
 *   centroids_out   DEVICE k x d fp32, original space
 *   assign_out_host HOST n int32 or NULL; dist_out_host HOST n fp32 or NULL
 *   params->R, if set, is a DEVICE pointer as elsewhere; params->init_idx a host
 *   array.  Not combined with ETR, the angular metric or sample_frac
 *   (SKM_EINVAL).  params->trace: one row per pass, stage times summed over
 *   the batches (time spent waiting for a copy shows in ms_step only).
 *   The call returns after its last copy has completed.
 */
int skm_fit_host(const float *X_host, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed,
                 const skm_params *params, int64_t batch_rows, float *centroids_out, int32_t *assign_out_host,
                 float *dist_out_host);

/*
 * skm_fit_hierarchical -- Hierarchical SuperKMeans (Section 6).
 *   MESO: Algorithm 1 with skm_hier_meso_count(k) = round(sqrt(k)) clusters on
 *   all points, meso_iters iterations (3 in the paper) and the final
 *   assignment pass.  FINE: Algorithm 1 inside every meso-cluster (its points
 *   in ascending row order) with skm_hier_alloc's share of the k clusters,
 *   fine_iters iterations (5 in the paper), seed `seed + 1 + i` for
 *   meso-cluster i.  The k fine centroids, in meso order, are the result;
 *   every point is then assigned to them by the two-phase step without a
 *   previous assignment.  X is rotated once; both phases run in the rotated
 *   space.  Not combined with ETR, sample_frac, init_idx or final_assign = 0
 *   (SKM_EINVAL).
 *   centroids_out        device k x d fp32, original space
 *   assign_out, dist_out device n int32 / n fp32 or NULL: the final assignment
 *   meso_sizes_out_host  HOST int64[round(sqrt(k))] or NULL: points per meso-cluster
 *   fine_counts_out_host HOST int32[round(sqrt(k))] or NULL: fine clusters per meso-cluster
 *   params->trace, if set, receives the rows of the meso phase, then the row
 *   of the final assignment; ms_init = rotation + meso phase, ms_etr_gt = the
 *   fine phase, ms_total = everything.
 */
int skm_fit_hierarchical(const float *X, int64_t n, int32_t d, int32_t k, int32_t meso_iters, int32_t fine_iters,
                         uint64_t seed, const skm_params *params, float *centroids_out, int32_t *assign_out,
                         float *dist_out, int64_t *meso_sizes_out_host, int32_t *fine_counts_out_host);

/* Host rules of the hierarchical fit (Section 6).  The paper gives sqrt(k)
 * meso-clusters and sqrt(n_i) fine clusters in meso-cluster i; so that the
 * total is exactly k, the k clusters are shared out in proportion to
 * sqrt(n_i): one to every non-empty meso-cluster, then the floors of the
 * quotas (k - non-empty) * sqrt(n_i) / sum_j sqrt(n_j), then the rest one by
 * one by largest fractional part (lowest index on ties); never more clusters
 * than points.  sizes_host / counts_out_host are HOST arrays of km entries;
 * SKM_EINVAL unless 1 <= km <= k <= sum of sizes. */
int32_t skm_hier_meso_count(int32_t k);
int skm_hier_alloc(const int64_t *sizes_host, int32_t km, int32_t k, int32_t *counts_out_host);

/*
 * skm_assign -- one two-phase assignment step (Section 3.2, "2nd -> n
 * iteration"; Section 3.3, final assignment) of X against given centroids,
 * both in the original space; the rotation is generated from seed 0 unless
 * the _ex form supplies one.
 *   prev_assign   device n int32 or NULL.  With a previous assignment the
 *                 initial threshold is the distance to that centroid
 *                 (Section 3.4); without it the incumbent is the centroid of
 *                 smallest partial distance on the first d' dimensions.
 */
int skm_assign(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k,
               const int32_t *prev_assign, int32_t *assign_out, float *dist_out);

/* As skm_assign, with parameters (R, eps0, dprime_frac, stream, trace: one row).
 * dprime > 0 overrides floor(d * dprime_frac); it is rounded to a multiple of 16. */
int skm_assign_ex(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k,
                  const int32_t *prev_assign, int32_t dprime, const skm_params *params,
                  int32_t *assign_out, float *dist_out);

/* Exact assignment over all d dimensions (Algorithm 1, iteration 1): the GEMM
 * with the ||y||^2 - 2 x.y epilogue and a fused row argmin, then the direct
 * distance to the winner.  No rotation involved. */
int skm_assign_exact(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k,
                     void *stream, int32_t *assign_out, float *dist_out);

/* skm_assign_exact for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same kernels, the same results, but the call's working memory (packed
 * minima, centroid norms, operand bounds, the split-fp16 copy of the centroids) is a fixed 16 MiB array in device
 * memory that every GPU the library runs on holds until the process ends.  No hipMalloc, hipFree or allocating
 * library routine is called.  Limits (SKM_EINVAL beyond them): 1 <= n <= 1 048 576, 1 <= k <= 16 384, d a
 * multiple of 16 in [16, 16384], X and centroids 16-byte aligned.  All calls on one GPU share that array: calls
 * that overlap on one GPU (other threads, other streams) race; calls one after the other do not, whatever their
 * sizes.  The call returns after `stream` has been synchronised. */
int skm_assign_exact_static(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k, void *stream,
                            int32_t *assign_out, float *dist_out);

/* Centroid update (Section 3.2): per-cluster mean of the assigned rows; empty
 * clusters keep the row already in `centroids`.  counts_out: device k int32. */
int skm_update(const float *X, int64_t n, int32_t d, const int32_t *assign, int32_t k,
               void *stream, float *centroids, int32_t *counts_out);

/* Ground truth of Early Termination by Recall (Section 3.3): for every query (device nq x d, original space) the
 * indices of its topk nearest points of X by L2, nearest first, lowest index on equal distances; -1 where fewer than
 * topk points exist.  gt_out: device nq x topk int64.  This is what skm_fit_ex computes when params->etr is set and
 * params->gt is NULL; 1 <= topk <= 256. */
int skm_etr_ground_truth(const float *X, int64_t n, int32_t d, const float *queries, int32_t nq, int32_t topk,
                         void *stream, int64_t *gt_out);

/* Random orthogonal d x d matrix (Algorithm 1, first line) written to device
 * memory R_out; Haar-distributed (Gram-Schmidt, in fp64 on the device, of a seeded Gaussian
 * matrix); a function of (d, seed) only, reproducible bit by bit. */
int skm_make_rotation(int32_t d, uint64_t seed, void *stream, float *R_out);

/* out = X R (n x d), the rotation GEMM (Algorithm 1, second line); with
 * transpose != 0 computes X R^T (the un-rotation of the last line). */
int skm_rotate(const float *X, int64_t n, int32_t d, const float *R, int32_t transpose,
               void *stream, float *out);

/* k distinct row indices in [0, n), host output: the library's own
 * initialisation draw (Section 3.1), exposed so that it can be compared. */
int skm_sample_rows(uint64_t seed, int64_t n, int32_t k, int64_t *idx_out_host);

/* theta(t, tau) / tau for d total dimensions (the pruning ratio). */
float skm_theta_ratio(int32_t d, int32_t t, float eps0);

/* d' rules: initial value and the Section 4.8 adjustment. */
int32_t skm_dprime_init(int32_t d, float frac);
int32_t skm_dprime_adjust(int32_t d, int32_t dprime, double prune_frac, float lo, float hi, float step);

/* Launch choices of the GEMM kernels, for tests (Algorithm 1's products are the same whatever is chosen; only tile
 * shape and launch banding change).  Process-wide, takes effect for later calls, not synchronised with running ones.
 *   tile256    -1 = chosen by shape (default), 0 = never the 256 x 256 tiles, 1 = whenever the operands allow them
 *   panel_cols 0 = default, > 0 = column tiles per panel of the tile walk
 *   max_tiles  0 = default, > 0 = tiles per launch (a tall product is cut into bands of row tiles) */
void skm_debug_gemm_config(int32_t tile256, int32_t panel_cols, int64_t max_tiles);

const char *skm_strerror(int rc);
const char *skm_last_error(void); /* text of the last failure on this thread */
const char *skm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SKM_H_ */
