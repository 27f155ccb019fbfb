// C ABI of libskm and the host-side driver of Algorithm 1 (SuperKMeans): every arithmetic step on the
// points runs in the HIP kernels of this library; the host keeps scalars only (d', prune fraction,
// recall history, the list of empty clusters and the integer PRNG that re-seeds them).
#include "../../include/skm.h"
#include "skm_internal.h"

#include <algorithm>
#include <atomic>
#include <chrono>
#include <mutex>
#include <thread>
#include <unordered_map>
#include <system_error>
#include <functional>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>
#include <string>
#include <vector>

using namespace skm;

namespace {

thread_local std::string g_last_error;

int fail(int rc, const char *what) {
  g_last_error = what;
  return rc;
}
int fail_hip(hipError_t e, const char *where) {
  g_last_error = std::string(where) + ": " + hipGetErrorString(e);
  return e == hipErrorOutOfMemory ? SKM_ENOMEM : SKM_EHIP;
}
#define HIPCHK(expr)                                              \
  do {                                                            \
    hipError_t e__ = (expr);                                      \
    if (e__ != hipSuccess) return fail_hip(e__, #expr);           \
  } while (0)

// device allocations released when the call ends, whichever way it ends
// A preallocated slab that Pools of nested calls carve their buffers from (the hierarchical fit runs hundreds of small
// fits; a hipMalloc per buffer would dominate them).  A Pool constructed while an arena is current takes memory from it
// and gives it back, stack-like, when it is destroyed; what does not fit falls back to hipMalloc.
struct Arena {
  char *base = nullptr;
  size_t cap = 0, off = 0;
  bool owned = true;     // false: the caller's memory (params->workspace)
  bool strict = false;   // true: what does not fit is an error, never a hipMalloc
  ~Arena() {
    if (base && owned) (void)hipFree(base);
  }
  hipError_t init(size_t bytes) {
    cap = bytes;
    return hipMalloc(reinterpret_cast<void **>(&base), bytes);
  }
  void lend(void *mem, size_t bytes) {
    base = static_cast<char *>(mem);
    cap = bytes;
    owned = false;
    strict = true;
  }
};
thread_local Arena *tl_arena = nullptr;
struct ArenaScope {
  Arena *saved;
  explicit ArenaScope(Arena *a) : saved(tl_arena) { tl_arena = a; }
  ~ArenaScope() { tl_arena = saved; }
};

struct Pool {
  std::vector<void *> ptrs;
  Arena *arena = tl_arena;
  size_t mark = tl_arena ? tl_arena->off : 0;
  bool count_only = false;   // plan mode: add up what would be taken (256-byte granules), hand out nothing
  size_t counted = 0;
  ~Pool() {
    for (void *p : ptrs) (void)hipFree(p);
    if (arena) arena->off = mark;
  }
  template <typename T>
  hipError_t get(T **out, size_t count) {
    void *p = nullptr;
    size_t bytes = std::max<size_t>(count, 1) * sizeof(T);
    if (count_only) {
      counted += (bytes + 255) & ~(size_t)255;
      *out = nullptr;
      return hipSuccess;
    }
    if (arena) {
      const size_t at = (arena->off + 255) & ~(size_t)255;
      if (at + bytes <= arena->cap) {
        arena->off = at + bytes;
        *out = reinterpret_cast<T *>(arena->base + at);
        return hipSuccess;
      }
      if (arena->strict) {   // a caller-owned workspace: the call allocates nothing
        *out = nullptr;
        return hipErrorOutOfMemory;
      }
    }
    hipError_t e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
      *out = nullptr;
      return e;
    }
    ptrs.push_back(p);
    *out = static_cast<T *>(p);
    return hipSuccess;
  }
};

// Page-locked host memory for the few numbers that every step reports to the host: copies into it are asynchronous,
// so one wait per step covers all of them (a copy into pageable memory waits for its own staging).  Blocks are kept
// in a per-thread cache and reused by later calls on that thread (the hierarchical fit runs hundreds of small fits);
// worker threads release their cache before they end, that of a caller's thread stays until the process ends.
struct PinnedCache {
  std::vector<std::pair<void *, size_t>> idle;
  void *take(size_t bytes, size_t *cap) {
    for (size_t i = 0; i < idle.size(); ++i)
      if (idle[i].second >= bytes) {
        void *p = idle[i].first;
        *cap = idle[i].second;
        idle.erase(idle.begin() + (std::ptrdiff_t)i);
        return p;
      }
    void *p = nullptr;
    const size_t want = std::max<size_t>(bytes, (size_t)1 << 16);
    if (hipHostMalloc(&p, want, hipHostMallocDefault) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    *cap = want;
    return p;
  }
  void give(void *p, size_t cap) { idle.emplace_back(p, cap); }
  void release() {
    for (auto &b : idle) (void)hipHostFree(b.first);
    idle.clear();
  }
};
thread_local PinnedCache tl_pinned;

struct Events {
  std::vector<hipEvent_t> ev;
  ~Events() {
    for (hipEvent_t e : ev) (void)hipEventDestroy(e);
  }
  hipEvent_t next() {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    ev.push_back(e);
    return e;
  }
};

// Records (stage, event) marks on the stream; after a synchronisation the time between two
// consecutive marks is charged to the stage of the later mark.
enum Stage { ST_NONE = 0, ST_TAU, ST_GEMM, ST_PRUNE, ST_UPDATE, ST_ETR, ST_COUNT };
struct StageTimer {
  Events pool;
  std::vector<std::pair<int, hipEvent_t>> marks;
  size_t used = 0;
  hipStream_t st;
  bool on;
  StageTimer(hipStream_t s, bool enable) : st(s), on(enable) {}
  void mark(int stage) {
    if (!on) return;
    hipEvent_t e;
    if (used < pool.ev.size()) e = pool.ev[used];
    else e = pool.next();
    if (!e) return;
    ++used;
    (void)hipEventRecord(e, st);
    marks.push_back({stage, e});
  }
  // call after the stream is synchronised
  void collect(float ms[ST_COUNT], float *total) {
    for (int s = 0; s < ST_COUNT; ++s) ms[s] = 0.f;
    *total = 0.f;
    for (size_t i = 1; i < marks.size(); ++i) {
      float t = 0.f;
      if (hipEventElapsedTime(&t, marks[i - 1].second, marks[i].second) == hipSuccess) {
        ms[marks[i].first] += t;
        *total += t;
      }
    }
    marks.clear();
    used = 0;
  }
};

// ---------------------------------------------------------------- integer PRNG (splitmix64)
struct Rng {
  uint64_t s;
  uint64_t next() {
    s += 0x9E3779B97F4A7C15ULL;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
  }
  double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); }
};
Rng rng_stream(uint64_t seed, uint64_t stream) { return Rng{seed + stream * 0xD1342543DE82EF95ULL}; }
enum { STREAM_INIT = 0, STREAM_SPLIT = 1, STREAM_QUERIES = 2, STREAM_ROTATION = 3, STREAM_SAMPLE = 4 };

// k distinct indices of [0, n): the first k steps of a Fisher-Yates shuffle of the identity
void sample_rows(uint64_t seed, uint64_t stream, int64_t n, int32_t k, int64_t *out) {
  Rng r = rng_stream(seed, stream);
  if ((int64_t)k * 8 >= n) {
    std::vector<int64_t> perm((size_t)n);
    for (int64_t i = 0; i < n; ++i) perm[(size_t)i] = i;
    for (int32_t i = 0; i < k; ++i) {
      const int64_t j = i + (int64_t)(r.next() % (uint64_t)(n - i));
      std::swap(perm[(size_t)i], perm[(size_t)j]);
      out[i] = perm[(size_t)i];
    }
    return;
  }
  // few draws from many rows: the same shuffle, keeping only the entries that no longer hold their own index (step i
  // reads positions i and j >= i and never looks at a position below i again, so position i itself need not be kept)
  std::unordered_map<int64_t, int64_t> moved;
  moved.reserve((size_t)k * 2);
  for (int32_t i = 0; i < k; ++i) {
    const int64_t j = i + (int64_t)(r.next() % (uint64_t)(n - i));
    const auto it_i = moved.find(i);
    const int64_t vi = it_i == moved.end() ? (int64_t)i : it_i->second;
    const auto it_j = moved.find(j);
    out[i] = it_j == moved.end() ? j : it_j->second;
    moved[j] = vi;
  }
}

// ---------------------------------------------------------------- scalar rules
double theta_ratio(int32_t d, int32_t t, double eps0) {
  if (t >= d) return 1.0;
  if (t <= 0) return 0.0;
  const double s = 1.0 + eps0 / std::sqrt((double)t);
  const double r = (double)t / (double)d * s * s;
  return r < 1.0 ? r : 1.0;
}
int32_t snap16(double v, int32_t d) {
  int32_t top = d / 16 * 16;
  if (top < 16) top = 16;
  int32_t r = (int32_t)std::floor(v / 16.0 + 0.5) * 16;
  return std::min(std::max(r, 16), top);
}
int32_t dprime_init(int32_t d, double frac) { return snap16(std::floor((double)d * frac), d); }
int32_t dprime_adjust(int32_t d, int32_t dp, double f, double lo, double hi, double step) {
  // nearest multiple of 16, but at least one step of 16 in the chosen direction
  if (f > hi) return std::min(snap16((double)dp - step * (double)dp, d), snap16((double)dp - 16.0, d));
  if (f < lo) return std::max(snap16((double)dp + step * (double)dp, d), snap16((double)dp + 16.0, d));
  return dp;
}
// Section 6: sqrt(k) meso-clusters; the k fine clusters are shared out in proportion to sqrt(n_i), one to every
// non-empty meso-cluster first, floors of the quotas next, the rest by largest fractional part (lowest index on ties),
// never more clusters than points.
int32_t hier_meso_count(int32_t k) {
  const int32_t km = (int32_t)std::floor(std::sqrt((double)k) + 0.5);
  return std::min(std::max(km, 1), k);
}
void hier_alloc(const int64_t *sizes, int32_t km, int32_t k, int32_t *counts) {
  std::vector<double> root((size_t)km), frac((size_t)km);
  double W = 0.0;
  int64_t given = 0;
  for (int32_t i = 0; i < km; ++i) {
    root[(size_t)i] = std::sqrt((double)sizes[i]);
    W += root[(size_t)i];
    counts[i] = sizes[i] > 0 ? 1 : 0;
    given += counts[i];
  }
  const int64_t r = std::max<int64_t>((int64_t)k - given, 0);
  for (int32_t i = 0; i < km; ++i) {
    const double q = W > 0.0 ? (double)r * root[(size_t)i] / W : 0.0;
    const double whole = std::floor(q);
    const int64_t g = std::min<int64_t>((int64_t)whole, sizes[i] - counts[i]);
    counts[i] += (int32_t)g;
    given += g;
    frac[(size_t)i] = q - whole;
  }
  std::vector<int32_t> order((size_t)km);
  for (int32_t i = 0; i < km; ++i) order[(size_t)i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return frac[(size_t)a] > frac[(size_t)b]; });
  int64_t left = (int64_t)k - given;
  while (left > 0) {
    bool progress = false;
    for (int32_t a = 0; a < km && left > 0; ++a) {
      const int32_t i = order[(size_t)a];
      if ((int64_t)counts[i] < sizes[i]) {
        ++counts[i];
        --left;
        progress = true;
      }
    }
    if (!progress) break;
  }
}
int32_t nprobe_of(int32_t k, double frac) {
  int32_t np = (int32_t)std::floor(frac * (double)k + 0.5);
  return std::min(std::max(np, 1), k);
}

// ---------------------------------------------------------------- rotation matrix (device, fp64)
int make_rotation_dev(Pool &pool, int32_t d, uint64_t seed, hipStream_t st, float *R_out) {
  double *Qw = nullptr, *Cw = nullptr, *Ww = nullptr, *Lw = nullptr;
  HIPCHK(pool.get(&Qw, (size_t)d * d + 2));
  HIPCHK(pool.get(&Cw, std::max<size_t>((size_t)12 * 64 * d, (size_t)((d + 63) / 64) * 64 * 64)));
  HIPCHK(pool.get(&Ww, (size_t)((d + 63) / 64) * 64 * d));
  HIPCHK(pool.get(&Lw, (size_t)64 * 64));
  HIPCHK(launch_make_rotation(d, rng_stream(seed, STREAM_ROTATION).s, Qw, Cw, Ww, Lw, R_out, st));
  return SKM_OK;
}

inline int32_t round_up(int32_t v, int32_t m) { return (v + m - 1) / m * m; }

// *slot = bit pattern of max |A| (the bound the split-fp16 GEMMs scale their operands by)
int measure_absmax(const float *A, int64_t lda, int64_t rows, int32_t cols, unsigned int *slot, hipStream_t st,
                   int max_blocks = 0) {
  HIPCHK(launch_fill_u32(slot, 1, 0u, st));
  HIPCHK(launch_absmax(A, lda, rows, cols, slot, st, max_blocks));
  return SKM_OK;
}
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// fit = false: an assignment of n points to k given centroids, where k may exceed n
int check_shape(const void *X, int64_t n, int32_t d, int32_t k, bool fit = true) {
  if (!X) return fail(SKM_EINVAL, "null input pointer");
  if (n < 1 || n >= (int64_t)1 << 31) return fail(SKM_EINVAL, "n out of range [1, 2^31)");
  if (d < 16 || d > 16384) return fail(SKM_EINVAL, "d out of range [16, 16384]");
  if (k < 1 || (fit && k > n) || k > (1 << 24)) return fail(SKM_EINVAL, "k out of range [1, min(n, 2^24)]");
  return SKM_OK;
}

// ---------------------------------------------------------------- one fit / assign context
struct Ctx {
  hipStream_t st = nullptr;
  Pool pool;
  int64_t n = 0;
  int32_t d = 0, ds = 0, k = 0;
  const float *Xr = nullptr;  // rotated (or original) points, row stride ldx, padded to ds
  int64_t ldx = 0;
  float *Y = nullptr;         // centroids k x ds (rotated space)
  float *Ypdx = nullptr;
  uint32_t *Xs = nullptr;     // [n][ds + 32] split-fp16 copy of Xr for the progressive kernel, made with xnp
  uint32_t *Ys = nullptr;     // [k][ds + 32] the same of Y, remade in every pruned step
  float *xnp = nullptr;       // [ds / 16][n] prefix norms of the points at every multiple of 16 dims, written by the
  bool xnp_valid = false;     // first pruned step (the points of a context never change)
  // Regrouping (a fit with several steps left): once the tables exist and a full update has just grouped the points
  // by their cluster, the next threshold pass rewrites the points, their split copy, their tables and every per-point
  // array in that order.  Row tiles then hold points of one or two clusters, whose challengers are the same few
  // centroids: the alive pairs of a step gather in few tiles, the others end at the first test, and the rows and
  // centroid blocks the gather kernel fetches are shared by neighbouring pairs.
  float *Xr2 = nullptr;          // [n][ds] the points in the new order (NULL: no regrouping in this context)
  int32_t *pos_to_id = nullptr;  // [n] point of every position
  unsigned char *subkey = nullptr;   // [n] scratch: the key that orders the points inside a cluster
  bool regroup_ok = false;       // the caller has enough steps left for it to pay
  int32_t max_cluster = -1;      // size of the largest cluster at the last update (-1: none yet)
  bool group_now = false;        // a single step that groups the points by their incumbents itself (assign_impl)
  int32_t *grp_cnt = nullptr;    // [k] sizes of those groups
  bool order_fresh = false;      // up.order groups the points by the labels now in `prev`
  bool permuted = false;
  unsigned long long *point_keys = nullptr;   // keys that name points (ETR ground truth): renumbered with the points
  int64_t n_point_keys = 0;
  float *ynp = nullptr;       // [nb + 1][k] prefix norms of the centroids at the checkpoints of the current step
  float *ynorm = nullptr;
  float *tau = nullptr, *dist = nullptr;
  unsigned long long *best = nullptr;
  int32_t *assign = nullptr, *prev = nullptr;
  Pair *pairs = nullptr;
  int64_t pair_cap = 0, sub_cap = 0, chunk_rows = 0;
  int32_t nchunks = 0;
  unsigned int emit_max = 0;         // a tile with at most this many alive pairs goes to the gather kernel
  unsigned int *counters = nullptr;  // per chunk the fill counters of the sub-lists, then [1] error flag (overflow / unset point)
  size_t ncounters = 0;              // words in `counters` before the flag
  float *ratio_dev = nullptr;        // [kMaxBlocks + 1]
  float *ratio_host = nullptr;       // [kMaxBlocks + 1] page-locked staging for ratio_dev (behind the read-back block)
  unsigned long long *scal = nullptr;  // [SC_COUNT]
  double *obj_partial = nullptr, *obj = nullptr;
  UpdateWs up{};
  IncUpdateWs inc{};                 // workspace of the incremental update
  double *S = nullptr;               // [k][ds] cluster sums of the last update (fp64), valid once S_valid
  bool S_valid = false;
  bool split_last = false;           // the last update re-seeded empty clusters (their donors' rows are perturbed)
  int32_t inc_updates = 0;           // update steps that took the incremental path
  int32_t *split_dev = nullptr;
  bool block_stats = false;
  // low-precision first filter (screen.hip): mode as params->screen; buffers for one chunk of rows
  int32_t screen_mode = 0;
  double last_prune_frac = -1.0;     // of the previous pruned step of this context (-1: none yet)
  uint32_t *colmask = nullptr;
  float *scr_arow = nullptr, *scr_ycol = nullptr;
  uint32_t *Xh = nullptr, *Yh = nullptr;   // [n][ds / 2 + 16], [k][ds / 2 + 16]: the hi halves of Xs, Ys as planes of their own
  int32_t pruned_steps = 0;                // pruned steps this context has completed
  bool exact_filter_off = false;           // iteration 1 takes the full GEMM (set after a candidate-list overflow)
  int32_t *scr_cnt = nullptr, *scr_first = nullptr, *scr_ntiles = nullptr, *scr_cols = nullptr, *scr_tile_rt = nullptr;
  unsigned int *amax = nullptr;      // [AM_COUNT] magnitude bounds of the GEMM operands
  enum { AM_XR = 0, AM_Y = 1, AM_X = 2, AM_Q = 3, AM_QR = 4, AM_COUNT = 8 };

  // what a step reports (page-locked, see PinnedCache): the step scalars, the objective, the error flag, the
  // cluster sizes
  void *rb_block = nullptr;
  size_t rb_cap = 0;
  Ctx() = default;
  Ctx(const Ctx &) = delete;
  Ctx &operator=(const Ctx &) = delete;
  ~Ctx() {
    if (rb_block) tl_pinned.give(rb_block, rb_cap);   // a context lives and dies on one thread
  }
  unsigned long long *rb_scal = nullptr;   // [SC_COUNT * kStatReplicas]
  double *rb_obj = nullptr;
  unsigned int *rb_flag = nullptr;
  int32_t *rb_cnt = nullptr;               // [k]
  bool rb_cnt_valid = false;               // rb_cnt holds the sizes of c.assign's clusters
  char *zblock = nullptr;                  // device: counters | flag | scal | obj | up.cnt (see alloc_common)
  size_t zbytes = 0, rb_off = 0;           // the part from rb_off on is what comes back to the host
  // start of a step: everything it counts into is cleared
  int clear_step_block() {
    HIPCHK(hipMemsetAsync(zblock, 0, zbytes, st));
    return SKM_OK;
  }
  // end of a step: flag, scalars, objective and cluster sizes in one copy; the caller waits on the stream
  int fetch_step_block() {
    HIPCHK(hipMemcpyAsync(rb_block, zblock + rb_off, zbytes - rb_off, hipMemcpyDeviceToHost, st));
    return SKM_OK;
  }
  int alloc_readback(size_t o_scal, size_t o_obj, size_t o_cnt) {
    const size_t o_ratio = (zbytes - rb_off + 15) & ~(size_t)15;
    if (!rb_block) rb_block = tl_pinned.take(o_ratio + sizeof(float) * ((size_t)kMaxBlocks + 1), &rb_cap);
    char *h = static_cast<char *>(rb_block);
    if (!h) return fail(SKM_EHIP, "hipHostMalloc failed for the step read-back block");
    rb_flag = reinterpret_cast<unsigned int *>(h);
    rb_scal = reinterpret_cast<unsigned long long *>(h + o_scal);
    rb_obj = reinterpret_cast<double *>(h + o_obj);
    rb_cnt = reinterpret_cast<int32_t *>(h + o_cnt);
    ratio_host = reinterpret_cast<float *>(h + o_ratio);
    return SKM_OK;
  }

  int alloc_bounds() {
    HIPCHK(pool.get(&amax, (size_t)AM_COUNT));
    return SKM_OK;
  }
  int measure_xr() { return measure_absmax(Xr, ldx, n, ds, amax + AM_XR, st); }
  bool y_amax_valid = false;   // amax[AM_Y] bounds the current Y (the update writes it; other changes of Y clear this)
  int measure_y() {
    if (y_amax_valid) return SKM_OK;
    y_amax_valid = true;
    return measure_absmax(Y, ds, k, ds, amax + AM_Y, st);
  }

  int alloc_common(int64_t pair_budget, float dense_frac, bool need_update) {
    HIPCHK(pool.get(&Y, (size_t)k * ds));
    const int32_t nbmax = (ds - 16 + kBlockDims - 1) / kBlockDims + 1;
    HIPCHK(pool.get(&Ypdx, (size_t)nbmax * k * kBlockDims));
    HIPCHK(pool.get(&xnp, (size_t)(ds / 16) * n));
    HIPCHK(pool.get(&Xs, (size_t)n * (ds + 32)));
    HIPCHK(pool.get(&Ys, (size_t)k * (ds + 32)));
    HIPCHK(pool.get(&ynp, (size_t)nbmax * k));
    HIPCHK(pool.get(&ynorm, (size_t)k));
    HIPCHK(pool.get(&tau, (size_t)n));
    HIPCHK(pool.get(&dist, (size_t)n));
    HIPCHK(pool.get(&best, (size_t)n));
    HIPCHK(pool.get(&assign, (size_t)n));
    HIPCHK(pool.get(&prev, (size_t)n));
    // Every tile hands over at most emit_max pairs, so a chunk of rows needs tiles * emit_max slots.
    const int64_t tile_pairs = progressive_tile_pairs();
    if (!(dense_frac >= 0.f)) dense_frac = 0.f;
    if (dense_frac > 1.f) dense_frac = 1.f;
    emit_max = (unsigned int)std::llround((double)dense_frac * (double)tile_pairs);
    const int64_t per_tile = std::max<int64_t>(emit_max, 1);
    if (pair_budget <= 0) pair_budget = (int64_t)1 << 29;
    const int64_t col_tiles = progressive_tiles(1, k);
    int64_t row_tiles = std::max<int64_t>(pair_budget / (per_tile * col_tiles), 1);
    row_tiles = std::min<int64_t>(row_tiles, std::max<int64_t>(((1 << 24) - 1) / col_tiles, 1));  // launch size limit
    chunk_rows = std::min<int64_t>(row_tiles * 128, (n + 127) / 128 * 128);
    nchunks = (int32_t)((n + chunk_rows - 1) / chunk_rows);
    // each of the kSubLists parts must hold what the tiles of one XCD can hand over
    const int64_t tiles_chunk = progressive_tiles(std::min<int64_t>(chunk_rows, n), k);
    sub_cap = ((tiles_chunk + kSubLists - 1) / kSubLists) * per_tile;
    // the filtered iteration 1 lists a few candidates per point in the same list (if it ever overflows, the step is
    // redone with the full GEMM): room for 16 per point of a chunk in each of the eight parts
    // (the kernels behind the filter address a listed centroid's row with 32-bit offsets: not for a centroid table of
    // 2^31 words or more, where the steps simply run unfiltered)
    const bool may_screen = (screen_mode > 0 || (screen_mode == 0 && k >= 2 * progressive_tile_cols())) &&
                            (int64_t)k * (ds + 32) < ((int64_t)1 << 31);
    if (may_screen) sub_cap = std::max<int64_t>(sub_cap, 16 * std::min<int64_t>(chunk_rows, n));
    pair_cap = sub_cap * kSubLists;
    if (pair_cap >= ((int64_t)1 << 32)) return fail(SKM_EINVAL, "pair_budget too large (must stay below 2^32 pairs)");
    HIPCHK(pool.get(&pairs, (size_t)pair_cap));
    ncounters = (size_t)nchunks * (kSubLists + 16) * kSubListStride;   // list fill counters, tile counters of the two tile kernels
    if (may_screen) {   // (unless forced: of no use below two column tiles)
      // one bit per (row tile, centroid); at most one tile of listed columns per (row tile, column tile) of the chunk
      const int64_t nrt_chunk = (std::min<int64_t>(chunk_rows, n) + 127) / 128;
      HIPCHK(pool.get(&colmask, (size_t)nrt_chunk * 4 * (size_t)col_tiles));
      HIPCHK(pool.get(&scr_cnt, (size_t)nrt_chunk));
      HIPCHK(pool.get(&scr_first, (size_t)nrt_chunk));
      HIPCHK(pool.get(&scr_ntiles, 2));   // the tile count, then a float scalar of the filter
      HIPCHK(pool.get(&scr_arow, (size_t)std::min<int64_t>(chunk_rows, n)));
      HIPCHK(pool.get(&scr_ycol, (size_t)k));
      HIPCHK(pool.get(&Xh, (size_t)n * (ds / 2 + 16)));
      HIPCHK(pool.get(&Yh, (size_t)k * (ds / 2 + 16)));
      HIPCHK(pool.get(&scr_cols, (size_t)tiles_chunk * 128));
      HIPCHK(pool.get(&scr_tile_rt, (size_t)tiles_chunk));
    }
    // Everything a step clears at its start and reports at its end is one block: counters | flag | step scalars |
    // objective | cluster sizes.  One memset, and one copy (from the flag on) into the page-locked mirror.
    {
      const size_t nscal = (size_t)SC_COUNT * kStatReplicas;
      const size_t off_flag = ncounters * sizeof(unsigned int);
      const size_t off_scal = (off_flag + sizeof(unsigned int) + 7) & ~(size_t)7;
      const size_t off_obj = off_scal + nscal * sizeof(unsigned long long);
      const size_t off_cnt = off_obj + sizeof(double);
      zbytes = off_cnt + sizeof(int32_t) * (size_t)k;
      HIPCHK(pool.get(&zblock, zbytes));
      rb_off = off_flag;
      if (zblock) {
        counters = reinterpret_cast<unsigned int *>(zblock);
        scal = reinterpret_cast<unsigned long long *>(zblock + off_scal);
        obj = reinterpret_cast<double *>(zblock + off_obj);
        up.cnt = reinterpret_cast<int32_t *>(zblock + off_cnt);
      }
      if (!pool.count_only)   // (a size query touches no device and no page-locked memory)
        if (int rc = alloc_readback(off_scal - off_flag, off_obj - off_flag, off_cnt - off_flag)) return rc;
    }
    HIPCHK(pool.get(&ratio_dev, (size_t)kMaxBlocks + 1));
    HIPCHK(pool.get(&obj_partial, (size_t)(n + 1023) / 1024));   // at least finalize_blocks(m) for every m <= n
    if (need_update) {
      HIPCHK(pool.get(&up.off, (size_t)k + 1));
      HIPCHK(pool.get(&up.cursor, (size_t)k));
      HIPCHK(pool.get(&up.segoff, (size_t)k + 1));
      HIPCHK(pool.get(&up.order, (size_t)n));
      up.max_segments = update_max_segments(n, k);
      HIPCHK(pool.get(&up.partial, (size_t)up.max_segments * ds));
      HIPCHK(pool.get(&split_dev, (size_t)3 * k + 2));   // (empty, donor) pairs | first split of every chain
      // the incremental update is used while at most one point in eight changes its label
      HIPCHK(pool.get(&S, (size_t)k * ds));
      inc.capacity = 2 * (n / 8) + 2;
      inc.max_segments = update_max_segments(inc.capacity, k);
      HIPCHK(pool.get(&inc.ent_id, (size_t)inc.capacity));
      HIPCHK(pool.get(&inc.ent_lab, (size_t)inc.capacity));
      HIPCHK(pool.get(&inc.order, (size_t)inc.capacity));
      HIPCHK(pool.get(&inc.cnt, (size_t)k));
      HIPCHK(pool.get(&inc.off, (size_t)k + 1));
      HIPCHK(pool.get(&inc.cursor, (size_t)k));
      HIPCHK(pool.get(&inc.segoff, (size_t)k + 1));
      HIPCHK(pool.get(&inc.counter, 1));
      HIPCHK(pool.get(&inc.partial, (size_t)inc.max_segments * ds));
    }
    return SKM_OK;
  }
};

// Bytes that a context of this shape takes from its pool (alloc_bounds + alloc_common), counted without allocating.
size_t plan_common_bytes(int64_t n, int32_t d, int32_t k, int64_t pair_budget, float dense_frac, bool need_update) {
  Ctx t;
  t.pool.count_only = true;
  t.n = n; t.d = d; t.k = k;
  t.ds = (d + 15) / 16 * 16;
  if (t.alloc_bounds() != SKM_OK || t.alloc_common(pair_budget, dense_frac, need_update) != SKM_OK) return 0;
  return t.pool.counted;
}

// One device allocation for the whole workspace of a top-level call instead of some forty (3.4 ms of allocation and
// release per fit of 1M x 1536 become 0.8 ms).  Declared before the context, so that the context's pool carves from it.
// A nested call (a worker of the hierarchical fit, the steps of the sampled fit) finds an arena in place and adds none;
// whatever does not fit, or the whole workspace if this allocation fails, comes from hipMalloc as before.
struct CallArena {
  Arena arena;
  bool on = false;
  bool too_small = false;   // a caller's workspace that cannot hold `bytes`
  explicit CallArena(size_t bytes, void *lent = nullptr, int64_t lent_bytes = 0) {
    if (tl_arena || bytes == 0) return;
    if (lent) {
      // the caller's memory: aligned up to the 256-byte granule of the pools
      const uintptr_t a = (reinterpret_cast<uintptr_t>(lent) + 255) & ~(uintptr_t)255;
      const size_t lost = (size_t)(a - reinterpret_cast<uintptr_t>(lent));
      if (lent_bytes < 0 || (size_t)lent_bytes < bytes + lost) {
        too_small = true;
        return;
      }
      arena.lend(reinterpret_cast<void *>(a), (size_t)lent_bytes - lost);
      tl_arena = &arena;
      on = true;
      return;
    }
    if (arena.init(bytes) != hipSuccess) {
      (void)hipGetLastError();
      arena.base = nullptr;
      arena.cap = 0;
      return;
    }
    tl_arena = &arena;
    on = true;
  }
  ~CallArena() {
    if (on) tl_arena = nullptr;
  }
  CallArena(const CallArena &) = delete;
  CallArena &operator=(const CallArena &) = delete;
};

// Host-clock readings of one call: entry, workspace ready, body done; the destructor (declared before the arena, so it
// runs after the arena's release) writes them to the caller's trace.
struct HostTimes {
  using clk = std::chrono::steady_clock;
  clk::time_point t0 = clk::now(), t_ws = t0, t_done = t0;
  skm_trace *tr = nullptr;
  bool done = false;
  static float ms(clk::time_point a, clk::time_point b) { return std::chrono::duration<float, std::milli>(b - a).count(); }
  void workspace_ready() { t_ws = clk::now(); }
  void body_done(skm_trace *t) {
    tr = t;
    t_done = clk::now();
    done = true;
  }
  ~HostTimes() {
    if (!tr || !done) return;
    const auto t1 = clk::now();
    tr->ms_host_alloc = ms(t0, t_ws);
    tr->ms_host_free = ms(t_done, t1);
    tr->ms_host_total = ms(t0, t1);
  }
};

// Upper bound of the device bytes one plain fit (or one assignment call) of this shape carves from its arena: the
// context's buffers, the rotated points and their regrouped copy, the rotation matrices and their generator, the ETR
// buffers.  What skm_workspace_bytes reports.
inline bool assign_groups(int64_t n, int32_t ds, int32_t k, int32_t screen_mode);
// ... of one assignment call (assign_impl)
size_t assign_workspace_need(int64_t n, int32_t d, int32_t k, const skm_params &p) {
  const size_t ds0 = (size_t)((d + 15) / 16 * 16);
  const size_t plan = plan_common_bytes(n, d, k, p.pair_budget, p.dense_frac, false);
  if (!plan) return 0;
  const size_t grouping = assign_groups(n, (int32_t)ds0, k, p.screen) ? (size_t)n * ds0 * 4 + (size_t)n * 9 + (size_t)k * 20 + 4096 : 0;
  return plan + grouping + (size_t)n * ds0 * 4 + 10 * (size_t)d * ds0 * 4 + (size_t)d * 16384 + ((size_t)32 << 20);
}
int64_t sample_size(int64_t n, int32_t k, float frac) {
  const int64_t s = (int64_t)std::llround((double)frac * (double)n);
  return std::min<int64_t>(std::max<int64_t>(s, k), n);
}
size_t fit_workspace_need(int64_t n, int32_t d, int32_t k, const skm_params &p) {
  const size_t ds0 = (size_t)((d + 15) / 16 * 16);
  if (p.sample_frac > 0.f && p.sample_frac < 1.f) {
    // the sampled fit: all rows rotated (and a dense copy of them when d is no multiple of 16), the sample, the
    // centroids, and below them first the fit on the sample, then the assignment of all rows
    skm_params q = p;
    q.sample_frac = 0.f;
    const int64_t s = sample_size(n, k, p.sample_frac);
    const size_t a = fit_workspace_need(s, d, k, q), b = assign_workspace_need(n, d, k, q);
    if (!a || !b) return 0;
    return std::max(a, b) + (size_t)n * ds0 * 4 + (ds0 != (size_t)d ? (size_t)n * d * 4 : 0) + (size_t)s * (8 + (size_t)d * 4) +
           (size_t)k * (d + ds0) * 4 + (size_t)n * 4 + 10 * (size_t)d * ds0 * 4 + (size_t)d * 16384 + ((size_t)32 << 20);
  }
  const size_t plan = plan_common_bytes(n, d, k, p.pair_budget, p.dense_frac, true);
  if (!plan) return 0;
  size_t need = plan + 2 * (size_t)n * ds0 * 4 + (size_t)n * 5 + 10 * (size_t)d * ds0 * 4 + (size_t)d * 16384 +
                (size_t)k * 16 + ((size_t)32 << 20);
  if (p.etr && p.nq > 0 && p.topk > 0) {
    const size_t nq = (size_t)p.nq;
    need += (size_t)n * 4 + nq * (size_t)std::min<int64_t>(n, 1 << 16) * 4 + nq * (size_t)p.topk * 8 + nq * (ds0 + d) * 4 +
            nq * 8 + nq * (size_t)k * 4 + (size_t)k * 4 + ((size_t)1 << 16);
  }
  return need;
}

struct StepStats {
  double objective = 0;
  int64_t survivors = 0, completed = 0, changed = 0, dense_dims = 0, dense_pair_blocks = 0;
  int64_t gather_pair_blocks = 0, gather_pairs = 0, screen_dims = 0, listed_tiles = 0;
  int64_t enter[SKM_MAX_BLOCKS] = {0};
  int32_t dprime = 0, nblocks = 0;
  bool pruned = false;  // false for the exact step of iteration 1
};

// Iteration 1 with the low-precision filter in front (screen.hip, exact mode): one fp16 product over all dimensions
// lists, for every point, the centroids that can be its nearest; the gather kernel takes their exact distances and the
// packed minimum is the exact nearest centroid (lowest index on ties).  A third of the matrix work of the full
// three-product GEMM; pays once there are enough centroids.
// c.best[i] = packed (squared distance over dims [0, K), centroid) of the centroid nearest to point i on those dims,
// exact (direct form, lowest index on ties): the one-product multiply over K dims lists the candidates, the gather
// kernel takes their distances.  K = ds: the nearest centroid; K = d': the incumbent of a step that comes without one.
// Clobbers ynorm, Ypdx, Ys / Yh, ratio_dev, tau; sets bit 0 of the step's flag word if the candidate list overflowed.
int filtered_nearest(Ctx &c, int32_t K, StageTimer *tm = nullptr) {
  const int32_t nbK = (K + kBlockDims - 1) / kBlockDims;
  if (nbK > kMaxBlocks) return fail(SKM_EINTERNAL, "too many blocks");
  if (!c.xnp_valid) {
    // the points' split copy, its hi plane and their norms do not exist before the first pruned step: the pass that
    // writes them runs now (its thresholds, against centroid 0, are discarded)
    HIPCHK(launch_fill_u32(reinterpret_cast<unsigned int *>(c.prev), c.n, 0u, c.st));
    HIPCHK(launch_tau_init(c.Xr, c.ldx, c.n, c.ds, c.Y, c.ds, c.prev, c.tau, nullptr, c.st, c.xnp, c.Xs,
                           c.amax + Ctx::AM_XR, nullptr, nullptr, nullptr, c.Xh));
    c.xnp_valid = true;
  }
  // ||y[0 : K)||^2 and the block-major copy of the first K dimensions, zero filled behind them (the gather kernel
  // starts every pair at dimension 0 and is told that rows end at K)
  HIPCHK(launch_prep_centroids(c.Y, c.ds, c.k, K, K, c.ynorm, 0, nbK, c.Ypdx, c.st));
  if (int rc = c.measure_y()) return rc;
  HIPCHK(launch_split_rows(c.Y, c.ds, c.k, c.ds, c.amax + Ctx::AM_Y, c.Ys, c.st, c.Yh));
  HIPCHK(launch_fill_u64(c.best, c.n, ~0ull, c.st));
  unsigned int *rowmin = reinterpret_cast<unsigned int *>(c.tau);   // (no thresholds while this runs)
  HIPCHK(launch_fill_u32(rowmin, c.n, 0xffffffffu, c.st));
  float *ratio = c.ratio_host;
  for (int m = 0; m <= nbK; ++m) ratio[m] = 1.f;   // nothing is dropped on the way
  HIPCHK(hipMemcpyAsync(c.ratio_dev, ratio, sizeof(float) * ((size_t)nbK + 1), hipMemcpyHostToDevice, c.st));
  if (tm) tm->mark(ST_TAU);
  for (int32_t ch = 0; ch < c.nchunks; ++ch) {
    const int64_t r0 = (int64_t)ch * c.chunk_rows;
    const int64_t rows = std::min<int64_t>(c.chunk_rows, c.n - r0);
    unsigned int *fill = c.counters + (size_t)ch * kSubLists * kSubListStride;
    ScreenLaunch sl{};
    sl.A = c.Xh + r0 * (c.ds / 2 + 16); sl.lda = c.ds / 2 + 16; sl.M = (int32_t)rows;
    sl.B = c.Yh; sl.ldb = c.ds / 2 + 16; sl.N = c.k;
    sl.a_absmax = c.amax + Ctx::AM_XR; sl.b_absmax = c.amax + Ctx::AM_Y;
    sl.ds = c.ds; sl.dprime = K; sl.ratio0 = 1.f;
    sl.tau = c.tau; sl.row_base = r0;
    sl.xn = c.xnp + (int64_t)(K / 16 - 1) * c.n;   // ||x[0 : K)||^2: row K / 16 - 1 of the prefix table
    sl.yn = c.ynorm;
    sl.arow = c.scr_arow; sl.ycol = c.scr_ycol;
    sl.colmask = c.colmask; sl.cnt = c.scr_cnt; sl.first = c.scr_first; sl.ntiles = c.scr_ntiles;
    sl.col_list = c.scr_cols; sl.tile_rt = c.scr_tile_rt;
    sl.scal = c.scal;
    sl.exact = 1; sl.rowmin = rowmin; sl.pairs = c.pairs; sl.pair_count = fill; sl.sub_capacity = (unsigned int)c.sub_cap;
    sl.overflow = c.counters + c.ncounters;
    HIPCHK(launch_screen(sl, c.st));
    PruneArgs pa{c.pairs, fill, (unsigned int)c.sub_cap, c.Xr, c.ldx, c.n, c.Ypdx, c.k, 0, K, nbK, c.ratio_dev,
                 c.best, c.scal, 0};
    HIPCHK(launch_prune(pa, c.st));
  }
  return SKM_OK;
}

int step_exact_filtered(Ctx &c, StageTimer &tm, StepStats &ss) {
  tm.mark(ST_NONE);
  if (int rc = c.clear_step_block()) return rc;
  if (int rc = filtered_nearest(c, c.ds, &tm)) return rc;
  tm.mark(ST_GEMM);
  // the packed minima already hold the direct distances
  HIPCHK(launch_finalize_assign(c.best, nullptr, c.n, c.assign, c.dist, c.up.cnt, c.k, c.obj_partial, nullptr,
                                c.counters + c.ncounters, c.st));
  HIPCHK(launch_sum_partials(c.obj_partial, finalize_blocks(c.n), c.obj, c.st));
  tm.mark(ST_TAU);
  if (int rc = c.fetch_step_block()) return rc;
  HIPCHK(hipStreamSynchronize(c.st));
  c.rb_cnt_valid = true;
  const size_t nscal = (size_t)SC_COUNT * kStatReplicas;
  ss = StepStats();
  for (int r = 0; r < kStatReplicas; ++r) {
    ss.gather_pair_blocks += (int64_t)c.rb_scal[(size_t)r * SC_COUNT + SC_GATHER_PB];
    ss.gather_pairs += (int64_t)c.rb_scal[(size_t)r * SC_COUNT + SC_GATHER_PAIRS];
    ss.screen_dims += (int64_t)c.rb_scal[(size_t)r * SC_COUNT + SC_SCREEN_DIMS];
  }
  (void)nscal;
  ss.objective = *c.rb_obj;
  ss.dprime = c.d;
  ss.changed = c.n;
  return SKM_OK;
}

// Iteration 1 of Algorithm 1: exact assignment over all dims.  Leaves assign, dist, cluster sizes.
int step_exact(Ctx &c, StageTimer &tm, StepStats &ss) {
  // many centroids: the low-precision filter first, exact distances for the few candidates it leaves
  if (c.colmask && !c.exact_filter_off && (c.screen_mode > 0 || c.k >= 2048)) {
    if (int rc = step_exact_filtered(c, tm, ss)) return rc;
    if ((*c.rb_flag & 1u) == 0) {
      if (*c.rb_flag != 0) return fail(SKM_EINTERNAL, "a point was left without a centroid");
      return SKM_OK;
    }
    c.exact_filter_off = true;   // the candidate list overflowed (never with the default capacities): the full GEMM instead
  }
  tm.mark(ST_NONE);
  if (int rc = c.clear_step_block()) return rc;
  HIPCHK(launch_prep_centroids(c.Y, c.ds, c.k, c.ds, c.ds, c.ynorm, 0, 0, nullptr, c.st));
  HIPCHK(launch_fill_u64(c.best, c.n, ~0ull, c.st));
  if (int rc = c.measure_y()) return rc;
  GemmOperands g{c.Xr, c.ldx, (int32_t)c.n, c.Y, c.ds, c.k, c.ds};
  g.a_absmax = c.amax + Ctx::AM_XR; g.b_absmax = c.amax + Ctx::AM_Y;
  g.b_split = c.Ys;   // every pruned step remakes it: free here
  HIPCHK(gemm_argmin(g, c.ynorm, c.best, c.st));
  tm.mark(ST_GEMM);
  // winners -> direct squared distances (also the objective of this step)
  HIPCHK(launch_finalize_assign(c.best, nullptr, c.n, c.assign, nullptr, nullptr, c.k, nullptr, nullptr, c.counters + c.ncounters, c.st));
  HIPCHK(launch_tau_init(c.Xr, c.ldx, c.n, c.ds, c.Y, c.ds, c.assign, nullptr, c.best, c.st));
  HIPCHK(launch_finalize_assign(c.best, nullptr, c.n, c.assign, c.dist, c.up.cnt, c.k, c.obj_partial, nullptr, nullptr, c.st));
  HIPCHK(launch_sum_partials(c.obj_partial, finalize_blocks(c.n), c.obj, c.st));
  tm.mark(ST_TAU);
  if (int rc = c.fetch_step_block()) return rc;
  HIPCHK(hipStreamSynchronize(c.st));
  c.rb_cnt_valid = true;
  if (*c.rb_flag != 0) return fail(SKM_EINTERNAL, "a point was left without a centroid");
  ss = StepStats();
  ss.objective = *c.rb_obj;
  ss.dprime = c.d;
  ss.changed = c.n;
  return SKM_OK;
}

// Iterations >= 2 of Algorithm 1: initial threshold, progressive-pruning GEMM, gather kernel for the
// pairs of sparse tiles, argmin.  On entry c.prev holds the incumbents (c.assign is overwritten);
// have_prev = false seeds the incumbent with the centroid of smallest partial distance.
int step_pruned(Ctx &c, StageTimer &tm, int32_t dprime, double eps0, bool have_prev, StepStats &ss) {
  const int32_t nb = (c.d - dprime + kBlockDims - 1) / kBlockDims;
  if (nb > kMaxBlocks) return fail(SKM_EINTERNAL, "too many trailing blocks");
  tm.mark(ST_NONE);
  bool found = false;   // the incumbents of a step that came without them are in c.prev
  if (!have_prev && c.colmask && !c.exact_filter_off && (c.screen_mode > 0 || c.k >= 2048)) {
    // many centroids: the nearest centroid on the first d' dimensions through the low-precision filter (a third of
    // the matrix work of the three-product GEMM below); if its candidate list overflows, that GEMM runs after all
    if (int rc = c.clear_step_block()) return rc;
    if (int rc = filtered_nearest(c, dprime, &tm)) return rc;
    HIPCHK(launch_finalize_assign(c.best, nullptr, c.n, c.prev, nullptr, nullptr, c.k, nullptr, nullptr, c.counters + c.ncounters, c.st));
    HIPCHK(hipMemcpyAsync(c.rb_flag, c.counters + c.ncounters, sizeof(unsigned int), hipMemcpyDeviceToHost, c.st));
    HIPCHK(hipStreamSynchronize(c.st));
    if (*c.rb_flag == 0) found = true;
    else if (*c.rb_flag & 1u) c.exact_filter_off = true;
    else return fail(SKM_EINTERNAL, "a point was left without a centroid");
    tm.mark(ST_GEMM);
  }
  HIPCHK(launch_prep_centroids(c.Y, c.ds, c.k, c.ds, dprime, c.ynorm, dprime, nb, c.Ypdx, c.st, c.ynp));
  if (int rc = c.measure_y()) return rc;
  // theta ratio at checkpoint m: t_m = min(d, d' + 64 m) dimensions seen
  float *ratio = c.ratio_host;
  for (int m = 0; m <= nb; ++m) ratio[m] = (float)theta_ratio(c.d, std::min(c.d, dprime + kBlockDims * m), eps0);
  HIPCHK(hipMemcpyAsync(c.ratio_dev, ratio, sizeof(float) * ((size_t)nb + 1), hipMemcpyHostToDevice, c.st));
  if (int rc = c.clear_step_block()) return rc;
  if (!have_prev && !found) {
    HIPCHK(launch_fill_u64(c.best, c.n, ~0ull, c.st));
    GemmOperands g0{c.Xr, c.ldx, (int32_t)c.n, c.Y, c.ds, c.k, dprime};
    g0.a_absmax = c.amax + Ctx::AM_XR; g0.b_absmax = c.amax + Ctx::AM_Y;
    g0.b_split = c.Ys;   // rewritten for all dimensions below
    HIPCHK(gemm_argmin(g0, c.ynorm, c.best, c.st));
    HIPCHK(launch_finalize_assign(c.best, nullptr, c.n, c.prev, nullptr, nullptr, c.k, nullptr, nullptr, c.counters + c.ncounters, c.st));
    tm.mark(ST_GEMM);
  }
  // (not before one pruned step has run: the labels of iteration 1, assigned against the initial rows, group the points
  // far less usefully than those of iteration 2)
  bool regroup = c.regroup_ok && !c.permuted && c.xnp_valid && c.order_fresh && c.Xr2 && have_prev && c.pruned_steps >= 1;
  if (c.group_now && !c.permuted && c.Xr2) {
    // A step on its own (no update before it left an order): the points are grouped by the incumbents they come with
    // (or were just given above), so that a row tile holds the points of one or two clusters and the first filter has
    // columns to drop.  One read-back of the group sizes decides whether the order is reproducible (see below).
    HIPCHK(launch_group_order(c.prev, c.n, c.k, c.grp_cnt, c.up.off, c.up.cursor, c.up.segoff, c.up.order, c.st));
    HIPCHK(hipMemcpyAsync(c.rb_cnt, c.grp_cnt, sizeof(int32_t) * (size_t)c.k, hipMemcpyDeviceToHost, c.st));
    HIPCHK(hipStreamSynchronize(c.st));
    c.max_cluster = *std::max_element(c.rb_cnt, c.rb_cnt + c.k);
    c.rb_cnt_valid = false;
    regroup = true;
    c.group_now = false;
  }
  if (regroup) {
    // The update leaves the members of a cluster sorted by index only up to a size (larger clusters keep the order in
    // which the scatter placed them, which depends on scheduling): with such a cluster the new order, and with it the
    // rounding of the results, would differ from run to run.  Those fits keep the input order.
    // (the sizes came back with the previous step's scalars: no copy, no wait here)
    regroup = c.max_cluster >= 0 && c.max_cluster <= update_sort_cap();
    if (!regroup) c.regroup_ok = false;
  }
  if (regroup) {
    // this pass reads every point anyway: it writes them back grouped by cluster (see Ctx)
    // Inside a cluster that spans several row tiles the points follow the signs of their first four dimensions, then
    // their index: which points of a cluster share a tile matters (measured: -3 % on a fit with 1000 points per
    // cluster, nothing to gain where a cluster is smaller than a tile).
    if (c.n / c.k >= 128)
      HIPCHK(launch_suborder(c.Xr, c.ldx, c.n, c.k, c.up.off, c.up.order, c.subkey, c.pos_to_id, c.st));
    else
      HIPCHK(hipMemcpyAsync(c.pos_to_id, c.up.order, sizeof(int32_t) * (size_t)c.n, hipMemcpyDeviceToDevice, c.st));
    HIPCHK(launch_tau_init(c.Xr, c.ldx, c.n, c.ds, c.Y, c.ds, c.prev, c.tau, c.best, c.st, c.xnp, c.Xs,
                           c.amax + Ctx::AM_XR, c.pos_to_id, c.Xr2, c.assign, c.Xh));
    std::swap(c.prev, c.assign);   // the incumbents in the new order; the other buffer receives this step's labels
    if (c.point_keys)   // (up.order is scratch until the next full update rebuilds it)
      HIPCHK(launch_remap_key_ids(c.point_keys, c.n_point_keys, c.pos_to_id, c.n, c.up.order, c.st));
    c.Xr = c.Xr2;
    c.ldx = c.ds;
    c.permuted = true;
  } else {
    // the first pruned step of a context also writes the tables that depend on the points only
    HIPCHK(launch_tau_init(c.Xr, c.ldx, c.n, c.ds, c.Y, c.ds, c.prev, c.tau, c.best, c.st, c.xnp_valid ? nullptr : c.xnp,
                           c.xnp_valid ? nullptr : c.Xs, c.amax + Ctx::AM_XR, nullptr, nullptr, nullptr,
                           c.xnp_valid ? nullptr : c.Xh));
  }
  c.order_fresh = false;
  c.xnp_valid = true;
  // Low-precision first filter: worth its pass over the front dimensions when most columns of a tile die at the
  // first test.  The previous step's prune fraction predicts that from below (the centroids only get better): the
  // step after one that cut half of the pairs cuts 85 to 99 % on the mixture workloads, and a wasted filter pass
  // costs a tenth of the poorly pruned step it precedes.
  const bool screen = c.colmask && nb > 0 &&
                      (c.screen_mode > 0 || (c.screen_mode == 0 && c.last_prune_frac >= 0.50));
  HIPCHK(launch_split_rows(c.Y, c.ds, c.k, c.ds, c.amax + Ctx::AM_Y, c.Ys, c.st, screen ? c.Yh : nullptr));
  tm.mark(ST_TAU);
  for (int32_t ch = 0; ch < c.nchunks; ++ch) {
    const int64_t r0 = (int64_t)ch * c.chunk_rows;
    const int64_t rows = std::min<int64_t>(c.chunk_rows, c.n - r0);
    ProgArgs g{};
    g.A = c.Xs + r0 * (c.ds + 32); g.lda = c.ds + 32; g.M = (int32_t)rows;
    g.B = c.Ys; g.ldb = c.ds + 32; g.N = c.k;
    g.a_absmax = c.amax + Ctx::AM_XR; g.b_absmax = c.amax + Ctx::AM_Y;
    g.ds = c.ds; g.d = c.d; g.dprime = dprime; g.nb = nb;
    g.ratio = c.ratio_dev; g.tau = c.tau; g.prev = c.prev; g.row_base = r0;
    g.xnp = c.xnp; g.xn_stride = c.n; g.ynp = c.ynp;
    unsigned int *fill = c.counters + (size_t)ch * kSubLists * kSubListStride;
    g.tile_counter = c.counters + ((size_t)c.nchunks * kSubLists + (size_t)ch * 8) * kSubListStride;
    g.pairs = c.pairs; g.pair_count = fill; g.sub_capacity = (unsigned int)c.sub_cap;
    g.overflow = c.counters + c.ncounters; g.emit_max = c.emit_max;
    g.best = c.best; g.scal = c.scal; g.block_stats = c.block_stats ? 1 : 0;
    if (screen) {
      ScreenLaunch sl{};
      sl.A = c.Xh + r0 * (c.ds / 2 + 16); sl.lda = c.ds / 2 + 16; sl.M = g.M;
      sl.B = c.Yh; sl.ldb = c.ds / 2 + 16; sl.N = g.N;
      sl.a_absmax = g.a_absmax; sl.b_absmax = g.b_absmax;
      sl.ds = c.ds; sl.dprime = dprime; sl.ratio0 = ratio[0];
      sl.tau = c.tau; sl.row_base = r0;
      sl.xn = c.xnp + (int64_t)(dprime / 16 - 1) * c.n;
      sl.yn = c.ynp;
      sl.arow = c.scr_arow; sl.ycol = c.scr_ycol;
      sl.colmask = c.colmask; sl.cnt = c.scr_cnt; sl.first = c.scr_first; sl.ntiles = c.scr_ntiles;
      sl.col_list = c.scr_cols; sl.tile_rt = c.scr_tile_rt;
      sl.tile_counter = c.counters + ((size_t)c.nchunks * (kSubLists + 8) + (size_t)ch * 8) * kSubListStride;
      sl.scal = c.scal;
      HIPCHK(launch_screen(sl, c.st));
      g.tile_rt = c.scr_tile_rt; g.col_list = c.scr_cols; g.ntiles = c.scr_ntiles;
    }
    HIPCHK(launch_progressive(g, c.st));
    tm.mark(ST_GEMM);
    if (c.emit_max > 0) {
      PruneArgs pa{c.pairs, fill, (unsigned int)c.sub_cap, c.Xr, c.ldx, c.n, c.Ypdx, c.k, dprime, c.ds, nb, c.ratio_dev,
                   c.best, c.scal, c.block_stats ? 1 : 0};
      HIPCHK(launch_prune(pa, c.st));
      tm.mark(ST_PRUNE);
    }
  }
  HIPCHK(launch_finalize_assign(c.best, c.prev, c.n, c.assign, c.dist, c.up.cnt, c.k, c.obj_partial, c.scal + SC_CHANGED,
                                nullptr, c.st));
  HIPCHK(launch_sum_partials(c.obj_partial, finalize_blocks(c.n), c.obj, c.st));
  tm.mark(ST_TAU);
  const size_t nscal = (size_t)SC_COUNT * kStatReplicas;
  if (int rc = c.fetch_step_block()) return rc;
  HIPCHK(hipStreamSynchronize(c.st));
  c.rb_cnt_valid = true;
  if (*c.rb_flag & 1u) return fail(SKM_EOVERFLOW, "the hand-over list of the dense tiles overflowed");
  if (*c.rb_flag != 0) return fail(SKM_EINTERNAL, "a point was left without a centroid");
  std::vector<unsigned long long> scal_h(c.rb_scal, c.rb_scal + nscal);
  const double obj = *c.rb_obj;
  for (int r = 1; r < kStatReplicas; ++r)   // fold the replicas into the first
    for (int q = 0; q < SC_COUNT; ++q) scal_h[(size_t)q] += scal_h[(size_t)r * SC_COUNT + q];
  ss = StepStats();
  ss.survivors = (int64_t)scal_h[SC_SURVIVORS];
  ss.completed = (int64_t)scal_h[SC_COMPLETED];
  ss.changed = (int64_t)scal_h[SC_CHANGED];
  ss.dense_dims = (int64_t)scal_h[SC_DENSE_DIMS];
  ss.dense_pair_blocks = (int64_t)scal_h[SC_DENSE_PB];
  ss.gather_pair_blocks = (int64_t)scal_h[SC_GATHER_PB];
  ss.gather_pairs = (int64_t)scal_h[SC_GATHER_PAIRS];
  ss.screen_dims = (int64_t)scal_h[SC_SCREEN_DIMS];
  ss.listed_tiles = (int64_t)scal_h[SC_LISTED_TILES];
  c.last_prune_frac = c.k > 1 ? 1.0 - (double)ss.survivors / ((double)c.n * (double)(c.k - 1)) : -1.0;
  ++c.pruned_steps;
  for (int m = 0; m < std::min<int>(nb, SKM_MAX_BLOCKS); ++m) ss.enter[m] = (int64_t)scal_h[SC_ENTER + (size_t)m];
  ss.objective = obj;
  ss.dprime = dprime;
  ss.nblocks = nb;
  ss.pruned = true;
  return SKM_OK;
}

// Update + split of empty clusters (Section 3.2).  c.up.cnt must hold the cluster sizes of c.assign.
// `changed` = points whose label differs from c.prev (c.n after the exact step).  While few points move, the cluster
// sums of the previous update are corrected by the rows that joined and left instead of being recomputed from all
// points (full = true forces the recomputation).
int split_empty(Ctx &c, StageTimer &tm, Rng &split_rng, float split_eps, int64_t *nempty_out);
int step_update(Ctx &c, StageTimer &tm, Rng &split_rng, float split_eps, int64_t *nempty_out, int64_t changed,
                bool full) {
  bool fresh = false;   // up.order rebuilt from the labels of this step
  if (!full && c.S_valid && changed == 0) {
    // no point changed its cluster: sums, sizes and therefore the means are those of the previous update.  If that
    // update was followed by a split, the donor's row still holds its perturbed copy: Algorithm 1's update puts the
    // mean of its members back before the next split, so the means are rewritten from the sums.
    ++c.inc_updates;
    if (c.split_last) {
      HIPCHK(launch_means_from_sums(c.S, c.up.cnt, c.k, c.ds, c.Y, c.ds, c.amax + Ctx::AM_Y, c.st));
    }
  } else if (!full && c.S_valid && 2 * changed <= c.inc.capacity - 2) {
    ++c.inc_updates;
    HIPCHK(launch_update_incremental(c.Xr, c.ldx, c.n, c.ds, c.assign, c.prev, changed, c.k, c.up, c.inc, c.S, c.Y, c.ds,
                                     c.st, c.amax + Ctx::AM_Y));
  } else {
    HIPCHK(launch_update(c.Xr, c.ldx, c.n, c.ds, c.assign, c.k, c.up, c.Y, c.ds, c.st, c.S, c.amax + Ctx::AM_Y));
    c.S_valid = true;
    fresh = true;
  }
  c.order_fresh = fresh;
  c.y_amax_valid = true;
  return split_empty(c, tm, split_rng, split_eps, nempty_out);
}

// Empty clusters after an update (Section 3.2): c.rb_cnt (if rb_cnt_valid) or c.up.cnt holds the cluster sizes.
int split_empty(Ctx &c, StageTimer &tm, Rng &split_rng, float split_eps, int64_t *nempty_out) {
  // the cluster sizes came back with the step's scalars; neither update changes them
  if (!c.rb_cnt_valid) {
    HIPCHK(hipMemcpyAsync(c.rb_cnt, c.up.cnt, sizeof(int32_t) * (size_t)c.k, hipMemcpyDeviceToHost, c.st));
    HIPCHK(hipStreamSynchronize(c.st));
  }
  c.rb_cnt_valid = false;
  std::vector<int32_t> cnt(c.rb_cnt, c.rb_cnt + c.k);
  int64_t nempty = 0;
  int32_t largest = 0;
  for (int32_t v : cnt) {
    nempty += (v == 0);
    largest = std::max(largest, v);
  }
  c.max_cluster = largest;   // of the labels the update just used (a split below moves a centroid, no label)
  *nempty_out = nempty;
  c.split_last = false;
  if (nempty > 0) {
    // empty clusters in increasing index; donor drawn with probability proportional to its size
    // among clusters of at least two points; the donor's points are shared floor(n/2) / rest.
    // The draw "first cluster whose cumulative weight exceeds r" runs on a Fenwick tree over the weights
    // (size if >= 2, else 0): O(log k) per empty cluster instead of a pass over all sizes.
    const int32_t k = c.k;
    std::vector<uint64_t> fen((size_t)k + 1, 0);
    auto weight = [](int32_t v) { return v >= 2 ? (uint64_t)v : 0ull; };
    for (int32_t j = 0; j < k; ++j) fen[(size_t)j + 1] = weight(cnt[(size_t)j]);
    for (int32_t j = 1; j <= k; ++j) {
      const int32_t up = j + (j & -j);
      if (up <= k) fen[(size_t)up] += fen[(size_t)j];
    }
    uint64_t total = 0;
    for (int32_t v : cnt) total += weight(v);
    auto fen_add = [&](int32_t j, int64_t delta) {
      for (int32_t i = j + 1; i <= k; i += i & -i) fen[(size_t)i] = (uint64_t)((int64_t)fen[(size_t)i] + delta);
    };
    int32_t top = 1;
    while ((top << 1) <= k) top <<= 1;
    auto fen_find = [&](uint64_t r) {   // smallest j with weight(0) + ... + weight(j) > r   (r < total)
      int32_t pos = 0;
      for (int32_t step = top; step > 0; step >>= 1)
        if (pos + step <= k && fen[(size_t)(pos + step)] <= r) {
          pos += step;
          r -= fen[(size_t)pos];
        }
      return pos;
    };
    std::vector<int32_t> pairs;
    for (int32_t e = 0; e < k; ++e) {
      if (cnt[(size_t)e] != 0) continue;
      if (total == 0) continue;
      const uint64_t r = split_rng.next() % total;
      const int32_t donor = fen_find(r);
      const int32_t give = cnt[(size_t)donor] / 2, keep = cnt[(size_t)donor] - give;
      const int64_t dd = (int64_t)weight(keep) - (int64_t)weight(cnt[(size_t)donor]);
      const int64_t de = (int64_t)weight(give);
      fen_add(donor, dd);
      fen_add(e, de);
      total = (uint64_t)((int64_t)total + dd + de);
      cnt[(size_t)e] = give;
      cnt[(size_t)donor] = keep;
      pairs.push_back(e);
      pairs.push_back(donor);
    }
    if (!pairs.empty()) {
      // Splits that share no cluster commute: they are grouped into chains (connected components of the clusters they
      // touch, in order of first appearance, every chain keeping the order above) and the device applies the chains
      // side by side.
      const size_t ns = pairs.size() / 2;
      std::vector<int32_t> parent((size_t)k);
      for (int32_t j = 0; j < k; ++j) parent[(size_t)j] = j;
      auto root = [&](int32_t v) {
        while (parent[(size_t)v] != v) v = parent[(size_t)v] = parent[(size_t)parent[(size_t)v]];
        return v;
      };
      for (size_t q = 0; q < ns; ++q) {
        const int32_t a = root(pairs[2 * q]), b = root(pairs[2 * q + 1]);
        if (a != b) parent[(size_t)a] = b;
      }
      std::vector<int32_t> chain_of((size_t)k, -1), chain(ns), len;
      for (size_t q = 0; q < ns; ++q) {
        const int32_t r0 = root(pairs[2 * q]);
        if (chain_of[(size_t)r0] < 0) {
          chain_of[(size_t)r0] = (int32_t)len.size();
          len.push_back(0);
        }
        chain[q] = chain_of[(size_t)r0];
        ++len[(size_t)chain[q]];
      }
      const size_t nchain = len.size();
      // upload: [2 ns] pairs sorted by chain | at word 2 k: [nchain + 1] first split of every chain
      std::vector<int32_t> up((size_t)2 * k + nchain + 1, 0);
      std::vector<int32_t> cursor(nchain + 1, 0);
      for (size_t q = 0; q < nchain; ++q) cursor[q + 1] = cursor[q] + len[q];
      for (size_t q = 0; q <= nchain; ++q) up[(size_t)2 * k + q] = cursor[q];
      for (size_t q = 0; q < ns; ++q) {
        const int32_t at = cursor[(size_t)chain[q]]++;
        up[(size_t)2 * at] = pairs[2 * q];
        up[(size_t)2 * at + 1] = pairs[2 * q + 1];
      }
      HIPCHK(hipMemcpyAsync(c.split_dev, up.data(), sizeof(int32_t) * up.size(), hipMemcpyHostToDevice, c.st));
      HIPCHK(launch_split(c.Y, c.ds, c.d, c.split_dev, c.split_dev + (size_t)2 * k, (int32_t)nchain, split_eps, c.st));
      c.y_amax_valid = false;
      c.split_last = true;
      HIPCHK(hipStreamSynchronize(c.st));  // `up` must outlive the copy
    }
  }
  tm.mark(ST_UPDATE);
  return SKM_OK;
}

void fill_row(skm_trace_row &r, const StepStats &ss, int64_t n, int32_t k, int64_t nempty, double recall,
              const float ms[ST_COUNT], float total) {
  std::memset(&r, 0, sizeof(r));
  r.objective = ss.objective;
  r.prune_frac = (ss.pruned && k > 1) ? 1.0 - (double)ss.survivors / ((double)n * (double)(k - 1)) : 0.0;
  r.recall = recall;
  r.survivors = ss.survivors;
  r.completed = ss.completed;
  r.changed = ss.changed;
  r.dense_dims = ss.dense_dims;
  r.dense_pair_blocks = ss.dense_pair_blocks;
  r.gather_pair_blocks = ss.gather_pair_blocks;
  r.gather_pairs = ss.gather_pairs;
  r.screen_dims = ss.screen_dims;
  r.listed_tiles = ss.listed_tiles;
  r.nempty = nempty;
  r.dprime = ss.dprime;
  r.nblocks = ss.nblocks;
  for (int m = 0; m < SKM_MAX_BLOCKS; ++m) r.enter[m] = ss.enter[m];
  r.ms_tau = ms[ST_TAU];
  r.ms_gemm = ms[ST_GEMM];
  r.ms_prune = ms[ST_PRUNE];
  r.ms_update = ms[ST_UPDATE];
  r.ms_etr = ms[ST_ETR];
  r.ms_step = total;
}

// Rotation buffers: Rp = R padded to row stride ds, Rtp = R^T padded likewise (both d rows).
struct Rot {
  float *Rp = nullptr, *Rtp = nullptr;
  unsigned int *amax = nullptr;   // [0] max |R|, [1] max |input| of the last rotate_into
  uint32_t *Rs = nullptr;         // workspace for the split-fp16 copy of R^T (tall rotations)
};
int setup_rotation(Pool &pool, hipStream_t st, int32_t d, int32_t ds, const float *R_dev, uint64_t seed, Rot &rot) {
  float *Rown = nullptr;
  if (!R_dev) {
    HIPCHK(pool.get(&Rown, (size_t)d * d));
    int rc = make_rotation_dev(pool, d, seed, st, Rown);
    if (rc) return rc;
    R_dev = Rown;
  }
  HIPCHK(pool.get(&rot.Rp, (size_t)d * ds));
  HIPCHK(pool.get(&rot.Rtp, (size_t)d * ds));
  HIPCHK(launch_pad_copy(R_dev, d, d, d, rot.Rp, ds, ds, 0, st));
  HIPCHK(launch_pad_copy(R_dev, d, d, d, rot.Rtp, ds, ds, 1, st));
  if (!rot.amax) HIPCHK(pool.get(&rot.amax, 2));
  if (d % 32 == 0) HIPCHK(pool.get(&rot.Rs, (size_t)d * ((size_t)d + 32)));
  return measure_absmax(R_dev, d, d, d, rot.amax, st);
}
// out (rows x ds, zero padded) = in (rows x d, stride ldin) * R
// out_absmax (optional) receives the bit pattern of max |out|
// (in_measured: rot.amax[1] already bounds |in|)
int rotate_into(const float *in, int64_t ldin, int64_t rows, int32_t d, int32_t ds, const Rot &rot, float *out,
                hipStream_t st, unsigned int *out_absmax = nullptr, bool in_measured = false) {
  if (!in_measured)
    if (int rc = measure_absmax(in, ldin, rows, d, rot.amax + 1, st)) return rc;
  if (out_absmax) HIPCHK(launch_fill_u32(out_absmax, 1, 0u, st));
  GemmOperands g{in, ldin, (int32_t)rows, rot.Rtp, ds, d, d};
  g.a_absmax = rot.amax + 1; g.b_absmax = rot.amax;
  g.b_split = rot.Rs;
  HIPCHK(gemm_store(g, out, ds, ds, 1.f, 0.f, st, out_absmax));
  return SKM_OK;
}
// out (rows x d) = Yr (rows x d, stride ldy) * R^T
int unrotate_into(const float *Yr, int64_t ldy, int32_t rows, int32_t d, int32_t ds, const Rot &rot, float *out,
                  hipStream_t st) {
  if (int rc = measure_absmax(Yr, ldy, rows, d, rot.amax + 1, st)) return rc;
  GemmOperands g{Yr, ldy, rows, rot.Rp, ds, d, d};
  g.a_absmax = rot.amax + 1; g.b_absmax = rot.amax;
  HIPCHK(gemm_store(g, out, d, d, 1.f, 0.f, st));
  return SKM_OK;
}

// Ground truth of ETR (Section 3.3): the K nearest points of every query by L2 over X (original space, lowest index
// on ties) as packed (distance, index) keys, ascending.  The scores q . x come from the GEMM in chunks of 65 536
// points; each chunk is merged into the running lists.  amax_x / amax_q: one word each for the operand bounds.
constexpr int64_t kGtChunk = 1 << 16;
int ground_truth_keys(Pool &pool, const float *X, int64_t n, int32_t d, const float *Q, int32_t nq, int32_t K,
                      unsigned int *amax_x, unsigned int *amax_q, unsigned long long *gt_keys, hipStream_t st) {
  float *xnorm = nullptr, *S = nullptr;
  const int64_t colchunk = std::min<int64_t>(n, kGtChunk);
  HIPCHK(pool.get(&xnorm, (size_t)n));
  HIPCHK(pool.get(&S, (size_t)nq * colchunk));
  HIPCHK(launch_row_norms(X, d, n, d, xnorm, st));
  HIPCHK(launch_fill_u64(gt_keys, (int64_t)nq * K, ~0ull, st));
  if (int rc = measure_absmax(X, d, n, d, amax_x, st)) return rc;
  if (int rc = measure_absmax(Q, d, nq, d, amax_q, st)) return rc;
  for (int64_t c0 = 0; c0 < n; c0 += colchunk) {
    const int64_t m = std::min<int64_t>(colchunk, n - c0);
    GemmOperands g{Q, d, nq, X + c0 * d, d, (int32_t)m, d};
    g.a_absmax = amax_q; g.b_absmax = amax_x;
    HIPCHK(gemm_store(g, S, colchunk, (int32_t)m, 1.f, 0.f, st));
    HIPCHK(launch_topk_merge(S, colchunk, nq, (int32_t)m, c0, xnorm, K, gt_keys, st));
  }
  return SKM_OK;
}

// A single assignment step regroups the points itself (see assign_impl) when there are thousands of centroids, several
// points per centroid, rows that the regrouping pass covers, and the first filter is not switched off.
inline bool assign_groups(int64_t n, int32_t ds, int32_t k, int32_t screen_mode) {
  return screen_mode >= 0 && k >= 4096 && n >= 8 * (int64_t)k && ds <= 2048 && n < ((int64_t)1 << 31);
}
int assign_impl(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k, const int32_t *prev_assign,
                int32_t dprime_in, const skm_params *pp, int32_t *assign_out, float *dist_out);
int fit_sampled(const float *X, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed, const skm_params &p,
                float *centroids_out, int32_t *assign_out, float *dist_out);
int fit_impl(const float *X, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed, const skm_params *pp,
             float *centroids_out, int32_t *assign_out, float *dist_out, int32_t *dprime_out);

// dprime_out (optional) receives the d' the next assignment step would use.
int fit_impl(const float *X, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed, const skm_params *pp,
             float *centroids_out, int32_t *assign_out, float *dist_out, int32_t *dprime_out) {
  int rc = check_shape(X, n, d, k);
  if (rc) return rc;
  if (!centroids_out) return fail(SKM_EINVAL, "centroids_out is null");
  if (iters < 1) return fail(SKM_EINVAL, "iters must be >= 1");
  HostTimes host;   // before the arena: its destructor runs after the workspace has been released
  skm_params p;
  if (pp) p = *pp; else skm_params_default(&p);
  if (!(p.dprime_frac > 0.f && p.dprime_frac <= 1.f)) return fail(SKM_EINVAL, "dprime_frac out of (0, 1]");
  if (!(p.eps0 >= 0.f)) return fail(SKM_EINVAL, "eps0 must be >= 0");
  if (p.tau_group != 0 && p.tau_group != k)
    return fail(SKM_EINVAL, "tau_group: only 0 (= k, the threshold frozen for the whole step) is implemented");
  if (!(p.conv_tol >= 0.f && p.conv_tol <= 1.f)) return fail(SKM_EINVAL, "conv_tol out of [0, 1]");
  skm_trace *tr = p.trace;
  if (tr && (!tr->row || tr->capacity < 1)) return fail(SKM_EINVAL, "trace without rows");
  if (p.angular && p.etr) return fail(SKM_EINVAL, "the angular metric is not combined with ETR");
  if (p.sample_frac > 0.f && p.sample_frac < 1.f) {
    if (p.angular) return fail(SKM_EINVAL, "the angular metric is not combined with sample_frac");
    return fit_sampled(X, n, d, k, iters, seed, p, centroids_out, assign_out, dist_out);
  }

  // the workspace in one piece (the caller's, if it lends one): the context's buffers, the rotated points, the rotation
  // matrices and their generator, the ETR buffers
  CallArena ws(fit_workspace_need(n, d, k, p), p.workspace, p.workspace_bytes);
  if (ws.too_small) return fail(SKM_ENOMEM, "params->workspace is smaller than skm_workspace_bytes() for this call");
  host.workspace_ready();
  Ctx c;
  c.st = (hipStream_t)p.stream;
  c.n = n; c.d = d; c.k = k;
  c.ds = round_up(d, 16);
  c.block_stats = p.block_stats != 0;
  c.screen_mode = p.screen;
  // stage times are taken only for a caller that asked for the trace (a small fit inside the hierarchical fit spends
  // a third of its host time creating and reading events otherwise)
  const bool timed = tr != nullptr;
  StageTimer tm(c.st, timed);
  Events evs;
  hipEvent_t e_begin = nullptr, e_rot = nullptr, e_init = nullptr, e_end0 = nullptr, e_end = nullptr;
  hipEvent_t e_gt0 = nullptr, e_gt1 = nullptr, e_rot0 = nullptr;
  if (timed) {
    e_begin = evs.next(); e_rot = evs.next(); e_init = evs.next(); e_end0 = evs.next(); e_end = evs.next();
    e_gt0 = evs.next(); e_gt1 = evs.next(); e_rot0 = evs.next();
    if (!e_begin || !e_rot || !e_init || !e_end0 || !e_end || !e_gt0 || !e_gt1 || !e_rot0)
      return fail(SKM_EHIP, "hipEventCreate failed");
  }
  if (timed) HIPCHK(hipEventRecord(e_begin, c.st));
  rc = c.alloc_bounds();
  if (rc) return rc;

  // ---- Algorithm 1: R, X~ = X R
  Rot rot;
  float *Xr_own = nullptr;
  if (p.rotate) {
    // The rotation matrix is made by a chain of small kernels that leaves most of the device idle: the pass over X
    // that bounds its magnitude (the scale of the split-fp16 product) runs beside it on a second stream.
    struct SideStream {
      hipStream_t s = nullptr;
      ~SideStream() {
        if (s) (void)hipStreamDestroy(s);
      }
    } side;
    hipEvent_t e_fork = nullptr, e_join = nullptr;
    const bool beside = !p.R && (int64_t)n * d >= ((int64_t)1 << 26);
    if (beside) {
      e_fork = evs.next();
      e_join = evs.next();
      if (!e_fork || !e_join) return fail(SKM_EHIP, "hipEventCreate failed");
      HIPCHK(hipStreamCreateWithFlags(&side.s, hipStreamNonBlocking));
      HIPCHK(c.pool.get(&rot.amax, 2));
      HIPCHK(hipEventRecord(e_fork, c.st));   // X is ready where the caller's stream stands now
      HIPCHK(hipStreamWaitEvent(side.s, e_fork, 0));
      rc = measure_absmax(X, d, n, d, rot.amax + 1, side.s, 1024);   // four workgroups per CU: the generator's kernels find room
      if (rc) return rc;
      HIPCHK(hipEventRecord(e_join, side.s));
    }
    rc = setup_rotation(c.pool, c.st, d, c.ds, p.R, seed, rot);
    if (rc) return rc;
    HIPCHK(c.pool.get(&Xr_own, (size_t)n * c.ds));
    if (beside) HIPCHK(hipStreamWaitEvent(c.st, e_join, 0));
    if (timed) HIPCHK(hipEventRecord(e_rot0, c.st));
    rc = rotate_into(X, d, n, d, c.ds, rot, Xr_own, c.st, c.amax + Ctx::AM_XR, beside);
    if (rc) return rc;
    if (beside) HIPCHK(hipStreamSynchronize(side.s));   // nothing is left on the side stream when it is destroyed
    if (timed) HIPCHK(hipEventRecord(e_rot, c.st));
    c.Xr = Xr_own; c.ldx = c.ds;
  } else if (d == c.ds && aligned16(X) && !p.angular) {
    c.Xr = X; c.ldx = d;
  } else {
    HIPCHK(c.pool.get(&Xr_own, (size_t)n * c.ds));
    HIPCHK(launch_pad_copy(X, d, n, d, Xr_own, c.ds, c.ds, 0, c.st));
    c.Xr = Xr_own; c.ldx = c.ds;
  }
  if (p.angular) HIPCHK(launch_normalize_rows(Xr_own, c.ds, n, c.ds, c.st));   // the library's own copy, in place
  if (!p.rotate || p.angular) {
    if (!p.rotate) {
      if (timed) HIPCHK(hipEventRecord(e_rot0, c.st));
      if (timed) HIPCHK(hipEventRecord(e_rot, c.st));
    }
    rc = c.measure_xr();
    if (rc) return rc;
  }
  rc = c.alloc_common(p.pair_budget, p.dense_frac, true);
  if (rc) return rc;
  // regrouping of the points by cluster (Ctx): not for rows that the batched table writes of the threshold pass do not
  // cover (it happens in the third step at the earliest and wants four steps, itself included, to pay)
  const bool may_regroup = c.ds <= 2048 && n < ((int64_t)1 << 31) && iters + (p.final_assign ? 1 : 0) >= 6;
  if (may_regroup) {
    HIPCHK(c.pool.get(&c.Xr2, (size_t)n * c.ds));
    HIPCHK(c.pool.get(&c.pos_to_id, (size_t)n));
    HIPCHK(c.pool.get(&c.subkey, (size_t)n));
  }

  // ---- InitCentroids: k distinct rows of X~
  {
    std::vector<int64_t> idx((size_t)k);
    if (p.init_idx) {
      for (int32_t i = 0; i < k; ++i) {
        idx[(size_t)i] = p.init_idx[i];
        if (idx[(size_t)i] < 0 || idx[(size_t)i] >= n) return fail(SKM_EINVAL, "init_idx out of range");
      }
    } else {
      sample_rows(seed, STREAM_INIT, n, k, idx.data());
    }
    int64_t *idx_dev = nullptr;
    HIPCHK(c.pool.get(&idx_dev, (size_t)k));
    HIPCHK(hipMemcpyAsync(idx_dev, idx.data(), sizeof(int64_t) * idx.size(), hipMemcpyHostToDevice, c.st));
    HIPCHK(launch_gather_rows(c.Xr, c.ldx, c.ds, idx_dev, k, c.Y, c.ds, c.ds, c.st));
    HIPCHK(hipStreamSynchronize(c.st));
  }

  // ---- ETR set-up (Section 3.3): queries, ground truth, rotated queries
  float *Qr = nullptr, *Sq = nullptr, *ynorm_full = nullptr;
  unsigned long long *gt_keys = nullptr, *etr_scal = nullptr;
  int32_t nprobe = 0;
  if (timed) HIPCHK(hipEventRecord(e_gt0, c.st));
  if (p.etr) {
    if (p.nq < 1 || p.topk < 1 || p.topk > 256) return fail(SKM_EINVAL, "ETR: nq >= 1 and 1 <= topk <= 256 required");
    nprobe = nprobe_of(k, p.probe_frac);
    if (nprobe > kMaxProbe) return fail(SKM_EINVAL, "ETR: probe_frac * k exceeds 8192");
    const float *Q = p.queries;
    float *Qown = nullptr;
    if (!Q) {
      if (p.nq > n) return fail(SKM_EINVAL, "ETR: nq > n");
      std::vector<int64_t> qi((size_t)p.nq);
      sample_rows(seed, STREAM_QUERIES, n, p.nq, qi.data());
      int64_t *qi_dev = nullptr;
      HIPCHK(c.pool.get(&qi_dev, (size_t)p.nq));
      HIPCHK(c.pool.get(&Qown, (size_t)p.nq * d));
      HIPCHK(hipMemcpyAsync(qi_dev, qi.data(), sizeof(int64_t) * qi.size(), hipMemcpyHostToDevice, c.st));
      HIPCHK(launch_gather_rows(X, d, d, qi_dev, p.nq, Qown, d, d, c.st));
      HIPCHK(hipStreamSynchronize(c.st));
      Q = Qown;
    }
    HIPCHK(c.pool.get(&gt_keys, (size_t)p.nq * p.topk));
    if (p.gt) {
      HIPCHK(launch_index_to_keys(p.gt, (int64_t)p.nq * p.topk, gt_keys, c.st));
    } else {
      rc = ground_truth_keys(c.pool, X, n, d, Q, p.nq, p.topk, c.amax + Ctx::AM_X, c.amax + Ctx::AM_Q, gt_keys, c.st);
      if (rc) return rc;
    }
    HIPCHK(c.pool.get(&Qr, (size_t)p.nq * c.ds));
    if (p.rotate) {
      rc = rotate_into(Q, d, p.nq, d, c.ds, rot, Qr, c.st, c.amax + Ctx::AM_QR);
      if (rc) return rc;
    } else {
      HIPCHK(launch_pad_copy(Q, d, p.nq, d, Qr, c.ds, c.ds, 0, c.st));
      rc = measure_absmax(Qr, c.ds, p.nq, c.ds, c.amax + Ctx::AM_QR, c.st);
      if (rc) return rc;
    }
    HIPCHK(c.pool.get(&Sq, (size_t)p.nq * k));
    HIPCHK(c.pool.get(&ynorm_full, (size_t)k));
    HIPCHK(c.pool.get(&etr_scal, 2));
    c.point_keys = gt_keys;   // the ground truth names points: it follows them if they are regrouped
    c.n_point_keys = (int64_t)p.nq * p.topk;
  }
  if (timed) HIPCHK(hipEventRecord(e_gt1, c.st));
  if (timed) HIPCHK(hipEventRecord(e_init, c.st));

  int32_t dprime = dprime_init(d, p.dprime_frac);
  Rng split_rng = rng_stream(seed, STREAM_SPLIT);
  int32_t run = 0, rows = 0, streak = 0;
  double best_recall = -1.0;
  // recall of (current centroids, current assignment): Section 3.3
  auto measure_recall = [&](double *out) -> int {
    HIPCHK(launch_prep_centroids(c.Y, c.ds, k, c.ds, c.ds, ynorm_full, 0, 0, nullptr, c.st));
    if (int mrc = c.measure_y()) return mrc;
    GemmOperands g{Qr, c.ds, p.nq, c.Y, c.ds, k, c.ds};
    g.a_absmax = c.amax + Ctx::AM_QR; g.b_absmax = c.amax + Ctx::AM_Y;
    HIPCHK(gemm_store(g, Sq, k, k, 1.f, 0.f, c.st));
    HIPCHK(hipMemsetAsync(etr_scal, 0, 2 * sizeof(unsigned long long), c.st));
    HIPCHK(launch_recall_scores(Sq, k, p.nq, k, ynorm_full, nprobe, gt_keys, p.topk, c.assign, etr_scal, etr_scal + 1,
                                c.st));
    unsigned long long h[2] = {0, 0};
    HIPCHK(hipMemcpyAsync(h, etr_scal, sizeof(h), hipMemcpyDeviceToHost, c.st));
    HIPCHK(hipStreamSynchronize(c.st));
    *out = h[1] ? (double)h[0] / (double)h[1] : 0.0;
    return SKM_OK;
  };

  for (int32_t t = 1; t <= iters; ++t) {
    StepStats ss;
    if (t == 1) {
      rc = step_exact(c, tm, ss);
    } else {
      std::swap(c.assign, c.prev);
      // the rewrite costs about as much as three threshold passes and saves a fraction of every later step
      c.regroup_ok = may_regroup && (iters - t + 1) + (p.final_assign ? 1 : 0) >= 4;
      rc = step_pruned(c, tm, dprime, (double)p.eps0, true, ss);
    }
    if (rc) return rc;
    double recall = -1.0;
    if (p.etr) {
      rc = measure_recall(&recall);
      if (rc) return rc;
      tm.mark(ST_ETR);
    }
    int64_t nempty = 0;
    rc = step_update(c, tm, split_rng, p.split_eps, &nempty, ss.changed, p.full_update != 0);
    if (rc) return rc;
    if (p.angular) {
      HIPCHK(launch_normalize_rows(c.Y, c.ds, k, c.ds, c.st));
      c.y_amax_valid = false;
    }
    HIPCHK(hipStreamSynchronize(c.st));
    float ms[ST_COUNT], total;
    tm.collect(ms, &total);
    run = t;
    if (tr && rows < tr->capacity) fill_row(tr->row[rows], ss, n, k, nempty, recall, ms, total);
    ++rows;
    if (t > 1 && p.adjust_dprime && k > 1) {
      const double f = 1.0 - (double)ss.survivors / ((double)n * (double)(k - 1));
      dprime = dprime_adjust(d, dprime, f, p.adj_lo, p.adj_hi, p.adj_step);
    }
    bool stop = false;
    if (p.etr) {
      if (t == 1) {
        best_recall = recall;
      } else {
        if (recall - best_recall <= (double)p.etr_tol) ++streak; else streak = 0;
        if (recall > best_recall) best_recall = recall;
        if (streak >= p.etr_patience) stop = true;
      }
    }
    // Section 3.3, second condition (convergence): hardly any point changed its cluster
    if (p.conv_tol > 0.f && t > 1 && (double)ss.changed <= (double)p.conv_tol * (double)n) stop = true;
    if (stop) break;
  }

  // ---- final assignment with the two-phase approach (Section 3.3)
  if (p.final_assign) {
    StepStats ss;
    std::swap(c.assign, c.prev);
    c.regroup_ok = false;
    rc = step_pruned(c, tm, dprime, (double)p.eps0, true, ss);
    if (rc) return rc;
    float ms[ST_COUNT], total;
    tm.collect(ms, &total);
    if (tr && rows < tr->capacity) fill_row(tr->row[rows], ss, n, k, 0, -1.0, ms, total);
    ++rows;
  }
  if (c.permuted) {   // per-point results back in the caller's order
    if (assign_out) HIPCHK(launch_scatter_by_index(c.assign, c.pos_to_id, n, assign_out, c.st));
    if (dist_out) HIPCHK(launch_scatter_by_index(c.dist, c.pos_to_id, n, dist_out, c.st));
  } else {
    if (assign_out) HIPCHK(hipMemcpyAsync(assign_out, c.assign, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToDevice, c.st));
    if (dist_out) HIPCHK(hipMemcpyAsync(dist_out, c.dist, sizeof(float) * (size_t)n, hipMemcpyDeviceToDevice, c.st));
  }

  // ---- Algorithm 1, last line: Y = Y~ R^T
  if (timed) HIPCHK(hipEventRecord(e_end0, c.st));
  if (p.rotate) {
    rc = unrotate_into(c.Y, c.ds, k, d, c.ds, rot, centroids_out, c.st);
    if (rc) return rc;
  } else {
    HIPCHK(hipMemcpy2DAsync(centroids_out, sizeof(float) * (size_t)d, c.Y, sizeof(float) * (size_t)c.ds,
                            sizeof(float) * (size_t)d, (size_t)k, hipMemcpyDeviceToDevice, c.st));
  }
  if (timed) HIPCHK(hipEventRecord(e_end, c.st));
  HIPCHK(hipStreamSynchronize(c.st));
  if (dprime_out) *dprime_out = dprime;
  if (tr) {
    tr->rows = std::min(rows, tr->capacity);
    tr->iters_run = run;
    tr->inc_updates = c.inc_updates;
    (void)hipEventElapsedTime(&tr->ms_rotate, e_rot0, e_rot);
    (void)hipEventElapsedTime(&tr->ms_init, e_begin, e_init);
    (void)hipEventElapsedTime(&tr->ms_etr_gt, e_gt0, e_gt1);
    (void)hipEventElapsedTime(&tr->ms_unrotate, e_end0, e_end);
    (void)hipEventElapsedTime(&tr->ms_total, e_begin, e_end);
  }
  host.body_done(tr);
  return SKM_OK;
}


// Algorithm 1 on points that stay in host memory (Section 7.1: batches of X pass through the device, copies and kernels
// overlap).  Every pass over the data (an iteration, or the final assignment) sends the rows through two device buffers
// of `W` rows: while batch g is rotated and assigned, batch g + 1 is already there and batch g + 2 follows as soon as the
// rotation has released its buffer.  A batch is rotated again in every pass (a d x d product per row, small next to the
// transfer), so nothing of size n x d is kept on the device: per point only its label, and its distance if asked for.
// An update adds the batch's cluster sums (fp64) to S; the means are taken once the pass is complete.
int fit_host_impl(const float *Xh, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed, const skm_params *pp,
                  int64_t batch_rows, float *centroids_out, int32_t *assign_out_host, float *dist_out_host) {
  int rc = check_shape(Xh, n, d, k);
  if (rc) return rc;
  if (!centroids_out) return fail(SKM_EINVAL, "centroids_out is null");
  if (iters < 1) return fail(SKM_EINVAL, "iters must be >= 1");
  if (batch_rows < 0) return fail(SKM_EINVAL, "batch_rows must be >= 0");
  skm_params p;
  if (pp) p = *pp; else skm_params_default(&p);
  if (!(p.dprime_frac > 0.f && p.dprime_frac <= 1.f)) return fail(SKM_EINVAL, "dprime_frac out of (0, 1]");
  if (!(p.eps0 >= 0.f)) return fail(SKM_EINVAL, "eps0 must be >= 0");
  if (p.etr || p.angular || (p.sample_frac > 0.f && p.sample_frac < 1.f))
    return fail(SKM_EINVAL, "the host-resident fit is not combined with ETR, the angular metric or sample_frac");
  skm_trace *tr = p.trace;
  if (tr && (!tr->row || tr->capacity < 1)) return fail(SKM_EINVAL, "trace without rows");

  // rows per batch: a multiple of 128 (whole tiles; the per-point arrays of a batch then start 512-byte aligned)
  int64_t W = batch_rows > 0 ? batch_rows : (int64_t)131072;
  W = std::min<int64_t>((W + 127) / 128 * 128, (n + 127) / 128 * 128);
  const int64_t nbatch = (n + W - 1) / W;
  const int npass = iters + (p.final_assign ? 1 : 0);

  // the workspace in one piece: the context of a batch, two raw batches and the rotated one, labels (and distances)
  // of all points, the rotation matrices and their generator, the initial rows
  const size_t ds0 = (size_t)round_up(d, 16);
  const size_t plan = plan_common_bytes(W, d, k, p.pair_budget, p.dense_frac, true);
  CallArena ws(plan ? plan + (size_t)W * (2 * (size_t)d + ds0) * 4 + 3 * (size_t)nbatch * W * 4 + 10 * (size_t)d * ds0 * 4 +
                          (size_t)d * 16384 + (size_t)k * d * 4 + ((size_t)32 << 20)
                    : 0);
  Ctx c;
  c.st = (hipStream_t)p.stream;
  c.n = W; c.d = d; c.k = k;
  c.ds = round_up(d, 16);
  c.block_stats = p.block_stats != 0;
  c.screen_mode = p.screen;
  StageTimer tm(c.st, true);
  Events evs;
  hipEvent_t e_begin = evs.next(), e_init = evs.next(), e_end0 = evs.next(), e_end = evs.next();
  hipEvent_t ev_copied[2] = {evs.next(), evs.next()}, ev_free[2] = {evs.next(), evs.next()};
  if (!e_begin || !e_init || !e_end0 || !e_end || !ev_copied[0] || !ev_copied[1] || !ev_free[0] || !ev_free[1])
    return fail(SKM_EHIP, "hipEventCreate failed");
  struct CopyStream {
    hipStream_t s = nullptr;
    ~CopyStream() {
      if (s) (void)hipStreamDestroy(s);
    }
  } cs;
  HIPCHK(hipStreamCreateWithFlags(&cs.s, hipStreamNonBlocking));
  HIPCHK(hipEventRecord(e_begin, c.st));
  rc = c.alloc_bounds();
  if (rc) return rc;
  rc = c.alloc_common(p.pair_budget, p.dense_frac, true);
  if (rc) return rc;
  const int64_t tile_rows = c.chunk_rows;   // rows per launch of the tile kernel inside a batch

  Rot rot;
  if (p.rotate) {
    rc = setup_rotation(c.pool, c.st, d, c.ds, p.R, seed, rot);
    if (rc) return rc;
  }
  float *raw[2] = {nullptr, nullptr}, *Xr_buf = nullptr, *dist_all = nullptr;
  int32_t *lab[2] = {nullptr, nullptr};
  HIPCHK(c.pool.get(&raw[0], (size_t)W * d));
  HIPCHK(c.pool.get(&raw[1], (size_t)W * d));
  HIPCHK(c.pool.get(&Xr_buf, (size_t)W * c.ds));
  HIPCHK(c.pool.get(&lab[0], (size_t)nbatch * W));
  HIPCHK(c.pool.get(&lab[1], (size_t)nbatch * W));
  if (dist_out_host) HIPCHK(c.pool.get(&dist_all, (size_t)nbatch * W));
  float *dist_batch = c.dist;
  int32_t *cnt_dev = c.up.cnt;

  // ---- InitCentroids: k distinct rows of X, rotated like the points
  {
    std::vector<int64_t> idx((size_t)k);
    if (p.init_idx) {
      for (int32_t i = 0; i < k; ++i) {
        idx[(size_t)i] = p.init_idx[i];
        if (idx[(size_t)i] < 0 || idx[(size_t)i] >= n) return fail(SKM_EINVAL, "init_idx out of range");
      }
    } else {
      sample_rows(seed, STREAM_INIT, n, k, idx.data());
    }
    std::vector<float> rows_h((size_t)k * d);
    for (int32_t i = 0; i < k; ++i)
      std::memcpy(rows_h.data() + (size_t)i * d, Xh + (size_t)idx[(size_t)i] * d, sizeof(float) * (size_t)d);
    float *rows_dev = nullptr;
    HIPCHK(c.pool.get(&rows_dev, (size_t)k * d));
    HIPCHK(hipMemcpyAsync(rows_dev, rows_h.data(), sizeof(float) * rows_h.size(), hipMemcpyHostToDevice, c.st));
    if (p.rotate) {
      rc = rotate_into(rows_dev, d, k, d, c.ds, rot, c.Y, c.st);
      if (rc) return rc;
    } else {
      HIPCHK(launch_pad_copy(rows_dev, d, k, d, c.Y, c.ds, c.ds, 0, c.st));
    }
    HIPCHK(hipStreamSynchronize(c.st));   // rows_h must outlive the copy
  }
  HIPCHK(hipEventRecord(e_init, c.st));

  // ---- the stream of batches: batch number g = pass * nbatch + b uses device buffer g & 1
  const int64_t gtotal = (int64_t)npass * nbatch;
  auto send = [&](int64_t g) -> int {   // enqueue the copy of batch g on the copy stream
    if (g >= gtotal) return SKM_OK;
    const int64_t b = g % nbatch, r0 = b * W, rows = std::min<int64_t>(W, n - r0);
    if (g >= 2) HIPCHK(hipStreamWaitEvent(cs.s, ev_free[g & 1], 0));
    HIPCHK(hipMemcpyAsync(raw[g & 1], Xh + (size_t)r0 * d, sizeof(float) * (size_t)rows * d, hipMemcpyHostToDevice, cs.s));
    HIPCHK(hipEventRecord(ev_copied[g & 1], cs.s));
    return SKM_OK;
  };
  if ((rc = send(0))) return rc;
  if ((rc = send(1))) return rc;

  int32_t dprime = dprime_init(d, p.dprime_frac);
  Rng split_rng = rng_stream(seed, STREAM_SPLIT);
  int32_t rows_out = 0;
  int cur = 0;   // lab[cur] receives the labels of the pass in work, lab[cur ^ 1] holds those of the pass before
  std::vector<int64_t> cnt_total((size_t)k);
  for (int pass = 0; pass < npass; ++pass) {
    const bool final_pass = pass >= iters;
    StepStats tot;
    tot.pruned = pass > 0;
    std::fill(cnt_total.begin(), cnt_total.end(), 0);
    if (!final_pass) HIPCHK(hipMemsetAsync(c.S, 0, sizeof(double) * (size_t)k * c.ds, c.st));
    for (int64_t b = 0; b < nbatch; ++b) {
      const int64_t g = (int64_t)pass * nbatch + b, r0 = b * W, rows = std::min<int64_t>(W, n - r0);
      HIPCHK(hipStreamWaitEvent(c.st, ev_copied[g & 1], 0));
      if (p.rotate) {
        rc = rotate_into(raw[g & 1], d, rows, d, c.ds, rot, Xr_buf, c.st, c.amax + Ctx::AM_XR);
        if (rc) return rc;
      } else {
        HIPCHK(launch_pad_copy(raw[g & 1], d, rows, d, Xr_buf, c.ds, c.ds, 0, c.st));
      }
      HIPCHK(hipEventRecord(ev_free[g & 1], c.st));
      if ((rc = send(g + 2))) return rc;
      c.n = rows;
      c.nchunks = (int32_t)((rows + tile_rows - 1) / tile_rows);
      c.Xr = Xr_buf; c.ldx = c.ds;
      c.xnp_valid = false;
      c.assign = lab[cur] + r0;
      c.prev = lab[cur ^ 1] + r0;
      c.dist = dist_all ? dist_all + r0 : dist_batch;
      if (!p.rotate) {
        rc = c.measure_xr();
        if (rc) return rc;
      }
      StepStats ss;
      rc = pass == 0 ? step_exact(c, tm, ss) : step_pruned(c, tm, dprime, (double)p.eps0, true, ss);
      if (rc) return rc;
      for (int32_t j = 0; j < k; ++j) cnt_total[(size_t)j] += c.rb_cnt[j];
      tot.objective += ss.objective;
      tot.survivors += ss.survivors;
      tot.completed += ss.completed;
      tot.changed += ss.changed;
      tot.dense_dims += ss.dense_dims;
      tot.dense_pair_blocks += ss.dense_pair_blocks;
      tot.gather_pair_blocks += ss.gather_pair_blocks;
      tot.gather_pairs += ss.gather_pairs;
      tot.screen_dims += ss.screen_dims;
      tot.listed_tiles += ss.listed_tiles;
      for (int m = 0; m < SKM_MAX_BLOCKS; ++m) tot.enter[m] += ss.enter[m];
      tot.dprime = ss.dprime;
      tot.nblocks = ss.nblocks;
      if (!final_pass) {
        HIPCHK(launch_update(c.Xr, c.ldx, rows, c.ds, c.assign, k, c.up, nullptr, c.ds, c.st, c.S, nullptr, 1));
        tm.mark(ST_UPDATE);
      }
    }
    int64_t nempty = 0;
    if (!final_pass) {
      // means of the whole pass, then the split of empty clusters on the total sizes
      for (int32_t j = 0; j < k; ++j) c.rb_cnt[j] = (int32_t)cnt_total[(size_t)j];
      HIPCHK(hipMemcpyAsync(cnt_dev, c.rb_cnt, sizeof(int32_t) * (size_t)k, hipMemcpyHostToDevice, c.st));
      HIPCHK(launch_means_from_sums(c.S, cnt_dev, k, c.ds, c.Y, c.ds, c.amax + Ctx::AM_Y, c.st));
      c.y_amax_valid = true;
      c.rb_cnt_valid = true;
      rc = split_empty(c, tm, split_rng, p.split_eps, &nempty);
      if (rc) return rc;
    }
    HIPCHK(hipStreamSynchronize(c.st));
    float ms[ST_COUNT], total;
    tm.collect(ms, &total);
    if (tr && rows_out < tr->capacity) fill_row(tr->row[rows_out], tot, n, k, nempty, -1.0, ms, total);
    ++rows_out;
    if (pass > 0 && !final_pass && p.adjust_dprime && k > 1) {
      const double f = 1.0 - (double)tot.survivors / ((double)n * (double)(k - 1));
      dprime = dprime_adjust(d, dprime, f, p.adj_lo, p.adj_hi, p.adj_step);
    }
    cur ^= 1;
  }
  const int last = cur ^ 1;   // labels of the last pass
  if (assign_out_host)
    HIPCHK(hipMemcpyAsync(assign_out_host, lab[last], sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost, c.st));
  if (dist_out_host)
    HIPCHK(hipMemcpyAsync(dist_out_host, dist_all, sizeof(float) * (size_t)n, hipMemcpyDeviceToHost, c.st));
  HIPCHK(hipEventRecord(e_end0, c.st));
  if (p.rotate) {
    rc = unrotate_into(c.Y, c.ds, k, d, c.ds, rot, centroids_out, c.st);
    if (rc) return rc;
  } else {
    HIPCHK(hipMemcpy2DAsync(centroids_out, sizeof(float) * (size_t)d, c.Y, sizeof(float) * (size_t)c.ds,
                            sizeof(float) * (size_t)d, (size_t)k, hipMemcpyDeviceToDevice, c.st));
  }
  HIPCHK(hipEventRecord(e_end, c.st));
  HIPCHK(hipStreamSynchronize(c.st));
  HIPCHK(hipStreamSynchronize(cs.s));
  if (tr) {
    tr->rows = std::min(rows_out, tr->capacity);
    tr->iters_run = iters;
    tr->inc_updates = 0;
    tr->ms_rotate = 0.f;
    tr->ms_etr_gt = 0.f;
    (void)hipEventElapsedTime(&tr->ms_init, e_begin, e_init);
    (void)hipEventElapsedTime(&tr->ms_unrotate, e_end0, e_end);
    (void)hipEventElapsedTime(&tr->ms_total, e_begin, e_end);
  }
  return SKM_OK;
}

// a label outside [0, k) would index past the centroid table: refuse it here
int labels_in_range(const int32_t *a, int64_t n, int32_t k, unsigned int *flag_dev, hipStream_t st) {
  unsigned int bad = 0;
  HIPCHK(hipMemsetAsync(flag_dev, 0, sizeof(unsigned int), st));
  HIPCHK(launch_check_labels(a, n, k, flag_dev, st));
  HIPCHK(hipMemcpyAsync(&bad, flag_dev, sizeof(bad), hipMemcpyDeviceToHost, st));
  HIPCHK(hipStreamSynchronize(st));
  if (bad) return fail(SKM_EINVAL, "assignment label outside [0, k)");
  return SKM_OK;
}

int assign_impl(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k, const int32_t *prev_assign,
                int32_t dprime_in, const skm_params *pp, int32_t *assign_out, float *dist_out) {
  int rc = check_shape(X, n, d, k, false);
  if (rc) return rc;
  if (!centroids || !assign_out) return fail(SKM_EINVAL, "null pointer");
  skm_params p;
  if (pp) p = *pp; else skm_params_default(&p);
  if (p.angular) return fail(SKM_EINVAL, "the angular metric is a fit option: normalise the inputs for a single step");
  if (p.tau_group != 0 && p.tau_group != k)
    return fail(SKM_EINVAL, "tau_group: only 0 (= k, the threshold frozen for the whole step) is implemented");
  skm_trace *tr = p.trace;
  HostTimes host;
  CallArena ws(assign_workspace_need(n, d, k, p), p.workspace, p.workspace_bytes);
  if (ws.too_small) return fail(SKM_ENOMEM, "params->workspace is smaller than skm_workspace_bytes() for this call");
  host.workspace_ready();
  Ctx c;
  c.st = (hipStream_t)p.stream;
  c.n = n; c.d = d; c.k = k;
  c.ds = round_up(d, 16);
  c.block_stats = p.block_stats != 0;
  c.screen_mode = p.screen;
  StageTimer tm(c.st, true);
  Rot rot;
  float *Xr_own = nullptr;
  rc = c.alloc_bounds();
  if (rc) return rc;
  rc = c.alloc_common(p.pair_budget, p.dense_frac, false);
  if (rc) return rc;
  if (p.rotate) {
    rc = setup_rotation(c.pool, c.st, d, c.ds, p.R, 0, rot);
    if (rc) return rc;
    HIPCHK(c.pool.get(&Xr_own, (size_t)n * c.ds));
    rc = rotate_into(X, d, n, d, c.ds, rot, Xr_own, c.st, c.amax + Ctx::AM_XR);
    if (rc) return rc;
    rc = rotate_into(centroids, d, k, d, c.ds, rot, c.Y, c.st);
    if (rc) return rc;
    c.Xr = Xr_own; c.ldx = c.ds;
  } else {
    if (d == c.ds && aligned16(X)) {
      c.Xr = X; c.ldx = d;
    } else {
      HIPCHK(c.pool.get(&Xr_own, (size_t)n * c.ds));
      HIPCHK(launch_pad_copy(X, d, n, d, Xr_own, c.ds, c.ds, 0, c.st));
      c.Xr = Xr_own; c.ldx = c.ds;
    }
    HIPCHK(launch_pad_copy(centroids, d, k, d, c.Y, c.ds, c.ds, 0, c.st));
    rc = c.measure_xr();
    if (rc) return rc;
  }
  if (prev_assign) {
    rc = labels_in_range(prev_assign, n, k, c.counters, c.st);
    if (rc) return rc;
    HIPCHK(hipMemcpyAsync(c.prev, prev_assign, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToDevice, c.st));
  }
  // Many centroids: a step on its own pays for what a fit does once in its third step.  The points are rewritten
  // grouped by their incumbents and the first filter runs in front of the exact kernel (a million tiles of two slabs
  // each otherwise: the fixed costs of a tile, not the arithmetic, are then the whole run time).
  if (assign_groups(n, c.ds, k, p.screen) && c.colmask) {
    HIPCHK(c.pool.get(&c.Xr2, (size_t)n * c.ds));
    HIPCHK(c.pool.get(&c.pos_to_id, (size_t)n));
    HIPCHK(c.pool.get(&c.subkey, (size_t)n));
    HIPCHK(c.pool.get(&c.up.off, (size_t)k + 1));
    HIPCHK(c.pool.get(&c.up.cursor, (size_t)k));
    HIPCHK(c.pool.get(&c.up.segoff, (size_t)k + 1));
    HIPCHK(c.pool.get(&c.up.order, (size_t)n));
    HIPCHK(c.pool.get(&c.grp_cnt, (size_t)k));
    c.group_now = true;
    c.last_prune_frac = 1.0;   // the filter runs: with points grouped and thousands of centroids it has columns to drop
  }
  const int32_t dprime = dprime_in > 0 ? snap16((double)dprime_in, d) : dprime_init(d, p.dprime_frac);
  StepStats ss;
  rc = step_pruned(c, tm, dprime, (double)p.eps0, prev_assign != nullptr, ss);
  if (rc) return rc;
  if (c.permuted) {   // per-point results back in the caller's order
    HIPCHK(launch_scatter_by_index(c.assign, c.pos_to_id, n, assign_out, c.st));
    if (dist_out) HIPCHK(launch_scatter_by_index(c.dist, c.pos_to_id, n, dist_out, c.st));
  } else {
    HIPCHK(hipMemcpyAsync(assign_out, c.assign, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToDevice, c.st));
    if (dist_out) HIPCHK(hipMemcpyAsync(dist_out, c.dist, sizeof(float) * (size_t)n, hipMemcpyDeviceToDevice, c.st));
  }
  HIPCHK(hipStreamSynchronize(c.st));
  float ms[ST_COUNT], total;
  tm.collect(ms, &total);
  if (tr && tr->row && tr->capacity >= 1) {
    fill_row(tr->row[0], ss, n, k, 0, -1.0, ms, total);
    tr->rows = 1;
    tr->iters_run = 0;
    tr->ms_total = total;
    host.body_done(tr);
  }
  return SKM_OK;
}

// Sampled fit (Section 4.4): Algorithm 1 runs on a uniform sample of the rows, then every point is assigned
// to the resulting centroids by the two-phase step without a previous assignment.
int fit_sampled(const float *X, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed, const skm_params &p,
                float *centroids_out, int32_t *assign_out, float *dist_out) {
  if (p.etr) return fail(SKM_EINVAL, "sample_frac and ETR cannot be combined");
  if (!p.final_assign) return fail(SKM_EINVAL, "sample_frac needs the final assignment pass");
  const int64_t s = sample_size(n, k, p.sample_frac);
  hipStream_t st = (hipStream_t)p.stream;
  const int32_t ds = round_up(d, 16);
  HostTimes host;
  // one workspace for the whole call (the caller's, if it lends one); the nested fit and the nested assignment carve
  // theirs from it, one after the other
  CallArena ws(fit_workspace_need(n, d, k, p), p.workspace, p.workspace_bytes);
  if (ws.too_small) return fail(SKM_ENOMEM, "params->workspace is smaller than skm_workspace_bytes() for this call");
  host.workspace_ready();
  Pool pool;
  Events evs;
  hipEvent_t e0 = evs.next(), e1 = evs.next();
  if (!e0 || !e1) return fail(SKM_EHIP, "hipEventCreate failed");
  HIPCHK(hipEventRecord(e0, st));
  // rotate everything once: the final pass needs all rows in the rotated space
  Rot rot;
  const float *Xr = X;
  int64_t ldx = d;
  float *Xr_own = nullptr;
  if (p.rotate) {
    int rc = setup_rotation(pool, st, d, ds, p.R, seed, rot);
    if (rc) return rc;
    HIPCHK(pool.get(&Xr_own, (size_t)n * ds));
    rc = rotate_into(X, d, n, d, ds, rot, Xr_own, st);
    if (rc) return rc;
    Xr = Xr_own; ldx = ds;
  }
  // the sample: s distinct rows, ascending
  std::vector<int64_t> idx((size_t)s);
  sample_rows(seed, STREAM_SAMPLE, n, (int32_t)std::min<int64_t>(s, 0x7fffffff), idx.data());
  std::sort(idx.begin(), idx.end());
  int64_t *idx_dev = nullptr;
  float *Xs = nullptr, *Yr = nullptr;
  HIPCHK(pool.get(&idx_dev, (size_t)s));
  HIPCHK(pool.get(&Xs, (size_t)s * d));
  HIPCHK(pool.get(&Yr, (size_t)k * d));
  HIPCHK(hipMemcpyAsync(idx_dev, idx.data(), sizeof(int64_t) * idx.size(), hipMemcpyHostToDevice, st));
  HIPCHK(launch_gather_rows(Xr, ldx, d, idx_dev, (int32_t)s, Xs, d, d, st));
  HIPCHK(hipStreamSynchronize(st));
  // Algorithm 1 on the sample, in the rotated space
  skm_params pin = p;
  pin.sample_frac = 0.f;
  pin.rotate = 0;
  pin.R = nullptr;
  pin.final_assign = 0;
  pin.workspace = nullptr;   // the nested calls carve from the arena of this call
  pin.workspace_bytes = 0;
  skm_trace inner{};
  skm_trace *tr = p.trace;
  if (tr) {
    inner = *tr;
    pin.trace = &inner;
  }
  int32_t dprime = 0;
  int rc = fit_impl(Xs, s, d, k, iters, seed, &pin, Yr, nullptr, nullptr, &dprime);
  if (rc) return rc;
  // every point against the final centroids, no previous assignment
  skm_params pfin = p;
  pfin.rotate = 0;
  pfin.R = nullptr;
  pfin.workspace = nullptr;
  pfin.workspace_bytes = 0;
  skm_trace last{};
  if (tr) {
    last.capacity = tr->capacity - inner.rows;
    last.row = tr->row + inner.rows;
    pfin.trace = last.capacity >= 1 ? &last : nullptr;
  }
  if (Xr_own && ds != d) {
    // the assignment call takes dense n x d rows; the rotated buffer has stride ds when d is no multiple of 16
    float *Xd = nullptr;
    HIPCHK(pool.get(&Xd, (size_t)n * d));
    HIPCHK(hipMemcpy2DAsync(Xd, sizeof(float) * (size_t)d, Xr_own, sizeof(float) * (size_t)ds, sizeof(float) * (size_t)d,
                            (size_t)n, hipMemcpyDeviceToDevice, st));
    Xr = Xd;
  }
  float *dist_tmp = dist_out;
  int32_t *assign_tmp = assign_out;
  if (!assign_tmp) HIPCHK(pool.get(&assign_tmp, (size_t)n));
  rc = assign_impl(Xr, n, d, Yr, k, nullptr, dprime, &pfin, assign_tmp, dist_tmp);
  if (rc) return rc;
  // centroids back in the original space
  if (p.rotate) {
    float *Yp = nullptr;
    HIPCHK(pool.get(&Yp, (size_t)k * ds));
    HIPCHK(launch_pad_copy(Yr, d, k, d, Yp, ds, ds, 0, st));
    rc = unrotate_into(Yp, ds, k, d, ds, rot, centroids_out, st);
    if (rc) return rc;
  } else {
    HIPCHK(hipMemcpyAsync(centroids_out, Yr, sizeof(float) * (size_t)k * d, hipMemcpyDeviceToDevice, st));
  }
  HIPCHK(hipEventRecord(e1, st));
  HIPCHK(hipStreamSynchronize(st));
  if (tr) {
    tr->rows = inner.rows + ((pfin.trace && last.rows > 0) ? 1 : 0);
    tr->iters_run = inner.iters_run;
    tr->ms_rotate = 0.f;
    tr->ms_init = inner.ms_init;
    tr->ms_etr_gt = 0.f;
    tr->ms_unrotate = 0.f;
    (void)hipEventElapsedTime(&tr->ms_total, e0, e1);
    host.body_done(tr);
  }
  return SKM_OK;
}

// Upper bound of what a hierarchical fit carves from its workspace: the rotated rows (and a dense copy when d is no
// multiple of 16), the meso and fine centroids, the membership arrays, and below them, one after the other, the meso
// fit, the fine phase and the final assignment.  The fine phase is bounded by its worst case, a single meso-cluster
// that holds nearly all rows and clusters; with balanced meso-clusters eight workers fit in that room many times over.
size_t hier_workspace_need(int64_t n, int32_t d, int32_t k, const skm_params &p) {
  const size_t ds0 = (size_t)((d + 15) / 16 * 16);
  skm_params q = p;
  q.sample_frac = 0.f;
  q.etr = 0;
  const size_t a = fit_workspace_need(n, d, k, q), b = assign_workspace_need(n, d, k, q);
  if (!a || !b) return 0;
  return std::max(a + (size_t)n * d * 4 + (size_t)n * 4 + 4096, b) + (size_t)n * ds0 * 4 + (ds0 != (size_t)d ? (size_t)n * d * 4 : 0) +
         (size_t)k * (2 * (size_t)d + ds0) * 4 + (size_t)n * 16 + 10 * (size_t)d * ds0 * 4 + (size_t)d * 16384 + ((size_t)32 << 20);
}

// Hierarchical SuperKMeans (Section 6): Algorithm 1 with sqrt(k) clusters on all points (MESO), then Algorithm 1 inside
// every meso-cluster with its share of the k clusters (FINE), then the two-phase assignment of every point to the k
// fine centroids.  Everything runs in the rotated space; X is rotated once.
int fit_hierarchical(const float *X, int64_t n, int32_t d, int32_t k, int32_t meso_iters, int32_t fine_iters, uint64_t seed,
                     const skm_params *pp, float *centroids_out, int32_t *assign_out, float *dist_out,
                     int64_t *meso_sizes_out, int32_t *fine_counts_out) {
  int rc = check_shape(X, n, d, k);
  if (rc) return rc;
  if (!centroids_out) return fail(SKM_EINVAL, "centroids_out is null");
  if (meso_iters < 1 || fine_iters < 1) return fail(SKM_EINVAL, "meso_iters and fine_iters must be >= 1");
  skm_params p;
  if (pp) p = *pp; else skm_params_default(&p);
  if (p.etr) return fail(SKM_EINVAL, "the hierarchical fit does not take ETR");
  if (p.angular) return fail(SKM_EINVAL, "the hierarchical fit does not take the angular metric");
  if (p.sample_frac > 0.f && p.sample_frac < 1.f) return fail(SKM_EINVAL, "the hierarchical fit does not take sample_frac");
  if (p.init_idx) return fail(SKM_EINVAL, "the hierarchical fit draws its initial rows from the seed");
  if (!p.final_assign) return fail(SKM_EINVAL, "the hierarchical fit needs the final assignment pass");
  skm_trace *tr = p.trace;
  if (tr && (!tr->row || tr->capacity < 1)) return fail(SKM_EINVAL, "trace without rows");
  hipStream_t st = (hipStream_t)p.stream;
  const int32_t ds = round_up(d, 16);
  HostTimes host;
  CallArena ws(hier_workspace_need(n, d, k, p), p.workspace, p.workspace_bytes);
  if (ws.too_small) return fail(SKM_ENOMEM, "params->workspace is smaller than skm_hier_workspace_bytes() for this call");
  host.workspace_ready();
  Pool pool;
  Events evs;
  hipEvent_t e0 = evs.next(), e1 = evs.next(), e_meso = evs.next(), e_fine = evs.next();
  if (!e0 || !e1 || !e_meso || !e_fine) return fail(SKM_EHIP, "hipEventCreate failed");
  HIPCHK(hipEventRecord(e0, st));
  Rot rot;
  const float *Xr = X;   // dense n x d rows in the rotated space
  if (p.rotate) {
    rc = setup_rotation(pool, st, d, ds, p.R, seed, rot);
    if (rc) return rc;
    float *Xp = nullptr;
    HIPCHK(pool.get(&Xp, (size_t)n * ds));
    rc = rotate_into(X, d, n, d, ds, rot, Xp, st);
    if (rc) return rc;
    Xr = Xp;
    if (ds != d) {
      float *Xd = nullptr;
      HIPCHK(pool.get(&Xd, (size_t)n * d));
      HIPCHK(hipMemcpy2DAsync(Xd, sizeof(float) * (size_t)d, Xp, sizeof(float) * (size_t)ds, sizeof(float) * (size_t)d,
                              (size_t)n, hipMemcpyDeviceToDevice, st));
      Xr = Xd;
    }
  }
  skm_params pin = p;
  pin.rotate = 0;
  pin.R = nullptr;
  pin.trace = nullptr;
  pin.workspace = nullptr;   // the nested calls carve from the arena of this call
  pin.workspace_bytes = 0;

  // ---- MESO
  const int32_t km = hier_meso_count(k);
  float *Ymeso = nullptr, *Yr = nullptr;
  int32_t *meso_assign = nullptr;
  HIPCHK(pool.get(&Ymeso, (size_t)km * d));
  HIPCHK(pool.get(&Yr, (size_t)k * d));
  HIPCHK(pool.get(&meso_assign, (size_t)n));
  skm_params pm = pin;
  skm_trace inner{};
  if (tr) {
    inner = *tr;
    pm.trace = &inner;
  }
  rc = fit_impl(Xr, n, d, km, meso_iters, seed, &pm, Ymeso, meso_assign, nullptr, nullptr);
  if (rc) return rc;
  HIPCHK(hipEventRecord(e_meso, st));
  // members of every meso-cluster in ascending row order (counting sort on the host)
  std::vector<int32_t> ma((size_t)n);
  HIPCHK(hipMemcpyAsync(ma.data(), meso_assign, sizeof(int32_t) * (size_t)n, hipMemcpyDeviceToHost, st));
  HIPCHK(hipStreamSynchronize(st));
  std::vector<int64_t> sizes((size_t)km, 0), start((size_t)km + 1, 0);
  for (int64_t i = 0; i < n; ++i) {
    if (ma[(size_t)i] < 0 || ma[(size_t)i] >= km) return fail(SKM_EINTERNAL, "meso assignment out of range");
    ++sizes[(size_t)ma[(size_t)i]];
  }
  for (int32_t c = 0; c < km; ++c) start[(size_t)c + 1] = start[(size_t)c] + sizes[(size_t)c];
  std::vector<int64_t> order((size_t)n), cursor(start.begin(), start.end() - 1);
  for (int64_t i = 0; i < n; ++i) order[(size_t)cursor[(size_t)ma[(size_t)i]]++] = i;
  std::vector<int32_t> counts((size_t)km, 0);
  hier_alloc(sizes.data(), km, k, counts.data());
  if (meso_sizes_out) std::copy(sizes.begin(), sizes.end(), meso_sizes_out);
  if (fine_counts_out) std::copy(counts.begin(), counts.end(), fine_counts_out);

  // ---- FINE: the meso-clusters are independent small problems; a few host threads, each with its own stream and
  // workspace arena, take them from a shared counter so that their short kernels overlap on the device.  The result
  // does not depend on who runs what: every fit writes its own block of Yr and draws from its own seed.
  const int64_t nmax = *std::max_element(sizes.begin(), sizes.end());
  const int32_t kmax = *std::max_element(counts.begin(), counts.end());
  std::vector<int32_t> koffs((size_t)km + 1, 0);
  for (int32_t c = 0; c < km; ++c) koffs[(size_t)c + 1] = koffs[(size_t)c] + counts[(size_t)c];
  if (koffs[(size_t)km] != k) return fail(SKM_EINTERNAL, "fine cluster counts do not add up to k");
  int64_t *order_dev = nullptr;
  HIPCHK(pool.get(&order_dev, (size_t)n));
  HIPCHK(hipMemcpyAsync(order_dev, order.data(), sizeof(int64_t) * (size_t)n, hipMemcpyHostToDevice, st));
  HIPCHK(hipStreamSynchronize(st));
  {
    struct Worker {
      hipStream_t st = nullptr;
      Arena arena;
      float *Xs = nullptr;
      int rc = SKM_OK;
      std::string err;
    };
    // The device exposes four hardware queues to a process; twice as many threads still gain a little (2 workers: 152 ms
    // for the fine phase of 1M x 1536 into 16 384 clusters, 4: 124, 8: 120, 12: 116), because the host side of one small
    // fit (some seventy launches and a dozen waits) then overlaps the device side of another.
    int nworkers = (int)std::min<int32_t>(8, km);
    // workspace of the largest fine fit (a bound for every other: the need grows with the rows and with the clusters)
    skm_params pneed = pin;
    pneed.final_assign = 0;
    const size_t want = fit_workspace_need(std::max<int64_t>(nmax, 1), d, std::max<int32_t>(kmax, 1), pneed);
    if (!want) return fail(SKM_EINVAL, "pair_budget too large (must stay below 2^32 pairs)");
    const size_t per_worker = want + (size_t)std::max<int64_t>(nmax, 1) * d * 4 + 1024;
    Arena *top = tl_arena;
    if (top && top->strict) {
      // a caller's workspace: every worker's share comes out of it, so there are as many workers as shares fit
      const size_t shares = (top->cap - std::min(top->cap, top->off + 512)) / per_worker;
      if (shares < 1) return fail(SKM_ENOMEM, "params->workspace cannot hold the largest fine fit");
      nworkers = (int)std::min<size_t>((size_t)nworkers, shares);
    }
    std::vector<Worker> workers((size_t)nworkers);
    Pool fine_pool;   // the workers' buffers and shares: given back to the arena when the fine phase ends
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    struct StreamGuard {
      std::vector<Worker> &w;
      ~StreamGuard() {
        for (Worker &x : w)
          if (x.st) (void)hipStreamDestroy(x.st);
      }
    } guard{workers};
    for (Worker &w : workers) {
      HIPCHK(hipStreamCreateWithFlags(&w.st, hipStreamNonBlocking));
      HIPCHK(fine_pool.get(&w.Xs, (size_t)std::max<int64_t>(nmax, 1) * d));
      if (top && top->cap - std::min(top->cap, top->off + 512) >= want) {
        char *share = nullptr;
        HIPCHK(fine_pool.get(&share, want));
        w.arena.lend(share, want);
        w.arena.strict = top->strict;   // the library's own arena: what does not fit may still come from hipMalloc
      } else if (w.arena.init(want) != hipSuccess) {
        (void)hipGetLastError();
        w.arena.base = nullptr;
        w.arena.cap = 0;   // every buffer of this worker then comes from hipMalloc
      }
    }
    std::atomic<int32_t> next_cluster{0};
    auto body = [&](Worker &w) {
      if (hipSetDevice(dev) != hipSuccess) {
        w.rc = fail(SKM_EHIP, "hipSetDevice failed in a worker thread");
        w.err = g_last_error;
        return;
      }
      ArenaScope scope(w.arena.base ? &w.arena : nullptr);
      skm_params pfine = pin;
      pfine.final_assign = 0;   // only the centroids of a fine fit are used
      pfine.stream = (void *)w.st;
      for (;;) {
        const int32_t c = next_cluster.fetch_add(1);
        if (c >= km) break;
        const int32_t kc = counts[(size_t)c];
        if (kc == 0) continue;
        const int64_t nc = sizes[(size_t)c];
        hipError_t e = launch_gather_rows(Xr, d, d, order_dev + start[(size_t)c], (int32_t)nc, w.Xs, d, d, w.st);
        int rcw = e == hipSuccess ? SKM_OK : fail_hip(e, "launch_gather_rows");
        if (!rcw)
          rcw = fit_impl(w.Xs, nc, d, kc, fine_iters, seed + 1 + (uint64_t)c, &pfine, Yr + (size_t)koffs[(size_t)c] * d,
                         nullptr, nullptr, nullptr);
        if (rcw) {
          w.rc = rcw;
          w.err = g_last_error;
          next_cluster.store(km);   // stop handing out work
          break;
        }
      }
    };
    std::vector<std::thread> threads;
    for (int t = 1; t < nworkers; ++t) {
      try {
        threads.emplace_back(
            [&body](Worker &w) {
              body(w);
              tl_pinned.release();   // this thread's page-locked blocks go with it
            },
            std::ref(workers[(size_t)t]));
      } catch (const std::system_error &) {
        break;   // fewer threads: the others take the work
      }
    }
    body(workers[0]);
    for (std::thread &t : threads) t.join();
    for (Worker &w : workers) {
      if (w.st) (void)hipStreamSynchronize(w.st);
    }
    for (Worker &w : workers) {
      if (w.rc) {
        g_last_error = w.err;
        return w.rc;
      }
    }
  }
  HIPCHK(hipEventRecord(e_fine, st));

  // ---- every point against the k fine centroids, no previous assignment
  skm_params pfin = pin;
  skm_trace last{};
  if (tr) {
    last.capacity = tr->capacity - inner.rows;
    last.row = tr->row + inner.rows;
    pfin.trace = last.capacity >= 1 ? &last : nullptr;
  }
  int32_t *assign_tmp = assign_out;
  if (!assign_tmp) HIPCHK(pool.get(&assign_tmp, (size_t)n));
  rc = assign_impl(Xr, n, d, Yr, k, nullptr, 0, &pfin, assign_tmp, dist_out);
  if (rc) return rc;
  if (p.rotate) {
    float *Yp = nullptr;
    HIPCHK(pool.get(&Yp, (size_t)k * ds));
    HIPCHK(launch_pad_copy(Yr, d, k, d, Yp, ds, ds, 0, st));
    rc = unrotate_into(Yp, ds, k, d, ds, rot, centroids_out, st);
    if (rc) return rc;
  } else {
    HIPCHK(hipMemcpyAsync(centroids_out, Yr, sizeof(float) * (size_t)k * d, hipMemcpyDeviceToDevice, st));
  }
  HIPCHK(hipEventRecord(e1, st));
  HIPCHK(hipStreamSynchronize(st));
  if (tr) {
    tr->rows = inner.rows + ((pfin.trace && last.rows > 0) ? 1 : 0);
    tr->iters_run = inner.iters_run;
    tr->ms_rotate = 0.f;
    (void)hipEventElapsedTime(&tr->ms_init, e0, e_meso);      // rotation + the whole meso phase
    (void)hipEventElapsedTime(&tr->ms_etr_gt, e_meso, e_fine);  // the whole fine phase
    tr->ms_unrotate = 0.f;
    (void)hipEventElapsedTime(&tr->ms_total, e0, e1);
    host.body_done(tr);
  }
  return SKM_OK;
}

}  // namespace

namespace skm {
int report_error(int rc, const char *what) { return fail(rc, what); }
int report_hip_error(hipError_t e, const char *where) { return fail_hip(e, where); }
}  // namespace skm

// ==================================================================== C ABI
extern "C" {
#pragma GCC visibility push(default)

void skm_params_default(skm_params *p) {
  if (!p) return;
  std::memset(p, 0, sizeof(*p));
  p->dprime_frac = 0.125f;
  p->eps0 = 2.1f;
  p->adjust_dprime = 1;
  p->adj_lo = 0.95f;
  p->adj_hi = 0.97f;
  p->adj_step = 0.20f;
  p->split_eps = 1.0f / 1024.0f;
  p->final_assign = 1;
  p->block_stats = 0;
  p->rotate = 1;
  p->etr = 0;
  p->nq = 1000;
  p->topk = 10;
  p->probe_frac = 0.01f;
  p->etr_tol = 0.005f;
  p->etr_patience = 2;
  p->pair_budget = 0;
  p->dense_frac = 0.0125f;
  p->sample_frac = 0.f;
  p->workspace = nullptr;
  p->workspace_bytes = 0;
  p->conv_tol = 0.f;
  p->screen = 0;
  p->tau_group = 0;
}

int64_t skm_workspace_bytes(int64_t n, int32_t d, int32_t k, const skm_params *params) {
  if (n < 1 || n >= (int64_t)1 << 31 || d < 16 || d > 16384 || k < 1 || k > (1 << 24))
    return fail(SKM_EINVAL, "shape out of range");
  skm_params p;
  if (params) p = *params; else skm_params_default(&p);
  const size_t need = fit_workspace_need(n, d, k, p);
  if (!need) return fail(SKM_EINVAL, "pair_budget too large (must stay below 2^32 pairs)");
  return (int64_t)need + 256;   // room to align the caller's pointer
}

int64_t skm_hier_workspace_bytes(int64_t n, int32_t d, int32_t k, const skm_params *params) {
  if (n < 1 || n >= (int64_t)1 << 31 || d < 16 || d > 16384 || k < 1 || k > (1 << 24) || k > n)
    return fail(SKM_EINVAL, "shape out of range");
  skm_params p;
  if (params) p = *params; else skm_params_default(&p);
  const size_t need = hier_workspace_need(n, d, k, p);
  if (!need) return fail(SKM_EINVAL, "pair_budget too large (must stay below 2^32 pairs)");
  return (int64_t)need + 256;   // room to align the caller's pointer
}

int skm_fit(const float *X, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed, float *centroids_out,
            int32_t *assign_out) {
  return fit_impl(X, n, d, k, iters, seed, nullptr, centroids_out, assign_out, nullptr, nullptr);
}

int skm_fit_ex(const float *X, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed, const skm_params *params,
               float *centroids_out, int32_t *assign_out, float *dist_out) {
  return fit_impl(X, n, d, k, iters, seed, params, centroids_out, assign_out, dist_out, nullptr);
}

int skm_fit_host(const float *X_host, int64_t n, int32_t d, int32_t k, int32_t iters, uint64_t seed,
                 const skm_params *params, int64_t batch_rows, float *centroids_out, int32_t *assign_out_host,
                 float *dist_out_host) {
  return fit_host_impl(X_host, n, d, k, iters, seed, params, batch_rows, centroids_out, assign_out_host, dist_out_host);
}

int skm_fit_hierarchical(const float *X, int64_t n, int32_t d, int32_t k, int32_t meso_iters, int32_t fine_iters,
                         uint64_t seed, const skm_params *params, float *centroids_out, int32_t *assign_out,
                         float *dist_out, int64_t *meso_sizes_out_host, int32_t *fine_counts_out_host) {
  return fit_hierarchical(X, n, d, k, meso_iters, fine_iters, seed, params, centroids_out, assign_out, dist_out,
                          meso_sizes_out_host, fine_counts_out_host);
}

int32_t skm_hier_meso_count(int32_t k) { return k >= 1 ? hier_meso_count(k) : 0; }

int skm_hier_alloc(const int64_t *sizes_host, int32_t km, int32_t k, int32_t *counts_out_host) {
  if (!sizes_host || !counts_out_host || km < 1 || k < km) return fail(SKM_EINVAL, "bad arguments");
  int64_t total = 0;
  for (int32_t i = 0; i < km; ++i) {
    if (sizes_host[i] < 0) return fail(SKM_EINVAL, "negative size");
    total += sizes_host[i];
  }
  if (total < k) return fail(SKM_EINVAL, "fewer points than clusters");
  hier_alloc(sizes_host, km, k, counts_out_host);
  return SKM_OK;
}

int skm_assign(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k, const int32_t *prev_assign,
               int32_t *assign_out, float *dist_out) {
  return assign_impl(X, n, d, centroids, k, prev_assign, 0, nullptr, assign_out, dist_out);
}

int skm_assign_ex(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k, const int32_t *prev_assign,
                  int32_t dprime, const skm_params *params, int32_t *assign_out, float *dist_out) {
  return assign_impl(X, n, d, centroids, k, prev_assign, dprime, params, assign_out, dist_out);
}

int skm_assign_exact(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k, void *stream,
                     int32_t *assign_out, float *dist_out) {
  int rc = check_shape(X, n, d, k, false);
  if (rc) return rc;
  if (!centroids || !assign_out) return fail(SKM_EINVAL, "null pointer");
  hipStream_t st = (hipStream_t)stream;
  Pool pool;
  const int32_t ds = round_up(d, 16);
  const float *Xp = X, *Yp = centroids;
  int64_t ldx = d, ldy = d;
  if (d != ds || !aligned16(X) || !aligned16(centroids)) {
    float *Xo = nullptr, *Yo = nullptr;
    HIPCHK(pool.get(&Xo, (size_t)n * ds));
    HIPCHK(pool.get(&Yo, (size_t)k * ds));
    HIPCHK(launch_pad_copy(X, d, n, d, Xo, ds, ds, 0, st));
    HIPCHK(launch_pad_copy(centroids, d, k, d, Yo, ds, ds, 0, st));
    Xp = Xo; Yp = Yo; ldx = ds; ldy = ds;
  }
  float *ynorm = nullptr;
  unsigned long long *best = nullptr;
  HIPCHK(pool.get(&ynorm, (size_t)k));
  HIPCHK(pool.get(&best, (size_t)n));
  HIPCHK(launch_prep_centroids(Yp, ldy, k, ds, ds, ynorm, 0, 0, nullptr, st));
  HIPCHK(launch_fill_u64(best, n, ~0ull, st));
  unsigned int *amax = nullptr;
  HIPCHK(pool.get(&amax, 2));
  rc = measure_absmax(Xp, ldx, n, ds, amax, st);
  if (rc) return rc;
  rc = measure_absmax(Yp, ldy, k, ds, amax + 1, st);
  if (rc) return rc;
  GemmOperands g{Xp, ldx, (int32_t)n, Yp, ldy, k, ds};
  g.a_absmax = amax; g.b_absmax = amax + 1;
  if (ds % 32 == 0) HIPCHK(pool.get(&g.b_split, (size_t)k * ((size_t)ds + 32)));
  HIPCHK(gemm_argmin(g, ynorm, best, st));
  HIPCHK(launch_finalize_assign(best, nullptr, n, assign_out, nullptr, nullptr, k, nullptr, nullptr, nullptr, st));
  if (dist_out) {
    HIPCHK(launch_tau_init(Xp, ldx, n, ds, Yp, ldy, assign_out, dist_out, nullptr, st));
  }
  HIPCHK(hipStreamSynchronize(st));
  return SKM_OK;
}

int skm_update(const float *X, int64_t n, int32_t d, const int32_t *assign, int32_t k, void *stream, float *centroids,
               int32_t *counts_out) {
  int rc = check_shape(X, n, d, k);
  if (rc) return rc;
  if (!assign || !centroids) return fail(SKM_EINVAL, "null pointer");
  hipStream_t st = (hipStream_t)stream;
  Pool pool;
  const int32_t ds = round_up(d, 16);
  const float *Xp = X;
  int64_t ldx = d;
  float *Yp = centroids;
  int64_t ldy = d;
  const bool padded = (d != ds) || !aligned16(X) || !aligned16(centroids);
  if (padded) {
    float *Xo = nullptr, *Yo = nullptr;
    HIPCHK(pool.get(&Xo, (size_t)n * ds));
    HIPCHK(pool.get(&Yo, (size_t)k * ds));
    HIPCHK(launch_pad_copy(X, d, n, d, Xo, ds, ds, 0, st));
    HIPCHK(launch_pad_copy(centroids, d, k, d, Yo, ds, ds, 0, st));
    Xp = Xo; ldx = ds; Yp = Yo; ldy = ds;
  }
  UpdateWs w{};
  HIPCHK(pool.get(&w.cnt, (size_t)k));
  HIPCHK(pool.get(&w.off, (size_t)k + 1));
  HIPCHK(pool.get(&w.cursor, (size_t)k));
  HIPCHK(pool.get(&w.segoff, (size_t)k + 1));
  HIPCHK(pool.get(&w.order, (size_t)n));
  w.max_segments = update_max_segments(n, k);
  HIPCHK(pool.get(&w.partial, (size_t)w.max_segments * ds));
  rc = labels_in_range(assign, n, k, reinterpret_cast<unsigned int *>(w.cursor), st);
  if (rc) return rc;
  HIPCHK(hipMemsetAsync(w.cnt, 0, sizeof(int32_t) * (size_t)k, st));
  HIPCHK(launch_histogram(assign, n, w.cnt, st));
  HIPCHK(launch_update(Xp, ldx, n, ds, assign, k, w, Yp, ldy, st));
  if (padded)
    HIPCHK(hipMemcpy2DAsync(centroids, sizeof(float) * (size_t)d, Yp, sizeof(float) * (size_t)ds,
                            sizeof(float) * (size_t)d, (size_t)k, hipMemcpyDeviceToDevice, st));
  if (counts_out) HIPCHK(hipMemcpyAsync(counts_out, w.cnt, sizeof(int32_t) * (size_t)k, hipMemcpyDeviceToDevice, st));
  HIPCHK(hipStreamSynchronize(st));
  return SKM_OK;
}

int skm_etr_ground_truth(const float *X, int64_t n, int32_t d, const float *queries, int32_t nq, int32_t topk,
                         void *stream, int64_t *gt_out) {
  if (!X || !queries || !gt_out) return fail(SKM_EINVAL, "null pointer");
  if (n < 1 || n >= (int64_t)1 << 31 || d < 1 || d > 16384) return fail(SKM_EINVAL, "shape out of range");
  if (nq < 1 || topk < 1 || topk > 256) return fail(SKM_EINVAL, "nq >= 1 and 1 <= topk <= 256 required");
  hipStream_t st = (hipStream_t)stream;
  Pool pool;
  unsigned int *amax = nullptr;
  unsigned long long *keys = nullptr;
  HIPCHK(pool.get(&amax, 2));
  HIPCHK(pool.get(&keys, (size_t)nq * topk));
  if (int rc = ground_truth_keys(pool, X, n, d, queries, nq, topk, amax, amax + 1, keys, st)) return rc;
  HIPCHK(launch_keys_to_index(keys, (int64_t)nq * topk, gt_out, st));
  HIPCHK(hipStreamSynchronize(st));
  return SKM_OK;
}

int skm_make_rotation(int32_t d, uint64_t seed, void *stream, float *R_out) {
  if (!R_out) return fail(SKM_EINVAL, "null pointer");
  if (d < 1 || d > 16384) return fail(SKM_EINVAL, "d out of range");
  hipStream_t st = (hipStream_t)stream;
  Pool pool;
  int rc = make_rotation_dev(pool, d, seed, st, R_out);
  if (rc) return rc;
  HIPCHK(hipStreamSynchronize(st));
  return SKM_OK;
}

int skm_rotate(const float *X, int64_t n, int32_t d, const float *R, int32_t transpose, void *stream, float *out) {
  if (!X || !R || !out) return fail(SKM_EINVAL, "null pointer");
  if (n < 1 || n >= (int64_t)1 << 31 || d < 1 || d > 16384) return fail(SKM_EINVAL, "shape out of range");
  hipStream_t st = (hipStream_t)stream;
  Pool pool;
  const int32_t ds = round_up(d, 16);
  float *B = nullptr;  // B[c][kk] = R[kk][c] for X R, R[c][kk] for X R^T
  HIPCHK(pool.get(&B, (size_t)d * ds));
  HIPCHK(launch_pad_copy(R, d, d, d, B, ds, ds, transpose ? 0 : 1, st));
  unsigned int *amax = nullptr;
  HIPCHK(pool.get(&amax, 2));
  int rc = measure_absmax(X, d, n, d, amax, st);
  if (rc) return rc;
  rc = measure_absmax(R, d, d, d, amax + 1, st);
  if (rc) return rc;
  GemmOperands g{X, d, (int32_t)n, B, ds, d, d};
  g.a_absmax = amax; g.b_absmax = amax + 1;
  if (d % 32 == 0) HIPCHK(pool.get(&g.b_split, (size_t)d * ((size_t)d + 32)));
  HIPCHK(gemm_store(g, out, d, d, 1.f, 0.f, st));
  HIPCHK(hipStreamSynchronize(st));
  return SKM_OK;
}

int skm_sample_rows(uint64_t seed, int64_t n, int32_t k, int64_t *idx_out_host) {
  if (!idx_out_host || n < 1 || k < 0 || k > n) return fail(SKM_EINVAL, "bad arguments");
  sample_rows(seed, STREAM_INIT, n, k, idx_out_host);
  return SKM_OK;
}

float skm_theta_ratio(int32_t d, int32_t t, float eps0) { return (float)theta_ratio(d, t, (double)eps0); }
int32_t skm_dprime_init(int32_t d, float frac) { return dprime_init(d, (double)frac); }
int32_t skm_dprime_adjust(int32_t d, int32_t dprime, double prune_frac, float lo, float hi, float step) {
  return dprime_adjust(d, dprime, prune_frac, (double)lo, (double)hi, (double)step);
}

void skm_debug_gemm_config(int32_t tile256, int32_t panel_cols, int64_t max_tiles) {
  gemm_debug_config(tile256, panel_cols, max_tiles);
}

const char *skm_strerror(int rc) {
  switch (rc) {
    case SKM_OK: return "ok";
    case SKM_EINVAL: return "invalid argument";
    case SKM_ENOMEM: return "out of memory";
    case SKM_EHIP: return "HIP runtime error";
    case SKM_EINTERNAL: return "internal error";
    case SKM_EOVERFLOW: return "hand-over list overflow";
    default: return "unknown error";
  }
}
const char *skm_last_error(void) { return g_last_error.c_str(); }
const char *skm_version(void) { return "skm 0.2 (gfx950)"; }

#pragma GCC visibility pop
}  // extern "C"
