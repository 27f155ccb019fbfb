// Low-precision first filter (the paper's closing remark of Section 4.14 on GEMM hardware; Algorithm 1's first test
// theta(d', tau) is what it screens for).
//
// The progressive kernel multiplies every (point tile, centroid tile) pair on the first d' dimensions with three fp16
// products per element, although in a well-pruned step all but a few columns of a tile die at the first test.  This
// pass finds those few columns at a third of the price: one fp16 product (the hi halves of the split operands only:
// half the bytes through L2 and LDS, a third of the matrix instructions), and the first test with its threshold
// widened by a bound of the error that the dropped lo halves can cause.  A pair that passes the exact test passes the
// widened one, so a column that no point of a row tile passes here is dead for that whole tile.  The output is one bit
// per (row tile, centroid); compaction turns the bits into a list of centroid ids per row tile, cut into tiles of 128
// listed columns, and the progressive kernel then runs on those tiles only, with the full arithmetic, the exact tests
// and the exact counters.  What is pruned here is pruned by Algorithm 1's first test as well: the result of the step
// does not depend on whether this pass ran.
//
// Error bound.  A scaled value v is hi + lo with |lo| <= 2^-11 |v| (fp16 rounding; values below the smallest normal
// fp16, 2^-14 in scaled units, are instead off by at most 2^-25).  For x.y = sum x_j y_j the dropped terms
// hi*lo' + lo*hi' + lo*lo' sum to at most (2^-10 + 2^-22) ||x|| ||y|| (Cauchy-Schwarz on the front dimensions), so
// the partial distance ||x'||^2 + ||y'||^2 - 2 x'.y' is off by at most 2 * 2^-10 ||x'|| ||y'|| (taken 10 % larger:
// the fp32 accumulation of up to 16384 / 16 matrix instructions adds 1.2e-4 of that product at most) plus a term for
// the subnormal halves; both prefix norms are at hand (they are the ones the exact test uses).  The test's own few
// fp32 operations are covered by a relative guard of 1e-6 on each of its terms.
#include "skm_internal.h"

#include <algorithm>

namespace skm {

namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 256, BN = 256, BK = 32;     // workgroup tile; a wavefront owns 128 x 64 of it
constexpr int RT = 128;                         // rows of a row tile of the exact kernel: what a bit of the output speaks for
constexpr int TM = 4, TN = 2;
constexpr int NT = 512;                         // 8 wavefronts: 2 (rows) x 4 (columns)
constexpr int ROW_WORDS = 16;                       // a tile row of a slab: the 32 hi halves = 64 bytes
constexpr int STAGE_WORDS = (BM + BN) * ROW_WORDS;  // one slab of both operands: 32 KB
constexpr int ROWS_PASS = NT / 4;                   // 4 lanes move one tile row: 128 rows per load instruction
constexpr int A_LD = BM / ROWS_PASS;                // 2 load instructions per thread, slab and operand
constexpr int B_LD = BN / ROWS_PASS;
constexpr float kWiden = 2.f * 1.1f / 1024.f;       // 2 * 1.1 * 2^-10, see the error bound above
constexpr float kGuard = 1e-6f;                     // relative guard for the fp32 rounding of the test's own terms

constexpr int DEPTH = 3, NSTAGE = 4;              // slabs requested ahead of the one being multiplied; LDS stages
// wait until at most n of this wavefront's vector memory operations are outstanding (LDS and export counters untouched)
#define SKM_SCREEN_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

}  // namespace

struct ScreenArgs {
  const uint32_t *A;   // hi halves of the split-fp16 copy of the chunk's points (launch_split_rows' out_hi), row stride lda words
  int64_t lda;
  int32_t M;
  const uint32_t *B;   // the same of the centroids
  int64_t ldb;
  int32_t N;
  const unsigned int *a_absmax, *b_absmax;
  int32_t dprime;
  const float *arow;       // [M] per point of the chunk: its widened threshold in accumulator units (screen_terms_kernel)
  const float *ycol;       // [N] per centroid: ||y_j[0 : d')||^2 in accumulator units
  uint32_t *colmask;       // [row tiles of 128][maskw]: bit j = some point of the row tile may pass the first test against j
  int32_t maskw;           // words per row tile: 4 per 128 centroids
  unsigned long long *scal;     // step scalars: SC_SCREEN_DIMS
  // exact mode (iteration 1): arow = the band of every row, ycol = ||y_j||^2 in accumulator units
  unsigned int *rowmin;         // [n] running minimum of every point over the tiles done so far (ordered float bits), by row_base + row
  int64_t row_base;
  Pair *pairs;                  // kSubLists parts of sub_capacity slots: the candidates
  unsigned int *pair_count;     // [kSubLists * kSubListStride]
  unsigned int sub_capacity;
  unsigned int *overflow;
};

// A workgroup of 8 wavefronts owns 256 points x 256 centroids; a wavefront owns 128 x 64 (4 x 2 accumulators of
// 32 x 32: per matrix instruction three quarters of the fragment bytes of a 64 x 64 arrangement), so the rows of a
// wavefront are exactly one row tile of the exact kernel and its verdict on a column needs no other wavefront.
// LDS rows are 64 bytes (four 16-byte pieces: dims 8 c .. 8 c + 7 of the slab, c = 2 h + kh for half-slab h and lane
// half kh); piece c of row r sits at position c ^ ((r >> 2) & 3), so that the 16-byte fragment reads of 16 consecutive
// rows fall into 16 different bank groups.  Staging is global -> LDS directly, 16 bytes per lane, four lanes per row:
// the lane that fills a position fetches the piece that belongs there.  In global memory the hi halves of a row are
// one contiguous plane (see launch_split_rows): a slab row is 64 contiguous bytes.  The kernel is persistent: every XCD walks a
// contiguous range of tiles (column tile fastest inside panels of 8 column tiles), its workgroups take every n-th;
// the first slab of a workgroup's next tile is requested before the finished tile is tested.
//
// EXACT (Algorithm 1, iteration 1, where nothing prunes): the same multiply over ALL dimensions finds, for every point,
// the centroids that can be its nearest.  With v~(i, j) = ||y_j||^2 - 2 (x_i.y_j)~ from the one product and b_i a
// bound of its error (twice the bound of the product: see the top of this file, with the full norms), the true
// nearest j* has v~(i, j*) <= min_j v~(i, j) + 2 b_i.  Every tile takes the minimum of each of its rows over its 256
// columns, lowers the point's running minimum by it (one atomic per row; the tiles of a row run in any order and a
// stale value is only larger), and emits the pairs within 2 b_i of the smaller of the two: j* is among them whenever
// its tile runs.  In random order a row emits in about ln(column tiles) tiles.  The gather kernel then takes the exact
// distance of every emitted pair, and the packed minimum over those is the exact nearest centroid.
template <bool EXACT>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) screen_kernel(ScreenArgs g) {
  extern __shared__ __align__(16) uint32_t smem[];   // [NSTAGE stages][A: BM rows | B: BN rows][ROW_WORDS]
  __shared__ __align__(16) float s_a[NSTAGE][BM];    // per row of a tile in flight: the widened threshold in accumulator units
  __shared__ __align__(16) float s_y[NSTAGE][BN];    // per column of a tile in flight: its prefix norm in the same units
  __shared__ unsigned int s_rmin[EXACT ? BM : 1];    // EXACT: minimum of every row of the tile (ordered float bits)
  __shared__ float s_thr[EXACT ? BM : 1];            // EXACT: emission threshold of every row

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int r32 = lane & 31, kh = lane >> 5;
  const int swz = (r32 >> 2) & 3;
  const int nrt = (g.M + BM - 1) / BM, nct = (g.N + BN - 1) / BN;
  const int ntiles = nrt * nct;
  constexpr int PC = 8;   // column tiles per panel of the tile walk (row tile slowest inside a panel)

  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, nslots = gridDim.x >> 3;
  const int tbase = ntiles >> 3, trem = ntiles & 7;
  const int xstart = xcd * tbase + (xcd < trem ? xcd : trem);
  const int xcount = tbase + (xcd < trem ? 1 : 0);
  const int panel_sz = PC * nrt;
  auto tile_rc = [&](int q, int &rt, int &ct) {   // q-th tile of this XCD -> (row tile, column tile)
    const int logical = xstart + q;
    const int p = logical / panel_sz;
    const int r = logical - p * panel_sz;
    const int pc = (nct - p * PC) < PC ? (nct - p * PC) : PC;
    rt = __builtin_amdgcn_readfirstlane(r / pc);
    ct = __builtin_amdgcn_readfirstlane(p * PC + (r - (r / pc) * pc));
  };

  const int lrow = lane >> 2, lpos = lane & 3;
  const int ld_row = 16 * wave + lrow;                        // + 128 j
  const int ld_c = lpos ^ ((ld_row >> 2) & 3);                // piece that belongs at this lane's position
  const int ld_words = 4 * ld_c;                              // its word offset inside the slab's 16 hi words
  const int koff = -((BK - g.dprime % BK) % BK);
  const int nslab = (g.dprime - koff) / BK;                   // slabs [koff, d')
  const int kw0 = 8 + koff / 2;                               // word of the hi plane where slab 0 starts

  // ---- the loading side runs DEPTH slabs ahead of the multiplying side, across tile boundaries (a tile of a
  // well-pruned step is two or three slabs: one tile's worth of loads in flight would leave the matrix cores waiting
  // for memory latency most of the time)
  int lq = slot, ls = 0;            // tile (per-XCD number) and slab the next request is for
  int ltile = 0;                    // tiles requested so far (ring slot of the row terms)
  int ljob = 0;                     // slabs requested so far (ring slot of the stage)
  const uint32_t *baseA = g.A, *baseB = g.B;
  unsigned int offA[A_LD], offB[B_LD];
  auto request = [&]() {            // one slab; at a tile's first slab also its row terms
    if (lq >= xcount) return;
    if (ls == 0) {
      int rt, ct;
      tile_rc(lq, rt, ct);
      const int row0 = rt * BM, col0 = ct * BN;
      baseA = g.A + (int64_t)row0 * g.lda;
      baseB = g.B + (int64_t)col0 * g.ldb;
      const int limA = g.M - 1 - row0, limB = g.N - 1 - col0;   // rows / columns past the end repeat the last one
#pragma unroll
      for (int j = 0; j < A_LD; ++j) offA[j] = (unsigned int)(min(ld_row + ROWS_PASS * j, limA) * (int)g.lda + ld_words);
#pragma unroll
      for (int j = 0; j < B_LD; ++j) offB[j] = (unsigned int)(min(ld_row + ROWS_PASS * j, limB) * (int)g.ldb + ld_words);
      // the tile's row terms (wavefronts 0-3) and column terms (4-7): one more 4-byte load each, straight into LDS
      {
        const int e = tid & (BM - 1);
        const float *src = wave < 4 ? g.arow + row0 + min(e, limA) : g.ycol + col0 + min(e, limB);
        float *dst = (wave < 4 ? s_a[ltile & (NSTAGE - 1)] : s_y[ltile & (NSTAGE - 1)]) + 64 * (wave & 3);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                         (__attribute__((address_space(3))) void *)dst, 4, 0, 0);
      }
      ++ltile;
    }
    uint32_t *sb = smem + (ljob & (NSTAGE - 1)) * STAGE_WORDS + 16 * wave * ROW_WORDS;
    const int kw = kw0 + (BK / 2) * ls;
#pragma unroll
    for (int j = 0; j < A_LD; ++j)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(baseA + offA[j] + kw),
                                       (__attribute__((address_space(3))) void *)(sb + ROWS_PASS * j * ROW_WORDS), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < B_LD; ++j)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(baseB + offB[j] + kw),
                                       (__attribute__((address_space(3))) void *)(sb + (BM + ROWS_PASS * j) * ROW_WORDS), 16, 0, 0);
    ++ljob;
    if (++ls == nslab) {
      ls = 0;
      lq += nslots;
    }
  };

  if (slot >= xcount) return;
#pragma unroll
  for (int i = 0; i < DEPTH; ++i) request();

  unsigned long long dims_done = 0ull;
  int cjob = 0, ctile = 0;
  for (int q = slot; q < xcount; q += nslots, ++ctile) {
    int rt, ct;
    tile_rc(q, rt, ct);
    const int col0 = ct * BN;
    bool colok[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) colok[b] = col0 + wn * 64 + b * 32 + r32 < g.N;
    f32x16 acc[TM][TN];
    for (int s = 0; s < nslab; ++s, ++cjob) {
      // slab cjob has arrived once at most the requests made after it are outstanding (DEPTH - 1 slabs of four loads
      // each; loads are counted in order, the tile terms in between only make the wait stricter); near the end fewer
      // requests follow, so everything is awaited
      if (lq < xcount) SKM_SCREEN_VMCNT((DEPTH - 1) * (A_LD + B_LD));
      else SKM_SCREEN_VMCNT(0);
      // ... for every wavefront's share of it; and the stage of slab cjob - 1 is free.  (A bare barrier: a fenced one
      // would first wait for every load in flight.  The only LDS traffic besides those loads are reads whose results
      // the matrix instructions before this point have consumed.)
      __builtin_amdgcn_s_barrier();
      request();         // slab cjob + DEPTH -> the stage slab cjob - 1 was in (NSTAGE = DEPTH + 1)
      if (s == 0 && EXACT) {
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
        if (tid < BM) s_rmin[tid] = 0xffffffffu;   // (read after this tile's slab barriers)
      }
      if (s == 0 && !EXACT) {      // every accumulator element starts from its row's term
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {   // accumulator elements 4 q4 .. 4 q4 + 3 are four consecutive rows
            const float4 a4 = *reinterpret_cast<const float4 *>(&s_a[ctile & (NSTAGE - 1)][wm * 128 + a * 32 + 8 * q4 + 4 * kh]);
#pragma unroll
            for (int b = 0; b < TN; ++b) {
              acc[a][b][4 * q4 + 0] = a4.x;
              acc[a][b][4 * q4 + 1] = a4.y;
              acc[a][b][4 * q4 + 2] = a4.z;
              acc[a][b][4 * q4 + 3] = a4.w;
            }
          }
      }
      const uint32_t *st = smem + (cjob & (NSTAGE - 1)) * STAGE_WORDS;
      const uint32_t *Ab = st + (wm * 128 + r32) * ROW_WORDS;
      const uint32_t *Bb = st + (BM + wn * 64 + r32) * ROW_WORDS;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        f16x8 ah[TM], bh[TN];
#pragma unroll
        for (int t = 0; t < TM; ++t)
          ah[t] = *reinterpret_cast<const f16x8 *>(Ab + t * 32 * ROW_WORDS + (((2 * h + kh) ^ swz) << 2));
#pragma unroll
        for (int t = 0; t < TN; ++t)
          bh[t] = *reinterpret_cast<const f16x8 *>(Bb + t * 32 * ROW_WORDS + (((2 * h + kh) ^ swz) << 2));
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
          for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ah[a], bh[b], acc[a][b], 0, 0, 0);
      }
    }
    dims_done += (unsigned long long)(BK * nslab);

    if (EXACT) {
      // ---- minimum of every row over the tile's columns
      const float *yc = s_y[ctile & (NSTAGE - 1)] + wn * 64 + r32;
      const float y0 = colok[0] ? yc[0] : 3.0e38f, y1 = colok[1] ? yc[32] : 3.0e38f;
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          if ((v & 3) == 0) asm volatile("" : : : "memory");   // (four rows at a time: see the registers note below)
          float m = fminf(y0 - acc[a][0][v], y1 - acc[a][1][v]);
          // over the 32 lanes that hold this row (same lane half): quads, half rows, rows, then the two rows of the half
          m = fminf(m, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, m), 0xB1, 0xF, 0xF, false)));
          m = fminf(m, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, m), 0x4E, 0xF, 0xF, false)));
          m = fminf(m, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, m), 0x141, 0xF, 0xF, false)));
          m = fminf(m, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, m), 0x140, 0xF, 0xF, false)));
          m = fminf(m, __shfl_xor(m, 16, 64));
          if (r32 == 0) atomicMin(&s_rmin[wm * 128 + a * 32 + 8 * (v >> 2) + 4 * kh + (v & 3)], f2ord(m));
        }
      __syncthreads();
      // ---- the point's running minimum takes it; the threshold is the smaller of the two plus the band
      if (tid < BM) {
        const int row = rt * BM + tid;
        float thr = -3.0e38f;
        if (row < g.M) {
          const unsigned int local = s_rmin[tid];
          const unsigned int old = atomicMin(g.rowmin + g.row_base + row, local);
          thr = ord2f(old < local ? old : local) + s_a[ctile & (NSTAGE - 1)][tid];
        }
        s_thr[tid] = thr;
      }
      __syncthreads();
      // ---- emit the pairs at or below the threshold of their row
      const int xsub = blockIdx.x & 7;
      int zero = 0;
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          // (a value the compiler cannot see through, renewed every four rows: the thresholds are then fetched four
          // at a time instead of all 64 ahead, which would not fit the registers next to the accumulators)
          if ((v & 3) == 0) asm volatile("" : "+v"(zero) : : "memory");
          const int rl = wm * 128 + a * 32 + 8 * (v >> 2) + 4 * kh + (v & 3) + zero;
          const float thr = s_thr[rl];
          // (v~ <= thr written from the accumulator's side: the differences of the first pass are not kept alive)
          const bool e0 = acc[a][0][v] >= y0 - thr, e1 = acc[a][1][v] >= y1 - thr;
          const unsigned long long b0 = __ballot(e0), b1 = __ballot(e1);
          if (b0 | b1) {
            const int n0 = __popcll(b0), tot = n0 + __popcll(b1);
            unsigned int base = 0;
            if (lane == 0) base = atomicAdd(g.pair_count + xsub * kSubListStride, (unsigned int)tot);
            base = __builtin_amdgcn_readfirstlane(base);
            if ((unsigned long long)base + tot > (unsigned long long)g.sub_capacity) {
              if (lane == 0) atomicOr(g.overflow, 1u);
            } else {
              const unsigned long long below = (1ull << lane) - 1ull;
              Pair pr;
              pr.i = (int32_t)(g.row_base + rt * BM + rl);
              pr.p = 0.f;
              pr.tau = 3.0e38f;
              Pair *dst = g.pairs + (size_t)xsub * g.sub_capacity + base;
              if (e0) {
                pr.j = col0 + wn * 64 + r32;
                dst[__popcll(b0 & below)] = pr;
              }
              if (e1) {
                pr.j = col0 + wn * 64 + 32 + r32;
                dst[n0 + __popcll(b1 & below)] = pr;
              }
            }
          }
        }
      continue;
    }

    // ---- widened first test: a column stays if any row of this wavefront's row tile may pass theta(d', tau) against it
    bool alive[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      float best = acc[0][b][0];
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) best = fmaxf(best, acc[a][b][v]);
      alive[b] = best >= s_y[ctile & (NSTAGE - 1)][wn * 64 + b * 32 + r32];
    }
    const int rtile = rt * (BM / RT) + wm;   // the row tile of 128 this wavefront speaks for
    if (rtile * RT < g.M) {
#pragma unroll
      for (int b = 0; b < TN; ++b) {
        const unsigned long long bal = __ballot(alive[b] && colok[b]);
        const unsigned int w = (unsigned int)bal | (unsigned int)(bal >> 32);   // column r32: lanes r32 and r32 + 32
        const int word = ct * (BN / 32) + wn * 2 + b;
        if (lane == 0 && word < g.maskw) g.colmask[(int64_t)rtile * g.maskw + word] = w;
      }
    }
  }
  if (tid == 0 && dims_done)   // (in units of the exact kernel's 128 x 128 tiles: four per tile of this kernel)
    atomicAdd(g.scal + (size_t)(blockIdx.x & (kStatReplicas - 1)) * SC_COUNT + SC_SCREEN_DIMS, 4ull * dims_done);
}

// ---------------------------------------------------------------- bits -> lists of listed columns per row tile
// cnt[rt] = set bits of row tile rt (one wavefront per row tile)
__global__ void __launch_bounds__(256) mask_count_kernel(const uint32_t *mask, int32_t nrt, int32_t maskw, int32_t *cnt) {
  const int lane = threadIdx.x & 63;
  const int rt = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (rt >= nrt) return;
  int c = 0;
  for (int w = lane; w < maskw; w += 64) c += __popc(mask[(int64_t)rt * maskw + w]);
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) c += __shfl_xor(c, m, 64);
  if (lane == 0) cnt[rt] = c;
}

// first[rt] = first tile of row tile rt (tiles of 128 listed columns, row tiles in order), *ntiles = their number
__global__ void __launch_bounds__(1024) mask_scan_kernel(const int32_t *cnt, int32_t nrt, int32_t *first, int32_t *ntiles,
                                                         unsigned long long *scal) {
  __shared__ int s_part[1024];
  const int tid = threadIdx.x;
  const int per = (nrt + 1023) / 1024;
  const int lo = min(tid * per, nrt), hi = min(lo + per, nrt);
  int sum = 0;
  for (int r = lo; r < hi; ++r) sum += (cnt[r] + 127) >> 7;
  s_part[tid] = sum;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {   // inclusive scan of the per-thread sums
    const int v = tid >= off ? s_part[tid - off] : 0;
    __syncthreads();
    s_part[tid] += v;
    __syncthreads();
  }
  int run = s_part[tid] - sum;
  for (int r = lo; r < hi; ++r) {
    first[r] = run;
    run += (cnt[r] + 127) >> 7;
  }
  if (tid == 1023) {
    *ntiles = s_part[1023];
    atomicAdd(scal + SC_LISTED_TILES, (unsigned long long)s_part[1023]);
  }
}

// One workgroup per row tile: the ids of its set bits in ascending order, padded with -1 to a multiple of 128, into
// col_list[128 * first[rt] ...]; tile_rt[t] = rt for each of its tiles.
__global__ void __launch_bounds__(256) mask_fill_kernel(const uint32_t *mask, int32_t maskw, const int32_t *cnt,
                                                        const int32_t *first, int32_t *col_list, int32_t *tile_rt) {
  __shared__ int s_wave[4];
  __shared__ int s_base;
  const int rt = blockIdx.x;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int total = cnt[rt];
  const int t0 = first[rt], nt = (total + 127) >> 7;
  int32_t *out = col_list + (int64_t)t0 * 128;
  if (tid == 0) s_base = 0;
  __syncthreads();
  for (int w0 = 0; w0 < maskw; w0 += 256) {
    const int w = w0 + tid;
    unsigned int bits = w < maskw ? mask[(int64_t)rt * maskw + w] : 0u;
    const int mine = __popc(bits);
    int incl = mine;   // inclusive prefix inside the wavefront
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, 64);
      if (lane >= off) incl += v;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int pos = s_base + incl - mine;
    for (int ww = 0; ww < wave; ++ww) pos += s_wave[ww];
    while (bits) {
      const int b = __builtin_ctz(bits);
      bits &= bits - 1u;
      out[pos++] = w * 32 + b;
    }
    __syncthreads();
    if (tid == 0) s_base += s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
    __syncthreads();
  }
  for (int p = total + tid; p < nt * 128; p += 256) out[p] = -1;
  for (int t = tid; t < nt; t += 256) tile_rt[t0 + t] = rt;
}

// The test of a pair, theta + widening - ||x'||^2 >= ||y'||^2 - 2 x'.y', in accumulator units (the accumulator holds
// x'.y' times the two scales; K = 2 / scales > 0):   acc + a_i >= y_j   with
//   a_i = (theta_i - ||x'_i||^2 + slack + guard + widening ||x'_i|| max_j ||y'_j||) / K,   y_j = ||y'_j||^2 (1 - guard) / K.
// a_i is what the row's accumulator elements START from, so after the last slab the verdict on a column is one maximum
// over its rows against one number.  (The widening uses the largest centroid norm instead of the column's own: looser
// only for centroids whose front part is small.)  slack: halves below the smallest normal fp16 (off by up to 2^-25
// scaled = 2^-39 of the bound each, times the other operand, two operands, d' terms, times 2 for the distance).
__global__ void __launch_bounds__(256) screen_terms_kernel(const float *tau, const float *xn, int64_t row_base, int32_t M,
                                                           const float *yn, int32_t N, const float *ynmax, float ratio0,
                                                           int32_t dprime, const unsigned int *a_absmax,
                                                           const unsigned int *b_absmax, float *arow, float *ycol,
                                                           int exact) {
  const float ax = __builtin_bit_cast(float, *a_absmax), ay = __builtin_bit_cast(float, *b_absmax);
  const float slack = (float)dprime * ax * ay * (1.f / 8589934592.f);   // d' * max|x| * max|y| * 2^-33
  const float inv_k = 0.5f * split_scale(*a_absmax) * split_scale(*b_absmax);
  const float symax = sqrtf(fmaxf(*ynmax, 0.f));
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (exact) {
    // exact mode: the band 2 b_i around the smallest v~ of a row inside which the true nearest centroid must lie:
    // b_i = 2 * (bound of the product's error) = widening ||x_i|| max_j ||y_j||, plus the slack and a guard for the
    // rounding of the values compared (their size is at most ||y||^2 + 2 ||x|| ||y||); y_j = ||y_j||^2 / K
    if (i < M) {
      const float xs = sqrtf(fmaxf(xn[row_base + i], 0.f));
      arow[i] = (2.f * kWiden * xs * symax + 2.f * slack + 4.f * kGuard * (symax * symax + 2.f * xs * symax)) * inv_k;
    }
    if (i < N) ycol[i] = yn[i] * inv_k;
    return;
  }
  if (i < M) {
    const float x2 = xn[row_base + i];
    const float th = ratio0 * tau[row_base + i];
    arow[i] = (th - x2 + slack + kGuard * (th + x2) + kWiden * sqrtf(fmaxf(x2, 0.f)) * symax) * inv_k;
  }
  if (i < N) ycol[i] = yn[i] * (1.f - kGuard) * inv_k;
}

// *out = max of v[0 .. n) (non-negative values: their bit patterns order like the numbers)
__global__ void __launch_bounds__(1024) max_value_kernel(const float *v, int32_t n, float *out) {
  __shared__ float red[16];
  float m = 0.f;
  for (int i = threadIdx.x; i < n; i += 1024) m = fmaxf(m, v[i]);
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 16; ++w) m = fmaxf(m, red[w]);
    *out = m;
  }
}

hipError_t launch_screen(const ScreenLaunch &a, hipStream_t st) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  if (a.dprime % 16 != 0 || a.dprime < 16 || a.dprime > a.ds || a.lda != a.ds / 2 + 16 || a.ldb != a.ds / 2 + 16 ||
      (reinterpret_cast<uintptr_t>(a.A) & 15u) || (reinterpret_cast<uintptr_t>(a.B) & 15u) || a.N > (1 << 24))
    return hipErrorInvalidValue;
  if (a.exact && (!a.rowmin || !a.pairs || !a.pair_count || !a.overflow)) return hipErrorInvalidValue;
  constexpr size_t smem = (size_t)NSTAGE * STAGE_WORDS * sizeof(uint32_t);
  struct Setup {
    hipError_t rc;
    int wgs = 0;
    Setup() {
      rc = hipFuncSetAttribute(reinterpret_cast<const void *>(screen_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (rc == hipSuccess)
        rc = hipFuncSetAttribute(reinterpret_cast<const void *>(screen_kernel<true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      int dev = 0, cus = 256;
      (void)hipGetDevice(&dev);
      (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
      wgs = cus;   // one workgroup of eight wavefronts per CU
    }
  };
  static const Setup setup;
  if (setup.rc != hipSuccess) return setup.rc;
  const int nrt = (a.M + RT - 1) / RT, nct = (a.N + 127) / 128;   // row tiles and column tiles of the exact kernel
  const int64_t ntiles = (int64_t)((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  if (ntiles > 0x7fffffffLL) return hipErrorInvalidValue;
  ScreenArgs g{};
  g.A = a.A; g.lda = a.lda; g.M = a.M; g.B = a.B; g.ldb = a.ldb; g.N = a.N;
  g.a_absmax = a.a_absmax; g.b_absmax = a.b_absmax;
  g.dprime = a.dprime;
  float *ynmax = reinterpret_cast<float *>(a.ntiles + 1);   // (the word after the tile count)
  hipLaunchKernelGGL(max_value_kernel, dim3(1), dim3(1024), 0, st, a.yn, a.N, ynmax);
  hipLaunchKernelGGL(screen_terms_kernel, dim3((unsigned)((std::max<int64_t>(a.M, a.N) + 255) / 256)), dim3(256), 0, st,
                     a.tau, a.xn, a.row_base, a.M, a.yn, a.N, (const float *)ynmax, a.ratio0, a.dprime, a.a_absmax,
                     a.b_absmax, a.arow, a.ycol, a.exact ? 1 : 0);
  g.arow = a.arow; g.ycol = a.ycol; g.colmask = a.colmask; g.maskw = 4 * nct;
  g.scal = a.scal;
  g.rowmin = a.rowmin; g.row_base = a.row_base; g.pairs = a.pairs; g.pair_count = a.pair_count;
  g.sub_capacity = a.sub_capacity; g.overflow = a.overflow;
  const int64_t grid = std::max<int64_t>(8, std::min<int64_t>(setup.wgs, (ntiles + 7) / 8 * 8));
  if (a.exact) {
    hipLaunchKernelGGL(screen_kernel<true>, dim3((unsigned)grid), dim3(NT), smem, st, g);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(screen_kernel<false>, dim3((unsigned)grid), dim3(NT), smem, st, g);
  hipError_t rc = hipGetLastError();
  if (rc != hipSuccess) return rc;
  hipLaunchKernelGGL(mask_count_kernel, dim3((unsigned)((nrt + 3) / 4)), dim3(256), 0, st, a.colmask, nrt, 4 * nct, a.cnt);
  hipLaunchKernelGGL(mask_scan_kernel, dim3(1), dim3(1024), 0, st, a.cnt, nrt, a.first, a.ntiles, a.scal);
  hipLaunchKernelGGL(mask_fill_kernel, dim3((unsigned)nrt), dim3(256), 0, st, a.colmask, 4 * nct, a.cnt, a.first,
                     a.col_list, a.tile_rt);
  return hipGetLastError();
}

}  // namespace skm
