// Progressive-pruning GEMM (Algorithm 1, iterations >= 2; Section 3.4 "Progressive Pruning").
//
// The paper multiplies only the first d' dimensions densely and finishes survivors one by one.
// On MI355X a 64-dimension step of a dense 128 x 128 tile on the matrix cores costs about as
// much as gathering the same step for 2 % of the tile's pairs, so this kernel keeps multiplying a
// tile densely, 64 dimensions at a time, while more than a small share of its pairs is alive, and
// hands the pairs over to the gather kernel (prune.hip) only once the tile is sparse.  The tests are
// the paper's: after t = d', d'+64, d'+128, ... dimensions a pair is dropped when its partial squared
// distance exceeds theta(t, tau_i); a pair that reaches t = d is offered to the point's packed
// (distance, centroid) minimum if it beats tau_i.
//
// Partial distances come from the norm expansion ||x_t||^2 + ||y_t||^2 - 2 x_t.y_t (Section 3.1).
// The prefix norms at the checkpoints are inputs (xnp, ynp): passes that read every point and every
// centroid anyway write them, and this kernel fetches one number per row and column and checkpoint.
//
// Operands arrive already split into fp16 pairs (the points once per fit, by the first threshold pass; the
// centroids once per step, by split_rows_kernel), in the very byte order of the LDS tiles, so staging is a
// copy: every lane moves 16 bytes from global memory straight into LDS and the vector unit is left to the tests.
//
// The kernel is persistent: two workgroups per CU take tiles from a per-XCD counter.  When a tile
// ends, the first slab and the per-row data of the next tile are already being fetched while the
// finished tile is written out, so the short tiles of a well-pruned step do not drain the pipeline.
#include "skm_internal.h"

#include <algorithm>
#include <cstdlib>

namespace skm {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// ---------------------------------------------------------------- split-fp16 copies of the operands
// Row r of a matrix scaled by split_scale(*absmax): granule g (dims 16 g .. 16 g + 15) is 16 words at word
// 16 (g + 1) of the row: 8 words of hi halves (fp16 of the scaled value, two per word), then 8 words of lo
// halves (fp16 of the remainder).  Granule positions 0 and ds / 16 + 1 are zero, so that a 32-dimension slab
// starting 16 dimensions before the row or ending 16 after it reads zeros.  Row stride ds + 32 words.
// out_hi (optional): the hi halves once more as a plane of their own, ds / 2 + 16 words a row (8 zero words, the row two
// dimensions a word, 8 zero words): what the low-precision first filter reads, 64 contiguous bytes per row and slab.
__global__ void __launch_bounds__(256) split_rows_kernel(const float *A, int64_t lda, int64_t rows, int32_t ds,
                                                         const unsigned int *absmax, uint32_t *out, uint32_t *out_hi) {
  const float scale = split_scale(*absmax);
  const int per_row = ds / 4 + 8;   // float4 pieces per output row, pads included
  const int64_t total = rows * per_row;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = e / per_row;
    const int piece = (int)(e - r * per_row);      // 4 dims each; pieces 0..3 and the last 4 are padding
    const int gpos = piece >> 2, q = piece & 3;    // granule position, quarter of the granule
    uint2 hi = make_uint2(0u, 0u), lo = hi;
    if (gpos >= 1 && gpos <= ds / 16) {
      const float4 v = *reinterpret_cast<const float4 *>(A + r * lda + 16 * (gpos - 1) + 4 * q);
      const f32x2 p0 = {v.x * scale, v.y * scale}, p1 = {v.z * scale, v.w * scale};
      const f16x2 h0 = __builtin_convertvector(p0, f16x2), h1 = __builtin_convertvector(p1, f16x2);
      const f16x2 l0 = __builtin_convertvector(p0 - __builtin_convertvector(h0, f32x2), f16x2);
      const f16x2 l1 = __builtin_convertvector(p1 - __builtin_convertvector(h1, f32x2), f16x2);
      hi.x = __builtin_bit_cast(unsigned int, h0); hi.y = __builtin_bit_cast(unsigned int, h1);
      lo.x = __builtin_bit_cast(unsigned int, l0); lo.y = __builtin_bit_cast(unsigned int, l1);
    }
    uint32_t *dst = out + r * (int64_t)(ds + 32) + 16 * gpos;
    *reinterpret_cast<uint2 *>(dst + 2 * q) = hi;
    *reinterpret_cast<uint2 *>(dst + 8 + 2 * q) = lo;
    if (out_hi) *reinterpret_cast<uint2 *>(out_hi + r * (int64_t)(ds / 2 + 16) + 2 * piece) = hi;
  }
}
hipError_t launch_split_rows(const float *A, int64_t lda, int64_t rows, int32_t ds, const unsigned int *absmax,
                             uint32_t *out, hipStream_t st, uint32_t *out_hi) {
  if (rows <= 0) return hipSuccess;
  if (ds % 16 != 0 || lda % 4 != 0 || (reinterpret_cast<uintptr_t>(A) & 15u) || (reinterpret_cast<uintptr_t>(out) & 15u))
    return hipErrorInvalidValue;
  const int64_t total = rows * (ds / 4 + 8);
  const int64_t blocks = std::min<int64_t>((total + 255) / 256, 1 << 16);
  if (reinterpret_cast<uintptr_t>(out_hi) & 15u) return hipErrorInvalidValue;
  hipLaunchKernelGGL(split_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, A, lda, rows, ds, absmax, out, out_hi);
  return hipGetLastError();
}

namespace {
constexpr int BM = 128, BN = 128, BK = 32;
constexpr int WTM = 64, WTN = 64, TM = 2, TN = 2;
constexpr int NT = 256;
constexpr int ROW_WORDS = BK;                       // a tile row of a slab: 32 hi + 32 lo halves = 128 bytes
constexpr int STAGE_WORDS = (BM + BN) * ROW_WORDS;  // one slab of both operands: 32 KB
constexpr int ROWS_PASS = NT / 8;                   // 8 lanes move one tile row: 32 rows per load instruction
constexpr int A_LD = BM / ROWS_PASS;                // 4 load instructions per thread, slab and operand
constexpr int B_LD = BN / ROWS_PASS;

// wait until at most n of this wavefront's vector memory operations are outstanding (LDS and export counters untouched)
#define SKM_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 0xF) | (((n) >> 4) << 14) | (0x7 << 4) | (0xF << 8))

// Sum over the 64 lanes of a wavefront through the data-parallel lane moves: within quads, mirrored
// within half rows and rows, then the row totals handed on to the following rows; lane 63 ends with the result.
#define SKM_WAVE_REDUCE(v, OP)                                                                \
  do {                                                                                        \
    v = v OP __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);  /* quad_perm [1,0,3,2] */ \
    v = v OP __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);  /* quad_perm [2,3,0,1] */ \
    v = v OP __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false); /* row_half_mirror */      \
    v = v OP __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, false); /* row_mirror */           \
    v = v OP __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false); /* row_bcast:15 */         \
    v = v OP __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false); /* row_bcast:31 */         \
  } while (0)
__device__ inline int wave_sum_i32(int v) {
  SKM_WAVE_REDUCE(v, +);
  return __builtin_amdgcn_readlane(v, 63);
}

}  // namespace

// Slabs of BK dimensions start at koff = -((BK - d' % BK) % BK), so that slab ends fall on every
// checkpoint d' + 64 m; the zero granules around every row of the split operands cover dimensions below 0
// or past ds.
template <bool LISTED>
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) progressive_kernel(ProgArgs g) {
  extern __shared__ __align__(16) uint32_t smem[];   // [2 stages][A: BM rows | B: BN rows][ROW_WORDS]
  __shared__ __align__(16) float s_tau[2][BM], s_thr[BM], s_xn[BM], s_yn[BN];   // s_tau: by tile parity
  __shared__ float s_ratio[kMaxBlocks + 1];
  __shared__ unsigned long long s_dead[NT];   // per thread: accumulator elements that start dead (the incumbent)
  __shared__ __align__(16) unsigned int s_wcnt[2][4];   // alive pairs of every wavefront at the last checkpoint (by checkpoint parity)
  __shared__ unsigned int s_base;         // first list slot of a tile that hands its pairs over
  __shared__ int s_q[4];   // ring of tile numbers drawn from the XCD's counter, two tiles ahead of the one in work
  __shared__ int s_cid[BN];   // listed columns: the centroid ids of the tile being committed (INT_MAX = none)

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int r32 = lane & 31, kh = lane >> 5;
  const int swz = (r32 >> 1) & 7;   // position swizzle of the tile rows this lane reads fragments from
  const int nrt = (g.M + BM - 1) / BM, nct = (g.N + BN - 1) / BN;
  // Listed columns (after the low-precision first filter): tile t is row tile tile_rt[t] against the 128 centroids
  // col_list[128 t ..]; the "column tile" of such a tile is its own number.
  constexpr bool listed = LISTED;
  const int ntiles = listed ? *g.ntiles : nrt * nct;
  // column tiles per panel of the tile walk: in the steady state only d' + a few blocks of every centroid are read,
  // so a panel of 16 column tiles fits one XCD's L2 and every point tile is read once per 16 column tiles
  constexpr int PC = 16;

  // This workgroup's share: the contiguous range of logical tile ids of its XCD (workgroups are dealt
  // round-robin to the 8 XCDs), walked through a per-XCD counter.
  const int xcd = blockIdx.x & 7;
  const int tbase = ntiles >> 3, trem = ntiles & 7;
  const int xstart = xcd * tbase + (xcd < trem ? xcd : trem);
  const int xcount = tbase + (xcd < trem ? 1 : 0);
  unsigned int *ctr = g.tile_counter + xcd * kSubListStride;
  const int panel_sz = PC * nrt;
  const float inv_panel = 1.0f / (float)panel_sz;
  auto tile_rc = [&](int q, int &rt, int &ct) {   // q-th tile of this XCD -> (row tile, column tile)
    const int logical = xstart + q;
    if (listed) {
      rt = g.tile_rt[logical];
      ct = logical;
      return;
    }
    // panel = logical / panel_sz without an integer division: the float estimate is within one of the quotient
    // (fewer than 2^20 panels), and the remainder says which way
    int p = (int)((float)logical * inv_panel);
    int r = logical - p * panel_sz;
    if (r < 0) {
      --p;
      r += panel_sz;
    } else if (r >= panel_sz) {
      ++p;
      r -= panel_sz;
    }
    const int pc = (nct - p * PC) < PC ? (nct - p * PC) : PC;
    rt = pc == PC ? r >> 4 : r / pc;   // only the last panel can be narrower
    ct = p * PC + (r - rt * pc);
  };
  static_assert(PC == 16, "the shift above");

  unsigned long long *sc = g.scal + (size_t)(blockIdx.x & (kStatReplicas - 1)) * SC_COUNT;
  for (int m = tid; m <= g.nb; m += NT) s_ratio[m] = g.ratio[m];
  s_dead[tid] = 0ull;

  // Staging: load instruction j of wavefront w moves tile rows 32 j + 8 w .. + 7 of a slab, 8 lanes per row and 16
  // bytes per lane, from global memory straight into LDS, where the lanes' pieces land one after the other: LDS rows
  // are 128 bytes without padding.  Piece c of a row (c = 4 h + 2 lo + kh: half-slab, hi or lo halves, dims 8 kh ..
  // + 7 of the half-slab) is kept at position c ^ swz(row), swz = (row >> 1) & 7, so that the 16-byte fragment reads
  // of 16 consecutive rows fall into 16 different bank groups; a lane therefore fetches the piece that belongs at
  // its own position.
  const int lrow = lane >> 3, lpos = lane & 7;
  const int ld_row = 8 * wave + lrow;                        // + 32 j
  const int ld_piece = lpos ^ ((ld_row >> 1) & 7);
  const int koff = -((BK - g.dprime % BK) % BK);
  const int nslab = (g.ds - koff + BK - 1) / BK;
  const int kw0 = 16 + koff;                                 // word of a split row where slab 0 starts (one zero granule leads)

  // Rows past the end are clamped to the last row (their accumulator elements start dead).
  unsigned int offA[A_LD], offB[B_LD];      // word offset of this lane's piece from the tile's first row / column
  float tau_reg = 0.f;
  int prev_reg = -1;
  const uint32_t *baseA = g.A, *baseB = g.B;   // first row / column of the tile being loaded (uniform)
  int limA = 0, limB = 0;                      // last valid row / column of that tile, relative to its first (uniform)
  // prefix norms: threads 0..127 fetch those of the tile's rows, threads 128..255 those of its columns
  const float *npre = g.xnp;                // &norm[0][this thread's row or column]
  const int64_t npre_stride = tid < BM ? g.xn_stride : (int64_t)g.N;
  float nreg = 0.f;
  int cid_reg = 0;   // listed columns, threads BM..: the centroid id of column tid - BM of the tile being loaded
  auto aim = [&](int row0, int col0) {
    baseA = g.A + (int64_t)row0 * g.lda;
    limA = g.M - 1 - row0;
#pragma unroll
    for (int j = 0; j < A_LD; ++j)
      offA[j] = (unsigned int)(min(ld_row + ROWS_PASS * j, limA) * (int)g.lda + 4 * ld_piece);
    if (listed) {
      // col0 is the tile's number: its columns are listed ids (a missing one loads centroid 0 and starts dead)
      const int32_t *ids = g.col_list + (int64_t)col0 * BN;
      baseB = g.B;
      limB = BN - 1;
#pragma unroll
      for (int j = 0; j < B_LD; ++j) {
        const int id = ids[ld_row + ROWS_PASS * j];
        offB[j] = (unsigned int)(max(id, 0) * (int)g.ldb + 4 * ld_piece);
      }
      cid_reg = tid >= BM ? ids[tid - BM] : 0;
      npre = tid < BM ? g.xnp + g.row_base + row0 + min(tid, limA) : g.ynp + max(cid_reg, 0);
      return;
    }
    baseB = g.B + (int64_t)col0 * g.ldb;
    limB = g.N - 1 - col0;
#pragma unroll
    for (int j = 0; j < B_LD; ++j)
      offB[j] = (unsigned int)(min(ld_row + ROWS_PASS * j, limB) * (int)g.ldb + 4 * ld_piece);
    npre = tid < BM ? g.xnp + g.row_base + row0 + min(tid, limA) : g.ynp + col0 + min(tid - BM, limB);
  };
  // slab s of the aimed tile -> LDS stage `stage` (asynchronous: SKM_VMCNT(0) and a barrier before it is read)
  auto issue = [&](int stage, int s) {
    uint32_t *sb = smem + stage * STAGE_WORDS + 8 * wave * ROW_WORDS;
    const int kw = kw0 + BK * s;
#pragma unroll
    for (int j = 0; j < A_LD; ++j)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(baseA + offA[j] + kw),
                                       (__attribute__((address_space(3))) void *)(sb + ROWS_PASS * j * ROW_WORDS), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < B_LD; ++j)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(baseB + offB[j] + kw),
                                       (__attribute__((address_space(3))) void *)(sb + (BM + ROWS_PASS * j) * ROW_WORDS), 16, 0, 0);
  };
  // Row of the norm tables that multiply step s needs if it ends on a checkpoint (any valid row otherwise): the
  // points' table has a row per 16 dimensions, the centroids' a row per checkpoint of this step.
  auto load_norm = [&](int s) {
    const int td = koff + BK * (s + 1);
    const bool end = s + 1 >= nslab;
    const int px = ((end ? g.ds : min(max(td, 16), g.ds)) >> 4) - 1;
    const int py = end ? g.nb : min(max((td - g.dprime) / kBlockDims, 0), g.nb);
    nreg = npre[(int64_t)(tid < BM ? px : py) * npre_stride];
  };
  auto load_rows = [&](int row0) {   // per-row data of a tile, one row per thread of the first two wavefronts
    if (tid < BM) {
      const int gr = min(row0 + tid, g.M - 1);
      tau_reg = g.tau[g.row_base + gr];
      prev_reg = row0 + tid < g.M ? g.prev[g.row_base + gr] : -1;
    }
  };
  const unsigned int amax = *g.a_absmax, bmax = *g.b_absmax;
  const float m2 = -2.f * split_unscale(amax) * split_unscale(bmax);   // accumulator -> -2 x.y
  // the prefix norms fetched during the previous step -> LDS, with the row's threshold theta(t_m, tau) - ||x_t||^2
  auto publish_norms = [&](float ratio) {
    if (tid < BM) {
      s_xn[tid] = nreg;
      s_thr[tid] = ratio * tau_reg - nreg;
    } else {
      s_yn[tid - BM] = nreg;
    }
  };
  auto row_of = [&](int a, int v) { return wm * WTM + a * 32 + 8 * (v >> 2) + 4 * kh + (v & 3); };

  // first tile of this workgroup
  __syncthreads();
  if (tid == 0) {
    s_q[0] = (int)atomicAdd(ctr, 1u);
    s_q[1] = (int)atomicAdd(ctr, 1u);
  }
  __syncthreads();
  int q = __builtin_amdgcn_readfirstlane(s_q[0]);
  if (q >= xcount) return;
  int rt, ct;
  tile_rc(q, rt, ct);
  rt = __builtin_amdgcn_readfirstlane(rt);
  ct = __builtin_amdgcn_readfirstlane(ct);
  // (listed columns: a tile's "first column" is its number, see aim and commit)
  auto col_arg = [&](int c) { return listed ? c : c * BN; };
  aim(rt * BM, col_arg(ct));
  int stg = 0;   // LDS stage that holds (or is receiving) the slab of the multiply step in work
  load_norm(0);
  issue(stg, 0);
  load_rows(rt * BM);
  // A tile is committed once its first slab and its per-row data have arrived: the thresholds go to LDS (two copies by
  // tile parity: the previous tile may still be handing pairs over), the incumbents are marked, and the number of the
  // tile after next is drawn (the counter's answer is stored at the end of the tile, so its round trip never stalls
  // the workgroup).  One barrier separates two tiles.
  unsigned int drawn = 0;
  auto commit = [&](int col0, int par) {
    SKM_VMCNT(0);
    if (listed) {   // the tile's centroid ids, ascending, for the search below
      if (tid >= BM) s_cid[tid - BM] = cid_reg < 0 ? 0x7fffffff : cid_reg;
      __syncthreads();
    }
    if (tid < BM) {
      s_tau[par][tid] = tau_reg;
      // the incumbent of this row, if it is a column of this tile, starts dead: find the thread and the
      // accumulator element that hold (row tid, column prev - col0).  (Every thread emptied its own marks right
      // after the previous commit's barrier, and has crossed a multiply step's barrier since.)
      int cl = prev_reg - col0;
      if (listed) {   // position of the incumbent among the listed ids, if it is one of them
        int lo = 0;
#pragma unroll
        for (int step = BN / 2; step > 0; step >>= 1)
          if (s_cid[lo + step] <= prev_reg) lo += step;
        cl = (prev_reg >= 0 && s_cid[lo] == prev_reg) ? lo : -1;
      }
      if (cl >= 0 && cl < BN) {
        const int rr = tid & 31;
        const int lane_t = ((rr >> 2) & 1) * 32 + (cl & 31);
        const int wave_t = (tid >> 6) * 2 + (cl >> 6);
        const int v_t = 4 * (rr >> 3) + (rr & 3);
        const int bit = ((((tid & 63) >> 5) * TN) + ((cl & 63) >> 5)) * 16 + v_t;
        atomicOr(&s_dead[wave_t * 64 + lane_t], 1ull << bit);
      }
    }
    if (tid == 0) drawn = atomicAdd(ctr, 1u);
    __syncthreads();
  };
  commit(col_arg(ct), 0);

  for (int tile_no = 0;; ++tile_no) {
    const int row0 = rt * BM, col0 = col_arg(ct);
    const int par = tile_no & 1;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    int gc[TN];   // centroid of this lane's accumulator columns (listed columns: from the committed ids, INT_MAX = none)
#pragma unroll
    for (int b = 0; b < TN; ++b) gc[b] = listed ? s_cid[wn * WTN + b * 32 + r32] : col0 + wn * WTN + b * 32 + r32;

    // one alive-bit per accumulator element
    unsigned long long bits = ~s_dead[tid];
    s_dead[tid] = 0ull;
    if (row0 + BM > g.M || (listed ? (gc[0] >= g.N || gc[1] >= g.N) : col0 + BN > g.N)) {
      // ragged edge tile: rows / columns past the end (or not listed) start dead
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const bool ok = (row0 + row_of(a, v) < g.M) && (gc[b] < g.N);
            bits &= ~((unsigned long long)(!ok) << ((a * TN + b) * 16 + v));
          }
    }

    int fin_mode = 0, fin_m = 0;   // how the tile ends: 0 = nothing alive, 1 = reached t = d, 2 = handed over at fin_m
    int wave_alive = 0;            // alive pairs of this wavefront at the last checkpoint
    unsigned int slot0 = 0;        // thread 0: reply of the list reservation
    float yn[TN] = {0.f, 0.f};
    // Fragments of half a slab (16 dims): lane half kh supplies the 8 consecutive dims 16 h + 8 kh .. + 7 of both
    // operands.  x.y ~ hi.hi' + lo.hi' + hi.lo' on the fp16 matrix cores, fp32 accumulation, in groups of four
    // matrix instructions; the fragments of the second half-slab are fetched as the first half releases registers.
    f16x8 ah[TM], al[TM], bh[TN], bl[TN];
    auto frag = [&](const uint32_t *base, int h, int lo, int t) {
      return *reinterpret_cast<const f16x8 *>(base + t * 32 * ROW_WORDS + (((4 * h + 2 * lo + kh) ^ swz) << 2));
    };
    auto mma4 = [&](const f16x8 (&x)[TM], const f16x8 (&y)[TN]) {
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x[a], y[b], acc[a][b], 0, 0, 0);
    };
    for (int s = 0; s < nslab; ++s) {
      const int tdone = koff + BK * (s + 1);   // dimensions multiplied after this step
      const bool last = (s + 1 == nslab);
      const bool check = !last && tdone >= g.dprime && tdone < g.d && ((tdone - g.dprime) & (kBlockDims - 1)) == 0;
      const bool cp = check || last;
      const int m = last ? g.nb : (tdone - g.dprime) / kBlockDims;   // checkpoint index, t_m = min(d, d' + 64 m)
      // the norms of checkpoint m were requested one step ago (or with the tile's first slab); every step requests
      // those of the step after it, needed or not, so that the request is never behind a branch
      if (cp) publish_norms(s_ratio[m]);
      load_norm(s + 1);
      // the next slab goes straight into the other stage, which every wavefront has finished reading (the barrier
      // that ended the previous step); it is complete, and visible, after the wait and the barrier below
      if (!last) issue(stg ^ 1, s + 1);
      const uint32_t *Ab = smem + stg * STAGE_WORDS + (wm * WTM + r32) * ROW_WORDS;
      const uint32_t *Bb = smem + stg * STAGE_WORDS + (BM + wn * WTN + r32) * ROW_WORDS;
      {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          ah[t] = frag(Ab, 0, 0, t); bh[t] = frag(Bb, 0, 0, t);
          al[t] = frag(Ab, 0, 1, t); bl[t] = frag(Bb, 0, 1, t);
        }
        __builtin_amdgcn_sched_barrier(0);
        mma4(ah, bh);
        mma4(al, bh);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 2; ++t) { al[t] = frag(Ab, 1, 1, t); bh[t] = frag(Bb, 1, 0, t); }
        mma4(ah, bl);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 2; ++t) { ah[t] = frag(Ab, 1, 0, t); bl[t] = frag(Bb, 1, 1, t); }
        mma4(al, bh);
        __builtin_amdgcn_sched_barrier(0);
        mma4(ah, bl);
        mma4(ah, bh);
        __builtin_amdgcn_sched_barrier(0);
      }
      stg ^= 1;
      SKM_VMCNT(0);
      __syncthreads();
      if (cp) {
#pragma unroll
        for (int b = 0; b < TN; ++b) yn[b] = s_yn[wn * WTN + b * 32 + r32];
        if (!last || g.nb == 0) {
          // test theta(t_m, tau_i): drop the pair when its partial distance exceeds it.  The sign of threshold minus
          // distance is the verdict (a difference of two floats is negative exactly when the second is larger); the
          // signs of the 32 elements of an accumulator row block are shifted into one word, last element first, one
          // funnel shift each.
#pragma unroll
          for (int a = 0; a < TM; ++a) {
            unsigned int dropped = 0u;
#pragma unroll
            for (int b = TN - 1; b >= 0; --b)
#pragma unroll
              for (int v = 15; v >= 0; --v) {
                const float margin = s_thr[row_of(a, v)] - fmaf(m2, acc[a][b][v], yn[b]);
                dropped = __builtin_amdgcn_alignbit(dropped, __builtin_bit_cast(unsigned int, margin), 31);
              }
            bits &= ~((unsigned long long)dropped << (32 * a));
          }
          static_assert(TN * 16 == 32, "one word per accumulator row block");
        }
        // alive pairs of this wavefront and of the whole tile
        wave_alive = wave_sum_i32(__popcll(bits));
        if (lane == 0) s_wcnt[m & 1][wave] = (unsigned int)wave_alive;
        __syncthreads();
        // (the counts of checkpoint m + 1 go to the other row: a wavefront that is already there cannot disturb this read)
        const uint4 wc = *reinterpret_cast<const uint4 *>(s_wcnt[m & 1]);
        const unsigned int total = wc.x + wc.y + wc.z + wc.w;
        if (tid == 0) {
          // a tile that hands its pairs over reserves their slots now (one reservation per tile in the sub-list of
          // this workgroup's XCD): the answer is not needed before the next tile's loads have been requested
          if (!last && total != 0u && total <= g.emit_max) slot0 = atomicAdd(g.pair_count + xcd * kSubListStride, total);
          if (total) {
            if (m == 0) atomicAdd(sc + SC_SURVIVORS, (unsigned long long)total);
            if (!last && g.block_stats) atomicAdd(sc + SC_ENTER + m, (unsigned long long)total);
            if (last) atomicAdd(sc + SC_COMPLETED, (unsigned long long)total);
          }
          if (total == 0u || last || total <= g.emit_max)   // the tile ends here
            atomicAdd(sc + SC_DENSE_DIMS, (unsigned long long)(BK * (s + 1)));
          else                                               // the next block of these pairs is done densely
            atomicAdd(sc + SC_DENSE_PB, (unsigned long long)total);
        }
        if (total == 0u) break;
        if (last) {
          fin_mode = 1;
          fin_m = m;
          break;
        }
        if (total <= g.emit_max) {
          fin_mode = 2;
          fin_m = m;
          break;
        }
      }
    }

    // ---- start fetching the next tile before this one is written out
    q = __builtin_amdgcn_readfirstlane(s_q[(tile_no + 1) & 3]);
    const bool more = q < xcount;
    int nrt_ = 0, nct_ = 0;
    if (more) {
      tile_rc(q, nrt_, nct_);
      nrt_ = __builtin_amdgcn_readfirstlane(nrt_);
      nct_ = __builtin_amdgcn_readfirstlane(nct_);
      aim(nrt_ * BM, col_arg(nct_));
      load_norm(0);
      issue(stg, 0);   // both stages are free: every wavefront has passed the barrier of the last multiply step
      load_rows(nrt_ * BM);
    }

    if (fin_mode == 1) {
      // finished distances: offer those below tau_i to the point's packed minimum
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int rl = row_of(a, v);
          unsigned long long key = ~0ull;
#pragma unroll
          for (int b = 0; b < TN; ++b) {
            if ((bits >> ((a * TN + b) * 16 + v)) & 1ull) {
              float dist = s_xn[rl] + fmaf(m2, acc[a][b][v], yn[b]);
              dist = dist > 0.f ? dist : 0.f;
              if (dist < s_tau[par][rl]) {
                const unsigned long long kb = pack_key(dist, gc[b]);
                key = kb < key ? kb : key;
              }
            }
          }
          if (__ballot(key != ~0ull)) {
#pragma unroll
            for (int sh = 1; sh < 32; sh <<= 1) {
              const unsigned long long o = __shfl_xor(key, sh, 64);
              key = o < key ? o : key;
            }
            if (r32 == 0 && key != ~0ull) atomicMin(g.best + g.row_base + row0 + rl, key);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
    } else if (fin_mode == 2) {
      // sparse enough: hand the alive pairs to the gather kernel, which resumes at block fin_m
      if (tid == 0) {
        const unsigned int tot = s_wcnt[fin_m & 1][0] + s_wcnt[fin_m & 1][1] + s_wcnt[fin_m & 1][2] + s_wcnt[fin_m & 1][3];
        unsigned int base = slot0;
        if ((unsigned long long)base + tot > (unsigned long long)g.sub_capacity) {
          atomicOr(g.overflow, 1u);
          base = 0xffffffffu;
        } else {
          base += xcd * g.sub_capacity;
        }
        s_base = base;
      }
      __syncthreads();
      unsigned int run = s_base;
      if (run != 0xffffffffu && wave_alive > 0) {
        for (int w = 0; w < wave; ++w) run += s_wcnt[fin_m & 1][w];
        // A sparse tile holds one or two alive pairs per lane.  Every lane walks its own alive bits; the accumulator
        // element behind a bit is found through LDS, where the lane parks its 32 values of a row block (a register
        // cannot be chosen per lane): the stage the last multiply step read is free, 8 KB per wavefront as [32][64].
        // List slots: the wavefront's range, then lane by lane (prefix sum of the lanes' counts), then bit by bit.
        int upto = __popcll(bits);
        const int mine = upto;
        upto += __builtin_amdgcn_update_dpp(0, upto, 0x111, 0xF, 0xF, false);   // row_shr:1
        upto += __builtin_amdgcn_update_dpp(0, upto, 0x112, 0xF, 0xF, false);   // row_shr:2
        upto += __builtin_amdgcn_update_dpp(0, upto, 0x114, 0xF, 0xF, false);   // row_shr:4
        upto += __builtin_amdgcn_update_dpp(0, upto, 0x118, 0xF, 0xF, false);   // row_shr:8
        upto += __builtin_amdgcn_update_dpp(0, upto, 0x142, 0xA, 0xF, false);   // row_bcast:15
        upto += __builtin_amdgcn_update_dpp(0, upto, 0x143, 0xC, 0xF, false);   // row_bcast:31
        unsigned int pos = run + (unsigned int)(upto - mine);
        float *park = reinterpret_cast<float *>(smem + (stg ^ 1) * STAGE_WORDS + wave * (32 * 64)) + lane;
        const int irow = wm * WTM + 4 * kh;   // + a * 32 + 8 * (v >> 2) + (v & 3)
#pragma unroll
        for (int a = 0; a < TM; ++a) {
#pragma unroll
          for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) park[(b * 16 + v) * 64] = acc[a][b][v];
          unsigned int left = (unsigned int)(bits >> (32 * a));
          while (left) {
            const int e = __builtin_ctz(left);   // b * 16 + v
            left &= left - 1u;
            const int v = e & 15, b = e >> 4;
            const int rl = irow + a * 32 + 8 * (v >> 2) + (v & 3);
            Pair pr;
            pr.i = (int32_t)g.row_base + row0 + rl;
            pr.j = (int32_t)((uint32_t)gc[b ? 1 : 0] | ((uint32_t)fin_m << 24));
            const float p = s_xn[rl] + fmaf(m2, park[e * 64], b ? yn[1] : yn[0]);
            pr.p = p > 0.f ? p : 0.f;
            pr.tau = s_tau[par][rl];
            g.pairs[pos++] = pr;
          }
        }
      }
    }

    if (!more) break;
    rt = nrt_;
    ct = nct_;
    if (tid == 0) s_q[(tile_no + 2) & 3] = (int)drawn;
    commit(col_arg(ct), par ^ 1);   // its barrier also ends this tile: everyone is done with the tile's LDS
  }
}

hipError_t launch_progressive(const ProgArgs &g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.ds % 16 != 0 || g.dprime % 16 != 0 || g.dprime < 16 || g.dprime > g.ds || g.lda != g.ds + 32 || g.ldb != g.ds + 32 ||
      g.nb > kMaxBlocks || (reinterpret_cast<uintptr_t>(g.A) & 15u) || (reinterpret_cast<uintptr_t>(g.B) & 15u) ||
      g.N > (1 << 24))
    return hipErrorInvalidValue;
  constexpr size_t smem = (size_t)2 * STAGE_WORDS * sizeof(uint32_t);
  // once per process (the initialisation of a function-local static is synchronised between threads): the kernel's LDS
  // size, and two workgroups per CU (LDS and registers allow no more)
  struct Setup {
    hipError_t rc;
    int wgs = 0;
    Setup() {
      rc = hipFuncSetAttribute(reinterpret_cast<const void *>(progressive_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      if (rc == hipSuccess)
        rc = hipFuncSetAttribute(reinterpret_cast<const void *>(progressive_kernel<true>),
                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
      int dev = 0, cus = 256;
      (void)hipGetDevice(&dev);
      (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
      wgs = 2 * cus;
    }
  };
  static const Setup setup;
  if (setup.rc != hipSuccess) return setup.rc;
  const int wgs = setup.wgs;
  if ((g.col_list != nullptr) != (g.tile_rt != nullptr) || (g.col_list != nullptr) != (g.ntiles != nullptr))
    return hipErrorInvalidValue;
  const int64_t ntiles = (int64_t)((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (ntiles > 0x7fffffffLL) return hipErrorInvalidValue;
  const int64_t grid = std::max<int64_t>(8, std::min<int64_t>(wgs, (ntiles + 7) / 8 * 8));
  if (g.col_list)
    hipLaunchKernelGGL(progressive_kernel<true>, dim3((unsigned)grid), dim3(NT), smem, st, g);
  else
    hipLaunchKernelGGL(progressive_kernel<false>, dim3((unsigned)grid), dim3(NT), smem, st, g);
  return hipGetLastError();
}

int64_t progressive_tiles(int64_t rows, int32_t k) { return ((rows + BM - 1) / BM) * (int64_t)((k + BN - 1) / BN); }
int32_t progressive_tile_pairs() { return BM * BN; }
int32_t progressive_tile_cols() { return BN; }

}  // namespace skm
