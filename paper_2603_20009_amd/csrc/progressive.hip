// Progressive-pruning GEMM (Algorithm 1, iterations >= 2; Section 3.4 "Progressive Pruning").
//
// The paper multiplies only the first d' dimensions densely and finishes survivors one by one.
// On MI355X a 64-dimension step of a dense 128 x 128 tile on the fp32 matrix cores costs about as
// much as gathering the same step for 2 % of the tile's pairs, so this kernel keeps multiplying a
// tile densely, 64 dimensions at a time, while more than a small share of its pairs is alive, and
// hands the pairs over to the gather kernel (prune.hip) only once the tile is sparse.  The tests are
// the paper's: after t = d', d'+64, d'+128, ... dimensions a pair is dropped when its partial squared
// distance exceeds theta(t, tau_i); a pair that reaches t = d is offered to the point's packed
// (distance, centroid) minimum if it beats tau_i.
//
// Partial distances come from the norm expansion ||x_t||^2 + ||y_t||^2 - 2 x_t.y_t (Section 3.1).
// The prefix norms at the checkpoints are inputs (xnp, ynp): passes that read every point and every
// centroid anyway write them, so that this kernel, whose vector unit is the busy one, only
// fetches one number per row and column and checkpoint.
//
// The kernel is persistent: two workgroups per CU take tiles from a per-XCD counter.  When a tile
// ends, the first slab and the per-row data of the next tile are already being fetched while the
// finished tile is written out, so the short tiles of a well-pruned step do not drain the pipeline.
#include "skm_internal.h"

#include <algorithm>
#include <cstdlib>
#include <type_traits>

namespace skm {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

namespace {
constexpr int BM = 128, BN = 128, BK = 32;
constexpr int WTM = 64, WTN = 64, TM = 2, TN = 2;
constexpr int NT = 256;
constexpr int LS = BK + 4;
constexpr int F4_ROW = BK / 4;              // 8 lanes stage one tile row
constexpr int ROWS_PASS = NT / F4_ROW;      // 32 tile rows per staging pass
constexpr int A_F4 = BM / ROWS_PASS;        // 4
constexpr int B_F4 = BN / ROWS_PASS;        // 4

// Sum / bitwise OR over the 64 lanes of a wavefront through the data-parallel lane moves: within quads, mirrored
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
__device__ inline int wave_or_i32(int v) {
  SKM_WAVE_REDUCE(v, |);
  return __builtin_amdgcn_readlane(v, 63);
}

}  // namespace

// Slabs of BK dimensions start at koff = -((BK - d' % BK) % BK), so that slab ends fall on every
// checkpoint d' + 64 m; dimensions below 0 or past ds are read as zero.
__global__ void __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(2, 2))) progressive_kernel(ProgArgs g) {
  extern __shared__ __align__(16) float smem[];
  float *As = smem;                  // [2][BM][LS]
  float *Bs = smem + 2 * BM * LS;    // [2][BN][LS]
  __shared__ __align__(16) float s_tau[BM], s_thr[BM], s_xn[BM], s_yn[BN];
  __shared__ int s_prev[BM];
  __shared__ float s_ratio[kMaxBlocks + 1];
  __shared__ unsigned long long s_dead[NT];   // per thread: accumulator elements that start dead (the incumbent)
  __shared__ unsigned int s_cnt[2];
  __shared__ unsigned int s_wcnt[2][4];   // alive pairs of every wavefront at the last checkpoint (by checkpoint parity)
  __shared__ unsigned int s_base;         // first list slot of a tile that hands its pairs over
  __shared__ int s_q[4];   // ring of tile numbers drawn from the XCD's counter, two tiles ahead of the one in work

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int r32 = lane & 31, kh = lane >> 5;
  const int nrt = (g.M + BM - 1) / BM, nct = (g.N + BN - 1) / BN;
  const int ntiles = nrt * nct;
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
  auto tile_rc = [&](int q, int &rt, int &ct) {   // q-th tile of this XCD -> (row tile, column tile)
    const int logical = xstart + q;
    const int panel_sz = PC * nrt;
    const int p = logical / panel_sz;
    const int r = logical - p * panel_sz;
    const int pc = (nct - p * PC) < PC ? (nct - p * PC) : PC;
    rt = r / pc;
    ct = p * PC + (r - rt * pc);
  };

  unsigned long long *sc = g.scal + (size_t)(blockIdx.x & (kStatReplicas - 1)) * SC_COUNT;
  for (int m = tid; m <= g.nb; m += NT) s_ratio[m] = g.ratio[m];
  if (tid < 2) s_cnt[tid] = 0u;
  s_dead[tid] = 0ull;

  // staging: thread (st_row, st_kq) moves dims 4 st_kq .. + 3 of tile rows st_row + 32 s.  The 8-lane groups of a
  // wavefront take rows 4 apart (group bits 0-1 and 2-3 swapped): with a row stride of 36 words the rows written by
  // 32 lanes then start 16 banks apart and their 8-byte LDS writes do not collide.
  const int grp = tid / F4_ROW, st_kq = tid % F4_ROW;
  const int st_row = (grp & 16) | ((grp & 3) << 2) | ((grp >> 2) & 3);
  const int koff = -((BK - g.dprime % BK) % BK);
  const int nslab = (g.ds - koff + BK - 1) / BK;

  // Global loads are unconditional: rows past the end are clamped to the last row (their accumulator elements start
  // dead), dimensions outside [0, ds) are clamped into the row and multiplied by zero when staged.  With nothing
  // conditional around them the compiler can keep the loads of a whole slab in flight across a multiply step.
  float4 ra[A_F4], rb[B_F4];
  float tau_reg = 0.f;
  int prev_reg = -1;
  const float *baseA = g.A, *baseB = g.B;   // first row / column of the tile being loaded (uniform)
  int limA = 0, limB = 0;                   // last valid row / column of that tile, relative to its first (uniform)
  // prefix norms: threads 0..127 fetch those of the tile's rows, threads 128..255 those of its columns
  const float *npre = g.xnp;                // &norm[0][this thread's row or column]
  const int64_t npre_stride = tid < BM ? g.xn_stride : (int64_t)g.N;
  float nreg = 0.f;
  auto aim = [&](int row0, int col0) {
    baseA = g.A + (int64_t)row0 * g.lda;
    baseB = g.B + (int64_t)col0 * g.ldb;
    limA = g.M - 1 - row0;
    limB = g.N - 1 - col0;
    npre = tid < BM ? g.xnp + g.row_base + row0 + min(tid, limA) : g.ynp + col0 + min(tid - BM, limB);
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
  auto kclamp = [&](int k0) { return (unsigned int)min(max(k0 + 4 * st_kq, 0), g.ds - 4); };
  auto klive = [&](int k0) { return k0 + 4 * st_kq >= 0 && k0 + 4 * st_kq < g.ds; };
  auto load_a = [&](int j, unsigned int kk) {
    const unsigned int off = (unsigned int)(min(st_row + ROWS_PASS * j, limA) * (int)g.lda) + kk;
    ra[j] = *reinterpret_cast<const float4 *>(baseA + off);
  };
  auto load_b = [&](int j, unsigned int kk) {
    const unsigned int off = (unsigned int)(min(st_row + ROWS_PASS * j, limB) * (int)g.ldb) + kk;
    rb[j] = *reinterpret_cast<const float4 *>(baseB + off);
  };
  auto gload = [&](int k0) {
    const unsigned int kk = kclamp(k0);
#pragma unroll
    for (int j = 0; j < A_F4; ++j) load_a(j, kk);
#pragma unroll
    for (int j = 0; j < B_F4; ++j) load_b(j, kk);
  };
  auto load_rows = [&](int row0) {   // per-row data of a tile, one row per thread of the first two wavefronts
    if (tid < BM) {
      const int gr = min(row0 + tid, g.M - 1);
      tau_reg = g.tau[g.row_base + gr];
      prev_reg = row0 + tid < g.M ? g.prev[g.row_base + gr] : -1;
    }
  };
  // Split-fp16 staging (see skm_internal.h): a scaled value v goes to LDS as hi = fp16(v) and lo = fp16(v - hi);
  // a tile row of a slab holds its 32 hi values (64 bytes), its 32 lo values, and 16 bytes of padding.
  const unsigned int amax = *g.a_absmax, bmax = *g.b_absmax;
  const float scale_a = split_scale(amax), scale_b = split_scale(bmax);
  const float m2 = -2.f * split_unscale(amax) * split_unscale(bmax);   // accumulator -> -2 x.y
  auto split_store = [&](float *dst_row, const float4 &v, float scale) {
    const f32x2 p0 = {v.x * scale, v.y * scale}, p1 = {v.z * scale, v.w * scale};
    const f16x2 h0 = __builtin_convertvector(p0, f16x2), h1 = __builtin_convertvector(p1, f16x2);
    const f16x2 l0 = __builtin_convertvector(p0 - __builtin_convertvector(h0, f32x2), f16x2);
    const f16x2 l1 = __builtin_convertvector(p1 - __builtin_convertvector(h1, f32x2), f16x2);
    uint2 hi, lo;
    hi.x = __builtin_bit_cast(unsigned int, h0); hi.y = __builtin_bit_cast(unsigned int, h1);
    lo.x = __builtin_bit_cast(unsigned int, l0); lo.y = __builtin_bit_cast(unsigned int, l1);
    *reinterpret_cast<uint2 *>(dst_row + 2 * st_kq) = hi;
    *reinterpret_cast<uint2 *>(dst_row + 16 + 2 * st_kq) = lo;
  };
  // float4 j of the staged slab -> LDS buffer `buf`, then the same registers are aimed at the slab after it (element
  // offset kk2), so that one register set carries two slabs: one being used, one in flight
  auto stage_a = [&](int j, int buf, float fa, unsigned int kk2) {
    split_store(As + (buf * BM + st_row + ROWS_PASS * j) * LS, ra[j], fa);
    load_a(j, kk2);
  };
  auto stage_b = [&](int j, int buf, float fb, unsigned int kk2) {
    split_store(Bs + (buf * BN + st_row + ROWS_PASS * j) * LS, rb[j], fb);
    load_b(j, kk2);
  };
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
  int q = s_q[0];
  if (q >= xcount) return;
  int rt, ct;
  tile_rc(q, rt, ct);
  rt = __builtin_amdgcn_readfirstlane(rt);
  ct = __builtin_amdgcn_readfirstlane(ct);
  aim(rt * BM, ct * BN);
  load_norm(0);
  gload(koff);
  load_rows(rt * BM);

  for (int tile_no = 0;; ++tile_no) {
    const int row0 = rt * BM, col0 = ct * BN;
    // ---- commit the prefetched first slab and per-row data of this tile
    {
      // slab 0 of this tile arrived while the previous tile was written out; slab 1 is requested as slab 0 is staged
      const bool live0 = klive(koff);
      const unsigned int kk1 = kclamp(koff + BK);
#pragma unroll
      for (int j = 0; j < A_F4; ++j) stage_a(j, 0, live0 ? scale_a : 0.f, kk1);
#pragma unroll
      for (int j = 0; j < B_F4; ++j) stage_b(j, 0, live0 ? scale_b : 0.f, kk1);
    }
    if (tid < BM) {
      s_tau[tid] = tau_reg;
      s_prev[tid] = prev_reg;
      // the incumbent of this row, if it is a column of this tile, starts dead: find the thread and the
      // accumulator element that hold (row tid, column prev - col0)
      const int cl = prev_reg - col0;
      if (cl >= 0 && cl < BN) {
        const int rr = tid & 31;
        const int lane_t = ((rr >> 2) & 1) * 32 + (cl & 31);
        const int wave_t = (tid >> 6) * 2 + (cl >> 6);
        const int v_t = 4 * (rr >> 3) + (rr & 3);
        const int bit = ((((tid & 63) >> 5) * TN) + ((cl & 63) >> 5)) * 16 + v_t;
        atomicOr(&s_dead[wave_t * 64 + lane_t], 1ull << bit);
      }
    }
    // Draw the number of the tile after next now; the answer of the counter is stored at the end of this tile, so
    // its round trip never stalls the workgroup.
    unsigned int drawn = 0;
    if (tid == 0) drawn = atomicAdd(ctr, 1u);
    __syncthreads();
    // The alive counter of checkpoint 0 may still hold the last total of the previous tile (a tile that ends at an
    // even checkpoint leaves it behind).  Every thread has read that total before the barrier above, and the first
    // add of this tile comes after the barrier of its first slab.
    if (tid == 0) s_cnt[0] = 0u;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;
    int gc[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) gc[b] = col0 + wn * WTN + b * 32 + r32;

    // one alive-bit per accumulator element
    unsigned long long bits = ~s_dead[tid];
    s_dead[tid] = 0ull;
    if (row0 + BM > g.M || col0 + BN > g.N) {   // ragged edge tile: rows / columns past the end start dead
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
    // matrix instructions between which the next slab is converted and the one after it requested.
    f16x8 ah[TM], al[TM], bh[TN], bl[TN];
    auto frag = [&](const float *base, int h, int lo, int t) {
      return *reinterpret_cast<const f16x8 *>(base + t * 32 * LS + kh * 4 + h * 8 + lo * 16);
    };
    auto mma4 = [&](const f16x8 (&x)[TM], const f16x8 (&y)[TN]) {
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x[a], y[b], acc[a][b], 0, 0, 0);
    };
    auto mix = [&](auto valu_per_mfma) {   // spread `valu` vector instructions behind each of the four matrix ones
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, decltype(valu_per_mfma)::value, 0);
      }
    };
    for (int s = 0; s < nslab; ++s) {
      const int buf = s & 1;
      const int tdone = koff + BK * (s + 1);   // dimensions multiplied after this step
      const bool last = (s + 1 == nslab);
      const bool check = !last && tdone >= g.dprime && tdone < g.d && ((tdone - g.dprime) & (kBlockDims - 1)) == 0;
      const bool cp = check || last;
      const int m = last ? g.nb : (tdone - g.dprime) / kBlockDims;   // checkpoint index, t_m = min(d, d' + 64 m)
      // the norms of checkpoint m were requested one step ago (or with the tile's first slab); every step requests
      // those of the step after it, needed or not, so that the request is never behind a branch
      if (cp) publish_norms(s_ratio[m]);
      load_norm(s + 1);
      const float *Ab = As + (buf * BM + wm * WTM + r32) * LS;
      const float *Bb = Bs + (buf * BN + wn * WTN + r32) * LS;
      {
        // (the last step of a tile stages a slab past the end: all zeros, into a buffer nobody reads again)
        const bool live1 = klive(koff + (s + 1) * BK);
        const float fa = live1 ? scale_a : 0.f, fb = live1 ? scale_b : 0.f;
        const unsigned int kk2 = kclamp(koff + (s + 2) * BK);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          ah[t] = frag(Ab, 0, 0, t); bh[t] = frag(Bb, 0, 0, t);
          al[t] = frag(Ab, 0, 1, t); bl[t] = frag(Bb, 0, 1, t);
        }
        __builtin_amdgcn_sched_barrier(0);
        mma4(ah, bh);
        stage_a(0, buf ^ 1, fa, kk2);
        mix(std::integral_constant<int, 6>());
        __builtin_amdgcn_sched_barrier(0);
        mma4(al, bh);
        stage_a(1, buf ^ 1, fa, kk2);
        mix(std::integral_constant<int, 6>());
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 2; ++t) { al[t] = frag(Ab, 1, 1, t); bh[t] = frag(Bb, 1, 0, t); }
        mma4(ah, bl);
        stage_a(2, buf ^ 1, fa, kk2);
        stage_a(3, buf ^ 1, fa, kk2);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
        mix(std::integral_constant<int, 11>());
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 2; ++t) { ah[t] = frag(Ab, 1, 0, t); bl[t] = frag(Bb, 1, 1, t); }
        mma4(al, bh);
        stage_b(0, buf ^ 1, fb, kk2);
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
        mix(std::integral_constant<int, 6>());
        __builtin_amdgcn_sched_barrier(0);
        mma4(ah, bl);
        stage_b(1, buf ^ 1, fb, kk2);
        mix(std::integral_constant<int, 6>());
        __builtin_amdgcn_sched_barrier(0);
        mma4(ah, bh);
        stage_b(2, buf ^ 1, fb, kk2);
        stage_b(3, buf ^ 1, fb, kk2);
        mix(std::integral_constant<int, 11>());
        __builtin_amdgcn_sched_barrier(0);
      }
      __syncthreads();
      if (cp) {
#pragma unroll
        for (int b = 0; b < TN; ++b) yn[b] = s_yn[wn * WTN + b * 32 + r32];
        if (!last || g.nb == 0) {
          // test theta(t_m, tau_i): drop the pair when its partial distance exceeds it
#pragma unroll
          for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const float th = s_thr[row_of(a, v)];
#pragma unroll
              for (int b = 0; b < TN; ++b) {
                const bool keep = fmaf(m2, acc[a][b][v], yn[b]) <= th;
                bits &= ~((unsigned long long)(!keep) << ((a * TN + b) * 16 + v));
              }
            }
        }
        // alive pairs of this wavefront and of the whole tile
        wave_alive = wave_sum_i32(__popcll(bits));
        if (lane == 0) {
          s_wcnt[m & 1][wave] = (unsigned int)wave_alive;
          if (wave_alive) atomicAdd(&s_cnt[m & 1], (unsigned int)wave_alive);
        }
        __syncthreads();
        const unsigned int total = s_cnt[m & 1];
        if (tid == 0) {
          s_cnt[(m + 1) & 1] = 0u;   // next checkpoint's counter; nobody reads it before the next barrier
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
    q = s_q[(tile_no + 1) & 3];
    const bool more = q < xcount;
    int nrt_ = 0, nct_ = 0;
    if (more) {
      tile_rc(q, nrt_, nct_);
      nrt_ = __builtin_amdgcn_readfirstlane(nrt_);
      nct_ = __builtin_amdgcn_readfirstlane(nct_);
      aim(nrt_ * BM, nct_ * BN);
      load_norm(0);
      gload(koff);
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
              if (dist < s_tau[rl]) {
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
          *g.overflow = 1u;
          base = 0xffffffffu;
        } else {
          base += xcd * g.sub_capacity;
        }
        s_base = base;
      }
      // element slots in which any lane of this wavefront holds an alive pair (a sparse tile has few): the others
      // are skipped by a scalar test each
      const unsigned long long any = ((unsigned long long)(unsigned int)wave_or_i32((int)(bits >> 32)) << 32) |
                                     (unsigned long long)(unsigned int)wave_or_i32((int)bits);
      __syncthreads();
      unsigned int run = s_base;
      if (run != 0xffffffffu && wave_alive > 0) {
        for (int w = 0; w < wave; ++w) run += s_wcnt[fin_m & 1][w];
#pragma unroll
        for (int a = 0; a < TM; ++a) {
          // per-row data of the 16 rows this lane holds in accumulator row block a: four aligned groups of four rows
          float4 xn4[4], tau4[4];
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            xn4[q4] = *reinterpret_cast<const float4 *>(&s_xn[wm * WTM + a * 32 + 8 * q4 + 4 * kh]);
            tau4[q4] = *reinterpret_cast<const float4 *>(&s_tau[wm * WTM + a * 32 + 8 * q4 + 4 * kh]);
          }
          auto pick = [](const float4 &f, int i) { return i == 0 ? f.x : i == 1 ? f.y : i == 2 ? f.z : f.w; };
#pragma unroll
          for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              if (!((any >> ((a * TN + b) * 16 + v)) & 1ull)) continue;
              const bool keep = (bits >> ((a * TN + b) * 16 + v)) & 1ull;
              const unsigned long long mk = __ballot(keep);
              if (keep) {
                const unsigned int pos =
                    run + __builtin_amdgcn_mbcnt_hi((unsigned int)(mk >> 32), __builtin_amdgcn_mbcnt_lo((unsigned int)mk, 0u));
                Pair pr;
                pr.i = (int32_t)(g.row_base + row0 + row_of(a, v));
                pr.j = (int32_t)((uint32_t)gc[b] | ((uint32_t)fin_m << 24));
                const float p = pick(xn4[v >> 2], v & 3) + fmaf(m2, acc[a][b][v], yn[b]);
                pr.p = p > 0.f ? p : 0.f;
                pr.tau = pick(tau4[v >> 2], v & 3);
                g.pairs[pos] = pr;
              }
              run += (unsigned int)__popcll(mk);
              __builtin_amdgcn_sched_barrier(0);
            }
        }
      }
    }

    if (!more) break;
    rt = nrt_;
    ct = nct_;
    if (tid == 0) s_q[(tile_no + 2) & 3] = (int)drawn;
    __syncthreads();   // everyone is done with this tile's LDS before the next one is committed
  }
}

hipError_t launch_progressive(const ProgArgs &g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  if (g.ds % 16 != 0 || g.dprime % 16 != 0 || g.dprime < 16 || g.dprime > g.ds || g.lda % 4 != 0 || g.ldb % 4 != 0 ||
      g.nb > kMaxBlocks || (reinterpret_cast<uintptr_t>(g.A) & 15u) || (reinterpret_cast<uintptr_t>(g.B) & 15u) ||
      g.N > (1 << 24))
    return hipErrorInvalidValue;
  constexpr size_t smem = (size_t)2 * (BM + BN) * LS * sizeof(float);
  static int wgs = 0;
  if (!wgs) {
    hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void *>(progressive_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (rc != hipSuccess) return rc;
    int dev = 0, cus = 256;
    (void)hipGetDevice(&dev);
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    wgs = 2 * cus;   // two workgroups per CU (LDS and registers allow no more)
  }
  const int64_t ntiles = (int64_t)((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  if (ntiles > 0x7fffffffLL) return hipErrorInvalidValue;
  const int64_t grid = std::max<int64_t>(8, std::min<int64_t>(wgs, (ntiles + 7) / 8 * 8));
  hipLaunchKernelGGL(progressive_kernel, dim3((unsigned)grid), dim3(NT), smem, st, g);
  return hipGetLastError();
}

int64_t progressive_tiles(int64_t rows, int32_t k) { return ((rows + BM - 1) / BM) * (int64_t)((k + BN - 1) / BN); }
int32_t progressive_tile_pairs() { return BM * BN; }

}  // namespace skm
