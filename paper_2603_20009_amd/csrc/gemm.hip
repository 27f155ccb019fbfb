// MFMA "NT" GEMM for gfx950 with two fused epilogues (store, row argmin).
//
// The GEMM phase of SuperKMeans (Algorithm 1: iteration 1 over all d dimensions, later iterations
// over the first d' dimensions; Section 3.1 for the rotation X R) is a product of two K-contiguous
// row-major matrices.  One workgroup of 256 threads (4 wavefronts, 2 x 2) owns a 128 x 128 tile of
// the score matrix; each wavefront owns 64 x 64 of it as 2 x 2 accumulators of 32 x 32.
// K is consumed in slabs that are staged global -> registers -> LDS (two LDS buffers, one barrier
// per slab) while the previous slab is multiplied.
//
// Two arithmetic forms share the tile shape and the epilogues:
//  - gemm_split_kernel: fp32 operands split into two fp16 numbers each, three v_mfma_f32_32x32x16_f16
//    per product, fp32 accumulation (fp32-class accuracy at a multiple of the fp32 matrix rate).  Used
//    whenever the operands are 16-byte aligned, K >= 32 and the caller supplies magnitude bounds.
//  - gemm_kernel: plain v_mfma_f32_32x32x2_f32, for unaligned operands and K = 16.
//
// The score matrix is never written for the distance use of iteration 1: the epilogue reduces it to
// a row argmin.  Iterations >= 2 use the progressive kernel of progressive.hip, built on the same tile.
#include "skm_internal.h"

#include <algorithm>
#include <atomic>
#include <cstdlib>
#include <type_traits>

namespace skm {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int BM = 128, BN = 128;  // workgroup tile
constexpr int WTM = 64, WTN = 64;  // wavefront tile
constexpr int TM = 2, TN = 2;      // 32 x 32 MFMA tiles per wavefront
constexpr int NTHREADS = 256;

enum { EPI_STORE = 0, EPI_ARGMIN = 1 };

struct StoreArgs {
  float *C;
  int64_t ldc;
  int32_t Nstore;
  float alpha, beta;
  unsigned int *c_absmax;   // optional: max |C| is folded into it
};
struct ArgminArgs {
  const float *ynorm;
  unsigned long long *best;
};

template <int EPI>
struct EpiArgs;
template <>
struct EpiArgs<EPI_STORE> {
  typedef StoreArgs type;
};
template <>
struct EpiArgs<EPI_ARGMIN> {
  typedef ArgminArgs type;
};

// Workgroups are dispatched round-robin over the 8 XCDs (each with its own L2).  Give every XCD a
// contiguous range of logical tile ids, and walk the tiles in panels of PC column tiles with the
// row tile advancing slowest inside a panel, so that the workgroups resident on one XCD share a
// few row tiles of A and one panel of B.
__device__ inline void tile_of_block(int nrt, int nct, int PC, int &rt, int &ct) {
  const int nwg = gridDim.x;
  const int bid = blockIdx.x;
  const int xcd = bid & 7, q = bid >> 3;
  const int base = nwg >> 3, rem = nwg & 7;
  const int logical = xcd * base + (xcd < rem ? xcd : rem) + q;
  const int panel_sz = PC * nrt;
  const int p = logical / panel_sz;
  const int r = logical - p * panel_sz;
  const int pc = (nct - p * PC) < PC ? (nct - p * PC) : PC;
  rt = r / pc;
  ct = p * PC + (r - rt * pc);
}

// Epilogues of a finished TB x TB tile (TB / 64 wavefronts each way).  `unscale` turns an accumulator into the
// score s(i, j).  Accumulator layout of the 32 x 32 MFMA results: register v of lane (r32, kh) holds
// row 8*(v/4) + 4*kh + (v%4), column r32 of the 32 x 32 tile.
template <int EPI, int TB = BM>
__device__ inline void tile_epilogue(f32x16 (&acc)[TM][TN], const GemmOperands &g, const typename EpiArgs<EPI>::type &e,
                                     int row0, int col0, float unscale, float *smem) {
  constexpr int NWN = TB / WTN;
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave / NWN, wn = wave % NWN;
  const int r32 = lane & 31, kh = lane >> 5;
  auto row_of = [&](int a, int v) { return wm * WTM + a * 32 + 8 * (v >> 2) + 4 * kh + (v & 3); };

  if constexpr (EPI == EPI_STORE) {
    const float alpha = e.alpha * unscale;
    float vmax = 0.f;
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int gr = row0 + row_of(a, v);
        if (gr >= g.M) continue;
#pragma unroll
        for (int b = 0; b < TN; ++b) {
          const int gc = col0 + wn * WTN + b * 32 + r32;
          if (gc >= e.Nstore) continue;
          float *dst = e.C + (int64_t)gr * e.ldc + gc;
          float val = 0.f;
          if (gc < g.N) {
            val = alpha * acc[a][b][v];
            if (e.beta != 0.f) val += e.beta * *dst;
            vmax = fmaxf(vmax, fabsf(val));
          }
          *dst = val;
        }
      }
    if (e.c_absmax) {
#pragma unroll
      for (int m = 1; m < 64; m <<= 1) vmax = fmaxf(vmax, __shfl_xor(vmax, m, 64));
      if (lane == 0 && vmax > 0.f) atomicMax(e.c_absmax, __builtin_bit_cast(unsigned int, vmax));
    }
  } else if constexpr (EPI == EPI_ARGMIN) {
    // per-row minimum of ynorm[j] - 2 s(i,j): lanes of one half share the rows, columns differ
    unsigned long long *red = reinterpret_cast<unsigned long long *>(smem);  // [NWN][TB], reuses the tile buffers
    const float m2 = -2.f * unscale;
    float yn[TN];
    int gc[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      gc[b] = col0 + wn * WTN + b * 32 + r32;
      yn[b] = gc[b] < g.N ? e.ynorm[gc[b]] : 0.f;
    }
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        unsigned long long key = ~0ull;
#pragma unroll
        for (int b = 0; b < TN; ++b) {
          if (gc[b] < g.N) {
            const unsigned long long kb = pack_key(fmaf(m2, acc[a][b][v], yn[b]), gc[b]);
            key = kb < key ? kb : key;
          }
        }
#pragma unroll
        for (int m = 1; m < 32; m <<= 1) {
          const unsigned long long o = __shfl_xor(key, m, 64);
          key = o < key ? o : key;
        }
        if (r32 == 0) red[wn * TB + row_of(a, v)] = key;
      }
    __syncthreads();
    if (tid < TB) {
      unsigned long long key = red[tid];
#pragma unroll
      for (int w = 1; w < NWN; ++w) {
        const unsigned long long o = red[w * TB + tid];
        key = o < key ? o : key;
      }
      const int gr = row0 + tid;
      // The minimum only goes down, so a key that does not beat what is there now never will: most tiles after the
      // first few column tiles of a row are settled by this plain read instead of an atomic.
      if (gr < g.M && key != ~0ull && key < __atomic_load_n(e.best + gr, __ATOMIC_RELAXED)) atomicMin(e.best + gr, key);
    }
  }
}

template <int BK, int EPI, bool ALIGNED>
__global__ void __launch_bounds__(NTHREADS) gemm_kernel(GemmOperands g, typename EpiArgs<EPI>::type e) {
  constexpr int LS = BK + 4;                       // LDS row stride in floats (16-byte aligned, conflict-free b128 reads)
  constexpr int F4_ROW = BK / 4;                   // float4 per tile row
  constexpr int A_F4 = BM * F4_ROW / NTHREADS;     // float4 staged per thread for A
  constexpr int B_F4 = BN * F4_ROW / NTHREADS;
  extern __shared__ __align__(16) float smem[];
  float *As = smem;                                // [2][BM][LS]
  float *Bs = smem + 2 * BM * LS;                  // [2][BN][LS]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int r32 = lane & 31, kh = lane >> 5;

  const int nrt = (g.M + BM - 1) / BM, nct = (g.N + BN - 1) / BN;
  int rt, ct;
  tile_of_block(nrt, nct, g.panel_cols, rt, ct);
  const int row0 = rt * BM, col0 = ct * BN;

  float4 ra[A_F4], rb[B_F4];
  auto gload = [&](int k0) {
#pragma unroll
    for (int s = 0; s < A_F4; ++s) {
      const int f = tid + s * NTHREADS;
      const int row = f / F4_ROW, kk = k0 + 4 * (f % F4_ROW);
      const int gr = row0 + row;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (gr < g.M) {
        const float *src = g.A + (int64_t)gr * g.lda + kk;
        if (ALIGNED) {
          if (kk < g.K) v = *reinterpret_cast<const float4 *>(src);
        } else {
          if (kk + 0 < g.K) v.x = src[0];
          if (kk + 1 < g.K) v.y = src[1];
          if (kk + 2 < g.K) v.z = src[2];
          if (kk + 3 < g.K) v.w = src[3];
        }
      }
      ra[s] = v;
    }
#pragma unroll
    for (int s = 0; s < B_F4; ++s) {
      const int f = tid + s * NTHREADS;
      const int row = f / F4_ROW, kk = k0 + 4 * (f % F4_ROW);
      const int gr = col0 + row;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (gr < g.N) {
        const float *src = g.B + (int64_t)gr * g.ldb + kk;
        if (ALIGNED) {
          if (kk < g.K) v = *reinterpret_cast<const float4 *>(src);
        } else {
          if (kk + 0 < g.K) v.x = src[0];
          if (kk + 1 < g.K) v.y = src[1];
          if (kk + 2 < g.K) v.z = src[2];
          if (kk + 3 < g.K) v.w = src[3];
        }
      }
      rb[s] = v;
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int s = 0; s < A_F4; ++s) {
      const int f = tid + s * NTHREADS;
      const int row = f / F4_ROW, kq = f % F4_ROW;
      *reinterpret_cast<float4 *>(As + (buf * BM + row) * LS + 4 * kq) = ra[s];
    }
#pragma unroll
    for (int s = 0; s < B_F4; ++s) {
      const int f = tid + s * NTHREADS;
      const int row = f / F4_ROW, kq = f % F4_ROW;
      *reinterpret_cast<float4 *>(Bs + (buf * BN + row) * LS + 4 * kq) = rb[s];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  const int nslab = (g.K + BK - 1) / BK;
  gload(0);
  sstore(0);
  __syncthreads();
  for (int s = 0; s < nslab; ++s) {
    const int buf = s & 1;
    if (s + 1 < nslab) gload((s + 1) * BK);
    const float *Ab = As + (buf * BM + wm * WTM + r32) * LS + kh * 4;
    const float *Bb = Bs + (buf * BN + wn * WTN + r32) * LS + kh * 4;
#pragma unroll
    for (int kg = 0; kg < BK / 8; ++kg) {
      float4 af[TM], bf[TN];
#pragma unroll
      for (int a = 0; a < TM; ++a) af[a] = *reinterpret_cast<const float4 *>(Ab + a * 32 * LS + kg * 8);
#pragma unroll
      for (int b = 0; b < TN; ++b) bf[b] = *reinterpret_cast<const float4 *>(Bb + b * 32 * LS + kg * 8);
      // the 8 k-values of this group are consumed as 4 MFMA steps; lane half kh supplies k = 4*kh + step
      // for both operands, which is a consistent permutation of the summation index.
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a].x, bf[b].x, acc[a][b], 0, 0, 0);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a].y, bf[b].y, acc[a][b], 0, 0, 0);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a].z, bf[b].z, acc[a][b], 0, 0, 0);
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[a].w, bf[b].w, acc[a][b], 0, 0, 0);
    }
    if (s + 1 < nslab) sstore(buf ^ 1);
    __syncthreads();
  }

  tile_epilogue<EPI>(acc, g, e, row0, col0, 1.f, smem);
}

// ---------------------------------------------------------------- split-fp16 form
// Same tile and wavefront layout, but every operand value is scaled and staged as two fp16 numbers hi and lo
// (see skm_internal.h) and a product is taken as lo*hi' + hi*lo' + hi*hi' on v_mfma_f32_32x32x16_f16: three
// matrix instructions of a quarter of the issue time replace eight fp32 ones.  A tile row of a slab of 32 dims
// holds its 32 hi values (64 bytes), then its 32 lo values, then 16 bytes of padding: the fp32 stride.
//
// With the matrix work five times shorter, staging decides the speed, so the loop is software pipelined by
// hand.  Global loads are unconditional (rows and the K tail are clamped to valid addresses; a clamped tail
// is multiplied by a zero scale, clamped rows only feed accumulators that are never stored), which lets the
// compiler keep the loads of two slabs in flight and count them.  While slab s is multiplied from one LDS
// buffer, slab s + 1 (requested one step earlier) is converted and written to the other buffer between the
// matrix instructions, and slab s + 2 is requested.
constexpr int SBK = 32, SLS = SBK + 4;
constexpr int S_F4 = BM * (SBK / 4) / NTHREADS;   // float4 staged per thread and operand: 4

template <int EPI>
__global__ void __launch_bounds__(NTHREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
gemm_split_kernel(GemmOperands g, typename EpiArgs<EPI>::type e) {
  extern __shared__ __align__(16) float smem[];
  float *As = smem;                    // [2][BM][SLS]
  float *Bs = smem + 2 * BM * SLS;     // [2][BN][SLS]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int r32 = lane & 31, kh = lane >> 5;

  const int nrt = (g.M + BM - 1) / BM, nct = (g.N + BN - 1) / BN;
  int rt, ct;
  tile_of_block(nrt, nct, g.panel_cols, rt, ct);
  const int row0 = rt * BM, col0 = ct * BN;

  const unsigned int ma = *g.a_absmax, mb = *g.b_absmax;
  const float scale_a = split_scale(ma), scale_b = split_scale(mb);
  const float unscale = split_unscale(ma) * split_unscale(mb);

  // staging: thread (st_row, kq) moves dims 4 kq .. 4 kq + 3 of tile rows st_row + 32 s.  The 8-lane groups of
  // a wavefront take rows 4 apart (group bits 0-1 and 2-3 swapped): with a row stride of 36 words the four rows
  // written by 32 lanes then start 16 banks apart and their 8-byte writes do not collide.
  const int grp = tid >> 3, kq = tid & 7;
  const int st_row = (grp & 16) | ((grp & 3) << 2) | ((grp >> 2) & 3);
  const float *pa[S_F4], *pb[S_F4];
#pragma unroll
  for (int s = 0; s < S_F4; ++s) {
    const int gr = min(row0 + st_row + 32 * s, g.M - 1);
    const int gc = min(col0 + st_row + 32 * s, g.N - 1);
    pa[s] = g.A + (int64_t)gr * g.lda;
    pb[s] = g.B + (int64_t)gc * g.ldb;
  }
  auto gload = [&](int k0, float4 *ra, float4 *rb) {
    const int kk = min(k0 + 4 * kq, g.K - 4);
#pragma unroll
    for (int s = 0; s < S_F4; ++s) ra[s] = *reinterpret_cast<const float4 *>(pa[s] + kk);
#pragma unroll
    for (int s = 0; s < S_F4; ++s) rb[s] = *reinterpret_cast<const float4 *>(pb[s] + kk);
  };
  auto split_store = [&](float *dst_row, const float4 &v, float scale) {
    const f32x2 p0 = {v.x * scale, v.y * scale}, p1 = {v.z * scale, v.w * scale};
    const f16x2 h0 = __builtin_convertvector(p0, f16x2), h1 = __builtin_convertvector(p1, f16x2);
    const f16x2 l0 = __builtin_convertvector(p0 - __builtin_convertvector(h0, f32x2), f16x2);
    const f16x2 l1 = __builtin_convertvector(p1 - __builtin_convertvector(h1, f32x2), f16x2);
    uint2 hi, lo;
    hi.x = __builtin_bit_cast(unsigned int, h0); hi.y = __builtin_bit_cast(unsigned int, h1);
    lo.x = __builtin_bit_cast(unsigned int, l0); lo.y = __builtin_bit_cast(unsigned int, l1);
    *reinterpret_cast<uint2 *>(dst_row + 2 * kq) = hi;
    *reinterpret_cast<uint2 *>(dst_row + 16 + 2 * kq) = lo;
  };
  auto store_slab = [&](int buf, int k0, const float4 *ra, const float4 *rb) {   // unpipelined (prologue)
    const bool live = k0 + 4 * kq < g.K;
#pragma unroll
    for (int s = 0; s < S_F4; ++s) {
      split_store(As + (buf * BM + st_row + 32 * s) * SLS, ra[s], live ? scale_a : 0.f);
      split_store(Bs + (buf * BN + st_row + 32 * s) * SLS, rb[s], live ? scale_b : 0.f);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  // Fragments of half a slab (16 dims): lane half kh supplies the 8 consecutive dims 16 h + 8 kh .. + 7 of both
  // operands.  Products are taken in three groups of four matrix instructions, hi*hi', lo*hi', hi*lo'.
  f16x8 ah[TM], al[TM], bh[TN], bl[TN];
  auto frag = [&](const float *base, int h, int lo, int t) {
    return *reinterpret_cast<const f16x8 *>(base + t * 32 * SLS + kh * 4 + h * 8 + lo * 16);
  };
  auto mma4 = [&](const f16x8 (&x)[TM], const f16x8 (&y)[TN]) {
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x[a], y[b], acc[a][b], 0, 0, 0);
  };
  // interleave the four matrix instructions of a group with `valu` vector instructions each
  auto mix = [&](auto valu_per_mfma) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, decltype(valu_per_mfma)::value, 0);
    }
  };
  auto multiply_only = [&](int buf) {
    const float *Ab = As + (buf * BM + wm * WTM + r32) * SLS;
    const float *Bb = Bs + (buf * BN + wn * WTN + r32) * SLS;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        ah[t] = frag(Ab, h, 0, t); al[t] = frag(Ab, h, 1, t);
        bh[t] = frag(Bb, h, 0, t); bl[t] = frag(Bb, h, 1, t);
      }
      mma4(ah, bh);
      mma4(al, bh);
      mma4(ah, bl);
    }
  };
  // One pipelined step: request slab k_load into (la, lb), multiply LDS buffer `buf`, and between the matrix
  // instructions convert the slab k_store held in (sa, sb) into the other buffer.  The fragments of the second
  // half are fetched into registers as the first half releases them, two groups before their first use.
  auto step = [&](int buf, int k_store, const float4 *sa, const float4 *sb, int k_load, float4 *la, float4 *lb) {
    const float *Ab = As + (buf * BM + wm * WTM + r32) * SLS;
    const float *Bb = Bs + (buf * BN + wn * WTN + r32) * SLS;
    float *Aw = As + ((buf ^ 1) * BM + st_row) * SLS;
    float *Bw = Bs + ((buf ^ 1) * BN + st_row) * SLS;
    const bool live = k_store + 4 * kq < g.K;
    const float fa = live ? scale_a : 0.f, fb = live ? scale_b : 0.f;
    __builtin_amdgcn_sched_barrier(0);
    gload(k_load, la, lb);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      ah[t] = frag(Ab, 0, 0, t); bh[t] = frag(Bb, 0, 0, t);
      al[t] = frag(Ab, 0, 1, t); bl[t] = frag(Bb, 0, 1, t);
    }
    __builtin_amdgcn_sched_barrier(0);
    mma4(ah, bh);
    split_store(Aw, sa[0], fa);
    split_store(Aw + 32 * SLS, sa[1], fa);
    mix(std::integral_constant<int, 6>());
    __builtin_amdgcn_sched_barrier(0);
    mma4(al, bh);
    split_store(Aw + 64 * SLS, sa[2], fa);
    mix(std::integral_constant<int, 3>());
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 2; ++t) { al[t] = frag(Ab, 1, 1, t); bh[t] = frag(Bb, 1, 0, t); }
    mma4(ah, bl);
    split_store(Aw + 96 * SLS, sa[3], fa);
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    mix(std::integral_constant<int, 3>());
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 2; ++t) { ah[t] = frag(Ab, 1, 0, t); bl[t] = frag(Bb, 1, 1, t); }
    mma4(al, bh);
    split_store(Bw, sb[0], fb);
    split_store(Bw + 32 * SLS, sb[1], fb);
    __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
    mix(std::integral_constant<int, 6>());
    __builtin_amdgcn_sched_barrier(0);
    mma4(ah, bl);
    split_store(Bw + 64 * SLS, sb[2], fb);
    mix(std::integral_constant<int, 3>());
    __builtin_amdgcn_sched_barrier(0);
    mma4(ah, bh);
    split_store(Bw + 96 * SLS, sb[3], fb);
    mix(std::integral_constant<int, 3>());
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
  };

  const int nslab = (g.K + SBK - 1) / SBK;
  float4 ra0[S_F4], rb0[S_F4], ra1[S_F4], rb1[S_F4];
  gload(0, ra0, rb0);
  store_slab(0, 0, ra0, rb0);
  gload(SBK, ra0, rb0);
  __syncthreads();
  // At the top of an even step LDS buffer 0 holds slab s and set 0 holds slab s + 1, in flight.
  int s = 0;
  for (; s + 2 < nslab; s += 2) {
    step(0, (s + 1) * SBK, ra0, rb0, (s + 2) * SBK, ra1, rb1);
    step(1, (s + 2) * SBK, ra1, rb1, (s + 3) * SBK, ra0, rb0);
  }
  if (s + 2 == nslab) {
    step(0, (s + 1) * SBK, ra0, rb0, (s + 2) * SBK, ra1, rb1);
    multiply_only(1);
  } else {
    multiply_only(0);
  }
  __syncthreads();
  tile_epilogue<EPI>(acc, g, e, row0, col0, unscale, smem);
}


// ---------------------------------------------------------------- split-fp16 form, 256 x 256 tile
// For tall products whose B operand is small enough to be split ahead of the multiply (the centroids of iteration 1,
// the rotation matrix).  One workgroup of 1024 threads (16 wavefronts, 4 x 4, 64 x 64 pairs each) owns 256 x 256
// scores: per matrix instruction half as many operand bytes travel from L2 to LDS as with the 128 x 128 tile, and
// half as many slabs' worth of barriers are crossed.  With 128 registers per lane the staging must be lean:
//  - B comes from a copy already split into fp16 pairs in the LDS byte order (split_rows_kernel), so every lane moves
//    16 bytes per load straight from global memory into LDS;
//  - A is fp32: a lane fetches 2 x 4 values of the next slab at the top of a step and converts them after the second
//    group of matrix instructions.
// LDS rows are 128 bytes, unpadded; the 16-byte piece c of a row (c = 4 h + 2 lo + kh: half-slab, hi or lo halves,
// dims 8 kh .. + 7 of the half-slab) sits at position c ^ ((row >> 1) & 7), which spreads the fragment reads of 16
// consecutive rows over all bank groups.  K must be a multiple of 32.
constexpr int T2 = 256, NT2 = 1024;
constexpr int T2_STAGE = 2 * T2 * 32;   // words of one slab of both operands (A rows, then B rows)
#define SKM_GEMM_VMCNT0() __builtin_amdgcn_s_waitcnt((0x7 << 4) | (0xF << 8))   // all vector memory operations done

template <int EPI>
__global__ void __launch_bounds__(NT2) gemm_split256_kernel(GemmOperands g, const uint32_t *Bsplit, int64_t ldbs,
                                                            typename EpiArgs<EPI>::type e) {
  extern __shared__ __align__(16) float smem[];
  uint32_t *lds = reinterpret_cast<uint32_t *>(smem);   // [2 stages][A 256 rows | B 256 rows][32 words]
  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int r32 = lane & 31, kh = lane >> 5;

  const int nrt = (g.M + T2 - 1) / T2, nct = (g.N + T2 - 1) / T2;
  int rt, ct;
  tile_of_block(nrt, nct, g.panel_cols, rt, ct);
  const int row0 = rt * T2, col0 = ct * T2;

  const unsigned int ma = *g.a_absmax, mb = *g.b_absmax;
  const float scale_a = split_scale(ma);
  const float unscale = split_unscale(ma) * split_unscale(mb);

  // B: load instruction j of wavefront w fills tile rows 128 j + 8 w .. + 7, 8 lanes a row; a lane fetches the piece
  // that belongs at its own position.  A: thread (arow, kq) converts dims 4 kq .. + 3 of tile rows arow and arow + 128.
  const int lrow = lane >> 3, lpos = lane & 7;
  const int kq = tid & 7, arow = tid >> 3;
  const int c_hi = 4 * (kq >> 2) + ((kq >> 1) & 1);   // piece that holds the hi halves of these four dims
  const uint32_t *gb[2];
  const float *ga[2];
  uint32_t *wa[2];
  int lo_off[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int rb = 8 * wave + 128 * j + lrow;
    gb[j] = Bsplit + (int64_t)min(col0 + rb, g.N - 1) * ldbs + 16 + 4 * (lpos ^ ((rb >> 1) & 7));   // one zero granule leads a row
    const int ra_ = arow + 128 * j, sw = (ra_ >> 1) & 7;
    ga[j] = g.A + (int64_t)min(row0 + ra_, g.M - 1) * g.lda + 4 * kq;
    wa[j] = lds + ra_ * 32 + ((c_hi ^ sw) << 2) + 2 * (kq & 1);
    lo_off[j] = (((c_hi + 2) ^ sw) - (c_hi ^ sw)) << 2;   // the lo halves: piece c_hi + 2
  }
  auto issue_b = [&](int stage, int k0) {
    uint32_t *sb = lds + stage * T2_STAGE + T2 * 32 + 8 * wave * 32;
#pragma unroll
    for (int j = 0; j < 2; ++j)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(gb[j] + k0),
                                       (__attribute__((address_space(3))) void *)(sb + 128 * j * 32), 16, 0, 0);
  };
  float4 ra[2];
  auto load_a = [&](int k0) {
#pragma unroll
    for (int j = 0; j < 2; ++j) ra[j] = *reinterpret_cast<const float4 *>(ga[j] + k0);
  };
  auto convert_a = [&](int stage) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float4 v = ra[j];
      const f32x2 p0 = {v.x * scale_a, v.y * scale_a}, p1 = {v.z * scale_a, v.w * scale_a};
      const f16x2 h0 = __builtin_convertvector(p0, f16x2), h1 = __builtin_convertvector(p1, f16x2);
      const f16x2 l0 = __builtin_convertvector(p0 - __builtin_convertvector(h0, f32x2), f16x2);
      const f16x2 l1 = __builtin_convertvector(p1 - __builtin_convertvector(h1, f32x2), f16x2);
      uint2 hi, lo;
      hi.x = __builtin_bit_cast(unsigned int, h0); hi.y = __builtin_bit_cast(unsigned int, h1);
      lo.x = __builtin_bit_cast(unsigned int, l0); lo.y = __builtin_bit_cast(unsigned int, l1);
      uint32_t *dst = wa[j] + stage * T2_STAGE;
      *reinterpret_cast<uint2 *>(dst) = hi;
      *reinterpret_cast<uint2 *>(dst + lo_off[j]) = lo;
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  const int swz = (r32 >> 1) & 7;
  const int fa = (wm * WTM + r32) * 32, fb = (T2 + wn * WTN + r32) * 32;
  auto frag = [&](const uint32_t *sb, int rowbase, int t, int h, int lo) {
    return *reinterpret_cast<const f16x8 *>(sb + rowbase + t * 32 * 32 + (((4 * h + 2 * lo + kh) ^ swz) << 2));
  };
  auto mma4 = [&](const f16x8 (&x)[TM], const f16x8 (&y)[TN]) {
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
      for (int b = 0; b < TN; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_f16(x[a], y[b], acc[a][b], 0, 0, 0);
  };

  const int nslab = g.K / 32;
  issue_b(0, 0);
  load_a(0);
  convert_a(0);
  SKM_GEMM_VMCNT0();
  __syncthreads();
  for (int s = 0; s < nslab; ++s) {
    const uint32_t *sb = lds + (s & 1) * T2_STAGE;
    const bool more = s + 1 < nslab;
    // the other stage was last read in the previous step, which ended with a barrier
    if (more) {
      issue_b((s + 1) & 1, (s + 1) * 32);
      load_a((s + 1) * 32);
    }
    f16x8 ah[TM], al[TM], bh[TN], bl[TN];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      ah[t] = frag(sb, fa, t, 0, 0); bh[t] = frag(sb, fb, t, 0, 0);
      al[t] = frag(sb, fa, t, 0, 1); bl[t] = frag(sb, fb, t, 0, 1);
    }
    __builtin_amdgcn_sched_barrier(0);
    mma4(ah, bh);
    mma4(al, bh);
    __builtin_amdgcn_sched_barrier(0);
    if (more) convert_a((s + 1) & 1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 2; ++t) { al[t] = frag(sb, fa, t, 1, 1); bh[t] = frag(sb, fb, t, 1, 0); }
    mma4(ah, bl);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int t = 0; t < 2; ++t) { ah[t] = frag(sb, fa, t, 1, 0); bl[t] = frag(sb, fb, t, 1, 1); }
    mma4(al, bh);
    __builtin_amdgcn_sched_barrier(0);
    mma4(ah, bl);
    mma4(ah, bh);
    __builtin_amdgcn_sched_barrier(0);
    SKM_GEMM_VMCNT0();
    __syncthreads();
  }
  tile_epilogue<EPI, T2>(acc, g, e, row0, col0, unscale, smem);
}

constexpr int64_t kMaxTilesPerLaunchFwd = (1 << 24) - 1;
template <int BK>
constexpr size_t smem_bytes() {
  return (size_t)2 * (BM + BN) * (BK + 4) * sizeof(float);
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool operands_aligned(const GemmOperands &g) {
  return aligned16(g.A) && aligned16(g.B) && (g.lda % 4 == 0) && (g.ldb % 4 == 0) && (g.K % 4 == 0);
}

template <int BK, int EPI, bool ALIGNED>
static hipError_t launch_one(const GemmOperands &g, const typename EpiArgs<EPI>::type &e, hipStream_t st) {
  auto kern = gemm_kernel<BK, EPI, ALIGNED>;
  // once per instantiation; the initialisation of a function-local static is synchronised between threads
  static const hipError_t attr_rc = hipFuncSetAttribute(
      reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<BK>());
  if (attr_rc != hipSuccess) return attr_rc;
  const int64_t nrt = (g.M + BM - 1) / BM, nct = (g.N + BN - 1) / BN;
  const int64_t nwg = nrt * nct;
  if (nwg <= 0) return hipSuccess;
  if (nwg > kMaxTilesPerLaunchFwd) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(NTHREADS), smem_bytes<BK>(), st, g, e);
  return hipGetLastError();
}

template <int EPI>
static hipError_t launch_split(const GemmOperands &g, const typename EpiArgs<EPI>::type &e, hipStream_t st) {
  auto kern = gemm_split_kernel<EPI>;
  static const hipError_t attr_rc = hipFuncSetAttribute(
      reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<SBK>());
  if (attr_rc != hipSuccess) return attr_rc;
  const int64_t nrt = (g.M + BM - 1) / BM, nct = (g.N + BN - 1) / BN;
  const int64_t nwg = nrt * nct;
  if (nwg <= 0) return hipSuccess;
  if (nwg > kMaxTilesPerLaunchFwd) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(NTHREADS), smem_bytes<SBK>(), st, g, e);
  return hipGetLastError();
}


// Launch choices a test can force (gemm_debug_config): nothing here changes what is computed.
static std::atomic<int> g_tile256{-1}, g_panel_cols{0};
static std::atomic<int64_t> g_max_tiles{0};
void gemm_debug_config(int tile256, int panel_cols, int64_t max_tiles) {
  g_tile256.store(tile256 < 0 ? -1 : (tile256 ? 1 : 0));
  g_panel_cols.store(panel_cols > 0 ? panel_cols : 0);
  g_max_tiles.store(max_tiles > 0 ? max_tiles : 0);
}

// The 256 x 256 form pays when the tall operand fills the device several times over and B can be split ahead.
static bool wants_split256(const GemmOperands &g) {
  const int forced = g_tile256.load(std::memory_order_relaxed);   // -1: by shape, 0: never, 1: whenever the operands allow it
  if (!g.b_split || !g.a_absmax || !g.b_absmax || g.K % 32 != 0 || g.K < 64 || forced == 0) return false;
  if (!aligned16(g.A) || !aligned16(g.B) || !aligned16(g.b_split) || g.lda % 4 != 0 || g.ldb % 4 != 0) return false;
  const int64_t tiles = (int64_t)((g.M + T2 - 1) / T2) * ((g.N + T2 - 1) / T2);
  // narrow B: a last column tile that is mostly padding costs more than the larger tile gains
  const int64_t ncols = (int64_t)((g.N + T2 - 1) / T2) * T2;
  return forced == 1 || (tiles >= 512 && ncols * 4 <= (int64_t)g.N * 5);
}

template <int EPI>
static hipError_t launch_split256(const GemmOperands &g, const typename EpiArgs<EPI>::type &e, hipStream_t st) {
  auto kern = gemm_split256_kernel<EPI>;
  constexpr size_t smem = (size_t)2 * T2_STAGE * sizeof(uint32_t);
  static const hipError_t attr_rc =
      hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (attr_rc != hipSuccess) return attr_rc;
  const int64_t nwg = (int64_t)((g.M + T2 - 1) / T2) * ((g.N + T2 - 1) / T2);
  if (nwg <= 0) return hipSuccess;
  if (nwg > (1 << 22) - 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(NT2), smem, st, g, (const uint32_t *)g.b_split, (int64_t)g.K + 32, e);
  return hipGetLastError();
}

// A launch may not exceed 2^32 threads in total: at 256 threads per tile that is 2^24 - 1 tiles, so
// tall problems are cut into bands of row tiles (the epilogue pointers move with the band).
constexpr int64_t kMaxTilesPerLaunch = (1 << 24) - 1;

// Column tiles per panel of the tile walk.  Measured on MI355X (rotation and iteration-1 GEMMs of the
// 1M x 1536 workload): the width moves the run time by less than the noise, but the bytes fetched from beyond L2
// drop by a quarter at 4 (the four centroid tiles of a panel then stay in one XCD's L2 while the point tiles
// stream past; every point tile is read once per panel).  With many column tiles the point tiles would be re-read
// too often, so wide problems keep 16.  gemm_debug_config overrides the width for experiments.
static int panel_cols_for(int64_t nct) {
  const int forced = g_panel_cols.load(std::memory_order_relaxed);
  return forced > 0 ? forced : (nct <= 16 ? 4 : 16);
}

inline void shift_rows(StoreArgs &e, int64_t r0) { e.C += r0 * e.ldc; }
inline void shift_rows(ArgminArgs &e, int64_t r0) { e.best += r0; }

template <int EPI>
static hipError_t launch_any(const GemmOperands &g, const typename EpiArgs<EPI>::type &e, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  const bool al = operands_aligned(g);
  // slabs of 32 for long K; slabs of 16 when K is short or not a multiple of 32 (d' is a multiple of 16)
  const bool bk32 = (g.K % 32 == 0) && g.K >= 256;
  const bool big = wants_split256(g);
  const int edge = big ? T2 : BM;
  const int64_t nct = (g.N + edge - 1) / edge;
  if (big) {   // B, split into fp16 pairs, K + 32 words a row
    hipError_t rc = launch_split_rows(g.B, g.ldb, g.N, g.K, g.b_absmax, g.b_split, st);
    if (rc != hipSuccess) return rc;
  }
  // gemm_debug_config lowers the limit so that the banding can be exercised on small inputs
  const int64_t forced_tiles = g_max_tiles.load(std::memory_order_relaxed);
  const int64_t max_tiles = (forced_tiles > 0 && forced_tiles < kMaxTilesPerLaunch) ? forced_tiles : kMaxTilesPerLaunch;
  const int64_t band_rows = std::max<int64_t>((big ? std::min<int64_t>(max_tiles, (1 << 22) - 1) : max_tiles) / nct, 1) * edge;
  for (int64_t r0 = 0; r0 < g.M; r0 += band_rows) {
    GemmOperands gb = g;
    gb.panel_cols = panel_cols_for(nct);
    gb.A = g.A + r0 * g.lda;
    gb.M = (int32_t)std::min<int64_t>(band_rows, g.M - r0);
    typename EpiArgs<EPI>::type eb = e;
    shift_rows(eb, r0);
    hipError_t rc;
    if (big) rc = launch_split256<EPI>(gb, eb, st);
    else if (al && g.K >= SBK && g.a_absmax && g.b_absmax) rc = launch_split<EPI>(gb, eb, st);
    else if (al) rc = bk32 ? launch_one<32, EPI, true>(gb, eb, st) : launch_one<16, EPI, true>(gb, eb, st);
    else rc = bk32 ? launch_one<32, EPI, false>(gb, eb, st) : launch_one<16, EPI, false>(gb, eb, st);
    if (rc != hipSuccess) return rc;
  }
  return hipSuccess;
}

hipError_t gemm_store(const GemmOperands &g, float *C, int64_t ldc, int32_t Nstore, float alpha, float beta,
                      hipStream_t st, unsigned int *c_absmax) {
  StoreArgs e{C, ldc, Nstore < g.N ? g.N : Nstore, alpha, beta, c_absmax};
  return launch_any<EPI_STORE>(g, e, st);
}

hipError_t gemm_argmin(const GemmOperands &g, const float *ynorm, unsigned long long *best, hipStream_t st) {
  ArgminArgs e{ynorm, best};
  return launch_any<EPI_ARGMIN>(g, e, st);
}

}  // namespace skm
