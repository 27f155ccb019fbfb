// fp32 MFMA "NT" GEMM for gfx950 with two fused epilogues (store, row argmin).
//
// The GEMM phase of SuperKMeans (Algorithm 1: iteration 1 over all d dimensions, later iterations
// over the first d' dimensions; Section 3.1 for the rotation X R) is a product of two K-contiguous
// row-major matrices.  One workgroup of 256 threads (4 wavefronts, 2 x 2) owns a 128 x 128 tile of
// the score matrix; each wavefront owns 64 x 64 of it as 2 x 2 v_mfma_f32_32x32x2_f32 accumulators.
// K is consumed in slabs of BK floats that are staged global -> registers -> LDS (two LDS buffers,
// one barrier per slab) while the previous slab is multiplied.
//
// The score matrix is never written for the distance use of iteration 1: the epilogue reduces it to
// a row argmin.  Iterations >= 2 use the progressive kernel of progressive.hip, built on the same tile.
#include "skm_internal.h"

#include <algorithm>
#include <cstdlib>

namespace skm {

typedef float f32x16 __attribute__((ext_vector_type(16)));

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

  // Accumulator layout of v_mfma_f32_32x32x2_f32: register v of lane (r32, kh) holds
  // row 8*(v/4) + 4*kh + (v%4), column r32 of the 32 x 32 tile.
  auto row_of = [&](int a, int v) { return wm * WTM + a * 32 + 8 * (v >> 2) + 4 * kh + (v & 3); };

  if constexpr (EPI == EPI_STORE) {
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
            val = e.alpha * acc[a][b][v];
            if (e.beta != 0.f) val += e.beta * *dst;
          }
          *dst = val;
        }
      }
  } else if constexpr (EPI == EPI_ARGMIN) {
    // per-row minimum of ynorm[j] - 2 s(i,j): lanes of one half share the rows, columns differ
    unsigned long long *red = reinterpret_cast<unsigned long long *>(smem);  // [2][BM], reuses the tile buffers
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
            const unsigned long long kb = pack_key(yn[b] - 2.f * acc[a][b][v], gc[b]);
            key = kb < key ? kb : key;
          }
        }
#pragma unroll
        for (int m = 1; m < 32; m <<= 1) {
          const unsigned long long o = __shfl_xor(key, m, 64);
          key = o < key ? o : key;
        }
        if (r32 == 0) red[wn * BM + row_of(a, v)] = key;
      }
    __syncthreads();
    if (tid < BM) {
      const unsigned long long k0 = red[tid], k1 = red[BM + tid];
      const unsigned long long key = k0 < k1 ? k0 : k1;
      const int gr = row0 + tid;
      if (gr < g.M && key != ~0ull) atomicMin(e.best + gr, key);
    }
  }
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
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)smem_bytes<BK>());
    if (rc != hipSuccess) return rc;
    attr_set = true;
  }
  const int64_t nrt = (g.M + BM - 1) / BM, nct = (g.N + BN - 1) / BN;
  const int64_t nwg = nrt * nct;
  if (nwg <= 0) return hipSuccess;
  if (nwg > kMaxTilesPerLaunchFwd) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(NTHREADS), smem_bytes<BK>(), st, g, e);
  return hipGetLastError();
}

// A launch may not exceed 2^32 threads in total: at 256 threads per tile that is 2^24 - 1 tiles, so
// tall problems are cut into bands of row tiles (the epilogue pointers move with the band).
constexpr int64_t kMaxTilesPerLaunch = (1 << 24) - 1;

// Column tiles per panel of the tile walk.  Measured on MI355X (rotation and iteration-1 GEMMs of the
// 1M x 1536 workload, widths 1..12): no effect on the run time, the kernel is bound by the matrix pipe;
// SKM_TEST_PANEL_COLS overrides the width for experiments.
static int panel_cols_for(int) {
  static const int forced = []() {
    const char *e = std::getenv("SKM_TEST_PANEL_COLS");
    return e ? std::atoi(e) : 0;
  }();
  return forced > 0 ? forced : 16;
}

inline void shift_rows(StoreArgs &e, int64_t r0) { e.C += r0 * e.ldc; }
inline void shift_rows(ArgminArgs &e, int64_t r0) { e.best += r0; }

template <int EPI>
static hipError_t launch_any(const GemmOperands &g, const typename EpiArgs<EPI>::type &e, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0) return hipSuccess;
  const bool al = operands_aligned(g);
  // slabs of 32 for long K; slabs of 16 when K is short or not a multiple of 32 (d' is a multiple of 16)
  const bool bk32 = (g.K % 32 == 0) && g.K >= 256;
  const int64_t nct = (g.N + BN - 1) / BN;
  // SKM_TEST_MAX_TILES lowers the limit so that the banding can be exercised on small inputs
  static const int64_t max_tiles = []() {
    const char *e = std::getenv("SKM_TEST_MAX_TILES");
    const int64_t v = e ? std::atoll(e) : 0;
    return (v > 0 && v < kMaxTilesPerLaunch) ? v : kMaxTilesPerLaunch;
  }();
  const int64_t band_rows = std::max<int64_t>(max_tiles / nct, 1) * BM;
  for (int64_t r0 = 0; r0 < g.M; r0 += band_rows) {
    GemmOperands gb = g;
    gb.panel_cols = panel_cols_for(g.K);
    gb.A = g.A + r0 * g.lda;
    gb.M = (int32_t)std::min<int64_t>(band_rows, g.M - r0);
    typename EpiArgs<EPI>::type eb = e;
    shift_rows(eb, r0);
    hipError_t rc;
    if (al) rc = bk32 ? launch_one<32, EPI, true>(gb, eb, st) : launch_one<16, EPI, true>(gb, eb, st);
    else rc = bk32 ? launch_one<32, EPI, false>(gb, eb, st) : launch_one<16, EPI, false>(gb, eb, st);
    if (rc != hipSuccess) return rc;
  }
  return hipSuccess;
}

hipError_t gemm_store(const GemmOperands &g, float *C, int64_t ldc, int32_t Nstore, float alpha, float beta,
                      hipStream_t st) {
  StoreArgs e{C, ldc, Nstore < g.N ? g.N : Nstore, alpha, beta};
  return launch_any<EPI_STORE>(g, e, st);
}

hipError_t gemm_argmin(const GemmOperands &g, const float *ynorm, unsigned long long *best, hipStream_t st) {
  ArgminArgs e{ynorm, best};
  return launch_any<EPI_ARGMIN>(g, e, st);
}

}  // namespace skm
