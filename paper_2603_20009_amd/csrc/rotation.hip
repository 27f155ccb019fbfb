// Random orthogonal matrix on the device (Algorithm 1, GenerateRandomRotationMatrix; Section 3.1).
//
// The rows of a d x d matrix of independent standard normals are orthonormalised by Gram-Schmidt, which
// gives a Haar-distributed orthogonal matrix.  Everything is fp64 (the result is rounded to fp32 at the
// end) and runs in panels of 64 rows (the chain of small dependent kernels per panel is what the run time is made of,
// so fewer, fatter panels are faster):
//   1. the panel is cleared of all finished rows (coefficients C = W Q^T, then W -= C Q);
//   2. the panel is orthonormalised in itself by Cholesky QR: G = W W^T = L L^T, W <- L^-1 W,
//      which is Gram-Schmidt inside the panel written as three dense steps.
// Both steps are done twice in the last rows, where the complement of the finished rows gets small.
// The normals come from a counter-based generator (splitmix64 of seed and element index, Box-Muller), so
// the matrix depends on (d, seed) only and no kernel uses atomics: the result is reproducible bit by bit.
#include "skm_internal.h"

namespace skm {

namespace {
constexpr int PB = 64;  // panel rows

__device__ inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ULL;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

__global__ void gauss_fill_kernel(double *Q, int64_t n_pairs, uint64_t seed) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_pairs) return;
  const uint64_t a = mix64(seed + 2 * (uint64_t)t), b = mix64(seed + 2 * (uint64_t)t + 1);
  double u1 = (double)(a >> 11) * (1.0 / 9007199254740992.0);
  const double u2 = (double)(b >> 11) * (1.0 / 9007199254740992.0);
  if (u1 < 1e-300) u1 = 1e-300;
  const double m = sqrt(-2.0 * log(u1));
  Q[2 * t] = m * cos(6.283185307179586 * u2);
  Q[2 * t + 1] = m * sin(6.283185307179586 * u2);
}

__device__ inline double wave_sum_f64(double v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// C = W Q_done^T as a small tiled product: workgroup (jt, ks) owns 32 finished rows j0 .. j0+31 and the
// ks-th part of the columns; Cpart[ks][r][j] holds its share of <W_r, Q_j>.
constexpr int KS = 12;   // column splits of the coefficient product
constexpr int JR = 64;   // finished rows per workgroup of the update (the row range is split into ceil(p0 / JR) parts)
__global__ void __launch_bounds__(256) coeff_kernel(const double *Q, int d, int p0, int nr, double *Cpart) {
  __shared__ double s_w[PB][65], s_q[32][65];
  const int j0 = blockIdx.x * 32, ks = blockIdx.y;
  const int kchunk = ((d + KS - 1) / KS + 63) / 64 * 64;
  const int kbeg = ks * kchunk, kend = min(d, kbeg + kchunk);
  const int r = threadIdx.x >> 3, jg = (threadIdx.x & 7) * 4;   // panel rows r and r + 32, finished rows j0 + jg .. + 3
  double a[2][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
  for (int c0 = kbeg; c0 < kend; c0 += 64) {
    __syncthreads();
    for (int t = threadIdx.x; t < PB * 64; t += 256) {
      const int rr = t >> 6, c = t & 63;
      s_w[rr][c] = (c0 + c < kend && rr < nr) ? Q[(int64_t)(p0 + rr) * d + c0 + c] : 0.0;
    }
    for (int t = threadIdx.x; t < 32 * 64; t += 256) {
      const int rr = t >> 6, c = t & 63;
      s_q[rr][c] = (c0 + c < kend && j0 + rr < p0) ? Q[(int64_t)(j0 + rr) * d + c0 + c] : 0.0;
    }
    __syncthreads();
#pragma unroll 8
    for (int c = 0; c < 64; ++c) {
      const double w0 = s_w[r][c], w1 = s_w[r + 32][c];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const double q = s_q[jg + u][c];
        a[0][u] = fma(w0, q, a[0][u]);
        a[1][u] = fma(w1, q, a[1][u]);
      }
    }
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    double *dst = Cpart + ((int64_t)ks * PB + r + 32 * h) * p0 + j0 + jg;
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (j0 + jg + u < p0) dst[u] = a[h][u];
  }
}
static_assert(PB == 64, "coeff_kernel: two panel rows per thread");

// Wpart[js][r][c] = sum over the js-th JR rows of the finished rows j of C[r][j] Q[j][c], with
// C[r][j] = sum_ks Cpart[ks][r][j].  Thread = (column, group of PB / 4 panel rows).
__global__ void __launch_bounds__(256) apply_kernel(const double *Q, int d, int p0, int nr, const double *Cpart,
                                                    double *Wpart) {
  __shared__ double s_c[PB][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  constexpr int RG = PB / 4;        // panel rows per thread
  const int rg = threadIdx.x >> 6;  // rows rg * RG .. + RG - 1
  const int js = blockIdx.y;
  const int jbeg = js * JR, jend = min(p0, jbeg + JR);
  double acc[RG];
#pragma unroll
  for (int u = 0; u < RG; ++u) acc[u] = 0.0;
  for (int j0 = jbeg; j0 < jend; j0 += 64) {
    __syncthreads();
    for (int t = threadIdx.x; t < PB * 64; t += 256) {
      const int r = t >> 6, jj = t & 63;
      double v = 0.0;
      if (r < nr && j0 + jj < jend)
        for (int ks = 0; ks < KS; ++ks) v += Cpart[((int64_t)ks * PB + r) * p0 + j0 + jj];
      s_c[r][jj] = v;
    }
    __syncthreads();
    if (c < d) {
      const int jn = min(64, jend - j0);
      for (int jb = 0; jb < jn; jb += 8) {
        double qv[8];
#pragma unroll
        for (int w = 0; w < 8; ++w) qv[w] = (jb + w < jn) ? Q[(int64_t)(j0 + jb + w) * d + c] : 0.0;
#pragma unroll
        for (int w = 0; w < 8; ++w)
#pragma unroll
          for (int u = 0; u < RG; ++u) acc[u] = fma(s_c[rg * RG + u][(jb + w) & 63], qv[w], acc[u]);
      }
    }
  }
  if (c < d)
#pragma unroll
    for (int u = 0; u < RG; ++u) Wpart[((int64_t)js * PB + rg * RG + u) * d + c] = acc[u];
}

// W[r][c] -= sum_js Wpart[js][r][c] (fixed order)
__global__ void __launch_bounds__(256) subtract_kernel(double *Q, int d, int p0, int nr, const double *Wpart, int njs) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  const int r = blockIdx.y;
  if (c >= d || r >= nr) return;
  double s = 0.0;
  for (int js = 0; js < njs; ++js) s += Wpart[((int64_t)js * PB + r) * d + c];
  Q[(int64_t)(p0 + r) * d + c] -= s;
}

// Partial Gram matrices: workgroup `chunk` covers GC columns and writes W_chunk W_chunk^T (PB x PB); a thread owns a
// 4 x 4 block of it.
constexpr int GC = 64;
__global__ void __launch_bounds__(256) gram_partial_kernel(const double *Q, int d, int p0, int nr, double *part) {
  __shared__ double s_w[PB][GC + 1];
  const int c0 = blockIdx.x * GC;
  for (int t = threadIdx.x; t < PB * GC; t += 256) {
    const int r = t / GC, c = t % GC;
    s_w[r][c] = (r < nr && c0 + c < d) ? Q[(int64_t)(p0 + r) * d + c0 + c] : 0.0;
  }
  __syncthreads();
  const int r4 = (threadIdx.x >> 4) * 4, g4 = (threadIdx.x & 15) * 4;   // entries (r4 .. r4+3, g4 .. g4+3)
  double a[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) a[i][j] = 0.0;
  for (int c = 0; c < GC; ++c) {
    double x[4], y[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[i] = s_w[r4 + i][c]; y[i] = s_w[g4 + i][c]; }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) a[i][j] = fma(x[i], y[j], a[i][j]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) part[((int64_t)blockIdx.x * PB + r4 + i) * PB + g4 + j] = a[i][j];
}
static_assert(PB == 64, "gram_partial_kernel: 16 x 16 threads of 4 x 4 entries");

__device__ inline double bcast_lane(double v, int src) {   // src is a compile-time constant after unrolling
  const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
  const unsigned int lo = __builtin_amdgcn_readlane((int)(unsigned int)u, src);
  const unsigned int hi = __builtin_amdgcn_readlane((int)(unsigned int)(u >> 32), src);
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// Cholesky factor and its inverse of a 32 x 32 matrix inside one wavefront.  Lane t (and its mirror t + 32) holds row
// t of the matrix in g[]; entries of other rows arrive by lane broadcast.  On return g[] holds row t of L and x[]
// column t of L^-1 (x[i] = Linv[i][t]).
constexpr int HB = 32;
__device__ inline void chol_inv32(double (&g)[HB], double (&x)[HB], int t) {
  // by columns: after step k, g[k] of lane t >= k holds L[t][k]
#pragma unroll
  for (int k = 0; k < HB; ++k) {
    double s = g[k];
#pragma unroll
    for (int m = 0; m < k; ++m) s = fma(-g[m], bcast_lane(g[m], k), s);
    const double dkk = sqrt(bcast_lane(s, k));
    g[k] = (t == k) ? dkk : s / dkk;
  }
  // forward substitution: lane j builds column j of L^-1
#pragma unroll
  for (int i = 0; i < HB; ++i) {
    double v = (i == t) ? 1.0 : 0.0;
#pragma unroll
    for (int m = 0; m < i; ++m) v = fma(-bcast_lane(g[m], i), x[m], v);
    x[i] = (i >= t) ? v / bcast_lane(g[i], i) : 0.0;
  }
}

// One workgroup: G = sum of the partials (fixed order) = [G11 G21^T; G21 G22] in blocks of 32, and the inverse of its
// Cholesky factor L = [L11 0; L21 L22] by blocks:
//   L11 = chol(G11), X11 = L11^-1;  L21 = G21 X11^T;  L22 = chol(G22 - L21 L21^T), X22 = L22^-1;
//   L^-1 = [X11 0; -X22 L21 X11, X22].
// The two 32 x 32 factorisations run in the registers of the first wavefront; the block products use all 256 threads
// (four results each) between barriers.
__global__ void __launch_bounds__(256) chol_inv_kernel(const double *part, int nchunks, int nr, double *Linv_out) {
  __shared__ double s_g[PB][PB + 1];    // G; its lower right block becomes X22, its upper right block L21 X11
  __shared__ double s_x11[HB][HB + 1];  // X11
  __shared__ double s_l21[HB][HB + 1];  // L21
  const int tid = threadIdx.x;
  {
    const int ti = tid >> 4, tj = tid & 15;
    double a[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) a[i][j] = 0.0;
    for (int ch = 0; ch < nchunks; ++ch)   // fixed order; the 16 loads of a chunk are independent
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) a[i][j] += part[((int64_t)ch * PB + 4 * ti + i) * PB + 4 * tj + j];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        // rows past nr are padding: make them the identity so that the factorisation stays defined
        const int row = 4 * ti + i, col = 4 * tj + j;
        s_g[row][col] = (row >= nr || col >= nr) ? ((row == col) ? 1.0 : 0.0) : a[i][j];
      }
  }
  __syncthreads();
  const int t = tid & 31;
  if (tid < 64) {   // L11, X11
    double g[HB], x[HB];
#pragma unroll
    for (int j = 0; j < HB; ++j) g[j] = s_g[t][j];
    chol_inv32(g, x, t);
    if (tid < HB)
#pragma unroll
      for (int i = 0; i < HB; ++i) s_x11[i][t] = x[i];
  }
  __syncthreads();
  const int r = tid >> 3, c4 = (tid & 7) * 4;   // block products: results (r, c4 .. c4 + 3)
  {   // L21 = G21 X11^T
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int m = 0; m < HB; ++m) {
      const double gv = s_g[HB + r][m];
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = fma(gv, s_x11[c4 + u][m], acc[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) s_l21[r][c4 + u] = acc[u];
  }
  __syncthreads();
  {   // G22 - L21 L21^T, in place
    double acc[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) acc[u] = s_g[HB + r][HB + c4 + u];
    for (int m = 0; m < HB; ++m) {
      const double lv = s_l21[r][m];
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = fma(-lv, s_l21[c4 + u][m], acc[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) s_g[HB + r][HB + c4 + u] = acc[u];
  }
  __syncthreads();
  if (tid < 64) {   // L22 (not kept), X22 over the block it came from
    double g[HB], x[HB];
#pragma unroll
    for (int j = 0; j < HB; ++j) g[j] = s_g[HB + t][HB + j];
    chol_inv32(g, x, t);
    if (tid < HB)
#pragma unroll
      for (int i = 0; i < HB; ++i) s_g[HB + i][HB + t] = x[i];
  }
  {   // meanwhile, by the other wavefronts too: L21 X11 into the unused upper right block
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int m = 0; m < HB; ++m) {
      const double lv = s_l21[r][m];
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = fma(lv, s_x11[m][c4 + u], acc[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) s_g[r][HB + c4 + u] = acc[u];
  }
  __syncthreads();
  {   // the result: [X11 0; -X22 (L21 X11), X22]
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int m = 0; m < HB; ++m) {
      const double xv = s_g[HB + r][HB + m];
#pragma unroll
      for (int u = 0; u < 4; ++u) acc[u] = fma(-xv, s_g[m][HB + c4 + u], acc[u]);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      Linv_out[(HB + r) * PB + c4 + u] = acc[u];
      Linv_out[r * PB + c4 + u] = s_x11[r][c4 + u];
      Linv_out[r * PB + HB + c4 + u] = 0.0;
      Linv_out[(HB + r) * PB + HB + c4 + u] = s_g[HB + r][HB + c4 + u];
    }
  }
}
static_assert(PB == 64 && HB * 2 == PB, "chol_inv_kernel: two blocks of 32");

// W <- Linv W on a tile of 64 columns: 16 x 16 threads, 4 x 4 results each, in place (the tile is read into LDS first).
__global__ void __launch_bounds__(256) tri_apply_kernel(double *Q, int d, int p0, int nr, const double *Linv) {
  __shared__ double s_l[PB][PB], s_w[PB][64];
  const int tid = threadIdx.x, ti = tid >> 4, tj = tid & 15;
  const int c0 = blockIdx.x * 64;
  for (int e = tid; e < PB * PB; e += 256) s_l[e / PB][e % PB] = Linv[e];
  for (int e = tid; e < PB * 64; e += 256) {
    const int r = e >> 6, c = e & 63;
    s_w[r][c] = (r < nr && c0 + c < d) ? Q[(int64_t)(p0 + r) * d + c0 + c] : 0.0;
  }
  __syncthreads();
  double acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0;
  const int kmax = 4 * ti + 4;   // Linv is lower triangular: rows 4 ti .. + 3 use columns below 4 ti + 4 only
#pragma unroll 4
  for (int k = 0; k < kmax; ++k) {
    double l[4], w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) l[i] = s_l[4 * ti + i][k];
#pragma unroll
    for (int j = 0; j < 4; ++j) w[j] = s_w[k][4 * tj + j];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = fma(l[i], w[j], acc[i][j]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = 4 * ti + i, c = c0 + 4 * tj + j;
      if (r < nr && c < d) Q[(int64_t)(p0 + r) * d + c] = acc[i][j];
    }
}
static_assert(PB == 64, "tri_apply_kernel: 16 x 16 threads of 4 x 4 entries");

__global__ void to_float_kernel(const double *Q, int64_t n, float *R) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) R[t] = (float)Q[t];
}
}  // namespace

// Qwork: d*d + 2 doubles; Cwork: max(12 * 64 * d, ceil(d/64) * 64 * 64); Wwork: ceil(d/64) * 64 * d; Lwork: 64 * 64.
hipError_t launch_make_rotation(int32_t d, uint64_t seed, double *Qwork, double *Cwork, double *Wwork, double *Lwork,
                                float *R_out, hipStream_t st) {
  const int64_t nel = (int64_t)d * d;
  const int64_t pairs = (nel + 1) / 2;
  hipLaunchKernelGGL(gauss_fill_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, st, Qwork, pairs, seed);
  for (int p0 = 0; p0 < d; p0 += PB) {
    const int nr = d - p0 < PB ? d - p0 : PB;
    // The rows are Gaussian: what a panel keeps after the projection has norm sqrt((d - p0) / d) of what it had, so one
    // projection and one Cholesky-QR already leave errors near fp64 rounding while the complement is large.  In the
    // last 256 rows, where the complement gets small and the panel ill-conditioned, both steps are done twice.
    const int passes = d - p0 <= 256 ? 2 : 1;
    if (p0 > 0) {
      for (int pass = 0; pass < passes; ++pass) {
        hipLaunchKernelGGL(coeff_kernel, dim3((unsigned)((p0 + 31) / 32), KS), dim3(256), 0, st, Qwork, d, p0, nr, Cwork);
        const int njs = (p0 + JR - 1) / JR;
        hipLaunchKernelGGL(apply_kernel, dim3((unsigned)((d + 63) / 64), (unsigned)njs), dim3(256), 0, st, Qwork, d, p0, nr,
                           Cwork, Wwork);
        hipLaunchKernelGGL(subtract_kernel, dim3((unsigned)((d + 255) / 256), PB), dim3(256), 0, st, Qwork, d, p0, nr,
                           Wwork, njs);
      }
    }
    for (int pass = 0; pass < passes; ++pass) {
      const int nchunks = (d + GC - 1) / GC;
      hipLaunchKernelGGL(gram_partial_kernel, dim3((unsigned)nchunks), dim3(256), 0, st, Qwork, d, p0, nr, Cwork);
      hipLaunchKernelGGL(chol_inv_kernel, dim3(1), dim3(256), 0, st, Cwork, nchunks, nr, Lwork);
      hipLaunchKernelGGL(tri_apply_kernel, dim3((unsigned)((d + 63) / 64)), dim3(256), 0, st, Qwork, d, p0, nr, Lwork);
    }
  }
  hipLaunchKernelGGL(to_float_kernel, dim3((unsigned)((nel + 255) / 256)), dim3(256), 0, st, Qwork, nel, R_out);
  return hipGetLastError();
}

}  // namespace skm
