// Random orthogonal matrix on the device (Algorithm 1, GenerateRandomRotationMatrix; Section 3.1).
//
// The rows of a d x d matrix of independent standard normals are orthonormalised by Gram-Schmidt, which
// gives a Haar-distributed orthogonal matrix.  Everything is fp64 (the result is rounded to fp32 at the
// end) and runs in panels of 32 rows:
//   1. the panel is cleared of all finished rows, twice (coefficients C = W Q^T, then W -= C Q);
//   2. the panel is orthonormalised in itself by two rounds of Cholesky QR: G = W W^T = L L^T, W <- L^-1 W,
//      which is Gram-Schmidt inside the panel written as three dense steps.
// The normals come from a counter-based generator (splitmix64 of seed and element index, Box-Muller), so
// the matrix depends on (d, seed) only and no kernel uses atomics: the result is reproducible bit by bit.
#include "skm_internal.h"

namespace skm {

namespace {
constexpr int PB = 32;  // panel rows

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
// ks-th quarter of the columns; Cpart[ks][r][j] holds its share of <W_r, Q_j>.
constexpr int KS = 12;   // column splits of the coefficient product
constexpr int JR = 64;   // finished rows per workgroup of the update (the row range is split into ceil(p0 / JR) parts)
__global__ void __launch_bounds__(256) coeff_kernel(const double *Q, int d, int p0, int nr, double *Cpart) {
  __shared__ double s_w[PB][65], s_q[32][65];
  const int j0 = blockIdx.x * 32, ks = blockIdx.y;
  const int kchunk = ((d + KS - 1) / KS + 63) / 64 * 64;
  const int kbeg = ks * kchunk, kend = min(d, kbeg + kchunk);
  const int r = threadIdx.x >> 3, jg = (threadIdx.x & 7) * 4;
  double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  for (int c0 = kbeg; c0 < kend; c0 += 64) {
    __syncthreads();
    for (int t = threadIdx.x; t < 32 * 64; t += 256) {
      const int rr = t >> 6, c = t & 63;
      const bool cok = c0 + c < kend;
      s_w[rr][c] = (cok && rr < nr) ? Q[(int64_t)(p0 + rr) * d + c0 + c] : 0.0;
      s_q[rr][c] = (cok && j0 + rr < p0) ? Q[(int64_t)(j0 + rr) * d + c0 + c] : 0.0;
    }
    __syncthreads();
#pragma unroll 8
    for (int c = 0; c < 64; ++c) {
      const double w = s_w[r][c];
      a0 = fma(w, s_q[jg + 0][c], a0);
      a1 = fma(w, s_q[jg + 1][c], a1);
      a2 = fma(w, s_q[jg + 2][c], a2);
      a3 = fma(w, s_q[jg + 3][c], a3);
    }
  }
  double *dst = Cpart + ((int64_t)ks * PB + r) * p0 + j0 + jg;
  if (j0 + jg + 0 < p0) dst[0] = a0;
  if (j0 + jg + 1 < p0) dst[1] = a1;
  if (j0 + jg + 2 < p0) dst[2] = a2;
  if (j0 + jg + 3 < p0) dst[3] = a3;
}

// Wpart[js][r][c] = sum over the js-th JR rows of the finished rows j of C[r][j] Q[j][c], with
// C[r][j] = sum_ks Cpart[ks][r][j].  Thread = (column, group of 8 panel rows).
__global__ void __launch_bounds__(256) apply_kernel(const double *Q, int d, int p0, int nr, const double *Cpart,
                                                    double *Wpart) {
  __shared__ double s_c[PB][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63);
  const int rg = threadIdx.x >> 6;  // rows rg*8 .. rg*8+7
  const int js = blockIdx.y;
  const int jbeg = js * JR, jend = min(p0, jbeg + JR);
  double acc[8];
#pragma unroll
  for (int u = 0; u < 8; ++u) acc[u] = 0.0;
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
          for (int u = 0; u < 8; ++u) acc[u] = fma(s_c[rg * 8 + u][(jb + w) & 63], qv[w], acc[u]);
      }
    }
  }
  if (c < d)
#pragma unroll
    for (int u = 0; u < 8; ++u) Wpart[((int64_t)js * PB + rg * 8 + u) * d + c] = acc[u];
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

// Partial Gram matrices: workgroup `chunk` covers GC columns and writes W_chunk W_chunk^T (PB x PB).
constexpr int GC = 128;
__global__ void __launch_bounds__(256) gram_partial_kernel(const double *Q, int d, int p0, int nr, double *part) {
  __shared__ double s_w[PB][GC + 1];
  const int c0 = blockIdx.x * GC;
  for (int t = threadIdx.x; t < PB * GC; t += 256) {
    const int r = t / GC, c = t % GC;
    s_w[r][c] = (r < nr && c0 + c < d) ? Q[(int64_t)(p0 + r) * d + c0 + c] : 0.0;
  }
  __syncthreads();
  const int r1 = threadIdx.x >> 3, g4 = (threadIdx.x & 7) * 4;   // entries (r1, g4 .. g4+3)
  double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  for (int c = 0; c < GC; ++c) {
    const double x = s_w[r1][c];
    a0 = fma(x, s_w[g4 + 0][c], a0);
    a1 = fma(x, s_w[g4 + 1][c], a1);
    a2 = fma(x, s_w[g4 + 2][c], a2);
    a3 = fma(x, s_w[g4 + 3][c], a3);
  }
  double *dst = part + ((int64_t)blockIdx.x * PB + r1) * PB + g4;
  dst[0] = a0; dst[1] = a1; dst[2] = a2; dst[3] = a3;
}

__device__ inline double bcast_lane(double v, int src) {   // src is a compile-time constant after unrolling
  const unsigned long long u = __builtin_bit_cast(unsigned long long, v);
  const unsigned int lo = __builtin_amdgcn_readlane((int)(unsigned int)u, src);
  const unsigned int hi = __builtin_amdgcn_readlane((int)(unsigned int)(u >> 32), src);
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}

// One wavefront: G = sum of the partials (fixed order), Cholesky G = L L^T and Linv = L^-1.
// Lane t keeps row t of G / L in registers; entries of other rows arrive by lane broadcast.
__global__ void __launch_bounds__(64) chol_inv_kernel(const double *part, int nchunks, int nr, double *Linv_out) {
  const int t = threadIdx.x & 31;   // lanes 32..63 mirror lanes 0..31 and write nothing
  double g[PB];
#pragma unroll
  for (int j = 0; j < PB; ++j) g[j] = 0.0;
  for (int ch = 0; ch < nchunks; ++ch)
#pragma unroll
    for (int j = 0; j < PB; ++j) g[j] += part[((int64_t)ch * PB + t) * PB + j];
  // rows past nr are padding: make them the identity so that the factorisation stays defined
  if (t >= nr)
#pragma unroll
    for (int j = 0; j < PB; ++j) g[j] = (j == t) ? 1.0 : 0.0;
  // Cholesky by columns: after step k, g[k] of lane t >= k holds L[t][k]
#pragma unroll
  for (int k = 0; k < PB; ++k) {
    double s = g[k];
#pragma unroll
    for (int m = 0; m < k; ++m) s = fma(-g[m], bcast_lane(g[m], k), s);
    const double dkk = sqrt(bcast_lane(s, k));
    g[k] = (t == k) ? dkk : s / dkk;
  }
  // forward substitution: lane j builds column j of L^-1 in x[]
  double x[PB];
#pragma unroll
  for (int i = 0; i < PB; ++i) {
    double v = (i == t) ? 1.0 : 0.0;
#pragma unroll
    for (int m = 0; m < i; ++m) v = fma(-bcast_lane(g[m], i), x[m], v);
    x[i] = (i >= t) ? v / bcast_lane(g[i], i) : 0.0;
  }
  if (threadIdx.x < 32)
#pragma unroll
    for (int i = 0; i < PB; ++i) Linv_out[i * PB + t] = x[i];
}

// W <- Linv W, one thread per column.
__global__ void __launch_bounds__(256) tri_apply_kernel(double *Q, int d, int p0, int nr, const double *Linv) {
  __shared__ double s_l[PB * PB];
  for (int t = threadIdx.x; t < PB * PB; t += 256) s_l[t] = Linv[t];
  __syncthreads();
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= d) return;
  double w[PB];
#pragma unroll
  for (int r = 0; r < PB; ++r) w[r] = r < nr ? Q[(int64_t)(p0 + r) * d + c] : 0.0;
#pragma unroll
  for (int r = PB - 1; r >= 0; --r) {   // row r of the product uses rows <= r: go downwards, in place
    double s = 0.0;
#pragma unroll
    for (int k = 0; k < PB; ++k)
      if (k <= r) s = fma(s_l[r * PB + k], w[k], s);
    if (r < nr) Q[(int64_t)(p0 + r) * d + c] = s;
  }
}

__global__ void to_float_kernel(const double *Q, int64_t n, float *R) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) R[t] = (float)Q[t];
}
}  // namespace

// Qwork: d*d + 2 doubles; Cwork: max(12 * 32 * d, ceil(d/128) * 32 * 32); Wwork: ceil(d/64) * 32 * d; Lwork: 32 * 32.
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
    const int passes = d - p0 <= 8 * PB ? 2 : 1;
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
      hipLaunchKernelGGL(chol_inv_kernel, dim3(1), dim3(64), 0, st, Cwork, nchunks, nr, Lwork);
      hipLaunchKernelGGL(tri_apply_kernel, dim3((unsigned)((d + 255) / 256)), dim3(256), 0, st, Qwork, d, p0, nr, Lwork);
    }
  }
  hipLaunchKernelGGL(to_float_kernel, dim3((unsigned)((nel + 255) / 256)), dim3(256), 0, st, Qwork, nel, R_out);
  return hipGetLastError();
}

}  // namespace skm
