// HBM-bound kernels around the two phases: initial threshold, centroid preparation (norms and the
// block-major copy of the trailing dimensions), unpacking of the argmin, and the centroid update as
// a segmented reduction (Section 3.2 "In between iterations", Section 3.4 "Initial threshold").
#include "skm_internal.h"

namespace skm {

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
  return v;
}
__device__ inline double wave_sum(double v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
  return v;
}

static int num_cus() {
  static const int cus = []() {   // (initialised once, synchronised between threads)
    int dev = 0, v = 0;
    (void)hipGetDevice(&dev);
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    return v;
  }();
  return cus;
}

// ------------------------------------------------------------------ initial threshold
// One wavefront per point: the rotated row and the row of its incumbent centroid are read as
// float4 per lane (1 KiB per wavefront load); squared differences over all dims give tau_i.
// NV = float4 loads per lane and operand (rows of up to 256 * NV floats): all loads of a row pair are
// issued before the first use, so that a wavefront keeps 2 * NV KiB in flight.
//
// The same pass can emit the prefix norms of the point that the progressive kernel tests against: every
// checkpoint t = d' + 64 m is a multiple of 16, so the table xnp[p][i] = ||x_i[0 : 16 (p + 1))||^2 serves any d',
// and the points do not change during a fit, so it is written once (PrefixOut), by the first pass that has the rows
// in registers anyway.  Lane l holds dims 4 l + 256 u .. + 3; a quad of lanes holds a 16-dim piece, and an
// inclusive scan over the 16 quads of the wavefront (then over u) gives every quad the norm of the row up to the
// end of its piece.
// With `xs` the pass also writes the split-fp16 copy of the row that the progressive kernel multiplies (the layout
// of launch_split_rows: row stride ds + 32 words, zero granules around the data).
struct PrefixOut {
  float *xnp;        // [ds / 16][n] or NULL
  int64_t n;
  int32_t ds;
  uint32_t *xs;      // [n][ds + 32] or NULL
  uint32_t *xh;      // [n][ds / 2 + 16] or NULL (with xs): the hi halves as a plane of their own
  const unsigned int *absmax;   // bound of |X| (bit pattern) that fixes the scale of xs
  float scale;       // split_scale(*absmax), set by the kernel
  // Regrouping (all three or none): output slot p takes point order[p]; its row is copied to xr_out (row stride ds)
  // and its label to label_out[p], so that every per-point array continues in the new order.
  const int32_t *order;
  float *xr_out;
  int32_t *label_out;
};

typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
// this lane's float4 at column c (a quarter of granule c / 16) -> hi and lo halves in the split copy of row i
__device__ inline void emit_split(const PrefixOut &po, int64_t i, int c, const float4 &v) {
  const f32x2_t p0 = {v.x * po.scale, v.y * po.scale}, p1 = {v.z * po.scale, v.w * po.scale};
  const f16x2_t h0 = __builtin_convertvector(p0, f16x2_t), h1 = __builtin_convertvector(p1, f16x2_t);
  const f16x2_t l0 = __builtin_convertvector(p0 - __builtin_convertvector(h0, f32x2_t), f16x2_t);
  const f16x2_t l1 = __builtin_convertvector(p1 - __builtin_convertvector(h1, f32x2_t), f16x2_t);
  uint32_t *dst = po.xs + i * (int64_t)(po.ds + 32) + 16 * (c / 16 + 1) + 2 * ((c / 4) & 3);
  *reinterpret_cast<uint2 *>(dst) = make_uint2(__builtin_bit_cast(unsigned int, h0), __builtin_bit_cast(unsigned int, h1));
  *reinterpret_cast<uint2 *>(dst + 8) = make_uint2(__builtin_bit_cast(unsigned int, l0), __builtin_bit_cast(unsigned int, l1));
  if (po.xh)
    *reinterpret_cast<uint2 *>(po.xh + i * (int64_t)(po.ds / 2 + 16) + 8 + c / 2) =
        make_uint2(__builtin_bit_cast(unsigned int, h0), __builtin_bit_cast(unsigned int, h1));
}
// the zero granules before and after the data of row i (lanes 0..3 and 4..7, 16 bytes each)
__device__ inline void emit_split_pads(const PrefixOut &po, int64_t i, int lane) {
  if (lane < 8) {
    uint32_t *dst = po.xs + i * (int64_t)(po.ds + 32) + (lane < 4 ? 4 * lane : po.ds + 16 + 4 * (lane - 4));
    *reinterpret_cast<uint4 *>(dst) = make_uint4(0u, 0u, 0u, 0u);
  } else if (lane < 12 && po.xh) {   // the 8 zero words at either end of the hi plane's row
    const int e = lane - 8;
    uint32_t *dst = po.xh + i * (int64_t)(po.ds / 2 + 16) + (e >> 1) * (8 + po.ds / 2) + 4 * (e & 1);
    *reinterpret_cast<uint4 *>(dst) = make_uint4(0u, 0u, 0u, 0u);
  }
}

// inclusive scan over the 16 quads of a wavefront of a value that is equal within each quad
__device__ inline float quad_scan64(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x114, 0xF, 0xF, false));  // row_shr:4
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x118, 0xF, 0xF, false));  // row_shr:8
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false));  // row_bcast:15 -> rows 1, 3
  v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false));  // row_bcast:31 -> rows 2, 3
  return v;
}
__device__ inline float quad_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  return v;
}
// q = sum of squares of this lane's float4 at column c0 = 4 lane + 256 u; base = norm of the row before column 256 u.
// Returns the norm of the row up to column 256 (u + 1).
// With `stage` (LDS, [ds / 16][64]) the value goes to column `slot` of it instead of the table: the caller writes the
// table 64 points at a time.
__device__ inline float emit_prefix(const PrefixOut &po, int64_t i, int lane, int u, float q, float base,
                                    float *stage = nullptr, int slot = 0) {
  const float upto = base + quad_scan64(quad_sum(q));   // norm up to the end of this quad's 16-dim piece
  const int t = 256 * u + 16 * (lane >> 2) + 16;          // that end
  if ((lane & 3) == 0 && t <= po.ds) {
    if (stage) stage[((t >> 4) - 1) * 64 + slot] = upto;
    else po.xnp[(int64_t)((t >> 4) - 1) * po.n + i] = upto;
  }
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, upto), 63));
}

// 16-byte load with the non-temporal hint (data read once)
__device__ inline float4 load_stream4(const float *p) {
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}

// BATCH (with po.xnp, NV > 0): a workgroup takes 64 consecutive points at a time and writes their prefix norms through
// LDS, 256 contiguous bytes per table row, instead of one 4-byte store per point and row.
constexpr int kPrefixStageRows = 128;   // ds <= 2048 in the batched form
template <int NV, bool BATCH>
__global__ void __launch_bounds__(256) tau_init_kernel(const float *Xr, int64_t ldx, int64_t n, int32_t ds,
                                                       const float *Y, int64_t ldy, const int32_t *assign, float *tau,
                                                       unsigned long long *best, PrefixOut po) {
  __shared__ float s_np[BATCH ? kPrefixStageRows * 64 : 1];
  if (po.xs) po.scale = split_scale(*po.absmax);
  const int lane = threadIdx.x & 63;
  auto point = [&](int64_t p, int slot) {   // output slot p <- point i
    const int64_t i = po.order ? (int64_t)po.order[p] : p;
    const int a = assign[i];
    const float *x = Xr + i * ldx;
    const float *y = Y + (int64_t)a * ldy;
    float s = 0.f;
    if (NV > 0) {
      float4 xv[NV > 0 ? NV : 1], yv[NV > 0 ? NV : 1];
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const int c = lane * 4 + 256 * u;
        // the points stream through once per step: keep them from displacing the centroids in the L2
        xv[u] = c < ds ? load_stream4(x + c) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const int c = lane * 4 + 256 * u;
        yv[u] = c < ds ? *reinterpret_cast<const float4 *>(y + c) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < NV; ++u) {
        const float dx = xv[u].x - yv[u].x, dy = xv[u].y - yv[u].y, dz = xv[u].z - yv[u].z, dw = xv[u].w - yv[u].w;
        s = fmaf(dx, dx, s);
        s = fmaf(dy, dy, s);
        s = fmaf(dz, dz, s);
        s = fmaf(dw, dw, s);
      }
      if (po.xnp) {
        float base = 0.f;
#pragma unroll
        for (int u = 0; u < NV; ++u) {
          if (256 * u >= ds) break;
          const float q = fmaf(xv[u].x, xv[u].x, fmaf(xv[u].y, xv[u].y, fmaf(xv[u].z, xv[u].z, xv[u].w * xv[u].w)));
          base = emit_prefix(po, p, lane, u, q, base, BATCH ? s_np : nullptr, slot);
        }
      }
      if (po.xs) {
        emit_split_pads(po, p, lane);
#pragma unroll
        for (int u = 0; u < NV; ++u)
          if (lane * 4 + 256 * u < ds) emit_split(po, p, lane * 4 + 256 * u, xv[u]);
      }
      if (po.xr_out) {
#pragma unroll
        for (int u = 0; u < NV; ++u)
          if (lane * 4 + 256 * u < ds) *reinterpret_cast<float4 *>(po.xr_out + p * (int64_t)ds + lane * 4 + 256 * u) = xv[u];
      }
    } else {
      float base = 0.f;
      for (int c0 = 0; c0 < ds; c0 += 256) {
        const int c = c0 + lane * 4;
        float4 xv = make_float4(0.f, 0.f, 0.f, 0.f), yv = xv;
        if (c < ds) {
          xv = *reinterpret_cast<const float4 *>(x + c);
          yv = *reinterpret_cast<const float4 *>(y + c);
        }
        const float dx = xv.x - yv.x, dy = xv.y - yv.y, dz = xv.z - yv.z, dw = xv.w - yv.w;
        s = fmaf(dx, dx, s);
        s = fmaf(dy, dy, s);
        s = fmaf(dz, dz, s);
        s = fmaf(dw, dw, s);
        if (po.xnp) {
          const float q = fmaf(xv.x, xv.x, fmaf(xv.y, xv.y, fmaf(xv.z, xv.z, xv.w * xv.w)));
          base = emit_prefix(po, p, lane, c0 >> 8, q, base);
        }
        if (po.xs) {
          if (c0 == 0) emit_split_pads(po, p, lane);
          if (c < ds) emit_split(po, p, c, xv);
        }
        if (po.xr_out && c < ds) *reinterpret_cast<float4 *>(po.xr_out + p * (int64_t)ds + c) = xv;
      }
    }
    s = wave_sum(s);
    if (lane == 0) {
      if (tau) tau[p] = s;
      if (best) best[p] = pack_key(s, a);
      if (po.label_out) po.label_out[p] = a;
    }
  };
  if (BATCH) {
    const int wave = threadIdx.x >> 6, rows = ds >> 4;
    for (int64_t b0 = (int64_t)blockIdx.x * 64; b0 < n; b0 += (int64_t)gridDim.x * 64) {
      for (int it = 0; it < 16; ++it) {
        const int slot = it * 4 + wave;
        if (b0 + slot < n) point(b0 + slot, slot);
      }
      __syncthreads();
      if (b0 + lane < n)
        for (int p = wave; p < rows; p += 4) po.xnp[(int64_t)p * po.n + b0 + lane] = s_np[p * 64 + lane];
      __syncthreads();
    }
  } else {
    const int64_t nwaves = (int64_t)gridDim.x * 4;
    for (int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); i < n; i += nwaves) point(i, 0);
  }
}

hipError_t launch_tau_init(const float *Xr, int64_t ldx, int64_t n, int32_t ds, const float *Y, int64_t ldy,
                           const int32_t *assign, float *tau, unsigned long long *best, hipStream_t st, float *xnp,
                           uint32_t *xs, const unsigned int *x_absmax, const int32_t *order, float *xr_out,
                           int32_t *label_out, uint32_t *xh) {
  if (n <= 0) return hipSuccess;
  const int nv = (ds + 255) / 256;
  const bool batch = xnp != nullptr && nv <= 8 && ds / 16 <= kPrefixStageRows;
  int64_t blocks = batch ? (n + 63) / 64 : (n + 3) / 4;
  const int64_t cap = (int64_t)num_cus() * 32;
  if (blocks > cap) blocks = cap;
  if (xs && (ds % 16 != 0 || !x_absmax)) return hipErrorInvalidValue;
  if ((order != nullptr) != (xr_out != nullptr) || (order != nullptr) != (label_out != nullptr)) return hipErrorInvalidValue;
  if (xr_out && (reinterpret_cast<uintptr_t>(xr_out) & 15u)) return hipErrorInvalidValue;
  if (xh && (!xs || (reinterpret_cast<uintptr_t>(xh) & 15u))) return hipErrorInvalidValue;
  const PrefixOut po{xnp, n, ds, xs, xh, x_absmax, 0.f, order, xr_out, label_out};
#define SKM_TAU_LAUNCH(NV)                                                                                      \
  do {                                                                                                          \
    if (batch && NV > 0)                                                                                        \
      hipLaunchKernelGGL((tau_init_kernel<NV, (NV > 0)>), dim3((unsigned)blocks), dim3(256), 0, st, Xr, ldx, n, ds, Y, \
                         ldy, assign, tau, best, po);                                                           \
    else                                                                                                        \
      hipLaunchKernelGGL((tau_init_kernel<NV, false>), dim3((unsigned)blocks), dim3(256), 0, st, Xr, ldx, n, ds, Y,   \
                         ldy, assign, tau, best, po);                                                           \
  } while (0)
  if (nv <= 1) SKM_TAU_LAUNCH(1);
  else if (nv <= 2) SKM_TAU_LAUNCH(2);
  else if (nv <= 3) SKM_TAU_LAUNCH(3);
  else if (nv <= 4) SKM_TAU_LAUNCH(4);
  else if (nv <= 6) SKM_TAU_LAUNCH(6);
  else if (nv <= 8) SKM_TAU_LAUNCH(8);
  else SKM_TAU_LAUNCH(0);
#undef SKM_TAU_LAUNCH
  return hipGetLastError();
}

// dst[idx[p]] = src[p] (4-byte items): per-point results back from a regrouped order to the caller's
__global__ void scatter_by_index_kernel(const uint32_t *src, const int32_t *idx, int64_t n, uint32_t *dst) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += (int64_t)gridDim.x * blockDim.x) dst[idx[p]] = src[p];
}
hipError_t launch_scatter_by_index(const void *src, const int32_t *idx, int64_t n, void *dst, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  const int64_t blocks = std::min<int64_t>((n + 255) / 256, (int64_t)num_cus() * 16);
  hipLaunchKernelGGL(scatter_by_index_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint32_t *)src, idx, n,
                     (uint32_t *)dst);
  return hipGetLastError();
}

// Sub-order of the points inside a cluster for the regrouping.  key[i] = the signs of the first four (rotated)
// dimensions of point i: four random hyperplanes through the origin cut every cluster into up to 16 pieces that are
// compact in space, and points of one piece share their challengers more than points of the whole cluster do.
__global__ void sign_key_kernel(const float *Xr, int64_t ldx, int64_t n, unsigned char *key) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const float4 v = *reinterpret_cast<const float4 *>(Xr + i * ldx);
    key[i] = (unsigned char)((v.x > 0.f) | ((v.y > 0.f) << 1) | ((v.z > 0.f) << 2) | ((v.w > 0.f) << 3));
  }
}
// order_out = order_in with every cluster's segment [off[c], off[c+1]) stably sorted by key (16 values): one
// workgroup per cluster, thread t takes the t-th contiguous part of the segment, so that the order inside a key is kept.
__global__ void __launch_bounds__(256) suborder_kernel(const int32_t *off, const int32_t *order_in, const unsigned char *key,
                                                       int32_t *order_out) {
  __shared__ int s_cnt[16][256];   // [key][thread]: count, then first output slot
  __shared__ int s_tot[16];
  const int c = blockIdx.x, t = threadIdx.x;
  const int lo = off[c], len = off[c + 1] - lo;
  const int part = (len + 255) / 256;
  const int p0 = min(t * part, len), p1 = min(p0 + part, len);
  for (int b = 0; b < 16; ++b) s_cnt[b][t] = 0;
  for (int p = p0; p < p1; ++p) s_cnt[key[order_in[lo + p]]][t] += 1;
  __syncthreads();
  if (t < 16) {   // exclusive scan of this key's counts over the threads
    int run = 0;
    for (int u = 0; u < 256; ++u) {
      const int v = s_cnt[t][u];
      s_cnt[t][u] = run;
      run += v;
    }
    s_tot[t] = run;
  }
  __syncthreads();
  if (t == 0) {   // first slot of every key
    int run = 0;
    for (int b = 0; b < 16; ++b) {
      const int v = s_tot[b];
      s_tot[b] = run;
      run += v;
    }
  }
  __syncthreads();
  for (int p = p0; p < p1; ++p) {
    const int id = order_in[lo + p];
    const int b = key[id];
    order_out[lo + s_tot[b] + s_cnt[b][t]] = id;
    s_cnt[b][t] += 1;
  }
}
hipError_t launch_suborder(const float *Xr, int64_t ldx, int64_t n, int32_t k, const int32_t *off, const int32_t *order_in,
                           unsigned char *key_scratch, int32_t *order_out, hipStream_t st) {
  if (n <= 0 || k <= 0) return hipSuccess;
  if ((reinterpret_cast<uintptr_t>(Xr) & 15u) || ldx % 4 != 0) return hipErrorInvalidValue;
  const int64_t blocks = std::min<int64_t>((n + 255) / 256, (int64_t)num_cus() * 16);
  hipLaunchKernelGGL(sign_key_kernel, dim3((unsigned)blocks), dim3(256), 0, st, Xr, ldx, n, key_scratch);
  hipLaunchKernelGGL(suborder_kernel, dim3((unsigned)k), dim3(256), 0, st, off, order_in, (const unsigned char *)key_scratch,
                     order_out);
  return hipGetLastError();
}

// inv[perm[p]] = p, then the point id in the low half of every key replaced by its position (keys of ~0 stay)
__global__ void invert_permutation_kernel(const int32_t *perm, int64_t n, int32_t *inv) {
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < n; p += (int64_t)gridDim.x * blockDim.x) inv[perm[p]] = (int32_t)p;
}
__global__ void remap_key_ids_kernel(unsigned long long *keys, int64_t m, const int32_t *inv, int64_t n) {
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < m; e += (int64_t)gridDim.x * blockDim.x) {
    const unsigned long long key = keys[e];
    const unsigned long long id = key & 0xffffffffull;
    if (key != ~0ull && (int64_t)id < n) keys[e] = (key & ~0xffffffffull) | (unsigned long long)(unsigned int)inv[id];
  }
}
hipError_t launch_remap_key_ids(unsigned long long *keys, int64_t m, const int32_t *perm, int64_t n, int32_t *inv_scratch,
                                hipStream_t st) {
  if (n <= 0 || m <= 0) return hipSuccess;
  const int64_t b1 = std::min<int64_t>((n + 255) / 256, (int64_t)num_cus() * 16);
  hipLaunchKernelGGL(invert_permutation_kernel, dim3((unsigned)b1), dim3(256), 0, st, perm, n, inv_scratch);
  const int64_t b2 = std::min<int64_t>((m + 255) / 256, (int64_t)num_cus() * 16);
  hipLaunchKernelGGL(remap_key_ids_kernel, dim3((unsigned)b2), dim3(256), 0, st, keys, m, (const int32_t *)inv_scratch, n);
  return hipGetLastError();
}

// ------------------------------------------------------------------ centroid preparation
// One workgroup per centroid: ynorm[c] over dims [0, dn), and the trailing dims from dprime on
// copied to Ypdx[m][c][0..63] (block m = dims dprime+64m ..), zero filled past the row.
__global__ void __launch_bounds__(256) prep_centroids_kernel(const float *Y, int64_t ldy, int32_t k, int32_t ds,
                                                             int32_t dn, float *ynorm, int32_t dprime, int32_t nb,
                                                             float *Ypdx, float *ynp) {
  __shared__ float red[4];
  __shared__ float piece[1024];   // ds <= 16384
  const int c = blockIdx.x;
  const float *y = Y + (int64_t)c * ldy;
  float s = 0.f;
  for (int j = threadIdx.x; j < dn; j += 256) s = fmaf(y[j], y[j], s);
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0 && ynorm) ynorm[c] = (red[0] + red[1]) + (red[2] + red[3]);
  if (ynp) {
    // ||y[0 : t_m)||^2 at the checkpoints t_m = min(ds, d' + 64 m): sums of squares of the 16-dim pieces of the row
    // in LDS, then thread m adds up the pieces below its checkpoint (d' is a multiple of 16; rows are short)
    const int np = (ds + 15) / 16;
    for (int p = threadIdx.x; p < np; p += 256) {
      float acc = 0.f;
      for (int j = 16 * p; j < min(ds, 16 * p + 16); ++j) acc = fmaf(y[j], y[j], acc);
      piece[p] = acc;
    }
    __syncthreads();
    for (int m = threadIdx.x; m <= nb; m += 256) {
      const int t = m == nb ? ds : min(ds, dprime + kBlockDims * m);
      float acc = 0.f;
      for (int p = 0; p < (t + 15) / 16; ++p) acc += piece[p];
      ynp[(int64_t)m * k + c] = acc;
    }
  }
  if (Ypdx) {
    for (int t = threadIdx.x; t < nb * kBlockDims; t += 256) {
      const int m = t / kBlockDims, qd = t % kBlockDims;
      const int col = dprime + t;
      Ypdx[((int64_t)m * k + c) * kBlockDims + qd] = col < ds ? y[col] : 0.f;
    }
  }
}

hipError_t launch_prep_centroids(const float *Y, int64_t ldy, int32_t k, int32_t ds, int32_t dn, float *ynorm,
                                 int32_t dprime, int32_t nb, float *Ypdx, hipStream_t st, float *ynp) {
  hipLaunchKernelGGL(prep_centroids_kernel, dim3(k), dim3(256), 0, st, Y, ldy, k, ds, dn, ynorm, dprime, nb, Ypdx, ynp);
  return hipGetLastError();
}

// ------------------------------------------------------------------ fills
template <typename T>
__global__ void fill_kernel(T *p, int64_t n, T v) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
template <typename T>
static hipError_t launch_fill(T *p, int64_t n, T v, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(fill_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}
hipError_t launch_fill_u64(unsigned long long *p, int64_t n, unsigned long long v, hipStream_t st) {
  return launch_fill<unsigned long long>(p, n, v, st);
}
hipError_t launch_fill_u32(unsigned int *p, int64_t n, unsigned int v, hipStream_t st) {
  return launch_fill<unsigned int>(p, n, v, st);
}

// ------------------------------------------------------------------ largest magnitude of a matrix
// Non-negative floats order like their bit patterns, so the maximum is kept with an unsigned atomicMax.
// max |v| over a workgroup of 256 threads into *out (bit pattern, unsigned order): one atomic per workgroup, and
// only if it would raise the word that thousands of workgroups share
__device__ inline void block_absmax(float v, unsigned int *out) {
  __shared__ unsigned int s_m[4];
  float m = fabsf(v);
#pragma unroll
  for (int w = 1; w < 64; w <<= 1) m = fmaxf(m, __shfl_xor(m, w, 64));
  if ((threadIdx.x & 63) == 0) s_m[threadIdx.x >> 6] = __builtin_bit_cast(unsigned int, m);
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned int mb = max(max(s_m[0], s_m[1]), max(s_m[2], s_m[3]));
    if (mb > __atomic_load_n(out, __ATOMIC_RELAXED)) atomicMax(out, mb);
  }
}

// Rows without gaps (lda == cols) are read as one array; otherwise an element index is split into row and column.
template <bool VEC4>
__global__ void __launch_bounds__(256) absmax_kernel(const float *A, int64_t lda, int64_t rows, int32_t cols,
                                                     unsigned int *out) {
  const int64_t per_row = VEC4 ? cols / 4 : cols;
  const int64_t total = rows * per_row;
  const bool flat = lda == cols;
  float m = 0.f;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += (int64_t)gridDim.x * blockDim.x) {
    int64_t at = e * (VEC4 ? 4 : 1);
    if (!flat) {
      const int64_t r = e / per_row;
      at = r * lda + (e - r * per_row) * (VEC4 ? 4 : 1);
    }
    if (VEC4) {
      const float4 v = *reinterpret_cast<const float4 *>(A + at);
      m = fmaxf(m, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    } else {
      m = fmaxf(m, fabsf(A[at]));
    }
  }
  block_absmax(m, out);
}

hipError_t launch_absmax(const float *A, int64_t lda, int64_t rows, int32_t cols, unsigned int *out, hipStream_t st,
                         int max_blocks) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  const bool vec = (reinterpret_cast<uintptr_t>(A) & 15u) == 0 && lda % 4 == 0 && cols % 4 == 0;
  const int64_t work = rows * (int64_t)(vec ? cols / 4 : cols);
  // at least four elements per thread where there are that many: fewer workgroups meet at the one result word
  const unsigned blocks = (unsigned)std::min<int64_t>((work + 1023) / 1024, max_blocks > 0 ? max_blocks : 256 * 16);
  if (vec) hipLaunchKernelGGL(absmax_kernel<true>, dim3(blocks), dim3(256), 0, st, A, lda, rows, cols, out);
  else hipLaunchKernelGGL(absmax_kernel<false>, dim3(blocks), dim3(256), 0, st, A, lda, rows, cols, out);
  return hipGetLastError();
}

// ------------------------------------------------------------------ unit-length rows (angular metric)
// One wavefront per row: sum of squares in fp32 over float4 loads, then the row is scaled in place.
// Rows of zeros are left alone.
__global__ void __launch_bounds__(256) normalize_rows_kernel(float *A, int64_t lda, int64_t rows, int32_t cols) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  float *row = A + r * lda;
  float s = 0.f;
  for (int c = 4 * lane; c < cols; c += 256) {
    const float4 v = *reinterpret_cast<const float4 *>(row + c);
    s = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, s))));
  }
#pragma unroll
  for (int w = 1; w < 64; w <<= 1) s += __shfl_xor(s, w, 64);
  if (!(s > 0.f)) return;
  const float inv = 1.0f / sqrtf(s);
  for (int c = 4 * lane; c < cols; c += 256) {
    float4 v = *reinterpret_cast<const float4 *>(row + c);
    v.x *= inv; v.y *= inv; v.z *= inv; v.w *= inv;
    *reinterpret_cast<float4 *>(row + c) = v;
  }
}

// cols and lda multiples of 4, A 16-byte aligned (the padded buffers of the library)
hipError_t launch_normalize_rows(float *A, int64_t lda, int64_t rows, int32_t cols, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if ((reinterpret_cast<uintptr_t>(A) & 15u) || lda % 4 || cols % 4) return hipErrorInvalidValue;
  const int64_t blocks = (rows + 3) / 4;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(normalize_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, A, lda, rows, cols);
  return hipGetLastError();
}

// ------------------------------------------------------------------ argmin unpack
// A workgroup takes 8192 consecutive points.  The cluster sizes are counted in LDS first when the k counters fit
// (k <= FIN_LDS_BINS) and flushed once per workgroup: a million atomic increments on the 64 cache lines that hold 1024
// counters took 0.2 ms per step; larger k spreads them over more lines and goes to memory directly.
// Small inputs (one small fit of many, as in the hierarchical fit) take 1024 points per workgroup instead: the
// launch is then a few workgroups side by side rather than one long loop.
constexpr int FIN_THREADS = 256;
constexpr int FIN_LDS_BINS = 8192;
static int finalize_per_block(int64_t n) { return n >= (int64_t)1 << 18 ? 8192 : 1024; }
int64_t finalize_blocks(int64_t n) { return (n + finalize_per_block(n) - 1) / finalize_per_block(n); }

__global__ void __launch_bounds__(FIN_THREADS) finalize_assign_kernel(const unsigned long long *best,
                                                                      const int32_t *prev, int64_t n, int32_t *assign,
                                                                      float *dist, int32_t *cnt, int32_t k,
                                                                      double *obj_partial, unsigned long long *changed,
                                                                      unsigned int *unset, int per_block) {
  __shared__ double red[4];
  __shared__ unsigned int redc[4];
  __shared__ int s_hist[FIN_LDS_BINS];
  const bool in_lds = cnt && k <= FIN_LDS_BINS && per_block > 1024;
  if (in_lds) {
    for (int b = threadIdx.x; b < k; b += FIN_THREADS) s_hist[b] = 0;
    __syncthreads();
  }
  double s = 0.0;
  unsigned int ch = 0;
  const int64_t base = (int64_t)blockIdx.x * per_block;
  for (int t = threadIdx.x; t < per_block; t += FIN_THREADS) {
    const int64_t i = base + t;
    if (i < n) {
      const unsigned long long key = best[i];
      int32_t a = (int32_t)(key & 0xffffffffull);
      float dv = ord2f((uint32_t)(key >> 32));
      if (key == ~0ull) {   // a point no kernel offered a centroid for: reported through `unset`, kept in range
        a = 0;
        dv = 0.f;
        if (unset) atomicOr(unset, 2u);   // bit 1: unset point (bit 0 is the hand-over list's overflow)
      }
      assign[i] = a;
      if (dist) dist[i] = dv;
      if (in_lds) atomicAdd(&s_hist[a], 1);
      else if (cnt) atomicAdd(cnt + a, 1);
      if (prev) ch += (prev[i] != a);
      s += (double)dv;
    }
  }
  s = wave_sum(s);
  for (int m = 1; m < 64; m <<= 1) ch += __shfl_xor(ch, m, 64);
  if ((threadIdx.x & 63) == 0) {
    red[threadIdx.x >> 6] = s;
    redc[threadIdx.x >> 6] = ch;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (obj_partial) obj_partial[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
    const unsigned int c4 = redc[0] + redc[1] + redc[2] + redc[3];
    if (changed && c4) atomicAdd(changed, (unsigned long long)c4);
  }
  if (in_lds) {   // (the barrier above has ordered the LDS increments before these reads)
    for (int b = threadIdx.x; b < k; b += FIN_THREADS) {
      const int v = s_hist[b];
      if (v) atomicAdd(cnt + b, v);
    }
  }
}

hipError_t launch_finalize_assign(const unsigned long long *best, const int32_t *prev, int64_t n, int32_t *assign,
                                  float *dist, int32_t *cnt, int32_t k, double *obj_partial,
                                  unsigned long long *changed, unsigned int *unset, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(finalize_assign_kernel, dim3((unsigned)finalize_blocks(n)), dim3(FIN_THREADS), 0, st, best, prev, n,
                     assign, dist, cnt, k, obj_partial, changed, unset, finalize_per_block(n));
  return hipGetLastError();
}

// fixed-order sum of the per-block partials (deterministic objective)
__global__ void __launch_bounds__(256) sum_partials_kernel(const double *part, int64_t m, double *out) {
  __shared__ double red[256];
  double s = 0.0;
  const int64_t per = (m + 255) / 256;
  const int64_t lo = (int64_t)threadIdx.x * per;
  for (int64_t i = lo; i < lo + per && i < m; ++i) s += part[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = red[0];
}
hipError_t launch_sum_partials(const double *part, int64_t m, double *out, hipStream_t st) {
  hipLaunchKernelGGL(sum_partials_kernel, dim3(1), dim3(256), 0, st, part, m, out);
  return hipGetLastError();
}

__global__ void histogram_kernel(const int32_t *assign, int64_t n, int32_t *cnt) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    atomicAdd(cnt + assign[i], 1);
}
hipError_t launch_histogram(const int32_t *assign, int64_t n, int32_t *cnt, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(histogram_kernel, dim3((unsigned)blocks), dim3(256), 0, st, assign, n, cnt);
  return hipGetLastError();
}

// sets *bad to 1 if any label is outside [0, k)
__global__ void check_labels_kernel(const int32_t *a, int64_t n, int32_t k, unsigned int *bad) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    if (a[i] < 0 || a[i] >= k) *bad = 1u;
}
hipError_t launch_check_labels(const int32_t *a, int64_t n, int32_t k, unsigned int *bad, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(check_labels_kernel, dim3((unsigned)blocks), dim3(256), 0, st, a, n, k, bad);
  return hipGetLastError();
}

// ------------------------------------------------------------------ centroid update
int64_t update_max_segments(int64_t n, int32_t k) { return (int64_t)k + n / kSegPoints + 1; }

// single workgroup: exclusive scans of the cluster sizes and of the segment counts
__global__ void __launch_bounds__(1024) scan_counts_kernel(const int32_t *cnt, int32_t k, int32_t *off, int32_t *cursor,
                                                           int32_t *segoff) {
  __shared__ int s_a[1024], s_b[1024];
  __shared__ int carry_a, carry_b;
  if (threadIdx.x == 0) { carry_a = 0; carry_b = 0; }
  __syncthreads();
  for (int base = 0; base < k; base += 1024) {
    const int c = base + threadIdx.x;
    const int va = c < k ? cnt[c] : 0;
    const int vb = (va + kSegPoints - 1) / kSegPoints;
    s_a[threadIdx.x] = va;
    s_b[threadIdx.x] = vb;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      int ta = 0, tb = 0;
      if ((int)threadIdx.x >= o) { ta = s_a[threadIdx.x - o]; tb = s_b[threadIdx.x - o]; }
      __syncthreads();
      s_a[threadIdx.x] += ta;
      s_b[threadIdx.x] += tb;
      __syncthreads();
    }
    if (c < k) {
      off[c] = carry_a + s_a[threadIdx.x] - va;
      segoff[c] = carry_b + s_b[threadIdx.x] - vb;
      cursor[c] = 0;
    }
    __syncthreads();
    if (threadIdx.x == 1023) { carry_a += s_a[1023]; carry_b += s_b[1023]; }
    __syncthreads();
  }
  if (threadIdx.x == 0) { off[k] = carry_a; segoff[k] = carry_b; }
}

// order[...] = i (or ids[i] when the labelled items are a list of ids), grouped by label
__global__ void scatter_order_kernel(const int32_t *assign, int64_t n, const int32_t *off, int32_t *cursor,
                                     int32_t *order, const int32_t *ids) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const int a = assign[i];
    const int pos = off[a] + atomicAdd(cursor + a, 1);
    order[pos] = ids ? ids[i] : (int32_t)i;
  }
}

// The cursor order above depends on scheduling; sorting every segment of `order` makes the
// summation order, and with it every bit of the result, independent of it.  One workgroup per
// cluster, odd-even merge in LDS for clusters up to SORT_CAP points; larger clusters are summed in
// fp64 in whatever order they were scattered (the fp64 sum of fp32 values then differs from the
// sorted-order sum by at most a few ulps of fp64, far below the fp32 rounding of the mean).
constexpr int SORT_CAP = 8192;
int32_t update_sort_cap() { return SORT_CAP; }
__global__ void __launch_bounds__(256) sort_segments_kernel(const int32_t *off, int32_t *order) {
  __shared__ int32_t s[SORT_CAP];
  const int c = blockIdx.x;
  const int lo = off[c], len = off[c + 1] - lo;
  if (len < 2 || len > SORT_CAP) return;
  int np2 = 1;
  while (np2 < len) np2 <<= 1;
  for (int t = threadIdx.x; t < np2; t += 256) s[t] = t < len ? order[lo + t] : 0x7fffffff;
  __syncthreads();
  for (int kk = 2; kk <= np2; kk <<= 1)
    for (int jj = kk >> 1; jj > 0; jj >>= 1) {
      for (int t = threadIdx.x; t < np2; t += 256) {
        const int p = t ^ jj;
        if (p > t) {
          const int32_t a = s[t], b = s[p];
          const bool up = (t & kk) == 0;
          if ((a > b) == up) { s[t] = b; s[p] = a; }
        }
      }
      __syncthreads();
    }
  for (int t = threadIdx.x; t < len; t += 256) order[lo + t] = s[t];
}

// One workgroup per (segment of <= kSegPoints points of one cluster, slice of 256 dims): rows are gathered through
// `order` (each a contiguous row read).  Wavefront w takes the points p0 + w, p0 + w + 4, ... of the segment, four
// rows in flight per thread, fp64 sums per thread; the four wavefronts' sums are added in a fixed order, so the
// result depends on the segment only.
// SIGNED: an entry i >= 0 adds row i, an entry ~i < 0 subtracts row i (a point that left the cluster).
template <bool SIGNED>
__global__ void __launch_bounds__(256) segment_sum_kernel(const float *Xr, int64_t ldx, int32_t ds, int32_t k,
                                                          const int32_t *off, const int32_t *segoff,
                                                          const int32_t *order, double *partial) {
  __shared__ double red[3][64][4];
  const int seg = blockIdx.x;
  if (seg >= segoff[k]) return;
  // cluster of this segment: last c with segoff[c] <= seg
  int lo = 0, hi = k;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (segoff[mid] <= seg) lo = mid; else hi = mid;
  }
  const int c = lo;
  const int s_in = seg - segoff[c];
  const int p0 = off[c] + s_in * kSegPoints;
  const int p1 = min(off[c + 1], p0 + kSegPoints);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int col = (blockIdx.y * 64 + lane) * 4;
  const bool live = col < ds;
  double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
  auto row = [&](int raw, float4 &v, double &sg) {
    const int i = SIGNED && raw < 0 ? ~raw : raw;
    sg = SIGNED && raw < 0 ? -1.0 : 1.0;
    v = *reinterpret_cast<const float4 *>(Xr + (int64_t)i * ldx + col);
  };
  auto add = [&](const float4 &v, double sg) {
    if (SIGNED) {
      a0 += sg * (double)v.x; a1 += sg * (double)v.y; a2 += sg * (double)v.z; a3 += sg * (double)v.w;
    } else {
      a0 += (double)v.x; a1 += (double)v.y; a2 += (double)v.z; a3 += (double)v.w;
    }
  };
  if (live) {
    int p = p0 + w;
    for (; p + 12 < p1; p += 16) {
      float4 v0, v1, v2, v3;
      double s0, s1, s2, s3;
      row(order[p], v0, s0);
      row(order[p + 4], v1, s1);
      row(order[p + 8], v2, s2);
      row(order[p + 12], v3, s3);
      add(v0, s0);
      add(v1, s1);
      add(v2, s2);
      add(v3, s3);
    }
    for (; p < p1; p += 4) {
      float4 v;
      double sg;
      row(order[p], v, sg);
      add(v, sg);
    }
  }
  if (w > 0) {
    red[w - 1][lane][0] = a0; red[w - 1][lane][1] = a1; red[w - 1][lane][2] = a2; red[w - 1][lane][3] = a3;
  }
  __syncthreads();
  if (w == 0 && live) {
    double *dst = partial + (int64_t)seg * ds + col;
    dst[0] = (a0 + red[0][lane][0]) + (red[1][lane][0] + red[2][lane][0]);
    dst[1] = (a1 + red[0][lane][1]) + (red[1][lane][1] + red[2][lane][1]);
    dst[2] = (a2 + red[0][lane][2]) + (red[1][lane][2] + red[2][lane][2]);
    dst[3] = (a3 + red[0][lane][3]) + (red[1][lane][3] + red[2][lane][3]);
  }
}

// One workgroup per (cluster, slice): partial sums added in segment order, divided by the size.
// S (optional, [k][ds] fp64) keeps the sum of every cluster between updates: it is overwritten by the total of the
// partials, or, with `accumulate`, the total (a signed change) is added to it.
// y_absmax (optional, zero before the launch) receives the bit pattern of max |Y| over all centroids, the bound
// that the split-fp16 GEMMs of the next step scale the centroids by.
__global__ void __launch_bounds__(256) centroid_mean_kernel(const double *partial, int32_t ds, const int32_t *cnt,
                                                            const int32_t *segoff, float *Y, int64_t ldy, double *S,
                                                            int accumulate, unsigned int *y_absmax) {
  const int c = blockIdx.x;
  const int n_c = cnt[c];
  const int col = blockIdx.y * 256 + threadIdx.x;
  float y = 0.f;
  if (col < ds) {
    double s = 0.0;
    for (int seg = segoff[c]; seg < segoff[c + 1]; ++seg) s += partial[(int64_t)seg * ds + col];
    if (S) {
      if (accumulate) s += S[(int64_t)c * ds + col];
      S[(int64_t)c * ds + col] = s;
    }
    if (!Y) {
      // sums only (a batch of a larger update: the means follow once all batches are in)
    } else if (n_c == 0) {   // an empty cluster keeps its centroid until the split
      y = Y[(int64_t)c * ldy + col];
    } else {
      y = (float)(s / (double)n_c);
      Y[(int64_t)c * ldy + col] = y;
    }
  }
  if (y_absmax) block_absmax(y, y_absmax);
}

// Y = S / size for every cluster with points (an empty one keeps its row), max |Y| into *y_absmax (zero before).
__global__ void __launch_bounds__(256) means_from_sums_kernel(const double *S, const int32_t *cnt, int32_t ds, float *Y,
                                                              int64_t ldy, unsigned int *y_absmax) {
  const int c = blockIdx.x;
  const int n_c = cnt[c];
  const int col = blockIdx.y * 256 + threadIdx.x;
  float y = 0.f;
  if (col < ds) {
    if (n_c == 0) {
      y = Y[(int64_t)c * ldy + col];
    } else {
      y = (float)(S[(int64_t)c * ds + col] / (double)n_c);
      Y[(int64_t)c * ldy + col] = y;
    }
  }
  if (y_absmax) block_absmax(y, y_absmax);
}
hipError_t launch_means_from_sums(const double *S, const int32_t *cnt, int32_t k, int32_t ds, float *Y, int64_t ldy,
                                  unsigned int *y_absmax, hipStream_t st) {
  if (y_absmax) {
    hipError_t rc = hipMemsetAsync(y_absmax, 0, sizeof(unsigned int), st);
    if (rc != hipSuccess) return rc;
  }
  hipLaunchKernelGGL(means_from_sums_kernel, dim3(k, (unsigned)((ds + 255) / 256)), dim3(256), 0, st, S, cnt, ds, Y, ldy,
                     y_absmax);
  return hipGetLastError();
}

// Points whose label changed: entry (i, new label) and entry (~i, old label), in any order (the segments are
// sorted afterwards).  *counter must be 0; entries past `cap` are dropped and show in the final *counter.
__global__ void __launch_bounds__(256) compact_changes_kernel(const int32_t *assign, const int32_t *prev, int64_t n,
                                                              int32_t *ent_id, int32_t *ent_lab, unsigned int *counter,
                                                              unsigned int cap) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const int a = assign[i], b = prev[i];
    if (a != b) {
      const unsigned int e = atomicAdd(counter, 2u);
      if (e + 2u <= cap) {
        ent_id[e] = (int32_t)i;
        ent_lab[e] = a;
        ent_id[e + 1] = ~(int32_t)i;
        ent_lab[e + 1] = b;
      }
    }
  }
}

hipError_t launch_update(const float *Xr, int64_t ldx, int64_t n, int32_t ds, const int32_t *assign, int32_t k,
                         const UpdateWs &w, float *Y, int64_t ldy, hipStream_t st, double *S, unsigned int *y_absmax,
                         int accumulate) {
  if ((accumulate && !S) || (!Y && y_absmax)) return hipErrorInvalidValue;
  if (y_absmax) {
    hipError_t rc = hipMemsetAsync(y_absmax, 0, sizeof(unsigned int), st);
    if (rc != hipSuccess) return rc;
  }
  hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(1024), 0, st, w.cnt, k, w.off, w.cursor, w.segoff);
  int64_t blocks = (n + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(scatter_order_kernel, dim3((unsigned)blocks), dim3(256), 0, st, assign, n, w.off, w.cursor,
                     w.order, (const int32_t *)nullptr);
  hipLaunchKernelGGL(sort_segments_kernel, dim3(k), dim3(256), 0, st, w.off, w.order);
  const unsigned slices4 = (unsigned)((ds + 255) / 256);   // 64 lanes x 4 dims per workgroup
  hipLaunchKernelGGL(segment_sum_kernel<false>, dim3((unsigned)w.max_segments, slices4), dim3(256), 0, st, Xr, ldx, ds, k,
                     w.off, w.segoff, w.order, w.partial);
  const unsigned slices1 = (unsigned)((ds + 255) / 256);
  hipLaunchKernelGGL(centroid_mean_kernel, dim3(k, slices1), dim3(256), 0, st, w.partial, ds, w.cnt, w.segoff, Y, ldy, S,
                     accumulate, y_absmax);
  return hipGetLastError();
}

// order[] = the point ids grouped by label (members of a cluster of at most SORT_CAP points in ascending order), off[] the
// start of every group, cnt[] the group sizes: the first half of launch_update, for callers that only want the grouping.
hipError_t launch_group_order(const int32_t *labels, int64_t n, int32_t k, int32_t *cnt, int32_t *off, int32_t *cursor,
                              int32_t *segoff, int32_t *order, hipStream_t st) {
  hipError_t rc = launch_fill_u32(reinterpret_cast<unsigned int *>(cnt), k, 0u, st);
  if (rc != hipSuccess) return rc;
  rc = launch_histogram(labels, n, cnt, st);
  if (rc != hipSuccess) return rc;
  hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(1024), 0, st, cnt, k, off, cursor, segoff);
  int64_t blocks = (n + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  hipLaunchKernelGGL(scatter_order_kernel, dim3((unsigned)blocks), dim3(256), 0, st, labels, n, off, cursor, order,
                     (const int32_t *)nullptr);
  hipLaunchKernelGGL(sort_segments_kernel, dim3(k), dim3(256), 0, st, off, order);
  return hipGetLastError();
}

// The same update from the points that changed label only: S (the cluster sums of the previous update) takes the
// rows of the points that joined minus those of the points that left, and every centroid is S / size again.
// w.cnt holds the new cluster sizes; `changed` is the number of points with assign != prev (known to the host from
// the assignment step), inc is a workspace for 2 * changed entries.
hipError_t launch_update_incremental(const float *Xr, int64_t ldx, int64_t n, int32_t ds, const int32_t *assign,
                                     const int32_t *prev, int64_t changed, int32_t k, const UpdateWs &w,
                                     const IncUpdateWs &inc, double *S, float *Y, int64_t ldy, hipStream_t st,
                                     unsigned int *y_absmax) {
  const int64_t m2 = 2 * changed;
  if (m2 > inc.capacity || !S) return hipErrorInvalidValue;
  hipError_t rc = hipMemsetAsync(inc.counter, 0, sizeof(unsigned int), st);
  if (rc != hipSuccess) return rc;
  if (y_absmax) {
    rc = hipMemsetAsync(y_absmax, 0, sizeof(unsigned int), st);
    if (rc != hipSuccess) return rc;
  }
  rc = hipMemsetAsync(inc.cnt, 0, sizeof(int32_t) * (size_t)k, st);
  if (rc != hipSuccess) return rc;
  int64_t blocks = std::min<int64_t>((n + 255) / 256, 16384);
  hipLaunchKernelGGL(compact_changes_kernel, dim3((unsigned)blocks), dim3(256), 0, st, assign, prev, n, inc.ent_id,
                     inc.ent_lab, inc.counter, (unsigned int)inc.capacity);
  if (m2 > 0) {
    rc = launch_histogram(inc.ent_lab, m2, inc.cnt, st);
    if (rc != hipSuccess) return rc;
  }
  hipLaunchKernelGGL(scan_counts_kernel, dim3(1), dim3(1024), 0, st, inc.cnt, k, inc.off, inc.cursor, inc.segoff);
  if (m2 > 0) {
    blocks = std::min<int64_t>((m2 + 255) / 256, 16384);
    hipLaunchKernelGGL(scatter_order_kernel, dim3((unsigned)blocks), dim3(256), 0, st, inc.ent_lab, m2, inc.off, inc.cursor,
                       inc.order, (const int32_t *)inc.ent_id);
    hipLaunchKernelGGL(sort_segments_kernel, dim3(k), dim3(256), 0, st, inc.off, inc.order);
    const unsigned slices4 = (unsigned)((ds + 255) / 256);   // 64 lanes x 4 dims per workgroup
    const int64_t segs = std::min<int64_t>(inc.max_segments, (int64_t)k + m2 / kSegPoints + 1);
    hipLaunchKernelGGL(segment_sum_kernel<true>, dim3((unsigned)segs, slices4), dim3(256), 0, st, Xr, ldx, ds, k, inc.off,
                       inc.segoff, inc.order, inc.partial);
  }
  const unsigned slices1 = (unsigned)((ds + 255) / 256);
  hipLaunchKernelGGL(centroid_mean_kernel, dim3(k, slices1), dim3(256), 0, st, inc.partial, ds, w.cnt, inc.segoff, Y, ldy,
                     S, 1, y_absmax);
  return hipGetLastError();
}

// ------------------------------------------------------------------ split of empty clusters
// pairs = (empty, donor) in the order decided on the host.  A donor may be used twice and a re-seeded cluster may
// itself donate later, so the splits of one chain (splits that share clusters, grouped by the host) are applied one
// after the other by one workgroup; chains touch disjoint rows and run side by side.
__global__ void __launch_bounds__(256) split_kernel(float *Y, int64_t ldy, int32_t d, const int32_t *pairs,
                                                    const int32_t *chain_first, float eps) {
  const int s0 = chain_first[blockIdx.x], s1 = chain_first[blockIdx.x + 1];
  for (int s = s0; s < s1; ++s) {
    const int e = pairs[2 * s], c = pairs[2 * s + 1];
    for (int j = threadIdx.x; j < d; j += 256) {
      const float sg = (j & 1) ? -1.f : 1.f;
      const float y = Y[(int64_t)c * ldy + j];
      Y[(int64_t)e * ldy + j] = y * (1.f + eps * sg);
      Y[(int64_t)c * ldy + j] = y * (1.f - eps * sg);
    }
    __syncthreads();
  }
}
hipError_t launch_split(float *Y, int64_t ldy, int32_t d, const int32_t *pairs_dev, const int32_t *chain_first_dev,
                        int32_t nchains, float eps, hipStream_t st) {
  if (nchains <= 0) return hipSuccess;
  hipLaunchKernelGGL(split_kernel, dim3((unsigned)nchains), dim3(256), 0, st, Y, ldy, d, pairs_dev, chain_first_dev, eps);
  return hipGetLastError();
}

// ------------------------------------------------------------------ small copies
__global__ void __launch_bounds__(256) gather_rows_kernel(const float *src, int64_t lds, int32_t d,
                                                          const int64_t *idx, float *dst, int64_t ldd, int32_t dpad) {
  const int c = blockIdx.x;
  const float *s = src + idx[c] * lds;
  for (int j = threadIdx.x; j < dpad; j += 256) dst[(int64_t)c * ldd + j] = j < d ? s[j] : 0.f;
}
hipError_t launch_gather_rows(const float *src, int64_t lds, int32_t d, const int64_t *idx_dev, int32_t k, float *dst,
                              int64_t ldd, int32_t dpad, hipStream_t st) {
  hipLaunchKernelGGL(gather_rows_kernel, dim3(k), dim3(256), 0, st, src, lds, d, idx_dev, dst, ldd, dpad);
  return hipGetLastError();
}

// dst[i][j] = src[i][j] (or src[j][i] when transpose) for j < d, 0 for d <= j < dpad
__global__ void __launch_bounds__(256) pad_copy_kernel(const float *src, int64_t lds, int64_t n, int32_t d, float *dst,
                                                       int64_t ldd, int32_t dpad, int32_t transpose) {
  const int64_t total = n * dpad;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t i = t / dpad;
    const int j = (int)(t - i * dpad);
    float v = 0.f;
    if (j < d) v = transpose ? src[(int64_t)j * lds + i] : src[i * lds + j];
    dst[i * ldd + j] = v;
  }
}
hipError_t launch_pad_copy(const float *src, int64_t lds, int64_t n, int32_t d, float *dst, int64_t ldd, int32_t dpad,
                           int32_t transpose, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n * dpad + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(pad_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, st, src, lds, n, d, dst, ldd, dpad,
                     transpose);
  return hipGetLastError();
}

}  // namespace skm
