// Selection kernels for Early Termination by Recall (Section 3.3): exact top-K ground truth of the
// queries over the points, and the recall of an IVF search that probes the nearest centroids.
// The score matrices come from the MFMA GEMM; these kernels only select.
#include "skm_internal.h"

namespace skm {

__device__ inline unsigned long long block_min_u64(unsigned long long v, unsigned long long *red) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) {
    const unsigned long long o = __shfl_xor(v, m, 64);
    v = o < v ? o : v;
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long r = red[0];
  for (int w = 1; w < (int)(blockDim.x >> 6); ++w) r = red[w] < r ? red[w] : r;
  return r;
}

// Keys are (order-preserving distance bits << 32 | index); the running list of each query and the new
// score row are treated as one candidate set, from which the K smallest keys are drawn one at a time
// (each round takes the smallest key above the previous one: ties resolve to the lowest index).
// Once the running list is full, a column can only enter it with a key below the list's largest: one pass over the
// row collects those columns in LDS (after the first chunks there are few) and the K rounds run over them instead of
// over the whole row; a row with more candidates than the buffer holds falls back to rounds over the row.
constexpr int TOPK_CAND = 4096;
__global__ void __launch_bounds__(256) topk_merge_kernel(const float *S, int64_t lds, int32_t m, int64_t col_base,
                                                         const float *colnorm, int32_t K, unsigned long long *top) {
  __shared__ unsigned long long red[4];
  __shared__ unsigned long long s_new[256];
  __shared__ unsigned long long s_cand[TOPK_CAND];
  __shared__ unsigned int s_ncand;
  const int q = blockIdx.x;
  const float *row = S + (int64_t)q * lds;
  unsigned long long *mine = top + (int64_t)q * K;
  auto key_of = [&](int c) {
    const float v = colnorm[col_base + c] - 2.f * row[c];
    return ((unsigned long long)f2ord(v) << 32) | (unsigned long long)(uint32_t)(col_base + c);
  };
  const unsigned long long kth = mine[K - 1];   // ~0 while the list is not full: then every column is a candidate
  if (threadIdx.x == 0) s_ncand = 0u;
  __syncthreads();
  bool filtered = false;
  if (kth != ~0ull) {
    for (int c = threadIdx.x; c < m; c += 256) {
      const unsigned long long key = key_of(c);
      if (key < kth) {
        const unsigned int pos = atomicAdd(&s_ncand, 1u);
        if (pos < (unsigned int)TOPK_CAND) s_cand[pos] = key;
      }
    }
    __syncthreads();
    filtered = s_ncand <= (unsigned int)TOPK_CAND;
  }
  const int ncand = filtered ? (int)s_ncand : m;
  unsigned long long last = 0ull;
  bool first = true;
  for (int r = 0; r < K; ++r) {
    unsigned long long best = ~0ull;
    for (int c = threadIdx.x; c < ncand; c += 256) {
      const unsigned long long key = filtered ? s_cand[c] : key_of(c);
      if ((first || key > last) && key < best) best = key;
    }
    if ((int)threadIdx.x < K) {
      const unsigned long long key = mine[threadIdx.x];
      if ((first || key > last) && key < best) best = key;
    }
    best = block_min_u64(best, red);
    if (threadIdx.x == 0) s_new[r] = best;
    last = best;
    first = false;
    if (best == ~0ull) {
      for (int rr = r + 1; rr < K; ++rr)
        if (threadIdx.x == 0) s_new[rr] = ~0ull;
      break;
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < K) mine[threadIdx.x] = s_new[threadIdx.x];
}

hipError_t launch_topk_merge(const float *S, int64_t lds, int32_t nq, int32_t m, int64_t col_base,
                             const float *colnorm, int32_t K, unsigned long long *top, hipStream_t st) {
  if (K > 256 || K < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(topk_merge_kernel, dim3(nq), dim3(256), 0, st, S, lds, m, col_base, colnorm, K, top);
  return hipGetLastError();
}

// One workgroup per query.  S[q][c] = q . y_c; the centroid order by distance is the order of
// ynorm[c] - 2 S[q][c].  The nprobe nearest centroids are drawn one at a time into LDS, then every
// ground-truth neighbour is looked up: it is retrieved iff its cluster is probed.
constexpr int MAX_PROBE = kMaxProbe;
__global__ void __launch_bounds__(256) recall_kernel(const float *S, int64_t lds, int32_t k, const float *ynorm,
                                                     int32_t nprobe, const unsigned long long *gt_keys, int32_t K,
                                                     const int32_t *assign, unsigned long long *hits,
                                                     unsigned long long *total) {
  __shared__ unsigned long long red[4];
  __shared__ int32_t s_probe[MAX_PROBE];
  __shared__ unsigned int s_hits, s_total;
  const int q = blockIdx.x;
  const float *row = S + (int64_t)q * lds;
  if (threadIdx.x == 0) { s_hits = 0; s_total = 0; }
  unsigned long long last = 0ull;
  for (int r = 0; r < nprobe; ++r) {
    unsigned long long best = ~0ull;
    for (int c = threadIdx.x; c < k; c += 256) {
      const unsigned long long key = ((unsigned long long)f2ord(ynorm[c] - 2.f * row[c]) << 32) | (unsigned long long)(uint32_t)c;
      if ((r == 0 || key > last) && key < best) best = key;
    }
    best = block_min_u64(best, red);
    if (threadIdx.x == 0) s_probe[r] = (int32_t)(best & 0xffffffffull);
    last = best;
  }
  __syncthreads();
  for (int g = 0; g < K; ++g) {
    const unsigned long long key = gt_keys[(int64_t)q * K + g];
    if (key == ~0ull) continue;
    const int32_t cl = assign[(int64_t)(key & 0xffffffffull)];
    bool found = false;
    for (int s = threadIdx.x; s < nprobe; s += 256) found |= (s_probe[s] == cl);
    if (__any(found) && (threadIdx.x & 63) == 0) atomicAdd(&s_hits, 1u);   // a cluster appears once in the list
    if (threadIdx.x == 0) s_total += 1;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    atomicAdd(hits, (unsigned long long)s_hits);
    atomicAdd(total, (unsigned long long)s_total);
  }
}

hipError_t launch_recall_scores(const float *S, int64_t lds, int32_t nq, int32_t k, const float *ynorm, int32_t nprobe,
                                const unsigned long long *gt_keys, int32_t K, const int32_t *assign,
                                unsigned long long *hits, unsigned long long *total, hipStream_t st) {
  if (nprobe > MAX_PROBE || nprobe < 1) return hipErrorInvalidValue;
  hipLaunchKernelGGL(recall_kernel, dim3(nq), dim3(256), 0, st, S, lds, k, ynorm, nprobe, gt_keys, K, assign, hits,
                     total);
  return hipGetLastError();
}

// ||row||^2 for n rows of length d (any alignment): one wavefront per row.
__global__ void __launch_bounds__(256) row_norms_kernel(const float *X, int64_t ldx, int64_t n, int32_t d, float *out) {
  const int lane = threadIdx.x & 63;
  const int64_t nw = (int64_t)gridDim.x * 4;
  for (int64_t i = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); i < n; i += nw) {
    const float *x = X + i * ldx;
    float s = 0.f;
    for (int j = lane; j < d; j += 64) s = fmaf(x[j], x[j], s);
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) s += __shfl_xor(s, m, 64);
    if (lane == 0) out[i] = s;
  }
}
hipError_t launch_row_norms(const float *X, int64_t ldx, int64_t n, int32_t d, float *out, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  int64_t blocks = (n + 3) / 4;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(row_norms_kernel, dim3((unsigned)blocks), dim3(256), 0, st, X, ldx, n, d, out);
  return hipGetLastError();
}

// keys (distance bits << 32 | index) -> int64 indices, -1 for missing
__global__ void keys_to_index_kernel(const unsigned long long *keys, int64_t n, int64_t *idx) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) idx[i] = keys[i] == ~0ull ? -1 : (int64_t)(keys[i] & 0xffffffffull);
}
__global__ void index_to_keys_kernel(const int64_t *idx, int64_t n, unsigned long long *keys) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) keys[i] = idx[i] < 0 ? ~0ull : (unsigned long long)idx[i];
}
hipError_t launch_keys_to_index(const unsigned long long *keys, int64_t n, int64_t *idx, hipStream_t st) {
  hipLaunchKernelGGL(keys_to_index_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, keys, n, idx);
  return hipGetLastError();
}
hipError_t launch_index_to_keys(const int64_t *idx, int64_t n, unsigned long long *keys, hipStream_t st) {
  hipLaunchKernelGGL(index_to_keys_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, idx, n, keys);
  return hipGetLastError();
}

}  // namespace skm
