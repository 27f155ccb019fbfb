// PRUNING phase (Algorithm 1, loop over PDX blocks; Section 3.4 "Progressive Pruning").
//
// Input is the list of (point, centroid) pairs that passed the first test.  A pair is owned by a
// group of 16 lanes: one 64-dimension block of the point (256 contiguous bytes of the rotated row)
// and of the centroid (256 contiguous bytes of the block-major centroid copy) is one float4 per
// lane, so every load instruction of a wavefront moves four full 256-byte segments.  After each
// block the group adds the block's squared distance, compares with theta(t, tau) and either drops
// the pair, goes on to the next block, or - at t = d - offers the finished distance to the point's
// packed (distance, centroid) minimum.  A group that is done with a pair takes the next one of its
// stride at once, so lanes do not idle while other groups of the wavefront are still busy.
#include "skm_internal.h"

namespace skm {

// Sum over the 16 lanes of a DPP row; every lane receives the same bits (symmetric butterfly:
// swap within pairs, within quads, mirror the half row, mirror the row).
__device__ inline float row16_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
  return v;
}

constexpr int PRUNE_THREADS = 256;

template <bool STATS>
__global__ void __launch_bounds__(PRUNE_THREADS) prune_kernel(PruneArgs a) {
  __shared__ float s_ratio[kMaxBlocks + 1];
  __shared__ unsigned int s_enter[kMaxBlocks + 1];
  __shared__ unsigned int s_completed;
  const int tid = threadIdx.x;
  for (int m = tid; m <= a.nb; m += PRUNE_THREADS) {
    s_ratio[m] = a.ratio[m];
    s_enter[m] = 0u;
  }
  if (tid == 0) s_completed = 0u;
  __syncthreads();

  // the list is kSubLists parts; a flat index p walks them in order
  unsigned int cum[kSubLists + 1];
  cum[0] = 0u;
#pragma unroll
  for (int sl = 0; sl < kSubLists; ++sl) cum[sl + 1] = cum[sl] + a.count[sl * kSubListStride];
  const unsigned int total = cum[kSubLists];
  const unsigned int ngroups = gridDim.x * (PRUNE_THREADS / 16);
  const int q = tid & 15;
  unsigned int p = blockIdx.x * (PRUNE_THREADS / 16) + (tid >> 4);
  bool active = p < total;
  int i = 0, j = 0, m = 0;
  float acc = 0.f, tau = 0.f;
  auto fetch = [&]() {
    unsigned int sl = 0;
#pragma unroll
    for (int t = 1; t < kSubLists; ++t) sl += (p >= cum[t]);
    const Pair pr = a.pairs[(size_t)sl * a.sub_capacity + (p - cum[sl])];
    const unsigned int jm = (unsigned int)pr.j;
    i = pr.i;
    j = (int)(jm & 0xffffffu);
    m = (int)(jm >> 24);   // first block still to be added
    acc = pr.p;
    tau = pr.tau;
  };
  if (active) fetch();
  while (__any(active)) {
    if (active) {
      if (m < a.nb) {
        const int col = a.dprime + kBlockDims * m + 4 * q;
        float4 xv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (col < a.ds) xv = *reinterpret_cast<const float4 *>(a.Xr + (int64_t)i * a.ldx + col);
        const float4 yv = *reinterpret_cast<const float4 *>(a.Ypdx + ((int64_t)m * a.k + j) * kBlockDims + 4 * q);
        const float dx = xv.x - yv.x, dy = xv.y - yv.y, dz = xv.z - yv.z, dw = xv.w - yv.w;
        float s = dx * dx;
        s = fmaf(dy, dy, s);
        s = fmaf(dz, dz, s);
        s = fmaf(dw, dw, s);
        acc += row16_sum(s);
        ++m;
      }
      const bool done = m >= a.nb;
      bool drop = false;
      if (done) {
        if (q == 0) {
          atomicAdd(&s_completed, 1u);
          if (acc < tau) atomicMin(a.best + i, pack_key(acc, j));
        }
      } else {
        drop = acc > s_ratio[m] * tau;   // checkpoint m: t = d' + 64 m dimensions seen
        if (STATS && !drop && q == 0) atomicAdd(&s_enter[m], 1u);
      }
      if (done || drop) {
        p += ngroups;
        active = p < total;
        if (active) fetch();
      }
    }
  }
  __syncthreads();
  unsigned long long *sc = a.scal + (size_t)(blockIdx.x & (kStatReplicas - 1)) * SC_COUNT;
  if (tid == 0 && s_completed) atomicAdd(sc + SC_COMPLETED, (unsigned long long)s_completed);
  if (STATS) {
    for (int mm = tid; mm < a.nb; mm += PRUNE_THREADS)
      if (s_enter[mm]) atomicAdd(sc + SC_ENTER + mm, (unsigned long long)s_enter[mm]);
  }
}

hipError_t launch_prune(const PruneArgs &a, hipStream_t st) {
  if (a.nb > kMaxBlocks) return hipErrorInvalidValue;
  int dev = 0, cus = 256;
  (void)hipGetDevice(&dev);
  (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  const unsigned grid = (unsigned)cus * 8u;  // 8 workgroups of 4 waves per CU = full occupancy at <= 64 VGPRs
  if (a.block_stats)
    hipLaunchKernelGGL(prune_kernel<true>, dim3(grid), dim3(PRUNE_THREADS), 0, st, a);
  else
    hipLaunchKernelGGL(prune_kernel<false>, dim3(grid), dim3(PRUNE_THREADS), 0, st, a);
  return hipGetLastError();
}

}  // namespace skm
