// PRUNING phase (Algorithm 1, loop over PDX blocks; Section 3.4 "Progressive Pruning").
//
// Input is the list of (point, centroid) pairs that passed the first test.  A pair is owned by a
// group of 8 lanes: one 64-dimension block of the point (256 contiguous bytes of the rotated row)
// and of the centroid (256 contiguous bytes of the block-major centroid copy) is two float4 per
// lane, taken so that each load instruction moves a full 128-byte line per pair.  After each
// block the group adds the block's squared distance, compares with theta(t, tau) and either drops
// the pair, goes on to the next block, or - at t = d - offers the finished distance to the point's
// packed (distance, centroid) minimum.  A group that is done with a pair takes the next one of its
// stride at once (its list entry was requested one pair earlier), so lanes do not idle while other
// groups of the wavefront are still busy.  The kernel is bound by memory latency times the number
// of pairs in flight: eight pairs per wavefront instead of four took a steady step of the 1M x 1536, k = 1024
// workload from 1.38 to 1.24 ms.
#include "skm_internal.h"

namespace skm {

// Sum over 8 consecutive lanes; every lane receives the same bits (symmetric butterfly: swap within
// pairs, within quads, mirror the half row).
__device__ inline float row8_sum(float v) {
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  v += __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
  return v;
}

constexpr int PRUNE_THREADS = 256;
constexpr int PAIR_LANES = 8;

template <bool STATS>
__global__ void __launch_bounds__(PRUNE_THREADS) prune_kernel(PruneArgs a) {
  __shared__ float s_ratio[kMaxBlocks + 1];
  __shared__ unsigned int s_enter[kMaxBlocks + 1];
  __shared__ unsigned int s_completed, s_steps, s_pairs;
  const int tid = threadIdx.x;
  for (int m = tid; m <= a.nb; m += PRUNE_THREADS) {
    s_ratio[m] = a.ratio[m];
    s_enter[m] = 0u;
  }
  if (tid == 0) {
    s_completed = 0u;
    s_steps = 0u;
    s_pairs = 0u;
  }
  __syncthreads();
  unsigned int my_steps = 0u, my_pairs = 0u;   // (lane 0 of a group) block steps gathered and pairs taken: the kernel's traffic

  // The list is kSubLists parts, one per XCD of the kernel that made it (workgroup id mod 8), each in the order in
  // which that XCD walked its tiles: neighbouring entries share point rows and centroid blocks.  A workgroup reads
  // the part of its own XCD, so those rows and blocks are fetched into one L2 only and found there again.
  static_assert(kSubLists == 8, "one part per XCD");
  const unsigned int part = blockIdx.x & 7u;
  // (a producer that ran out of room has still counted what it could not write: never read past the part's end)
  const unsigned int total = min(a.count[part * kSubListStride], a.sub_capacity);
  const Pair *list = a.pairs + (size_t)part * a.sub_capacity;
  const unsigned int ngroups = (gridDim.x >> 3) * (PRUNE_THREADS / PAIR_LANES);
  const int q = tid & (PAIR_LANES - 1);
  unsigned int p = (blockIdx.x >> 3) * (PRUNE_THREADS / PAIR_LANES) + (tid / PAIR_LANES);
  bool active = p < total;
  int i = 0, j = 0, m = 0;
  float acc = 0.f, tau = 0.f;
  auto unpack = [&](const Pair &pr) {
    const unsigned int jm = (unsigned int)pr.j;
    i = pr.i;
    j = (int)(jm & 0xffffffu);
    m = (int)(jm >> 24);   // first block still to be added
    acc = pr.p;
    tau = pr.tau;
    // An entry that names no point or centroid is skipped (finished at once, offering nothing).  Every producer
    // writes valid entries only; but after a producer's overflow, which the host answers by redoing the step another
    // way, slots inside the counted range may never have been written.
    if ((unsigned int)i >= (unsigned int)a.n || j >= a.k || m > a.nb) {
      i = 0;
      j = 0;
      m = a.nb;
      acc = 1.f;
      tau = 0.f;
    }
  };
  if (active) {
    unpack(list[p]);
    ++my_pairs;
  }
  unsigned int pn = p + ngroups;   // the entry after this one, requested ahead of its use
  Pair nx = {0, 0, 0.f, 0.f};
  if (pn < total) nx = list[pn];
  while (__any(active)) {
    if (active) {
      if (m < a.nb) {
        // lane q holds float4 q and float4 q + 8 of the 16 in a block
        const int col = a.dprime + kBlockDims * m + 4 * q;
        const float *xp = a.Xr + (int64_t)i * a.ldx + col;
        const float *yp = a.Ypdx + ((int64_t)m * a.k + j) * kBlockDims + 4 * q;
        float4 x0 = make_float4(0.f, 0.f, 0.f, 0.f), x1 = x0;
        if (col < a.ds) x0 = *reinterpret_cast<const float4 *>(xp);
        if (col + 32 < a.ds) x1 = *reinterpret_cast<const float4 *>(xp + 32);
        const float4 y0 = *reinterpret_cast<const float4 *>(yp);
        const float4 y1 = *reinterpret_cast<const float4 *>(yp + 32);
        float dx = x0.x - y0.x, dy = x0.y - y0.y, dz = x0.z - y0.z, dw = x0.w - y0.w;
        float s = dx * dx;
        s = fmaf(dy, dy, s);
        s = fmaf(dz, dz, s);
        s = fmaf(dw, dw, s);
        dx = x1.x - y1.x; dy = x1.y - y1.y; dz = x1.z - y1.z; dw = x1.w - y1.w;
        s = fmaf(dx, dx, s);
        s = fmaf(dy, dy, s);
        s = fmaf(dz, dz, s);
        s = fmaf(dw, dw, s);
        acc += row8_sum(s);
        ++m;
        ++my_steps;
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
        p = pn;
        active = p < total;
        if (active) {
          unpack(nx);
          ++my_pairs;
          pn = p + ngroups;
          if (pn < total) nx = list[pn];
        }
      }
    }
  }
  if (q == 0) {
    if (my_steps) atomicAdd(&s_steps, my_steps);
    if (my_pairs) atomicAdd(&s_pairs, my_pairs);
  }
  __syncthreads();
  unsigned long long *sc = a.scal + (size_t)(blockIdx.x & (kStatReplicas - 1)) * SC_COUNT;
  if (tid == 0 && s_completed) atomicAdd(sc + SC_COMPLETED, (unsigned long long)s_completed);
  if (tid == 0 && s_steps) atomicAdd(sc + SC_GATHER_PB, (unsigned long long)s_steps);
  if (tid == 0 && s_pairs) atomicAdd(sc + SC_GATHER_PAIRS, (unsigned long long)s_pairs);
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
  const unsigned grid = (unsigned)cus * 8u;  // 8 workgroups of 4 waves per CU = full occupancy at <= 64 VGPRs; a multiple of 8
  if (a.block_stats)
    hipLaunchKernelGGL(prune_kernel<true>, dim3(grid), dim3(PRUNE_THREADS), 0, st, a);
  else
    hipLaunchKernelGGL(prune_kernel<false>, dim3(grid), dim3(PRUNE_THREADS), 0, st, a);
  return hipGetLastError();
}

}  // namespace skm
