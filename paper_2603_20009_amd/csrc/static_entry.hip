// Entry point that allocates nothing: the exact assignment step (Algorithm 1, iteration 1) for callers that cannot
// call hipMalloc (code under HIP graph capture, tight serving loops, harnesses that forbid it).  It runs the kernels of
// skm_assign_exact; what that call takes from hipMalloc (the packed minima, the centroid norms, the operand bounds and
// the split-fp16 copy of the centroids) lives here in a file-scope device array instead.
#include "../../include/skm.h"
#include "skm_internal.h"

#include <mutex>

namespace {

constexpr size_t kScratchBytes = (size_t)16 << 20;          // held by every device the library runs on, for good
constexpr size_t kOffBest = 0;                               // [n] packed (distance, centroid), n <= kMaxPoints
constexpr size_t kOffYnorm = (size_t)8 << 20;                // [k] centroid norms, k <= kMaxCentroids
constexpr size_t kOffAmax = kOffYnorm + ((size_t)64 << 10);  // [2] magnitude bounds of the two operands
constexpr size_t kOffSplit = kOffAmax + ((size_t)64 << 10);  // split-fp16 copy of the centroids, if it fits
constexpr int64_t kMaxPoints = (int64_t)1 << 20;
constexpr int32_t kMaxCentroids = 1 << 14;
constexpr size_t kSplitWords = (kScratchBytes - kOffSplit) / sizeof(uint32_t);
static_assert(kOffYnorm >= (size_t)kMaxPoints * sizeof(unsigned long long), "best[] fits");
static_assert(kOffAmax - kOffYnorm >= (size_t)kMaxCentroids * sizeof(float), "ynorm[] fits");

// In host code this name is only a handle for hipGetSymbolAddress: the device address is looked up once per device
// (every device holds its own copy of the array) and only that address is ever handed to a kernel or a copy.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_mu;
unsigned char *g_scratch_ptr[kMaxDevices] = {nullptr};

// device address of `scratch` on the current device
int scratch_address(unsigned char **out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return skm::report_hip_error(e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return skm::report_error(SKM_EINVAL, "device ordinal out of range");
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return skm::report_hip_error(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
  }
  *out = g_scratch_ptr[dev];
  return SKM_OK;
}

#define HIPCHK(expr)                                                     \
  do {                                                                   \
    hipError_t e__ = (expr);                                             \
    if (e__ != hipSuccess) return skm::report_hip_error(e__, #expr);     \
  } while (0)

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int skm_assign_exact_static(const float *X, int64_t n, int32_t d, const float *centroids, int32_t k, void *stream,
                            int32_t *assign_out, float *dist_out) {
  using namespace skm;
  if (!X || !centroids || !assign_out) return report_error(SKM_EINVAL, "null pointer");
  if (n < 1 || n > kMaxPoints) return report_error(SKM_EINVAL, "skm_assign_exact_static: n out of range [1, 1048576]");
  if (k < 1 || k > kMaxCentroids) return report_error(SKM_EINVAL, "skm_assign_exact_static: k out of range [1, 16384]");
  if (d < 16 || d > 16384 || d % 16 != 0)
    return report_error(SKM_EINVAL, "skm_assign_exact_static: d must be a multiple of 16 in [16, 16384]");
  if ((reinterpret_cast<uintptr_t>(X) & 15u) || (reinterpret_cast<uintptr_t>(centroids) & 15u))
    return report_error(SKM_EINVAL, "skm_assign_exact_static: X and centroids must be 16-byte aligned");
  unsigned char *base = nullptr;
  if (int rc = scratch_address(&base)) return rc;
  hipStream_t st = (hipStream_t)stream;
  unsigned long long *best = reinterpret_cast<unsigned long long *>(base + kOffBest);
  float *ynorm = reinterpret_cast<float *>(base + kOffYnorm);
  unsigned int *amax = reinterpret_cast<unsigned int *>(base + kOffAmax);
  uint32_t *split = reinterpret_cast<uint32_t *>(base + kOffSplit);
  // the array keeps what the last call left: everything read below is written first (fill kernels, no memset nodes)
  HIPCHK(launch_prep_centroids(centroids, d, k, d, d, ynorm, 0, 0, nullptr, st));
  HIPCHK(launch_fill_u64(best, n, ~0ull, st));
  HIPCHK(launch_fill_u32(amax, 2, 0u, st));
  HIPCHK(launch_absmax(X, d, n, d, amax, st));
  HIPCHK(launch_absmax(centroids, d, k, d, amax + 1, st));
  GemmOperands g{X, d, (int32_t)n, centroids, d, k, d};
  g.a_absmax = amax;
  g.b_absmax = amax + 1;
  if (d % 32 == 0 && (size_t)k * ((size_t)d + 32) <= kSplitWords) g.b_split = split;
  HIPCHK(gemm_argmin(g, ynorm, best, st));
  HIPCHK(launch_finalize_assign(best, nullptr, n, assign_out, nullptr, nullptr, k, nullptr, nullptr, nullptr, st));
  if (dist_out) HIPCHK(launch_tau_init(X, d, n, d, centroids, d, assign_out, dist_out, nullptr, st));
  HIPCHK(hipStreamSynchronize(st));
  return SKM_OK;
}

#pragma GCC visibility pop
}
