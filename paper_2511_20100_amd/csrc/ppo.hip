// Clipped surrogate of the PPO update over scored samples (value and two diagnostics, no gradient).
// Two launches: per-workgroup partial sums in double, then one workgroup adds the partials; both
// reductions run in a fixed order, so the result does not depend on scheduling.
#include <mutex>

#include "common.h"
#include "kernels.h"

namespace mtmc {

namespace {

constexpr int kPpoBlocks = 1024;   // partial results at most
constexpr int kPpoThreads = 256;

struct PpoSums {
  double surrogate, clipped, kl, count;
};

__device__ __forceinline__ PpoSums ppo_add(const PpoSums& a, const PpoSums& b) {
  return PpoSums{a.surrogate + b.surrogate, a.clipped + b.clipped, a.kl + b.kl, a.count + b.count};
}

// Sum over the workgroup in a fixed tree; the result is valid in thread 0.
__device__ __forceinline__ PpoSums ppo_block_sum(PpoSums v, PpoSums* red) {
  red[threadIdx.x] = v;
  __syncthreads();
  for (int w = kPpoThreads / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] = ppo_add(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  return red[0];
}

__global__ __launch_bounds__(kPpoThreads) void k_ppo_partial(const float* new_logp, const float* old_logp,
                                                             const float* adv, const int* mask, long long n,
                                                             double eps, PpoSums* partial) {
  __shared__ PpoSums red[kPpoThreads];
  PpoSums s{0.0, 0.0, 0.0, 0.0};
  for (long long i = (long long)blockIdx.x * kPpoThreads + threadIdx.x; i < n; i += (long long)gridDim.x * kPpoThreads) {
    if (mask && mask[i] == 0) continue;
    const double d = (double)new_logp[i] - (double)old_logp[i];
    const double r = exp(d), a = (double)adv[i];
    const double rc = fmin(fmax(r, 1.0 - eps), 1.0 + eps);
    s.surrogate += fmin(r * a, rc * a);
    s.clipped += (fabs(r - 1.0) > eps) ? 1.0 : 0.0;
    s.kl -= d;
    s.count += 1.0;
  }
  s = ppo_block_sum(s, red);
  if (threadIdx.x == 0) partial[blockIdx.x] = s;
}

__global__ __launch_bounds__(kPpoThreads) void k_ppo_final(const PpoSums* partial, int n_partial, double* out) {
  __shared__ PpoSums red[kPpoThreads];
  PpoSums s{0.0, 0.0, 0.0, 0.0};
  for (int i = threadIdx.x; i < n_partial; i += kPpoThreads) s = ppo_add(s, partial[i]);
  s = ppo_block_sum(s, red);
  if (threadIdx.x == 0) {
    const double c = s.count > 0.0 ? s.count : 1.0;
    out[0] = -s.surrogate / c;
    out[1] = s.clipped / c;
    out[2] = s.kl / c;
    out[3] = s.count;
  }
}

// Partial sums of the entry point that takes no workspace: one copy of this array per GPU, part of the loaded
// code object, alive until the process ends.  Host code never uses the array's name as an address: it asks the
// runtime for the device address once per device (ppo_static_scratch) and passes that to the kernels.
static __device__ __align__(256) unsigned char scratch[kPpoBlocks * sizeof(PpoSums)];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

}  // namespace

size_t ppo_workspace_bytes() { return kPpoBlocks * sizeof(PpoSums); }

// Device address of this GPU's copy of `scratch` (looked up on the first call on a device, with that device current).
int ppo_static_scratch(void** out) {
  int dev = -1;
  MTMC_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) {
    set_error("device index " + std::to_string(dev) + " is beyond the " + std::to_string(kMaxDevices) +
              " devices the static scratch table covers");
    return MTMC_EINVAL;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    MTMC_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) {
      set_error("hipGetSymbolAddress returned no address for the static scratch array");
      return MTMC_EHIP;
    }
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return MTMC_OK;
}

void launch_ppo_clip_loss(const float* new_logp, const float* old_logp, const float* adv, const int* mask,
                          long long n, double eps, double* out, void* workspace, hipStream_t st) {
  const long long want = (n + 4 * kPpoThreads - 1) / (4 * kPpoThreads);
  const int blocks = (int)(want < 1 ? 1 : want > kPpoBlocks ? kPpoBlocks : want);
  PpoSums* partial = reinterpret_cast<PpoSums*>(workspace);
  k_ppo_partial<<<blocks, kPpoThreads, 0, st>>>(new_logp, old_logp, adv, mask, n, eps, partial);
  k_ppo_final<<<1, kPpoThreads, 0, st>>>(partial, blocks, out);
}

}  // namespace mtmc
