// Small kernels: residual update + RMS normalisation between blocks (wiring of
// the multi-layer workloads, not part of the paper's method) and the update of
// the device-side residency table.
#include "device_utils.h"
#include "launch.h"
#include "norm_core.h"

namespace adapmoe {

// h[b] += gamma * y[b]; x[b] = h[b] / sqrt(mean(h[b]^2) + 1e-6), one workgroup per token.
template <bool BF16>
__global__ __launch_bounds__(kNormThreads) void residual_rmsnorm_kernel(float* h, const float* y, float gamma, void* x, int H) {
  __shared__ float part[kNormThreads / kWave];
  const int b = blockIdx.x;
  void* xrow = static_cast<char*>(x) + (size_t)b * H * (BF16 ? 2 : 4);
  uint4 xk[kNormKeep];
  (void)residual_rmsnorm_row<BF16>(h + (size_t)b * H, y ? y + (size_t)b * H : nullptr, gamma, xrow, H, part, xk);
}

hipError_t launch_residual_rmsnorm(float* h, const float* y, float gamma, void* x, bool bf16, int B, int H, hipStream_t s) {
  if (bf16) hipLaunchKernelGGL(residual_rmsnorm_kernel<true>, dim3(B), dim3(kNormThreads), 0, s, h, y, gamma, x, H);
  else hipLaunchKernelGGL(residual_rmsnorm_kernel<false>, dim3(B), dim3(kNormThreads), 0, s, h, y, gamma, x, H);
  return hipGetLastError();
}

// *addr[i] = value[i]: residency changes (table entries, resolved expert
// pointers) are ordered on the compute stream with the kernels that read them.
__global__ void poke_kernel(PokeArgs p) {
  const int i = threadIdx.x;
  if (i < p.n) *p.addr[i] = p.value[i];
}

hipError_t launch_poke(const PokeArgs& p, hipStream_t s) {
  hipLaunchKernelGGL(poke_kernel, dim3(1), dim3(64), 0, s, p);
  return hipGetLastError();
}

}  // namespace adapmoe
