// Small kernels: residual update + RMS normalisation between blocks (wiring of
// the multi-layer workloads, not part of the paper's method) and the update of
// the device-side residency table.
#include "device_utils.h"
#include "launch.h"

namespace adapmoe {

constexpr int kNormThreads = 256;

// h[b] += gamma * y[b]; x[b] = h[b] / sqrt(mean(h[b]^2) + 1e-6), one workgroup per token.
template <bool BF16>
__global__ __launch_bounds__(kNormThreads) void residual_rmsnorm_kernel(float* h, const float* y, float gamma, void* x, int H) {
  __shared__ float part[kNormThreads / kWave];
  const int b = blockIdx.x, tid = threadIdx.x;
  float* hr = h + (size_t)b * H;
  const float* yr = y ? y + (size_t)b * H : nullptr;
  float ss = 0.f;
  for (int i = tid; i < H; i += kNormThreads) {
    float v = hr[i];
    if (yr) {
      v = fmaf(gamma, yr[i], v);
      hr[i] = v;
    }
    ss = fmaf(v, v, ss);
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) part[tid >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < kNormThreads / kWave; ++i) tot += part[i];
  const float inv = 1.0f / sqrtf(tot / (float)H + 1e-6f);
  for (int i = tid; i < H; i += kNormThreads) {
    const float v = hr[i] * inv;
    if (BF16) static_cast<uint16_t*>(x)[(size_t)b * H + i] = f32_to_bf16_bits(v);
    else static_cast<float*>(x)[(size_t)b * H + i] = v;
  }
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
