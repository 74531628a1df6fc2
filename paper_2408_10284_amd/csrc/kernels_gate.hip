// Gate kernel: router product, softmax, top-2 and the adaptive activation test
// in one workgroup per (token, router); the decision itself is taken by one
// wavefront with DPP reductions and ballots.  Sec. 2.1 Eq.1 and Sec. 4.2 Eq.3, Eq.4,
// Eq.8 of the AdapMoE paper; router 1 is the following layer's, applied to the
// same input to predict its experts (Sec. 4.3).
#include "device_utils.h"
#include "launch.h"
#include "norm_core.h"

namespace adapmoe {

constexpr int kGateWaves = 8;
constexpr int kGateThreads = kGateWaves * kWave;

// One workgroup per (token, router).  The H axis is cut into 1 KiB runs dealt
// round-robin to the wavefronts, so all loads of a router matrix are in flight
// at once (the kernel is latency-bound: 2*N*H bytes per token).  Each wavefront
// reduces its partial logits with DPP, wavefront 0 adds the partials in a fixed
// order and takes the decision.
// xk != nullptr (bfloat16 only): the caller already holds this thread's 16-byte pieces of x, piece i
// being the one at element (threadIdx.x + i * kGateThreads) * 8, and x is not read from memory.
template <bool BF16>
__device__ __forceinline__ void gate_body(const GateArgs& a, int b, int r, float (*part)[64], const uint4* xk = nullptr) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int N = a.N, H = a.H;

  int32_t* ids_out = a.ids[r] + 2 * b;
  int32_t* k_out = a.k[r] + b;
  if (a.Wg[r] == nullptr) {  // no following layer: empty prediction
    if (threadIdx.x == 0) { ids_out[0] = -1; ids_out[1] = -1; *k_out = 0; }
    return;
  }

  // Requested now, used after the decision (a dependent load there would add a memory round trip
  // to a kernel that is all latency): the threshold and, for router 0, the residency-table entry of
  // expert e in lane e of the deciding wavefront.
  const float tau = a.tau[r];
  const bool want_table = r == 0 && a.res != nullptr;
  const void* tab = (want_table && wave == 0 && lane < N) ? a.table[lane] : nullptr;

  constexpr int VEC = BF16 ? 8 : 4;      // elements per 16-byte vector
  const size_t esz = BF16 ? 2 : 4;
  const char* xrow = static_cast<const char*>(a.x) + (size_t)b * H * esz;
  const char* W = static_cast<const char*>(a.Wg[r]);

  // partial z_e = sum over this wavefront's runs of x_h W_g[e,h], eight experts at a time
  for (int e0 = 0; e0 < N; e0 += 8) {
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    auto piece = [&](int c, const uint4& xv) {   // the 16-byte piece of x at element c against 8 router rows
      uint4 wv[8];
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e0 + e < N) wv[e] = *reinterpret_cast<const uint4*>(W + ((size_t)(e0 + e) * H + c) * esz);
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (e0 + e < N) {
          if (BF16) acc[e] = dot16_bf16(wv[e], xv, acc[e]);
          else acc[e] = dot16_f32(wv[e], __builtin_bit_cast(float4, xv), acc[e]);
        }
    };
    if (BF16 && xk != nullptr) {
#pragma unroll
      for (int i = 0; i < kNormKeep; ++i) {
        const int c = (threadIdx.x + i * kGateThreads) * VEC;
        if (c < H) piece(c, xk[i]);
      }
    } else {
      for (int c = (wave * kWave + lane) * VEC; c < H; c += kGateThreads * VEC)
        piece(c, *reinterpret_cast<const uint4*>(xrow + (size_t)c * esz));
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float s = wave_sum(acc[e]);
      if (lane == 0 && e0 + e < N) part[wave][e0 + e] = s;
    }
  }
  __syncthreads();
  if (wave != 0) return;

  // lane e holds logit e; top-1 / top-2 by wave maximum + ballot (lowest index wins ties)
  const bool live = lane < N;
  float z = -INFINITY;
  if (live) {
    z = 0.f;
#pragma unroll
    for (int w = 0; w < kGateWaves; ++w) z += part[w][lane];
  }
  const float m1 = wave_max(z);
  const uint64_t mask1 = __builtin_amdgcn_ballot_w64(live && z == m1);
  const int e1 = mask1 ? __builtin_ctzll(mask1) : 0;
  const float zr = (lane == e1) ? -INFINITY : z;
  const float m2 = wave_max(zr);
  const uint64_t mask2 = __builtin_amdgcn_ballot_w64(live && lane != e1 && zr == m2);
  const int e2 = mask2 ? __builtin_ctzll(mask2) : (e1 == 0 ? 1 : 0);

  // full softmax over the N logits, then the two selected scores renormalised
  const float ex = live ? expf(z - m1) : 0.f;
  const float S = wave_sum(ex);
  const float p1 = 1.0f / S;               // exp(m1 - m1) / S
  const float p2 = expf(m2 - m1) / S;
  const float alpha = p1 / (p1 + p2);
  const float v = p2 / (p1 + p2);          // weight of the second expert, the test value
  const int k = (v <= tau) ? 1 : 2;       // Eq.8 with tau = sqrt(T / sum diag(F))

  const void* tab1 = readlane_ptr(tab, e1);
  const void* tab2 = readlane_ptr(tab, e2);
  if (lane == 0) {
    ids_out[0] = e1;
    ids_out[1] = e2;
    *k_out = k;
    const float w0 = (k == 1) ? 1.0f : alpha, w1 = (k == 1) ? 0.0f : v;   // Eq.4 / Eq.3
    if (r == 0 && a.w != nullptr) {
      a.w[2 * b + 0] = w0;
      a.w[2 * b + 1] = w1;
    }
    if (want_table) {
      ResolvedExperts out;
      out.base[0] = tab1;
      out.base[1] = (k == 2) ? tab2 : nullptr;
      out.w[0] = w0;
      out.w[1] = w1;
      out.k = k;
      out.pad = 0;
      a.res[b] = out;
    }
  }
}

template <bool BF16>
__global__ __launch_bounds__(kGateThreads) void gate_kernel(GateArgs a) {
  __shared__ float part[kGateWaves][64];
  gate_body<BF16>(a, blockIdx.x, blockIdx.y, part);
}

// Residual update and RMS normalisation of the block input (the wiring between blocks of the
// multi-layer workloads) followed by the gate of one router, in one launch: the workgroup runs
// exactly the arithmetic of the separate normalisation kernel, then the gate on the x it has just
// written.  Same results as the two launches.
static_assert(kNormThreads == kGateThreads, "the normalisation and the gate share one workgroup shape");
template <bool BF16>
__global__ __launch_bounds__(kGateThreads) void norm_gate_kernel(GateArgs a, NormArgs n) {
  __shared__ float part[kGateWaves][64];
  __shared__ float npart[kNormThreads / kWave];
  const int b = blockIdx.x;
  const int H = a.H;
  void* xrow = static_cast<char*>(n.x) + (size_t)b * H * (BF16 ? 2 : 4);
  uint4 xk[kNormKeep];
  const bool kept = residual_rmsnorm_row<BF16>(n.h + (size_t)b * H, n.y ? n.y + (size_t)b * H : nullptr, n.gamma, xrow, H, npart, xk);
  if (BF16 && kept) {
    gate_body<BF16>(a, b, 0, part, xk);   // every thread holds its pieces of x already
  } else {
    __syncthreads();   // x of this token is written and visible to the workgroup
    gate_body<BF16>(a, b, 0, part);
  }
}

hipError_t launch_norm_gate(const GateArgs& a, const NormArgs& n, bool bf16, hipStream_t s, const KernelTiming& t) {
  dim3 grid(a.B), block(kGateThreads);
  if (bf16) launch_kernel(norm_gate_kernel<true>, grid, block, 0, s, t, a, n);
  else launch_kernel(norm_gate_kernel<false>, grid, block, 0, s, t, a, n);
  return hipGetLastError();
}

hipError_t launch_gate(const GateArgs& a, bool bf16, int routers, hipStream_t s, const KernelTiming& t) {
  dim3 grid(a.B, routers), block(kGateThreads);
  if (bf16) launch_kernel(gate_kernel<true>, grid, block, 0, s, t, a);
  else launch_kernel(gate_kernel<false>, grid, block, 0, s, t, a);
  return hipGetLastError();
}

}  // namespace adapmoe
