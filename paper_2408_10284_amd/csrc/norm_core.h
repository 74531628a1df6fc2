// Residual update and RMS normalisation of one token by one workgroup, shared by the stand-alone
// kernel and by the kernel that goes on to the gate, so that both produce the same bits:
//   h += gamma * y (y may be null),  x = store( h / sqrt(mean(h^2) + 1e-6) ).
// This wiring between MoE blocks is the build's own (the paper's model has attention and its own
// normalisation there).  Thread t owns the 8-element chunks t, t + 512, ... of the row; up to
// kNormKeep chunks stay in registers between the two passes (rows of up to 8192 elements), longer
// rows are read again.  Sums are taken in a fixed order: along the thread's elements, then across
// the wavefront, then over the eight wavefronts.
#pragma once
#include "device_utils.h"

namespace adapmoe {

constexpr int kNormThreads = 512;
constexpr int kNormKeep = 2;

struct NormChunk {
  float4 lo, hi;
};

__device__ __forceinline__ float sumsq8(const NormChunk& c, float ss) {
  ss = fmaf(c.lo.x, c.lo.x, ss);
  ss = fmaf(c.lo.y, c.lo.y, ss);
  ss = fmaf(c.lo.z, c.lo.z, ss);
  ss = fmaf(c.lo.w, c.lo.w, ss);
  ss = fmaf(c.hi.x, c.hi.x, ss);
  ss = fmaf(c.hi.y, c.hi.y, ss);
  ss = fmaf(c.hi.z, c.hi.z, ss);
  ss = fmaf(c.hi.w, c.hi.w, ss);
  return ss;
}

__device__ __forceinline__ float4 axpy4(float g, const float4& y, const float4& h) {
  return make_float4(fmaf(g, y.x, h.x), fmaf(g, y.y, h.y), fmaf(g, y.z, h.z), fmaf(g, y.w, h.w));
}

// Returns the chunk as stored when the storage type is bfloat16 (eight packed values).
template <bool BF16>
__device__ __forceinline__ uint4 store_x8(void* xrow, int ci, const NormChunk& c, float inv) {
  const float v[8] = {c.lo.x * inv, c.lo.y * inv, c.lo.z * inv, c.lo.w * inv, c.hi.x * inv, c.hi.y * inv, c.hi.z * inv, c.hi.w * inv};
  if (BF16) {
    uint4 o;
    o.x = f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
    o.y = f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
    o.z = f32_to_bf16_bits(v[4]) | ((uint32_t)f32_to_bf16_bits(v[5]) << 16);
    o.w = f32_to_bf16_bits(v[6]) | ((uint32_t)f32_to_bf16_bits(v[7]) << 16);
    static_cast<uint4*>(xrow)[ci] = o;
    return o;
  } else {
    float4* x4 = static_cast<float4*>(xrow) + 2 * (size_t)ci;
    x4[0] = make_float4(v[0], v[1], v[2], v[3]);
    x4[1] = make_float4(v[4], v[5], v[6], v[7]);
    return make_uint4(0, 0, 0, 0);
  }
}

// Called by all kNormThreads threads of the workgroup; `part` is LDS for kNormThreads / 64 floats.
// H is a multiple of 8.  Ends with every store issued but without a barrier.  Returns true when
// the row was short enough to stay in registers; xk[i] then holds, for bfloat16 storage, the
// stored chunk tid + i * kNormThreads (what a 16-byte load of x at that place would return).
template <bool BF16>
__device__ __forceinline__ bool residual_rmsnorm_row(float* hr, const float* yr, float gamma, void* xrow, int H, float* part,
                                                     uint4 (&xk)[kNormKeep]) {
  const int tid = threadIdx.x;
  const int nchunks = H >> 3;
  float4* h4 = reinterpret_cast<float4*>(hr);
  const float4* y4 = reinterpret_cast<const float4*>(yr);
  auto update = [&](int ci) -> NormChunk {   // reads the chunk, applies the residual update, writes h back
    NormChunk c{h4[2 * (size_t)ci], h4[2 * (size_t)ci + 1]};
    if (yr) {
      c.lo = axpy4(gamma, y4[2 * (size_t)ci], c.lo);
      c.hi = axpy4(gamma, y4[2 * (size_t)ci + 1], c.hi);
      h4[2 * (size_t)ci] = c.lo;
      h4[2 * (size_t)ci + 1] = c.hi;
    }
    return c;
  };
  const bool keep = nchunks <= kNormKeep * kNormThreads;
  NormChunk kept[kNormKeep];
  float ss = 0.f;
  if (keep) {
#pragma unroll
    for (int i = 0; i < kNormKeep; ++i) {
      const int ci = tid + i * kNormThreads;
      if (ci < nchunks) {
        kept[i] = update(ci);
        ss = sumsq8(kept[i], ss);
      }
    }
  } else {
    for (int ci = tid; ci < nchunks; ci += kNormThreads) ss = sumsq8(update(ci), ss);
  }
  ss = wave_sum(ss);
  if ((tid & 63) == 0) part[tid >> 6] = ss;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int i = 0; i < kNormThreads / kWave; ++i) tot += part[i];
  const float inv = 1.0f / sqrtf(tot / (float)H + 1e-6f);
  if (keep) {
#pragma unroll
    for (int i = 0; i < kNormKeep; ++i) {
      const int ci = tid + i * kNormThreads;
      if (ci < nchunks) xk[i] = store_x8<BF16>(xrow, ci, kept[i], inv);
    }
  } else {
    for (int ci = tid; ci < nchunks; ci += kNormThreads) {
      const NormChunk c{h4[2 * (size_t)ci], h4[2 * (size_t)ci + 1]};   // this thread's own earlier stores
      store_x8<BF16>(xrow, ci, c, inv);
    }
  }
  return keep;
}

}  // namespace adapmoe
