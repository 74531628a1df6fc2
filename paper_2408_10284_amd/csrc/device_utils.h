// Device-side helpers shared by the kernels: wavefront reductions on DPP,
// bfloat16 unpacking, 16-byte streaming loads.  gfx950 only (64-lane waves).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adapmoe {

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;

constexpr int kWave = 64;

// Index of the wavefront inside its workgroup, as a scalar: told that it is the same for all
// lanes, the compiler keeps row numbers and row addresses derived from it in scalar registers and
// computes them on the scalar unit instead of once per lane.
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)); }

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also orders global memory,
// which makes every wavefront wait for all of its outstanding global loads - in the streaming
// kernels that is the first burst of weight loads, microseconds at the start of a launch.  This
// one waits for the wavefront's LDS operations only.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// DPP controls (GCN3+ encoding)
constexpr int kDppQuadSwap1 = 0xB1;      // quad_perm:[1,0,3,2]
constexpr int kDppQuadSwap2 = 0x4E;      // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141;
constexpr int kDppRowMirror = 0x140;

// Value of `v` in the lane the control selects.  All patterns used here read inside a row of 16
// lanes of a fully active wavefront, so no lane is without a source; "old" = 0 with bound_ctrl
// lets the compiler fold the move into the add or max that follows (one v_add_f32_dpp per step
// instead of a move, a DPP move and the add).
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  int i = __builtin_bit_cast(int, v);
  i = __builtin_amdgcn_update_dpp(0, i, CTRL, 0xf, 0xf, true);
  return __builtin_bit_cast(float, i);
}

__device__ __forceinline__ float readlane_f32(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}

// The pointer held by lane `lane` (the same for the whole wavefront), for every lane.
__device__ __forceinline__ const void* readlane_ptr(const void* v, int lane) {
  const uint64_t u = reinterpret_cast<uint64_t>(v);
  const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)u, lane);
  const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), lane);
  return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}

// Sum over the 64 lanes of a fully active wavefront; every lane gets the result.
// Four DPP steps give each row of 16 lanes its row sum, the four row sums are
// then read as scalars.  The order of additions is fixed, so results are
// reproducible from run to run.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f32<kDppQuadSwap1>(v);
  v += dpp_f32<kDppQuadSwap2>(v);
  v += dpp_f32<kDppRowHalfMirror>(v);
  v += dpp_f32<kDppRowMirror>(v);
  float r0 = readlane_f32(v, 0), r1 = readlane_f32(v, 16), r2 = readlane_f32(v, 32), r3 = readlane_f32(v, 48);
  return (r0 + r1) + (r2 + r3);
}

// A pointer that is the same in every lane, moved into scalar registers: addresses derived from it
// with wavefront-uniform offsets are then computed on the scalar unit, and loads take the form
// "scalar base + 32-bit lane offset" instead of a 64-bit address per lane.
__device__ __forceinline__ const char* uniform_ptr(const void* p) {
  const uint64_t u = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)u), hi = __builtin_amdgcn_readfirstlane((uint32_t)(u >> 32));
  return reinterpret_cast<const char*>(((uint64_t)hi << 32) | lo);
}

// Sums of two values over the 64 lanes at once: returns sum(g) in lanes 0..31 and sum(u) in lanes
// 32..63.  v_permlane32_swap exchanges the upper half of its first operand with the lower half of
// its second, so one swap and one add leave 32 partial sums of g in the lower and of u in the upper
// half; four DPP steps sum inside rows of 16 lanes and a row swap adds neighbouring rows.  11
// instructions for both sums (the order of additions is fixed).
__device__ __forceinline__ float pair_sum(float g, float u) {
  const auto h = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, g), __builtin_bit_cast(unsigned, u), false, false);
  float v = __builtin_bit_cast(float, (unsigned)h[0]) + __builtin_bit_cast(float, (unsigned)h[1]);
  v += dpp_f32<kDppQuadSwap1>(v);
  v += dpp_f32<kDppQuadSwap2>(v);
  v += dpp_f32<kDppRowHalfMirror>(v);
  v += dpp_f32<kDppRowMirror>(v);
  const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, v), __builtin_bit_cast(unsigned, v), false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}
// lane l (< 32) gets the value of lane l + 32 and the other way round
__device__ __forceinline__ float swap_halves(float v) {
  const auto h = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, v), __builtin_bit_cast(unsigned, v), false, false);
  // h[0] = (lower, lower), h[1] = (upper, upper)
  return (threadIdx.x & 32) ? __builtin_bit_cast(float, (unsigned)h[0]) : __builtin_bit_cast(float, (unsigned)h[1]);
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_f32<kDppQuadSwap1>(v));
  v = fmaxf(v, dpp_f32<kDppQuadSwap2>(v));
  v = fmaxf(v, dpp_f32<kDppRowHalfMirror>(v));
  v = fmaxf(v, dpp_f32<kDppRowMirror>(v));
  float r0 = readlane_f32(v, 0), r1 = readlane_f32(v, 16), r2 = readlane_f32(v, 32), r3 = readlane_f32(v, 48);
  return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// bfloat16 pair packed in a dword -> two floats (exact)
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

// float -> bfloat16 bits, round to nearest even (NaN kept quiet)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// acc += a.lo*b.lo + a.hi*b.hi for two packed bfloat16 pairs, fp32 accumulate
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc, false);
}

// 16-byte load of read-once data (weights): non-temporal so that the stream
// does not displace the small reused vectors from the caches.
__device__ __forceinline__ uint4 load_stream16(const void* p) {
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  typedef const __attribute__((address_space(1))) u32x4* gptr_t;  // expert images always live in global memory
  u32x4 v = __builtin_nontemporal_load((gptr_t)(uintptr_t)p);
  return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint32_t load_stream4(const void* p) {
  typedef const __attribute__((address_space(1))) uint32_t* gptr_t;
  return __builtin_nontemporal_load((gptr_t)(uintptr_t)p);
}

// fp16 bit pattern -> float
__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

// Elements of type T in a 16-byte vector and the dot product of a weight
// vector with an activation vector, for the storage types of the library.
// Weights float32 x activations float32:
__device__ __forceinline__ float dot16_f32(const uint4& w, const float4& x, float acc) {
  acc = fmaf(__builtin_bit_cast(float, w.x), x.x, acc);
  acc = fmaf(__builtin_bit_cast(float, w.y), x.y, acc);
  acc = fmaf(__builtin_bit_cast(float, w.z), x.z, acc);
  acc = fmaf(__builtin_bit_cast(float, w.w), x.w, acc);
  return acc;
}
// Weights bfloat16 (8 per vector) x activations bfloat16 (8 per vector):
__device__ __forceinline__ float dot16_bf16(const uint4& w, const uint4& x, float acc) {
  acc = dot2_bf16(w.x, x.x, acc);
  acc = dot2_bf16(w.y, x.y, acc);
  acc = dot2_bf16(w.z, x.z, acc);
  acc = dot2_bf16(w.w, x.w, acc);
  return acc;
}
// Weights bfloat16 (8 per vector) x activations float32 (two float4):
__device__ __forceinline__ float dot16_bf16_f32(const uint4& w, const float4& a0, const float4& a1, float acc) {
  acc = fmaf(bf16_lo(w.x), a0.x, acc);
  acc = fmaf(bf16_hi(w.x), a0.y, acc);
  acc = fmaf(bf16_lo(w.y), a0.z, acc);
  acc = fmaf(bf16_hi(w.y), a0.w, acc);
  acc = fmaf(bf16_lo(w.z), a1.x, acc);
  acc = fmaf(bf16_hi(w.z), a1.y, acc);
  acc = fmaf(bf16_lo(w.w), a1.z, acc);
  acc = fmaf(bf16_hi(w.w), a1.w, acc);
  return acc;
}

}  // namespace adapmoe
