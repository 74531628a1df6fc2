// Internal interface between the host library and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

namespace adapmoe {

// What the gate leaves for the expert kernels of the same token: the image
// base pointers of the activated experts (already looked up in the residency
// table), their weights and k, so that the FFN kernels need one small load
// instead of a chain of three dependent ones.
struct ResolvedExperts {
  const void* base[2];
  float w[2];
  int32_t k;
  int32_t pad;
};

struct GateArgs {
  const void* x;        // [B,H] activation type
  const void* Wg[4];    // router of this layer, routers of the following layers (look-ahead; null = none)
  float tau[4];
  int32_t* ids[4];      // [B,2] each
  int32_t* k[4];        // [B] each
  float* w;             // [B,2], decision of router 0 only
  ResolvedExperts* res; // [B] or null; written for router 0 from `table`
  const void* const* table;  // residency table row of the layer (N pointers), used with res
  int B, H, N;
};

// Residual update and normalisation in front of a gate: h[b] += gamma * y[b] (y may be null),
// x[b] = h[b] / sqrt(mean(h[b]^2) + 1e-6) in the activation type.
struct NormArgs {
  float* h;
  const float* y;
  float gamma;
  void* x;
};

struct FfnArgs {
  const void* const* table;  // residency table row of the layer: N image base pointers, null = absent
  const ResolvedExperts* res;  // [B] resolved by the gate (then ids/w/k/table are not read) or null
  const void* x;             // [B,H] activation type
  const int32_t* ids;        // [B,2]
  const float* w;            // [B,2]
  const int32_t* k;          // [B]
  float* a;                  // scratch [B][2][a_stride]: w_j * silu(W1 x) * (W3 x) per activated expert
  size_t a_stride;           // floats per (token, expert slot) in the scratch, >= F
  float* y;                  // [B,H]
  int32_t* err;              // device flag word (bit 0: non-resident expert, bit 1: id out of range)
  int B, H, F, N;
  size_t w2_offset;          // byte offset of W2 inside an expert image
  // Window of a tile-wise launch (Alg.1, tile-wise scheduling): j_only >= 0 restricts the launch
  // to the activated expert of that rank and to rows [r0, r1) of its gate/up pairs (gate/up
  // kernels) or of W2 (down kernels); accumulate != 0 adds onto y instead of overwriting it.
  // j_only < 0: all activated experts, all rows, overwrite.
  int j_only, r0, r1, accumulate;
  // Dynamic tail (null = every row is assigned statically).  The last `dyn_pct` percent of the
  // passes over the grid are not dealt out in advance but drawn one row at a time from
  // kDynQueues shared counters, so that compute-unit groups that reach memory faster during a
  // launch end up doing more rows.  Every queue is shared by wavefronts of all compute-unit
  // groups; a wavefront draws from one queue only and stops when it is empty, so a launch
  // costs one atomic per drawn row plus one per wavefront.  Counters sit kDynStride words apart
  // (different memory channels: same-address atomics serialise at about 90 per microsecond).
  // dyn_ctr[b][kDynQueues * kDynStride] is read by the gate/up kernel and must be zero at its
  // launch; the down kernel, which runs after it, clears dyn_clear (the same array) again.
  unsigned* dyn_ctr;
  unsigned* dyn_clear;
  int dyn_pct;
};

constexpr int kDynQueues = 64;
constexpr int kDynStride = 128;   // unsigned words between two counters (512 bytes)

// Batched path (several tokens, experts streamed once each on the matrix cores)
struct BatchArgs {
  const void* const* table;  // residency table row of the layer
  const void* x;             // [B,H] bfloat16
  const int32_t* ids;        // [B,2]
  const float* w;            // [B,2]
  const int32_t* k;          // [B]
  float* y;                  // [B,H], cleared then accumulated
  int32_t* err;
  int B, H, F, N;
  size_t w2_offset;
  // scratch owned by the context
  int32_t* bkt_count;        // [N] tokens per expert
  int32_t* bkt_tok;          // [N][16] token index
  float* bkt_w;              // [N][16] routing weight
  const void** bkt_base;     // [N] image base pointer
  int32_t* bkt_active;       // [N+1] experts with at least one token, ascending; entry N = how many
  uint16_t* xop;             // [N][H/32][64][8] x of the bucket's tokens in MFMA operand order
  uint16_t* a_hi;            // [N][F/32][64][8] A in operand order, high bfloat16 part
  uint16_t* a_lo;            //                                      low part
  int two_terms;             // 1: A = hi + lo (fp32 accuracy), 0: A rounded to bfloat16
};

// Grid-wide barrier of the fused FFN kernel: a counter that only grows; launch n
// waits until it reaches n * grid size.  The intermediate vector a_j crosses the
// barrier through device-coherent stores and loads, so that the barrier itself
// needs no cache write-back or invalidate.
struct FusedSync {
  unsigned* counter;
  unsigned target;
  unsigned spin_limit;
};

// Events tied to one kernel dispatch (start and end of its execution, the interval a profiler
// reports); null = plain launch.  Events recorded on the stream around a launch also cover the
// processing of the event packets themselves, 1-2 us per side.
struct KernelTiming {
  hipEvent_t start = nullptr, stop = nullptr;
};

template <class K, class... A>
inline void launch_kernel(K kernel, dim3 grid, dim3 block, size_t lds, hipStream_t s, const KernelTiming& t, A... args) {
  if (t.start) hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds, s, t.start, t.stop, 0, args...);
  else hipLaunchKernelGGL(kernel, grid, block, lds, s, args...);
}

struct LaunchCfg {
  int gateup_blocks;  // workgroups of the gate/up GEMV (256 threads each)
  int down_blocks;    // workgroups of the down GEMV (1024 threads each)
  int batch_min;      // smallest number of tokens per call that takes the batched (MFMA) path
  int batch_two_terms;  // batched path: intermediate activation as hi + lo bfloat16 (1) or bfloat16 only (0)
  int fused_blocks;   // workgroups of the fused single-token FFN kernel (0 = fused path off)
  int dyn_pct;        // percent of the row passes of the GEMV kernels that are scheduled dynamically (0 = none)
  int batch_direct;   // batched gate/up GEMM: 2 = wavefronts stream through their tiles without a break, 1 = one tile per
                      // workgroup with the token operand loaded per wavefront, 0 = one tile per workgroup, operand staged in LDS
  KernelTiming timing;  // set for one launch when the context is profiling
};

hipError_t launch_gate(const GateArgs& a, bool bf16, int routers, hipStream_t s, const KernelTiming& t = KernelTiming{});
hipError_t launch_norm_gate(const GateArgs& a, const NormArgs& n, bool bf16, hipStream_t s, const KernelTiming& t = KernelTiming{});
hipError_t launch_ffn_gateup(const FfnArgs& p, int dtype, const LaunchCfg& lc, hipStream_t s);
hipError_t launch_ffn_down(const FfnArgs& p, int dtype, const LaunchCfg& lc, hipStream_t s);
int down_waves_per_workgroup(int rows, int blocks);   // 16, or 12 if that deals the rows out more evenly
hipError_t ffn_kernels_init(int dtype);
hipError_t ffn_fused_init(int dtype);
int ffn_fused_capacity(int dtype, int H, int F, int device);
hipError_t launch_ffn_fused(const FfnArgs& p, int dtype, const FusedSync& sy, int grid_blocks, hipStream_t s);
// group-quantised experts, bits = 4 or 2
hipError_t launch_ffn_gateup_quant(const FfnArgs& p, int bits, const LaunchCfg& lc, hipStream_t s);
hipError_t launch_ffn_down_quant(const FfnArgs& p, int bits, const LaunchCfg& lc, hipStream_t s);
hipError_t quant_kernels_init(int bits);
hipError_t batched_kernels_init();
hipError_t launch_stream_probe(const void* buf, long nrows, int row_bytes, int R, int C, int workgroups, unsigned* sink, hipStream_t s);
hipError_t launch_bucket_gather(const BatchArgs& p, hipStream_t s, const KernelTiming& t = KernelTiming{});
hipError_t launch_grouped_gateup(const BatchArgs& p, int mode, hipStream_t s, const KernelTiming& t = KernelTiming{});
hipError_t launch_grouped_down(const BatchArgs& p, bool two_terms, hipStream_t s, const KernelTiming& t = KernelTiming{});
hipError_t launch_residual_rmsnorm(float* h, const float* y, float gamma, void* x, bool bf16, int B, int H, hipStream_t s);

struct PokeArgs {   // up to 8 pointer-sized stores, ordered on the stream
  int n;
  const void** addr[8];
  const void* value[8];
};
hipError_t launch_poke(const PokeArgs& p, hipStream_t s);

}  // namespace adapmoe
