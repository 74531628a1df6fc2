// Shared by the expert-FFN kernels: the two-buffer part streamer, expert
// resolution through the residency table, SiLU.
#pragma once
#include "device_utils.h"
#include "launch.h"

namespace adapmoe {

constexpr int kChunkBytes = kWave * 16;  // bytes one wavefront reads per load instruction

__device__ __forceinline__ float silu_f32(float g) { return g / (1.0f + expf(-g)); }

// Resolves the image base pointers of the (up to two) activated experts of
// token b: from the record the gate left (one load) or, for callers that bring
// their own ids/w/k, through the residency table.
__device__ __forceinline__ int resolve_experts(const FfnArgs& p, int b, const char* base[2], float w[2]) {
  if (p.res != nullptr) {
    const ResolvedExperts r = p.res[b];
    const int kk = r.k < 1 ? 1 : (r.k > 2 ? 2 : r.k);
    for (int j = 0; j < 2; ++j) {
      base[j] = j < kk ? static_cast<const char*>(r.base[j]) : nullptr;
      w[j] = j < kk ? r.w[j] : 0.f;
      if (j < kk && base[j] == nullptr && threadIdx.x == 0) atomicOr(p.err, 1);
    }
    return kk;
  }
  // k, both ids and both weights are requested together (ids[B,2] and w[B,2] always exist); only
  // the table entries depend on a previous load
  int kk = p.k[b];
  const int e_in[2] = {p.ids[2 * b], p.ids[2 * b + 1]};
  const float w_in[2] = {p.w[2 * b], p.w[2 * b + 1]};
  kk = kk < 1 ? 1 : (kk > 2 ? 2 : kk);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    base[j] = nullptr;
    w[j] = 0.f;
    if (j < kk) {
      const int e = e_in[j];
      if (e < 0 || e >= p.N) {
        if (threadIdx.x == 0) atomicOr(p.err, 2);
      } else {
        base[j] = static_cast<const char*>(p.table[e]);
        w[j] = w_in[j];
        if (base[j] == nullptr && threadIdx.x == 0) atomicOr(p.err, 1);
      }
    }
  }
  return kk;
}

// a[j] for a run-time j in {0, 1}.  A local array indexed with a run-time value is placed in
// scratch memory, which costs the kernel a private segment at dispatch and memory round trips;
// a select keeps both elements in registers.
template <class T>
__device__ __forceinline__ T pick2(const T (&a)[2], int j) { return j ? a[1] : a[0]; }

// ----------------------------------------------------------- part streaming --

// Both GEMVs read, per wavefront, a known sequence of "parts": NV consecutive
// 1 KiB runs of a matrix row (16 bytes per lane each).  Two register buffers
// alternate: while part q is consumed, part q+1 is already in flight and part
// q+2 is requested as soon as q's buffer is free, so a wavefront keeps NV to
// 2*NV loads outstanding.  The steady loop has no conditional loads (those
// would make the compiler copy the buffers); the tail is peeled.
// next_addr() returns the lane's address of the next part in sequence,
// consume(buf) uses the next part in sequence; both keep their own cursor.
template <int NV>
__device__ __forceinline__ void load_vecs(const char* p, uint4 (&buf)[NV]) {
#pragma unroll
  for (int c = 0; c < NV; ++c) buf[c] = load_stream16(p + (size_t)c * kChunkBytes);
}

// The first two loads are issued whatever Q is (with Q < 2 the second buffer re-reads the first
// part, with Q == 0 nothing is loaded and nothing consumed): the compiler counts outstanding loads
// per path and takes the most cautious count where paths join, so a buffer that is loaded on some
// paths into the loop only would make every wait inside the loop wait for the younger buffer too
// (measured on the down GEMV: 1 us of 39 lost to that).
template <int NV, class AddrFn, class ConsumeFn, class MidFn>
__device__ __forceinline__ void stream_parts(int Q, AddrFn next_addr, ConsumeFn consume, MidFn after_first_loads) {
  if (Q <= 0) {
    after_first_loads();
    return;
  }
  uint4 A[NV], B[NV];
  const char* a0 = next_addr();
  const char* a1 = next_addr();   // only dereferenced when a second part exists
  load_vecs<NV>(a0, A);
  load_vecs<NV>(Q > 1 ? a1 : a0, B);
  after_first_loads();  // e.g. staging the activation vector in LDS while the first weights travel
  int q = 0;
  for (; q + 3 < Q; q += 2) {
    consume(A);
    load_vecs<NV>(next_addr(), A);
    consume(B);
    load_vecs<NV>(next_addr(), B);
  }
  // 1, 2 or 3 parts left; A holds part q, B part q+1
  consume(A);
  if (q + 2 < Q) load_vecs<NV>(next_addr(), A);
  if (q + 1 < Q) consume(B);
  if (q + 2 < Q) consume(A);
}

// Same pipeline for parts that are not a plain run of vectors: load_next(buf, advance) fills a
// buffer with the part under its cursor and then moves the cursor on if `advance` is set.
// The first loads are issued without conditions (a wavefront with fewer parts than buffers reads
// its last part again): the compiler counts outstanding loads per control-flow path and takes the
// most cautious count where paths join, so with conditional first loads every wait that follows -
// in particular the wait for small loads that after_first_loads() depends on, issued BEFORE these
// - would wait for the whole first burst of weights (measured: 5 us at the start of the quantised
// kernels).  A wavefront without any part only runs after_first_loads().
// EARLY = number of buffers requested before after_first_loads(), the others right after it.  A
// load instruction is held back while the memory pipeline of the compute unit is full, so a
// wavefront that requests all of its buffers first reaches after_first_loads() only when the
// opening burst of the whole workgroup has been accepted - microseconds, when every wavefront of
// the chip starts the same way.  EARLY = 1 keeps the memory system busy while the staging runs and
// lets the rest of the burst follow it.
template <class Buf, int EARLY = 2, class LoadFn, class ConsumeFn, class MidFn>
__device__ __forceinline__ void stream_bufs(int Q, LoadFn load_next, ConsumeFn consume, MidFn after_first_loads) {
  if (Q <= 0) {
    after_first_loads();
    return;
  }
  Buf A, B;
  load_next(A, Q > 1);
  if (EARLY > 1) load_next(B, true);
  after_first_loads();
  if (EARLY <= 1) load_next(B, true);
  int q = 0;
  for (; q + 3 < Q; q += 2) {
    consume(A);
    load_next(A, true);
    consume(B);
    load_next(B, true);
  }
  consume(A);
  if (q + 2 < Q) load_next(A, true);
  if (q + 1 < Q) consume(B);
  if (q + 2 < Q) consume(A);
}

// The same with four buffers in flight, for parts that are small (a few registers each): a
// wavefront keeps up to four parts outstanding.
template <class Buf, int EARLY = 4, class LoadFn, class ConsumeFn, class MidFn>
__device__ __forceinline__ void stream_bufs4(int Q, LoadFn load_next, ConsumeFn consume, MidFn after_first_loads) {
  if (Q <= 0) {
    after_first_loads();
    return;
  }
  Buf A, B, C, D;
  load_next(A, Q > 1);
  if (EARLY > 1) load_next(B, Q > 2);
  if (EARLY > 2) load_next(C, Q > 3);
  if (EARLY > 3) load_next(D, true);
  after_first_loads();
  if (EARLY <= 1) load_next(B, Q > 2);
  if (EARLY <= 2) load_next(C, Q > 3);
  if (EARLY <= 3) load_next(D, true);
  int q = 0;
  for (; q + 7 < Q; q += 4) {   // at least four more parts to request beyond the four in flight
    consume(A);
    load_next(A, true);
    consume(B);
    load_next(B, true);
    consume(C);
    load_next(C, true);
    consume(D);
    load_next(D, true);
  }
  // 1 to 7 parts left, the first min(left, 4) of them in A, B, C, D
  const int left = Q - q;
  consume(A);
  if (left > 4) load_next(A, true);
  if (left > 1) consume(B);
  if (left > 5) load_next(B, true);
  if (left > 2) consume(C);
  if (left > 6) load_next(C, true);
  if (left > 3) consume(D);
  if (left > 4) consume(A);
  if (left > 5) consume(B);
  if (left > 6) consume(C);
}

}  // namespace adapmoe
