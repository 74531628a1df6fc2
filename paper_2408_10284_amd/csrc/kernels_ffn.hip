// Expert FFN for decode (one or a few tokens): weight-streaming GEMVs.
//
//   y = sum_{j<k} w_j * W2_j ( silu(W1_j x) * (W3_j x) )      (Sec. 2.1 Eq.2; Sec. 4.2 Eq.3-4)
//
// Two launches, both bound by HBM bandwidth (one multiply-add per weight read):
//   gate/up  one wavefront per row pair (W1[f,:], W3[f,:]) of an activated
//            expert; rows of W1 and W3 are interleaved in the image so the pair
//            is one contiguous 2*H-element read; writes a_j[f] = w_j silu(g) u.
//   down     one wavefront per output element y[h]: dot of W2_j[h,:] with a_j
//            (staged in LDS) for every activated expert, summed in a fixed order.
// Every lane reads 16 bytes per load and a wavefront reads 1 KiB contiguous.
// No atomics: results are bit-reproducible.
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include "device_utils.h"
#include "launch.h"
#include "stream_parts.h"
#include "../../include/adapmoe.h"

namespace adapmoe {

constexpr int kGateUpThreads = 256;
constexpr int kDownThreads = 1024;
// ------------------------------------------------------------------ gate/up --

template <bool BF16, int NV>
__device__ __forceinline__ float dot_x(const uint4 (&buf)[NV], const uint4* xs, int c0, int lane, float acc) {
#pragma unroll
  for (int c = 0; c < NV; ++c) {
    const uint4 xv = xs[(c0 + c) * kWave + lane];
    if (BF16) acc = dot16_bf16(buf[c], xv, acc);
    else acc = dot16_f32(buf[c], __builtin_bit_cast(float4, xv), acc);
  }
  return acc;
}

// Row length not known at compile time, or an expert missing: plain loop.
template <bool BF16>
__device__ __forceinline__ float dot_row_generic(const char* row, const uint4* xs, int lane, int nch) {
  float acc = 0.f;
  for (int c = 0; c < nch; ++c) {
    uint4 buf[1];
    buf[0] = load_stream16(row + (size_t)c * kChunkBytes + lane * 16);
    acc = dot_x<BF16, 1>(buf, xs, c, lane, acc);
  }
  return acc;
}

// Each wavefront walks over row pairs r = first, first + stride, ...; a part
// is one row (W1[f,:] then W3[f,:], adjacent in the image).
template <bool BF16, int NCH>
__global__ __launch_bounds__(kGateUpThreads) void ffn_gateup_kernel(FfnArgs p) {
  extern __shared__ uint4 xs[];  // x[b,:] in its storage type
  const int b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const size_t esz = BF16 ? 2 : 4;
  const size_t row_bytes = (size_t)p.H * esz;
  const int nch = (int)(row_bytes / kChunkBytes);

  const uint4* xg = reinterpret_cast<const uint4*>(static_cast<const char*>(p.x) + (size_t)b * row_bytes);
  // x is staged in two steps: its loads are issued first of all - before the expert pointers are
  // fetched, so that they are ahead of every weight request of the launch (a small load issued
  // among the weight requests of the whole chip comes back microseconds later) - and its LDS
  // writes come after the first weight loads.  The barrier that follows orders LDS only: a full
  // __syncthreads() would also wait for those weight loads.
  constexpr int kStageX = 4;
  const int nsx = nch * kWave;
  struct StageX {   // passed by value (an array written through a captured reference ends up in scratch memory)
    uint4 v[kStageX];
  };
  auto stage_x_issue = [&]() -> StageX {
    StageX sx;
#pragma unroll
    for (int u = 0; u < kStageX; ++u) sx.v[u] = xg[min(tid + u * kGateUpThreads, nsx - 1)];
    return sx;
  };
  auto stage_x_finish = [&](const StageX& sx) {
#pragma unroll
    for (int u = 0; u < kStageX; ++u) xs[min(tid + u * kGateUpThreads, nsx - 1)] = sx.v[u];   // unconditional, see the down kernel
    for (int i = tid + kStageX * kGateUpThreads; i < nsx; i += kGateUpThreads) xs[i] = xg[i];
    lds_barrier();
  };
  const StageX sxv = stage_x_issue();

  const char* base[2];
  float wj[2];
  const int kk = resolve_experts(p, b, base, wj);
  const int F = p.F;
  const bool windowed = p.j_only >= 0;
  if (windowed && p.j_only >= kk) return;
  const int lo = windowed ? p.j_only * F + p.r0 : 0;        // rows are numbered expert-major: r = j*F + f
  const int total = windowed ? p.j_only * F + p.r1 : kk * F;
  const int stride = gridDim.x * (kGateUpThreads / kWave);
  const int first = lo + blockIdx.x * (kGateUpThreads / kWave) + wave;
  float* a_out = p.a + (size_t)b * 2 * p.a_stride;

  const bool need0 = !windowed || p.j_only == 0, need1 = kk > 1 && (!windowed || p.j_only == 1);
  const bool all_resident = (!need0 || base[0] != nullptr) && (!need1 || base[1] != nullptr);

  if (NCH > 0 && all_resident && p.dyn_ctr != nullptr && !windowed) {
    // Static passes first, then rows drawn from the shared counters (see FfnArgs::dyn_ctr).
    constexpr int NV = NCH > 0 ? NCH : 1;
    unsigned* ctr = p.dyn_ctr + (size_t)b * kDynQueues * kDynStride;
    const int nfull = total / stride;
    const int npool = nfull >= 2 ? max(1, (nfull * p.dyn_pct + 50) / 100) : nfull;
    const int nstatic = nfull - npool;
    const int pool_start = nstatic * stride, pool_len = total - pool_start;
    // queue q of nq holds pool rows pool_start + q + nq * t; workgroups 8m .. 8m+7 (one per
    // compute-unit group under round-robin dispatch) share queue m % nq, so every queue in use
    // has wavefronts drawing from it
    const int nq = min(kDynQueues, (int)(gridDim.x + 7) >> 3);
    const int q = (blockIdx.x >> 3) % nq;
    const int qlen = (pool_len - q + nq - 1) / nq;
    int it = 0;
    bool pool_open = true;
    auto grab = [&]() -> int {
      if (!pool_open) return -1;
      unsigned old = 0;
      if (lane == 0) old = __hip_atomic_fetch_add(ctr + q * kDynStride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      old = __builtin_amdgcn_readfirstlane(old);
      if ((int)old < qlen) return pool_start + q + nq * (int)old;
      pool_open = false;
      return -1;
    };
    auto next_row = [&]() -> int {
      if (it < nstatic) return (it++) * stride + first;
      return grab();
    };
    auto load_half = [&](uint4(&buf)[NV], int r, int half) {
      const int j = r >= F ? 1 : 0;
      load_vecs<NV>(pick2(base, j) + ((size_t)(r - j * F) * 2 + half) * row_bytes + lane * 16, buf);
    };
    uint4 A[NV], B[NV];
    int cur = next_row();
    if (cur >= 0) {
      load_half(A, cur, 0);
      load_half(B, cur, 1);
    }
    stage_x_finish(sxv);
    while (cur >= 0) {
      const int nxt = next_row();
      const float g = wave_sum(dot_x<BF16, NV>(A, xs, 0, lane, 0.f));
      if (nxt >= 0) load_half(A, nxt, 0);
      const float u = wave_sum(dot_x<BF16, NV>(B, xs, 0, lane, 0.f));
      if (lane == 0) a_out[(cur >= F ? p.a_stride - F : 0) + cur] = pick2(wj, cur >= F) * silu_f32(g) * u;
      if (nxt >= 0) load_half(B, nxt, 1);
      cur = nxt;
    }
  } else if (NCH > 0 && all_resident) {
    const int nrows = first < total ? (total - first + stride - 1) / stride : 0;
    int ra = first, half_a = 0;  // load cursor
    auto next_addr = [&]() -> const char* {
      const int j = ra >= F ? 1 : 0;
      const char* q = pick2(base, j) + ((size_t)(ra - j * F) * 2 + half_a) * row_bytes + lane * 16;
      if (half_a) ra += stride;
      half_a ^= 1;
      return q;
    };
    int rc = first, half_c = 0;  // consume cursor
    float g = 0.f;
    auto consume = [&](const uint4(&buf)[NCH > 0 ? NCH : 1]) {
      const float d = dot_x<BF16, (NCH > 0 ? NCH : 1)>(buf, xs, 0, lane, 0.f);
      if (!half_c) {
        g = d;
      } else {
        const float gs = wave_sum(g), us = wave_sum(d);
        if (lane == 0) a_out[(rc >= F ? p.a_stride - F : 0) + rc] = pick2(wj, rc >= F) * silu_f32(gs) * us;
        rc += stride;
      }
      half_c ^= 1;
    };
    stream_parts<(NCH > 0 ? NCH : 1)>(2 * nrows, next_addr, consume, [&, sxv]() { stage_x_finish(sxv); });
  } else {
    [&, sxv]() { stage_x_finish(sxv); }();
    for (int r = first; r < total; r += stride) {
      const int j = r >= F ? 1 : 0;
      float val = 0.f;
      const char* bj = pick2(base, j);
      if (bj) {
        const char* row = bj + (size_t)(r - j * F) * 2 * row_bytes;
        const float g = wave_sum(dot_row_generic<BF16>(row, xs, lane, nch));
        const float u = wave_sum(dot_row_generic<BF16>(row + row_bytes, xs, lane, nch));
        val = pick2(wj, j) * silu_f32(g) * u;
      }
      if (lane == 0) a_out[(size_t)j * p.a_stride + (r - j * F)] = val;
    }
  }
}

// --------------------------------------------------------------------- down --

// LDS position of a_j[f] for the bfloat16 path: a lane reads the eight values
// matching its 16-byte weight vector as two float4; placing the two halves of
// all 64 lanes in separate 1 KiB runs makes both reads bank-conflict free.
__device__ __forceinline__ int lds_pos_bf16(int f4 /* float4 index, f = 4*f4 */) {
  const int c = f4 >> 7;          // chunk of 512 elements = 128 float4
  const int r = f4 & 127;
  const int ln = r >> 1, half = r & 1;
  return (c << 7) + (half << 6) + ln;
}

template <bool BF16, int NV>
__device__ __forceinline__ float dot_a(const uint4 (&buf)[NV], const float4* aj, int c0, int lane, float acc) {
#pragma unroll
  for (int u = 0; u < NV; ++u) {
    const int c = c0 + u;
    if (BF16) acc = dot16_bf16_f32(buf[u], aj[(c << 7) + lane], aj[(c << 7) + 64 + lane], acc);
    else acc = dot16_f32(buf[u], aj[(c << 6) + lane], acc);
  }
  return acc;
}

// One wavefront per output element y[h]; a part is UN vectors of a row
// W2_j[h,:].  UN == 0 selects the plain loop (row length not a multiple of the
// part size).  A missing expert also takes the plain loop.  THREADS = 1024 or 768: the launcher
// takes 12 wavefronts per workgroup when that deals the rows out evenly and 16 do not (H = 6144
// over 256 workgroups: two rows per wavefront instead of two for one half and one for the other).
template <bool BF16, int UN, int THREADS>
__global__ __launch_bounds__(THREADS) void ffn_down_kernel(FfnArgs p) {
  extern __shared__ float4 as4[];  // a[j][F] of the activated experts
  const int b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const size_t esz = BF16 ? 2 : 4;
  const size_t row_bytes = (size_t)p.F * esz;
  const int nch = (int)(row_bytes / kChunkBytes);
  const int F4 = p.F >> 2;
  const int H = p.H;
  constexpr int kWaves = THREADS / kWave;
  constexpr int NV = UN > 0 ? UN : 1;

  const bool windowed = p.j_only >= 0;
  const int j0 = windowed ? p.j_only : 0;   // experts j0 .. j0 + nj - 1 take part
  const float4* ag = reinterpret_cast<const float4*>(p.a + (size_t)b * 2 * p.a_stride);
  const int S4 = (int)(p.a_stride >> 2);
  // Staging of a_j in two steps.  The loads of the first kStageA vectors per thread are issued first
  // of all - before the expert pointers are fetched, hence for both slots of the token whatever its
  // k (an unused slot holds old values that nothing reads) - so that they are ahead of every weight
  // request of the launch: a small load issued among the weight requests of the whole chip comes
  // back microseconds later, and a loop of load, wait, write would cost seven such round trips.
  // The LDS writes come after the first weight loads, and the barrier behind them orders LDS only
  // (a full __syncthreads() would also wait for those weight loads).
  constexpr int kStageA = (8192 + THREADS - 1) / THREADS;   // covers both slots of F = 16384 without the loop below
  const int nst = (windowed ? 1 : 2) * F4;
  struct StageA {   // passed by value: an array written through a captured reference ends up in scratch memory
    float4 v[kStageA];
  };
  auto a_src = [&](int i) -> const float4* {
    const int jr = i >= F4 ? 1 : 0;
    return ag + (j0 + jr) * S4 + (i - jr * F4);
  };
  auto a_dst = [&](int i) -> float4* {
    const int jr = i >= F4 ? 1 : 0;
    const int f4 = i - jr * F4;
    return as4 + jr * F4 + (BF16 ? lds_pos_bf16(f4) : f4);
  };
  auto stage_a_issue = [&]() -> StageA {
    StageA st;
#pragma unroll
    for (int u = 0; u < kStageA; ++u) st.v[u] = *a_src(min(tid + u * THREADS, nst - 1));   // unconditional: a clamped repeat is dropped below
    return st;
  };
  auto stage_a_finish = [&](const StageA& st) {
    // unconditional as well (threads beyond the end rewrite the last vector with its own value):
    // under a condition the compiler would move each load down to its write again
#pragma unroll
    for (int u = 0; u < kStageA; ++u) *a_dst(min(tid + u * THREADS, nst - 1)) = st.v[u];
    for (int i = tid + kStageA * THREADS; i < nst; i += THREADS) *a_dst(i) = *a_src(i);   // very long rows only
    lds_barrier();
  };
  const StageA sta = stage_a_issue();

  const char* base[2];
  float wj[2];
  const int kk = resolve_experts(p, b, base, wj);
  if (windowed && p.j_only >= kk) return;
  const int nj = windowed ? 1 : kk;
  const int hlo = windowed ? p.r0 : 0, hhi = windowed ? p.r1 : H;
  // the experts taking part, in order: one of the window, or all kk
  const char* part[2] = {pick2(base, j0), nj > 1 ? base[1] : nullptr};
  const bool all_resident = part[0] != nullptr && (nj < 2 || part[1] != nullptr);

  const int first = hlo + blockIdx.x * kWaves + wave;
  const int hstride = gridDim.x * kWaves;
  float* y = p.y + (size_t)b * H;
  const bool accumulate = p.accumulate != 0;
  // the gate/up kernel's row counters are cleared here, ready for its next launch
  if (blockIdx.x == 0 && tid < kDynQueues && p.dyn_clear && !windowed) p.dyn_clear[((size_t)b * kDynQueues + tid) * kDynStride] = 0u;

  if (UN > 0 && all_resident) {
    const int nbp = nch / NV;        // parts per row of one expert
    const int nb = nj * nbp;         // parts per output element
    const int nrows = first < hhi ? (hhi - first + hstride - 1) / hstride : 0;
    const char* w2[2] = {part[0] + p.w2_offset, nj > 1 ? part[1] + p.w2_offset : nullptr};
    int ha = first, ba = 0;  // load cursor
    auto next_addr = [&]() -> const char* {
      const int j = ba >= nbp ? 1 : 0;
      const char* q = pick2(w2, j) + (size_t)ha * row_bytes + (size_t)(ba - j * nbp) * NV * kChunkBytes + lane * 16;
      if (++ba == nb) { ba = 0; ha += hstride; }
      return q;
    };
    int hc = first, bc = 0;  // consume cursor
    float acc = 0.f;
    auto consume = [&](const uint4(&buf)[NV]) {
      const int j = bc >= nbp ? 1 : 0;
      acc = dot_a<BF16, NV>(buf, as4 + j * F4, (bc - j * nbp) * NV, lane, acc);
      if (++bc == nb) {
        const float s = wave_sum(acc);
        if (lane == 0) y[hc] = accumulate ? y[hc] + s : s;
        acc = 0.f;
        bc = 0;
        hc += hstride;
      }
    };
    stream_parts<NV>(nrows * nb, next_addr, consume, [&, sta]() { stage_a_finish(sta); });
  } else {
    [&, sta]() { stage_a_finish(sta); }();   // through a by-value capture like the other branch, or the array lands in scratch memory
    for (int h = first; h < hhi; h += hstride) {
      float acc = 0.f;
      for (int jr = 0; jr < nj; ++jr) {
        const char* bj = pick2(part, jr);
        if (!bj) continue;
        const char* row = bj + p.w2_offset + (size_t)h * row_bytes + lane * 16;
        for (int c = 0; c < nch; ++c) {
          uint4 buf[1];
          buf[0] = load_stream16(row + (size_t)c * kChunkBytes);
          acc = dot_a<BF16, 1>(buf, as4 + jr * F4, c, lane, acc);
        }
      }
      acc = wave_sum(acc);
      if (lane == 0) y[h] = accumulate ? y[h] + acc : acc;
    }
  }
}

// -------------------------------------------------------------------- fused --

// Both GEMVs of one token in a single launch.  The grid is one workgroup of 16
// wavefronts per compute unit, all co-resident; between the two phases every
// workgroup passes a grid-wide barrier (a counter in global memory), and the
// first W2 loads are already in flight while it waits, so the HBM stream does
// not drain between gate/up and down.  Measured slower than two launches all the
// same (114 vs 108 us per Mixtral-shaped step), so it is an opt-in.  The barrier wait is bounded: a
// workgroup that does not see all arrivals within `spin_limit` polls raises
// error bit 2 and goes on, so the kernel always terminates.
// Requirements checked by the launcher: one token, H row of 8 vector runs,
// W2 rows a multiple of UN runs, grid <= number of compute units.
constexpr int kFusedThreads = 1024;

__device__ __forceinline__ void grid_barrier(const FusedSync& sy, int* s_ok, int32_t* err) {
  __syncthreads();  // this workgroup's a_j stores are issued
  if (threadIdx.x == 0) {
    // a_j is written with device-coherent stores, which have completed at device scope once the
    // barrier above has waited for them, and read back with device-coherent loads, which do not
    // see stale cache lines: arrival and wait need no cache write-back or invalidate (with a
    // release / acquire pair here every workgroup paid both, 11 us more per step)
    __hip_atomic_fetch_add(sy.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0;
    int ok = 1;
    while ((int)(__hip_atomic_load(sy.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - sy.target) < 0) {
      if (++spins > sy.spin_limit) {
        ok = 0;
        atomicOr(err, 4);
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    *s_ok = ok;
  }
  __syncthreads();
}

template <bool BF16, int UN>
__global__ __launch_bounds__(kFusedThreads) void ffn_fused_kernel(FfnArgs p, FusedSync sy) {
  extern __shared__ uint4 smem[];  // x row, then a[j][F]
  __shared__ int s_ok;
  constexpr int NCH = 8;
  constexpr int kWaves = kFusedThreads / kWave;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const size_t esz = BF16 ? 2 : 4;
  const int H = p.H, F = p.F;

  const char* base[2];
  float wj[2];
  const int kk = resolve_experts(p, 0, base, wj);
  if (base[0] == nullptr || (kk > 1 && base[1] == nullptr)) {
      // flagged by resolve_experts; the same for every workgroup, so nobody waits at the barrier,
      // but the arrival is still counted to keep the counter in step with the launch number
      if (tid == 0) __hip_atomic_fetch_add(sy.counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
  }

  const int first = blockIdx.x * kWaves + wave;
  const int stride = gridDim.x * kWaves;

  // ---- phase 1: a_j[f] = w_j silu(W1_j[f,:] x) (W3_j[f,:] x)
  {
    const size_t row_bytes = (size_t)H * esz;
    uint4* xs = smem;
    const uint4* xg = reinterpret_cast<const uint4*>(p.x);
    auto stage_x = [&]() {
      for (int i = tid; i < NCH * kWave; i += kFusedThreads) xs[i] = xg[i];
      __syncthreads();
    };
    const int total = kk * F;
    const int nrows = first < total ? (total - first + stride - 1) / stride : 0;
    int ra = first, half_a = 0;
    auto next_addr = [&]() -> const char* {
      const int j = ra >= F ? 1 : 0;
      const char* q = pick2(base, j) + ((size_t)(ra - j * F) * 2 + half_a) * row_bytes + lane * 16;
      if (half_a) ra += stride;
      half_a ^= 1;
      return q;
    };
    int rc = first, half_c = 0;
    float g = 0.f;
    auto consume = [&](const uint4(&buf)[NCH]) {
      const float d = dot_x<BF16, NCH>(buf, xs, 0, lane, 0.f);
      if (!half_c) {
        g = d;
      } else {
        const float gs = wave_sum(g), us = wave_sum(d);
        if (lane == 0) {
          float* dst = p.a + (rc >= F ? p.a_stride - F : 0) + rc;
          const float val = pick2(wj, rc >= F) * silu_f32(gs) * us;
          __hip_atomic_store(dst, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        rc += stride;
      }
      half_c ^= 1;
    };
    stream_parts<NCH>(2 * nrows, next_addr, consume, stage_x);
  }

  // ---- phase 2: y[h] = sum_j W2_j[h,:] a_j
  {
    const size_t row_bytes = (size_t)F * esz;
    const int nch = (int)(row_bytes / kChunkBytes);
    const int F4 = F >> 2, S4 = (int)(p.a_stride >> 2);
    float4* as4 = reinterpret_cast<float4*>(smem + NCH * kWave);
    const float4* ag = reinterpret_cast<const float4*>(p.a);
    auto barrier_and_stage_a = [&]() {
      grid_barrier(sy, &s_ok, p.err);
      for (int i = tid; i < kk * F4; i += kFusedThreads) {
        const int j = i >= F4 ? 1 : 0;
        const int f4 = i - j * F4;
        const uint64_t* src = reinterpret_cast<const uint64_t*>(ag + j * S4 + f4);
        const uint64_t lo = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t hi = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        as4[j * F4 + (BF16 ? lds_pos_bf16(f4) : f4)] =
            make_float4(__builtin_bit_cast(float, (uint32_t)lo), __builtin_bit_cast(float, (uint32_t)(lo >> 32)),
                        __builtin_bit_cast(float, (uint32_t)hi), __builtin_bit_cast(float, (uint32_t)(hi >> 32)));
      }
      __syncthreads();
    };
    const int nbp = nch / UN, nb = kk * nbp;
    const int nrows = first < H ? (H - first + stride - 1) / stride : 0;
    const char* w2[2] = {base[0] + p.w2_offset, kk > 1 ? base[1] + p.w2_offset : nullptr};
    int ha = first, ba = 0;
    auto next_addr = [&]() -> const char* {
      const int j = ba >= nbp ? 1 : 0;
      const char* q = pick2(w2, j) + (size_t)ha * row_bytes + (size_t)(ba - j * nbp) * UN * kChunkBytes + lane * 16;
      if (++ba == nb) { ba = 0; ha += stride; }
      return q;
    };
    int hc = first, bc = 0;
    float acc = 0.f;
    auto consume = [&](const uint4(&buf)[UN]) {
      const int j = bc >= nbp ? 1 : 0;
      acc = dot_a<BF16, UN>(buf, as4 + j * F4, (bc - j * nbp) * UN, lane, acc);
      if (++bc == nb) {
        const float sum = wave_sum(acc);
        if (lane == 0) p.y[hc] = sum;
        acc = 0.f;
        bc = 0;
        hc += stride;
      }
    };
    stream_parts<UN>(nrows * nb, next_addr, consume, barrier_and_stage_a);
  }
}

// ------------------------------------------------------------------ launch ---

template <typename K>
static hipError_t allow_big_lds(K kernel) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

template <bool BF16, int THREADS>
static hipError_t init_down_t() {
  hipError_t e;
  if ((e = allow_big_lds(ffn_down_kernel<BF16, 7, THREADS>)) != hipSuccess) return e;
  if ((e = allow_big_lds(ffn_down_kernel<BF16, 8, THREADS>)) != hipSuccess) return e;
  if ((e = allow_big_lds(ffn_down_kernel<BF16, 4, THREADS>)) != hipSuccess) return e;
  return allow_big_lds(ffn_down_kernel<BF16, 0, THREADS>);
}
template <bool BF16>
static hipError_t init_down() {
  const hipError_t e = init_down_t<BF16, kDownThreads>();
  return e != hipSuccess ? e : init_down_t<BF16, 768>();
}

hipError_t ffn_kernels_init(int dtype) {
  if (dtype == ADAPMOE_INT4G64 || dtype == ADAPMOE_INT2G64) return quant_kernels_init(dtype == ADAPMOE_INT4G64 ? 4 : 2);
  return dtype == ADAPMOE_F32 ? init_down<false>() : init_down<true>();
}

template <bool BF16>
static void launch_gateup_t(const FfnArgs& p, int nch, dim3 grid, size_t lds, hipStream_t s, const KernelTiming& t) {
  dim3 block(kGateUpThreads);
  if (nch == 8) launch_kernel(ffn_gateup_kernel<BF16, 8>, grid, block, lds, s, t, p);         // H = 4096 bf16, 2048 fp32
  else if (nch == 12) launch_kernel(ffn_gateup_kernel<BF16, 12>, grid, block, lds, s, t, p);  // H = 6144 bf16 (8x22B)
  else if (nch == 4) launch_kernel(ffn_gateup_kernel<BF16, 4>, grid, block, lds, s, t, p);
  else launch_kernel(ffn_gateup_kernel<BF16, 0>, grid, block, lds, s, t, p);
}

hipError_t launch_ffn_gateup(const FfnArgs& p, int dtype, const LaunchCfg& lc, hipStream_t s) {
  const bool bf16 = dtype != ADAPMOE_F32;
  const size_t row_bytes = (size_t)p.H * (bf16 ? 2 : 4);
  const int nch = (int)(row_bytes / kChunkBytes);
  dim3 grid(lc.gateup_blocks, p.B);
  if (p.j_only >= 0) grid.x = std::max(1, std::min(lc.gateup_blocks, (p.r1 - p.r0 + 3) / (kGateUpThreads / kWave)));
  if (bf16) launch_gateup_t<true>(p, nch, grid, row_bytes, s, lc.timing);
  else launch_gateup_t<false>(p, nch, grid, row_bytes, s, lc.timing);
  return hipGetLastError();
}

template <bool BF16, int THREADS>
static void launch_down_t(const FfnArgs& p, int nch, dim3 grid, size_t lds, hipStream_t s, const KernelTiming& t) {
  dim3 block(THREADS);
  if (nch % 7 == 0) launch_kernel(ffn_down_kernel<BF16, 7, THREADS>, grid, block, lds, s, t, p);
  else if (nch % 8 == 0) launch_kernel(ffn_down_kernel<BF16, 8, THREADS>, grid, block, lds, s, t, p);
  else if (nch % 4 == 0) launch_kernel(ffn_down_kernel<BF16, 4, THREADS>, grid, block, lds, s, t, p);
  else launch_kernel(ffn_down_kernel<BF16, 0, THREADS>, grid, block, lds, s, t, p);
}

// Wavefronts per workgroup of a down GEMV that walks `rows` rows with `blocks` workgroups, one row per
// wavefront and pass.  A compute unit streams at the same rate with 12 as with 16 wavefronts, so the
// launch lasts (passes x wavefronts per workgroup) row times: 16 unless 12 makes that product smaller
// (H = 6144 over 256 workgroups: 2 x 12 against 2 x 16, the second pass of 16 being half empty).
int down_waves_per_workgroup(int rows, int blocks) {
  if (rows < blocks * 16) return 16;
  auto passes = [&](int w) { return (rows + blocks * w - 1) / (blocks * w); };
  return passes(12) * 12 < passes(16) * 16 ? 12 : 16;
}

hipError_t launch_ffn_down(const FfnArgs& p, int dtype, const LaunchCfg& lc, hipStream_t s) {
  const bool bf16 = dtype != ADAPMOE_F32;
  const int nch = (int)((size_t)p.F * (bf16 ? 2 : 4) / kChunkBytes);
  dim3 grid(lc.down_blocks, p.B);
  if (p.j_only >= 0) grid.x = std::max(1, std::min(lc.down_blocks, (p.r1 - p.r0 + 15) / (kDownThreads / kWave)));
  const size_t lds = (size_t)2 * p.F * sizeof(float);
  const bool twelve = p.j_only < 0 && down_waves_per_workgroup(p.H, (int)grid.x) == 12;
  if (bf16) {
    if (twelve) launch_down_t<true, 768>(p, nch, grid, lds, s, lc.timing);
    else launch_down_t<true, kDownThreads>(p, nch, grid, lds, s, lc.timing);
  } else {
    if (twelve) launch_down_t<false, 768>(p, nch, grid, lds, s, lc.timing);
    else launch_down_t<false, kDownThreads>(p, nch, grid, lds, s, lc.timing);
  }
  return hipGetLastError();
}

// the fused kernel also has a few bytes of static LDS, which count against the 160 KiB
constexpr size_t kFusedMaxDynLds = 160 * 1024 - 256;

// Fused launch; returns hipErrorNotSupported when the shape does not fit the fused kernel.
template <bool BF16>
static hipError_t launch_fused_t(const FfnArgs& p, const FusedSync& sy, int grid_blocks, hipStream_t s) {
  const size_t esz = BF16 ? 2 : 4;
  const int nch_up = (int)((size_t)p.H * esz / kChunkBytes);
  const int nch_dn = (int)((size_t)p.F * esz / kChunkBytes);
  const size_t lds = (size_t)p.H * esz + (size_t)2 * p.F * sizeof(float);
  if (p.B != 1 || nch_up != 8 || lds > kFusedMaxDynLds) return hipErrorNotSupported;
  dim3 grid(grid_blocks), block(kFusedThreads);
  if (nch_dn % 7 == 0) hipLaunchKernelGGL((ffn_fused_kernel<BF16, 7>), grid, block, lds, s, p, sy);
  else if (nch_dn % 8 == 0) hipLaunchKernelGGL((ffn_fused_kernel<BF16, 8>), grid, block, lds, s, p, sy);
  else return hipErrorNotSupported;
  return hipGetLastError();
}

hipError_t launch_ffn_fused(const FfnArgs& p, int dtype, const FusedSync& sy, int grid_blocks, hipStream_t s) {
  return dtype == ADAPMOE_F32 ? launch_fused_t<false>(p, sy, grid_blocks, s) : launch_fused_t<true>(p, sy, grid_blocks, s);
}

// Number of workgroups of the fused kernel that are guaranteed to be resident at once
// for this shape (one per compute unit), or 0 if the shape does not fit.
int ffn_fused_capacity(int dtype, int H, int F, int device) {
  const bool bf16 = dtype != ADAPMOE_F32;
  const size_t esz = bf16 ? 2 : 4;
  const size_t lds = (size_t)H * esz + (size_t)2 * F * sizeof(float);
  const int nch_up = (int)((size_t)H * esz / kChunkBytes), nch_dn = (int)((size_t)F * esz / kChunkBytes);
  if (nch_up != 8 || lds > kFusedMaxDynLds || (nch_dn % 7 != 0 && nch_dn % 8 != 0)) return 0;
  int cus = 0, per_cu = 0;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) return 0;
  const void* k = nch_dn % 7 == 0 ? (bf16 ? reinterpret_cast<const void*>(ffn_fused_kernel<true, 7>) : reinterpret_cast<const void*>(ffn_fused_kernel<false, 7>))
                                  : (bf16 ? reinterpret_cast<const void*>(ffn_fused_kernel<true, 8>) : reinterpret_cast<const void*>(ffn_fused_kernel<false, 8>));
  const hipError_t oe = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k, kFusedThreads, lds);
  if (getenv("ADAPMOE_VERBOSE")) fprintf(stderr, "adapmoe: fused occupancy query %s: %d per CU, %d CUs, lds %zu\n", hipGetErrorString(oe), per_cu, cus, lds);
  if (oe != hipSuccess || per_cu < 1) return 0;
  return cus;
}

template <typename K>
static hipError_t allow_fused_lds(K kernel) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)kFusedMaxDynLds);
}

hipError_t ffn_fused_init(int dtype) {
  hipError_t e;
  if (dtype == ADAPMOE_F32) {
    if ((e = allow_fused_lds(ffn_fused_kernel<false, 7>)) != hipSuccess) return e;
    return allow_fused_lds(ffn_fused_kernel<false, 8>);
  }
  if ((e = allow_fused_lds(ffn_fused_kernel<true, 7>)) != hipSuccess) return e;
  return allow_fused_lds(ffn_fused_kernel<true, 8>);
}

}  // namespace adapmoe
