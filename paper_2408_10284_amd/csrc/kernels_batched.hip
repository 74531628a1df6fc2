// Batched decode (several tokens per step): the activated (token, expert)
// pairs are bucketed by expert and every touched expert is streamed from HBM
// once, as a grouped GEMM on the matrix cores
//
//   A_e[f, n] = w_n silu(W1_e[f,:] . x_n) (W3_e[f,:] . x_n)     n over the tokens of bucket e
//   y_n      += W2_e A_e[:, n]                                   (Sec. 2.1 Eq.2 per token)
//
// with v_mfma_f32_16x16x32_bf16: 16 weight rows x 32 reduction elements per
// instruction against up to 16 tokens.  The work is still bound by HBM (each
// weight is used for at most 16 multiply-adds), so the layout follows the
// weight stream: a wavefront owns 16 rows and walks the reduction axis; the
// token-side operand (x, or A split into two bfloat16 terms so that it keeps
// fp32 accuracy) is small, lives in global memory in MFMA operand order and is
// staged through LDS slab by slab for all wavefronts of the workgroup.
//
// Operand order: for reduction step s (32 elements) lane l = 16 q + n holds the
// 8 elements k = 32 s + 8 q + i of token column n.
#include <algorithm>
#include "../../include/adapmoe.h"
#include "stream_parts.h"

namespace adapmoe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kBTok = 16;            // token columns of one MFMA
constexpr int kBThreads = 256;       // 4 wavefronts, 16 rows each
constexpr int kBWaves = kBThreads / kWave;

__device__ __forceinline__ f32x4_t mfma16(const uint4& a, const uint4& b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// ------------------------------------------------------------------ buckets --

// Every workgroup recomputes the (tiny) bucket lists, workgroup (0,0) publishes
// them; then the grid gathers x into operand order per expert and clears y.
// grid = (H/32/4, N): workgroup (i, e) writes 4 reduction steps of expert e.
__global__ __launch_bounds__(kBThreads) void bucket_gather_kernel(BatchArgs p) {
  __shared__ int s_count[64];
  __shared__ int s_tok[64][kBTok];
  const int tid = threadIdx.x, lane = tid & 63;
  const int e_mine = blockIdx.y;
  if (tid < 64) {
    // lane l < 2B is the pair (token l/2, rank l%2)
    const int b = lane >> 1, j = lane & 1;
    int e = -1;
    float w = 0.f;
    if (b < p.B) {
      int kk = p.k[b];
      const int e_in = p.ids[2 * b + j];   // read together with k, not after it
      const int e_other = p.ids[2 * b + (j ^ 1)];
      const float w_in = p.w[2 * b + j];
      kk = kk < 1 ? 1 : (kk > 2 ? 2 : kk);
      if (j < kk) {
        e = e_in;
        w = w_in;
        // a bucket has room for one pair per token: the same expert twice for one token is not a
        // gate decision and would overflow it, so the second pair is dropped and flagged
        if (e < 0 || e >= p.N || (j == 1 && e == e_other)) {
          e = -1;
          if (blockIdx.x == 0 && blockIdx.y == 0) atomicOr(p.err, 2);
        }
      }
    }
    // residency of all experts in one load per lane (a load per loop pass below would be N memory
    // round trips one after the other)
    const void* mine = lane < p.N ? p.table[lane] : nullptr;
    const uint64_t resmask = __builtin_amdgcn_ballot_w64(mine != nullptr);
    for (int ex = 0; ex < p.N; ++ex) {
      const uint64_t m = __builtin_amdgcn_ballot_w64(e == ex);
      const int rank = __builtin_popcountll(m & ((1ull << lane) - 1));
      const bool resident = (resmask >> ex) & 1;
      if (m && !resident && lane == 0 && blockIdx.x == 0 && blockIdx.y == 0) atomicOr(p.err, 1);
      if (lane == 0) s_count[ex] = resident ? __builtin_popcountll(m) : 0;
      if (e == ex && resident) {
        s_tok[ex][rank] = b;
        if (blockIdx.x == 0 && blockIdx.y == 0) {
          p.bkt_tok[ex * kBTok + rank] = b;
          p.bkt_w[ex * kBTok + rank] = w;
        }
      }
    }
    if (blockIdx.x == 0 && blockIdx.y == 0) {
      if (lane < p.N) {
        p.bkt_count[lane] = s_count[lane];
        p.bkt_base[lane] = mine;
      }
      // the experts that have tokens, in ascending order, and how many they are
      const bool active = lane < p.N && s_count[lane] > 0;
      const uint64_t am = __builtin_amdgcn_ballot_w64(active);
      if (active) p.bkt_active[__builtin_popcountll(am & ((1ull << lane) - 1))] = lane;
      if (lane == 0) p.bkt_active[p.N] = __builtin_popcountll(am);
    }
  }
  __syncthreads();

  // clear this workgroup's share of y
  {
    const int nwg = gridDim.x * gridDim.y, wg = blockIdx.y * gridDim.x + blockIdx.x;
    const int total4 = p.B * p.H / 4;
    float4* y4 = reinterpret_cast<float4*>(p.y);
    for (int i = wg * kBThreads + tid; i < total4; i += nwg * kBThreads) y4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
  }

  // gather x: 4 reduction steps = 256 lane slots of 16 bytes, one per thread
  const int cnt = s_count[e_mine];
  if (cnt == 0) return;
  const int step = blockIdx.x * 4 + (tid >> 6);
  if (step * 32 >= p.H) return;
  const int n = lane & 15, q = lane >> 4;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (n < cnt) {
    const uint16_t* xr = static_cast<const uint16_t*>(p.x) + (size_t)s_tok[e_mine][n] * p.H;
    v = *reinterpret_cast<const uint4*>(xr + step * 32 + q * 8);
  }
  reinterpret_cast<uint4*>(p.xop)[((size_t)e_mine * (p.H / 32) + step) * 64 + lane] = v;
}

// -------------------------------------------------------------- grouped GEMM --

// C[16 rows per wavefront, 16 tokens] += W[rows, :] . Bop, reduction in slabs of
// KS steps (KS * 64 bytes of every row).  NMAT = 2 reads two interleaved
// matrices (W1 and W3 rows of the same index, gate/up); NTERM = 2 multiplies by
// two operand arrays (hi and lo halves of A) and adds.
// Weight path: coalesced 16-byte loads (32 lanes cover the slab's contiguous
// KS*64 bytes of one row, an instruction covers two rows), two slabs in flight
// in registers; at use the slab is turned into MFMA operand order through a
// wavefront-private LDS tile whose rows are padded by 16 bytes so that the
// operand reads (16 rows x 16 bytes per pass) hit all banks once.
// Token operand: staged in LDS slab by slab by the whole workgroup.
template <int NMAT, int RT, int NB>
struct WSlab {
  uint4 a[NMAT][RT][8];   // instruction i of matrix t, row tile rt: rows 16 rt + 2i, 16 rt + 2i + 1
  uint4 b[NB > 0 ? NB : 1];  // DIRECT mode: the lane's token-operand vectors of the slab, [term][step]
};

template <int KS>
constexpr int wtile_row_bytes() { return KS * 64 + 16; }

// DB = 2: the token operand slab is double-buffered in LDS (one barrier per slab instead of two;
// measured 5 % slower on MI355X for the down GEMM, so both GEMMs use DB = 1)
template <int KS, int NMAT, int NTERM, int NW, int DB>
constexpr size_t grouped_lds_bytes() {
  return (size_t)DB * KS * 64 * NTERM * 16 + (size_t)NW * NMAT * 16 * wtile_row_bytes<KS>();
}
// DIRECT mode (DB = 0): no operand slab in LDS, every wavefront loads its operand vectors itself
// (1 KiB contiguous per instruction, served by L2) and runs without workgroup barriers.

// RT = row tiles of 16 per wavefront (they share the token operand and the LDS tile).
template <int KS, int NMAT, int NTERM, int RT, int NW, int DB, class Epilogue>
__device__ __forceinline__ void grouped_gemm_tile_loop(const char* wbase, size_t row_stride, size_t mat_stride, int nsteps,
                                                       int ntiles_rows, int tile0, int tile_stride,
                                                       const uint4* bop0, const uint4* bop1, uint4* lds, Epilogue epilogue) {
  static_assert(KS * 64 == 32 * 16, "a slab row must be 32 lanes x 16 bytes");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int m = lane & 15, q = lane >> 4;
  const int nslabs = nsteps / KS;
  constexpr int kThreads = NW * kWave;
  constexpr int kSlabVecs = KS * 64 * NTERM;            // 16-byte vectors of one operand slab
  constexpr int kVecsPerThread = kSlabVecs / kThreads;
  static_assert(kSlabVecs % kThreads == 0, "operand slab must divide evenly over the workgroup");
  constexpr int kRowB = wtile_row_bytes<KS>();
  char* wt = reinterpret_cast<char*>(lds + DB * kSlabVecs) + (size_t)wave * NMAT * 16 * kRowB;   // this wavefront's tile(s)
  char* wt_store = wt + (lane >> 5) * kRowB + (lane & 31) * 16;    // where this lane's loaded pieces go (row 2i + lane/32)
  const char* wt_read = wt + m * kRowB + q * 16;                   // operand read: row m, bytes 64 s + 16 q

  for (int tile = tile0; tile < ntiles_rows; tile += tile_stride) {
    const int row0 = (tile * NW + wave) * 16 * RT;
    const char* wsrc = wbase + (size_t)(row0 + (lane >> 5)) * row_stride + (lane & 31) * 16;
    f32x4_t acc[RT][NMAT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int t = 0; t < NMAT; ++t) acc[rt][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    constexpr bool DIRECT = DB == 0;
    using Slab = WSlab<NMAT, RT, DIRECT ? NTERM * KS : 0>;
    int sa = 0;
    auto load_next = [&](Slab& buf, bool advance) {
#pragma unroll
      for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int t = 0; t < NMAT; ++t)
#pragma unroll
          for (int i = 0; i < 8; ++i)
            buf.a[t][rt][i] = load_stream16(wsrc + t * mat_stride + (size_t)(16 * rt + 2 * i) * row_stride + (size_t)sa * KS * 64);
      if constexpr (DIRECT) {
#pragma unroll
        for (int term = 0; term < NTERM; ++term)
#pragma unroll
          for (int s = 0; s < KS; ++s) buf.b[term * KS + s] = (term == 0 ? bop0 : bop1)[((size_t)sa * KS + s) * 64 + lane];
      }
      if (advance) ++sa;
    };
    int sc = 0;
    // the workgroup's next operand slab on its way from L2 to LDS, a value (not an array written
    // in place under a condition, which the compiler keeps in scratch memory)
    struct Stage { uint4 v[kVecsPerThread]; };
    auto fetch_operand = [&](int slab) -> Stage {
      Stage st;
#pragma unroll
      for (int v = 0; v < kVecsPerThread; ++v) {
        const int idx = v * kThreads + tid;                // vector index inside the slab: [term][step][lane]
        const int term = idx / (KS * 64), r = idx - term * (KS * 64);
        const uint4* src = term == 0 ? bop0 : bop1;
        st.v[v] = src[(size_t)slab * KS * 64 + r];
      }
      return st;
    };
    Stage stage;
    auto consume = [&](const Slab& buf) {
      // single buffer: wait until everyone is done with the previous slab; double buffer: the
      // other half was last read two slabs ago and every wavefront has passed a barrier since
      uint4* bslab = lds + (DB == 2 ? (sc & 1) * kSlabVecs : 0);
      if constexpr (!DIRECT) {
        // both barriers order LDS only: a full __syncthreads() would also wait for the weight loads of the
        // next slab, which are already in flight, and with that undo the double buffering
        if (DB == 1) lds_barrier();
#pragma unroll
        for (int v = 0; v < kVecsPerThread; ++v) bslab[v * kThreads + tid] = stage.v[v];
        lds_barrier();
        if (sc + 1 < nslabs) stage = fetch_operand(sc + 1);
      }
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        // the wavefront's own LDS tile: written and read by this wavefront only, program order suffices
#pragma unroll
        for (int t = 0; t < NMAT; ++t)
#pragma unroll
          for (int i = 0; i < 8; ++i)
            *reinterpret_cast<uint4*>(wt_store + (size_t)t * 16 * kRowB + (size_t)(2 * i) * kRowB) = buf.a[t][rt][i];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          uint4 a[NMAT];
#pragma unroll
          for (int t = 0; t < NMAT; ++t) a[t] = *reinterpret_cast<const uint4*>(wt_read + (size_t)t * 16 * kRowB + s * 64);
#pragma unroll
          for (int term = 0; term < NTERM; ++term) {
            const uint4 b = DIRECT ? buf.b[term * KS + s] : bslab[(term * KS + s) * 64 + lane];
#pragma unroll
            for (int t = 0; t < NMAT; ++t) acc[rt][t] = mfma16(a[t], b, acc[rt][t]);
          }
        }
      }
      ++sc;
    };
    if constexpr (!DIRECT) stage = fetch_operand(0);
    stream_bufs<Slab>(nslabs, load_next, consume, [] {});
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) epilogue(row0 + 16 * rt, acc[rt]);
  }
}

// gate/up: rows f of W1 and W3 (interleaved in the image), reduction over H
template <int KS, int DB>
__global__ __launch_bounds__(kBThreads) void grouped_gateup_mfma_kernel(BatchArgs p) {
  extern __shared__ uint4 lds[];
  const int e = blockIdx.y;
  const int cnt = p.bkt_count[e];
  if (cnt == 0) return;
  const char* base = static_cast<const char*>(p.bkt_base[e]);
  const int lane = threadIdx.x & 63, n = lane & 15, q = lane >> 4;
  const float wn = n < cnt ? p.bkt_w[e * kBTok + n] : 0.f;
  const size_t row_bytes = (size_t)p.H * 2;
  uint16_t* ahi = p.a_hi + (size_t)e * p.F * kBTok;
  uint16_t* alo = p.a_lo + (size_t)e * p.F * kBTok;
  auto epilogue = [&](int f0, const f32x4_t (&acc)[2]) {
    // lane holds rows f0 + 4 q + r (r = 0..3) of token column n; A goes out in the operand
    // order of the down GEMM (reduction index f), split into hi + lo bfloat16
    uint16_t hi[4], lo[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float v = wn * silu_f32(acc[0][r]) * acc[1][r];
      if (p.two_terms) {
        const uint32_t h = __builtin_bit_cast(uint32_t, v) & 0xffff0000u;   // truncated high part, v - hi is exact
        hi[r] = (uint16_t)(h >> 16);
        lo[r] = f32_to_bf16_bits(v - __builtin_bit_cast(float, h));
      } else {
        hi[r] = f32_to_bf16_bits(v);   // single term: round to nearest
        lo[r] = 0;
      }
    }
    const int f = f0 + 4 * q;                              // first of the lane's four consecutive rows
    const size_t pos = ((size_t)(f >> 5) * 64 + ((f >> 3) & 3) * 16 + n) * 8 + (f & 7);
    *reinterpret_cast<uint2*>(ahi + pos) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
    *reinterpret_cast<uint2*>(alo + pos) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
  };
  const uint4* xop = reinterpret_cast<const uint4*>(p.xop) + (size_t)e * (p.H / 32) * 64;
  grouped_gemm_tile_loop<KS, 2, 1, 1, kBWaves, DB>(base, 2 * row_bytes, row_bytes, p.H / 32, p.F / (16 * kBWaves), blockIdx.x, gridDim.x,
                                   xop, xop, lds, epilogue);
}

// gate/up without a break between tiles.  With one tile per workgroup a compute unit starts from an
// empty pipeline seven times per launch at Mixtral size (1792 workgroups of one wavefront per SIMD each):
// the last loads of a tile are issued two slabs before its end and the next workgroup's first loads
// only after it has been dispatched.  Here a launch has one workgroup per compute unit and every
// wavefront walks its own sequence of units (16 row pairs of one active expert, all slabs) as one
// stream of slabs: the loads of the next unit are in flight while the current one is finished.
// Units are dealt out round robin over the experts that have tokens (bucket_gather_kernel lists
// them), so that experts without tokens cost nothing.  Same arithmetic, same order of additions
// and same results as the tile-per-workgroup kernel.
template <int KS>
__global__ __launch_bounds__(kBThreads) void grouped_gateup_stream_kernel(BatchArgs p) {
  extern __shared__ uint4 lds[];
  __shared__ int s_act[64];
  __shared__ const char* s_base[64];
  __shared__ float s_w[64 * kBTok];
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int nact = p.bkt_active[p.N];
  if (tid < 64) {
    const int e = tid < nact ? p.bkt_active[tid] : 0;
    s_act[tid] = e;
    s_base[tid] = tid < nact ? static_cast<const char*>(p.bkt_base[e]) : nullptr;
  }
  for (int i = tid; i < nact * kBTok; i += kBThreads) {
    const int e = p.bkt_active[i / kBTok], n = i % kBTok;
    s_w[i] = n < p.bkt_count[e] ? p.bkt_w[e * kBTok + n] : 0.f;
  }
  __syncthreads();

  const int m = lane & 15, q = lane >> 4;
  constexpr int kRowB = wtile_row_bytes<KS>();
  char* wt = reinterpret_cast<char*>(lds) + (size_t)wave * 2 * 16 * kRowB;   // this wavefront's tiles (W1 rows, W3 rows)
  char* wt_store = wt + (lane >> 5) * kRowB + (lane & 31) * 16;
  const char* wt_read = wt + m * kRowB + q * 16;
  const size_t row_bytes = (size_t)p.H * 2;
  const int nslabs = p.H / 32 / KS, upe = p.F / 16;       // slabs per unit, units per expert
  const int total = nact * upe, nwaves = gridDim.x * kBWaves, w0 = blockIdx.x * kBWaves + wave;
  const int nunits = w0 < total ? (total - w0 + nwaves - 1) / nwaves : 0;
  const uint4* xop_all = reinterpret_cast<const uint4*>(p.xop);
  const size_t xop_stride = (size_t)(p.H / 32) * 64;      // 16-byte vectors per expert

  using Slab = WSlab<2, 1, KS>;
  // load cursor: unit ua (its expert's position among the active ones and its first row pair), slab sa
  int ua = w0, sa = 0;
  const char* wsrc = nullptr;
  const uint4* bsrc = nullptr;
  auto open_load_unit = [&](int u) {
    const int a = u / upe, f0 = (u - a * upe) * 16;
    wsrc = s_base[a] + (size_t)(f0 + (lane >> 5)) * 2 * row_bytes + (lane & 31) * 16;
    bsrc = xop_all + (size_t)s_act[a] * xop_stride + lane;
  };
  if (nunits > 0) open_load_unit(ua);
  auto load_next = [&](Slab& buf, bool advance) {
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        buf.a[t][0][i] = load_stream16(wsrc + t * row_bytes + (size_t)(2 * i) * 2 * row_bytes + (size_t)sa * KS * 64);
#pragma unroll
    for (int s = 0; s < KS; ++s) buf.b[s] = bsrc[((size_t)sa * KS + s) * 64];
    if (advance && ++sa == nslabs) {
      sa = 0;
      ua += nwaves;
      if (ua < total) open_load_unit(ua);
    }
  };
  // consume cursor
  int uc = w0, sc = 0;
  f32x4_t acc[2];
  auto consume = [&](const Slab& buf) {
    if (sc == 0) acc[0] = acc[1] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // the wavefront's own LDS tile: written and read by this wavefront only, program order suffices
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        *reinterpret_cast<uint4*>(wt_store + (size_t)t * 16 * kRowB + (size_t)(2 * i) * kRowB) = buf.a[t][0][i];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint4 a = *reinterpret_cast<const uint4*>(wt_read + (size_t)t * 16 * kRowB + s * 64);
        acc[t] = mfma16(a, buf.b[s], acc[t]);
      }
    }
    if (++sc == nslabs) {
      // lane holds rows f0 + 4 q + r (r = 0..3) of token column m; A goes out in the operand order of
      // the down GEMM (reduction index f), as hi + lo bfloat16 or rounded to bfloat16
      const int a = uc / upe, f0 = (uc - a * upe) * 16;
      const int e = s_act[a];
      const float wn = s_w[a * kBTok + m];
      uint16_t hi[4], lo[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = wn * silu_f32(acc[0][r]) * acc[1][r];
        if (p.two_terms) {
          const uint32_t h = __builtin_bit_cast(uint32_t, v) & 0xffff0000u;   // truncated high part, v - hi is exact
          hi[r] = (uint16_t)(h >> 16);
          lo[r] = f32_to_bf16_bits(v - __builtin_bit_cast(float, h));
        } else {
          hi[r] = f32_to_bf16_bits(v);
          lo[r] = 0;
        }
      }
      const int f = f0 + 4 * q;
      const size_t pos = (size_t)e * p.F * kBTok + ((size_t)(f >> 5) * 64 + ((f >> 3) & 3) * 16 + m) * 8 + (f & 7);
      *reinterpret_cast<uint2*>(p.a_hi + pos) = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
      *reinterpret_cast<uint2*>(p.a_lo + pos) = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
      sc = 0;
      uc += nwaves;
    }
  };
  stream_bufs<Slab>(nunits * nslabs, load_next, consume, [] {});
}

// down: rows h of W2, reduction over F, result added into y of the bucket's tokens
template <int KS, int RT, int NW, int NTERM>
__global__ __launch_bounds__(NW * kWave) void grouped_down_mfma_kernel(BatchArgs p) {
  extern __shared__ uint4 lds[];
  const int e = blockIdx.y;
  const int cnt = p.bkt_count[e];
  if (cnt == 0) return;
  const char* base = static_cast<const char*>(p.bkt_base[e]) + p.w2_offset;
  const int lane = threadIdx.x & 63, n = lane & 15, q = lane >> 4;
  const int tok = n < cnt ? p.bkt_tok[e * kBTok + n] : -1;
  auto epilogue = [&](int h0, const f32x4_t (&acc)[1]) {
    if (tok < 0) return;
    float* yr = p.y + (size_t)tok * p.H + h0 + 4 * q;
    // a token receives at most two contributions (its two experts) onto a cleared row:
    // the sum does not depend on their order
#pragma unroll
    for (int r = 0; r < 4; ++r) atomicAdd(yr + r, acc[0][r]);
  };
  const uint4* ahi = reinterpret_cast<const uint4*>(p.a_hi) + (size_t)e * (p.F / 32) * 64;
  const uint4* alo = reinterpret_cast<const uint4*>(p.a_lo) + (size_t)e * (p.F / 32) * 64;
  grouped_gemm_tile_loop<KS, 1, NTERM, RT, NW, 1>(base, (size_t)p.F * 2, 0, p.F / 32, p.H / (16 * NW * RT), blockIdx.x, gridDim.x, ahi, alo, lds,
                                   epilogue);
}

// ------------------------------------------------------------------ launch ---

constexpr int kGateUpKS = 8;
constexpr int kDownKS = 8;

template <typename K>
static hipError_t big_lds(K k) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(k), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
}

hipError_t batched_kernels_init() {
  hipError_t e;
  if ((e = big_lds(grouped_gateup_mfma_kernel<kGateUpKS, 1>)) != hipSuccess) return e;
  if ((e = big_lds(grouped_gateup_mfma_kernel<kGateUpKS, 0>)) != hipSuccess) return e;
  // this kernel also has static LDS arrays: ask for what its wavefront tiles need, not for all of the LDS
  if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(grouped_gateup_stream_kernel<kGateUpKS>), hipFuncAttributeMaxDynamicSharedMemorySize,
                               (int)grouped_lds_bytes<kGateUpKS, 2, 1, kBWaves, 0>())) != hipSuccess) return e;
  if ((e = big_lds(grouped_down_mfma_kernel<kDownKS, 1, 8, 2>)) != hipSuccess) return e;
  return big_lds(grouped_down_mfma_kernel<kDownKS, 1, 8, 1>);
}

hipError_t launch_bucket_gather(const BatchArgs& p, hipStream_t s, const KernelTiming& t) {
  dim3 grid((p.H / 32 + 3) / 4, p.N), block(kBThreads);
  launch_kernel(bucket_gather_kernel, grid, block, 0, s, t, p);
  return hipGetLastError();
}

hipError_t launch_grouped_gateup(const BatchArgs& p, int mode, hipStream_t s, const KernelTiming& t) {
  // mode 1: every wavefront loads its own operand vectors (no workgroup barriers), measured 10 %
  // faster than staging them per workgroup (mode 0); mode 2: the same with one workgroup per compute
  // unit, every wavefront streaming through its units without a break (needs at least two slabs per unit)
  if (mode == 2 && p.H / 32 / kGateUpKS >= 2) {
    static int cus = 0;
    if (cus == 0) {
      int dev = 0, n = 0;
      if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
      cus = n;
    }
    const int units = p.N * (p.F / 16);
    dim3 grid(std::max(1, std::min(cus, (units + kBWaves - 1) / kBWaves))), block(kBThreads);   // two workgroups per compute unit measured no faster
    constexpr size_t lds = grouped_lds_bytes<kGateUpKS, 2, 1, kBWaves, 0>();
    launch_kernel(grouped_gateup_stream_kernel<kGateUpKS>, grid, block, lds, s, t, p);
    return hipGetLastError();
  }
  dim3 grid(p.F / (16 * kBWaves), p.N), block(kBThreads);
  if (mode != 0) {
    constexpr size_t lds = grouped_lds_bytes<kGateUpKS, 2, 1, kBWaves, 0>();
    launch_kernel(grouped_gateup_mfma_kernel<kGateUpKS, 0>, grid, block, lds, s, t, p);
  } else {
    constexpr size_t lds = grouped_lds_bytes<kGateUpKS, 2, 1, kBWaves, 1>();
    launch_kernel(grouped_gateup_mfma_kernel<kGateUpKS, 1>, grid, block, lds, s, t, p);
  }
  return hipGetLastError();
}

// down: 8 wavefronts x 16 rows per workgroup, operand slab staged in LDS (the barrier-free variant
// and 4 x 32 rows measured slower here).  `two_terms` multiplies by A = hi + lo (fp32 accuracy);
// otherwise by A rounded to bfloat16 only.
hipError_t launch_grouped_down(const BatchArgs& p, bool two_terms, hipStream_t s, const KernelTiming& t) {
  dim3 grid(p.H / 128, p.N), block(512);
  if (two_terms) {
    constexpr size_t lds = grouped_lds_bytes<kDownKS, 1, 2, 8, 1>();
    launch_kernel(grouped_down_mfma_kernel<kDownKS, 1, 8, 2>, grid, block, lds, s, t, p);
  } else {
    constexpr size_t lds = grouped_lds_bytes<kDownKS, 1, 1, 8, 1>();
    launch_kernel(grouped_down_mfma_kernel<kDownKS, 1, 8, 1>, grid, block, lds, s, t, p);
  }
  return hipGetLastError();
}

}  // namespace adapmoe
