// Expert FFN for decode with 4-bit group-quantised weights (groups of 64 along
// the reduction axis, fp16 scale and zero per group; weight = code*scale+zero).
// The paper runs its experts in 4 bit (Sec. 6.3); dequantisation is fused into
// the GEMVs of Eq.2 so that only the packed image crosses HBM (9/16 byte per
// weight).
//
// Image of one expert (n = row length, G = n/64 groups per row):
//   row   = [codes, n/2 bytes][G x (fp16 scale, fp16 zero)]
//   codes = blocks of up to 64 groups; a block of nb groups is
//           [first 16 bytes of every group (nb x 16)][second 16 bytes of every group]
//           so that lane l of a wavefront owns group l of the block and every
//           load instruction reads a contiguous run;
//   inside a group's 32 bytes, dword d holds elements 8d..8d+7 with nibble s
//           (s < 4) = element 8d+2s and nibble s+4 = element 8d+2s+1.
//   image = rows of W1 and W3 interleaved (W1[0], W3[0], W1[1], ...) then rows of W2.
//
// The 2-bit variant (the paper's second setting stores MoE blocks in 2 bit, Sec. 6.3) uses the
// same scheme with 2-bit codes: a group's 64 codes are one 16-byte vector, a block of nb groups
// is nb x 16 bytes, and inside a dword field s (s < 8, bits 2s) is element 2s and field s+8 is
// element 2s+1 of the dword's 16 elements; 5/16 byte per weight.
//
// Arithmetic: codes are turned into half-precision numbers without being moved.  A code field
// that lies inside the 10 mantissa bits of a half whose exponent is 2^10 reads as 1024 + code
// if it starts at bit 0 and as 1024 + 2^p * code if it starts at bit p, so one mask-and-or per
// field position yields a packed pair of halves; the fields of the upper byte of each half are
// brought down by one shift of the dword.  v_dot2_f32_f16 multiplies the pair with a packed pair
// of activations (held as halves) and accumulates in fp32, one accumulator per field position p
// ("class": 2 for 4-bit, 4 for 2-bit codes).  Per group, with xs_p the sum of the activations
// that meet class p,
//   sum (q s + z) x = s * sum_p 2^-p (acc_p - 1024 xs_p) + z * sum_p xs_p.
// That is 9 vector operations per 8 weights (4-bit) instead of 11 with one shift per field.
// Activations: x arrives as bfloat16 and is converted to half (exact for 6.1e-5 <= |x| <= 65504,
// clamped above, truncated to the half subnormal grid of 6e-8 below); the gate/up kernel writes
// a_j = w_j silu(g) u as halves for the down kernel.
#include <algorithm>
#include "../../include/adapmoe.h"
#include "stream_parts.h"

namespace adapmoe {

typedef __attribute__((ext_vector_type(2))) _Float16 f16x2_t;

// gate/up workgroup: 4 wavefronts (16 per workgroup measured 1 us slower per launch at Mixtral size)
template <int NBLK>
constexpr int gateup_threads() { return 256; }
constexpr int kQDownThreads = 1024;   // 16 wavefronts, one output row at a time each

template <int BITS>
__device__ __forceinline__ size_t q_row_bytes(int n) { return (size_t)n * BITS / 8 + (size_t)n / 16; }

// field positions inside a byte that are used without a shift ("classes"): 4-bit codes at bits 0 and 4,
// 2-bit codes at bits 0, 2, 4, 6
template <int BITS>
struct QTraits {
  static constexpr int NC = 8 / BITS;
};

// The masks and the exponent pattern live in registers (fetched through opaque
// moves) so that (v & mask) | pattern is a single v_and_or_b32; as literals the
// compiler has to split it into two instructions (VOP3 takes no literals here).
template <int BITS>
struct QConsts {
  uint32_t mask[QTraits<BITS>::NC];
  uint32_t magic;
};
template <int BITS>
__device__ __forceinline__ QConsts<BITS> q_consts() {
  QConsts<BITS> k;
  if constexpr (BITS == 4) {
    asm("s_mov_b32 %0, 0x000F000F" : "=s"(k.mask[0]));
    asm("s_mov_b32 %0, 0x00F000F0" : "=s"(k.mask[1]));
  } else {
    asm("s_mov_b32 %0, 0x00030003" : "=s"(k.mask[0]));
    asm("s_mov_b32 %0, 0x000C000C" : "=s"(k.mask[1]));
    asm("s_mov_b32 %0, 0x00300030" : "=s"(k.mask[2]));
    asm("s_mov_b32 %0, 0x00C000C0" : "=s"(k.mask[3]));
  }
  asm("v_mov_b32 %0, 0x64006400" : "=v"(k.magic));   // two halves of value 1024
  return k;
}

// acc += a.lo*b.lo + a.hi*b.hi for two packed half pairs, fp32 accumulate
__device__ __forceinline__ float dot2_f16(uint32_t a, uint32_t b, float acc) {
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2_t, a), __builtin_bit_cast(f16x2_t, b), acc, false);
}

__device__ __forceinline__ uint32_t pick(const uint4& v, int c) { return c == 0 ? v.x : c == 1 ? v.y : c == 2 ? v.z : v.w; }

// Accumulators of one group, one per class.
template <int BITS>
struct QAcc {
  float v[QTraits<BITS>::NC];
};

// One 16-byte vector of codes against the matching activations (packed half pairs):
// 4-bit: 32 codes, x[0..3] (dword d meets x[d]: pairs .x .y .z .w are its nibble positions 0..3);
// 2-bit: 64 codes, x[0..7] (dword d meets x[2d] with its fields 0..3 and x[2d+1] with its fields 4..7).
template <int BITS>
__device__ __forceinline__ void dot_codes16(const uint4& c, const uint4* x, QAcc<BITS>& acc, const QConsts<BITS>& k) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint32_t t = w[d] >> 8;
    if constexpr (BITS == 4) {
      const uint4 xv = x[d];
      acc.v[0] = dot2_f16((w[d] & k.mask[0]) | k.magic, xv.x, acc.v[0]);
      acc.v[1] = dot2_f16((w[d] & k.mask[1]) | k.magic, xv.y, acc.v[1]);
      acc.v[0] = dot2_f16((t & k.mask[0]) | k.magic, xv.z, acc.v[0]);
      acc.v[1] = dot2_f16((t & k.mask[1]) | k.magic, xv.w, acc.v[1]);
    } else {
      const uint4 xa = x[2 * d], xb = x[2 * d + 1];
#pragma unroll
      for (int cl = 0; cl < 4; ++cl) {
        acc.v[cl] = dot2_f16((w[d] & k.mask[cl]) | k.magic, pick(xa, cl), acc.v[cl]);
        acc.v[cl] = dot2_f16((t & k.mask[cl]) | k.magic, pick(xb, cl), acc.v[cl]);
      }
    }
  }
}

// What a group's activations contribute besides the code products: xsum = sum of its 64 values,
// nxq = -1024 * sum_p 2^-p xs_p (minus the offsets that the mantissa trick adds, see the file
// comment; the accumulator of class 0 starts from it).
struct GroupSums {
  float xsum, nxq;
};
// x: the group's 64 halves as 8 vectors of packed pairs.  In both formats component c of every vector
// meets class c mod NC.
template <int BITS>
__device__ __forceinline__ GroupSums group_sums(const uint4* x) {
  const uint32_t ones = 0x3C003C00u;
  float s[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    s[0] = dot2_f16(x[j].x, ones, s[0]);
    s[1] = dot2_f16(x[j].y, ones, s[1]);
    s[2] = dot2_f16(x[j].z, ones, s[2]);
    s[3] = dot2_f16(x[j].w, ones, s[3]);
  }
  GroupSums g;
  g.xsum = (s[0] + s[1]) + (s[2] + s[3]);
  if constexpr (BITS == 4) g.nxq = -1024.f * ((s[0] + s[2]) + 0.0625f * (s[1] + s[3]));
  else g.nxq = -1024.f * ((s[0] + 0.25f * s[1]) + (0.0625f * s[2] + 0.015625f * s[3]));
  return g;
}

template <int BITS>
struct QGroup {  // what one lane holds of one row block: its group's codes (BITS/2 vectors) and (scale, zero)
  uint4 c[BITS / 2];
  uint32_t sz;
};

// Byte offsets of a lane inside a row block of nb groups: its 16-byte code vectors and its
// (scale, zero) pair.  Lanes beyond nb take the block's last group (no branch around the loads, so
// the compiler can count outstanding loads exactly); their activations are zero, so they add nothing.
struct LaneOff {
  uint32_t c16, s4;
};
__device__ __forceinline__ LaneOff lane_off(int lane, int nb) {
  const int l = min(lane, nb - 1);
  return LaneOff{(uint32_t)l * 16u, (uint32_t)l * 4u};
}

// lane's share of block `blk` (nb groups) of the row starting at `row`.  `row`, n and blk are the
// same for all lanes (the address is a scalar base plus the lane's 32-bit offset).
template <int BITS>
__device__ __forceinline__ void q_load_group(const char* row, int n, int blk, int nb, const LaneOff& lo, QGroup<BITS>& g) {
  // every uniform part of an address is folded into a scalar base first (pinned to scalar registers
  // by the empty asm statement), so that each load is "scalar base + the lane's 32-bit offset"
#pragma unroll
  for (int v = 0; v < BITS / 2; ++v) {
    const char* pv = row + ((size_t)blk * (64 * BITS * 8) + (size_t)(v * nb * 16));
    asm volatile("" : "+s"(pv));
    g.c[v] = load_stream16(pv + lo.c16);
  }
  const char* ps = row + ((size_t)n * BITS / 8 + (size_t)blk * 256);
  asm volatile("" : "+s"(ps));
  g.sz = load_stream4(ps + lo.s4);
}

// The lane offsets, opaque to the optimiser from here on: the instruction selector forms "scalar
// base + 32-bit lane offset" addresses only if it sees the widening of the offset in the same block
// as the load; a widening hoisted out of the streaming loop costs a 64-bit vector addition per load.
__device__ __forceinline__ LaneOff fresh(LaneOff lo) {
  asm volatile("" : "+v"(lo.c16), "+v"(lo.s4));
  return lo;
}

// value of the lane's group: sum (q s + z) x.  Activations of lanes without a group must be zero.
template <int BITS>
__device__ __forceinline__ float q_group_dot(const QGroup<BITS>& g, const uint4* x, const GroupSums& gs, const QConsts<BITS>& k) {
  QAcc<BITS> acc;
  acc.v[0] = gs.nxq;
#pragma unroll
  for (int c = 1; c < QTraits<BITS>::NC; ++c) acc.v[c] = 0.f;
  if constexpr (BITS == 4) {
    dot_codes16<4>(g.c[0], x, acc, k);
    dot_codes16<4>(g.c[1], x + 4, acc, k);
  } else {
    dot_codes16<2>(g.c[0], x, acc, k);
  }
  float d;
  if constexpr (BITS == 4) d = fmaf(0.0625f, acc.v[1], acc.v[0]);
  else d = fmaf(0.015625f, acc.v[3], fmaf(0.0625f, acc.v[2], fmaf(0.25f, acc.v[1], acc.v[0])));
  const float s = half_bits_to_float(g.sz & 0xffffu), z = half_bits_to_float(g.sz >> 16);
  return fmaf(s, d, z * gs.xsum);
}

// float -> half bits, round to nearest even, clamped to the finite range
__device__ __forceinline__ uint32_t f32_to_f16_bits(float f) {
  f = __builtin_fminf(__builtin_fmaxf(f, -65504.f), 65504.f);
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);
}
// a packed pair of bfloat16 -> a packed pair of halves.  A bfloat16 has fewer mantissa bits than a
// half, so inside the half's normal range the conversion is exact whatever the rounding; the
// round-toward-zero pack instruction is used because it also clamps: magnitudes beyond the range
// come out as 65504 instead of infinity (below 6.1e-5 it truncates to the subnormal grid of 6e-8).
__device__ __forceinline__ uint32_t bf16x2_to_f16x2(uint32_t u) {
  return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(bf16_lo(u), bf16_hi(u)));
}
__device__ __forceinline__ uint4 bf16x8_to_f16x8(const uint4& v) {
  return make_uint4(bf16x2_to_f16x2(v.x), bf16x2_to_f16x2(v.y), bf16x2_to_f16x2(v.z), bf16x2_to_f16x2(v.w));
}

// position (in 16-bit elements) of a_j[f] in the scratch vector the down kernel reads:
// [block of 64 groups][vector c of 8][lane = group in block][8 elements]
__device__ __forceinline__ int i4_a_pos(int f) {
  const int g = f >> 6, i = f & 63;
  return (((g >> 6) * 8 + (i >> 3)) * 64 + (g & 63)) * 8 + (i & 7);
}

// ------------------------------------------------------------------ gate/up --

template <int BITS, int NBLK>
struct I4RowPair {
  QGroup<BITS> g1[NBLK], g3[NBLK];
};

// One wavefront per row pair; lane l owns group l (+64 per further block) of
// both rows, its share of x stays in registers for the whole kernel.  Row numbers and row
// addresses are wavefront-uniform and kept on the scalar unit: the kernel sits close to the
// vector-ALU limit, so whatever is not arithmetic on the codes is kept off the vector unit.
template <int BITS, int NBLK>
__global__ __launch_bounds__(gateup_threads<NBLK>()) void ffn_gateup_quant_kernel(FfnArgs p) {
  constexpr int kI4GateUpThreads = gateup_threads<NBLK>();
  const int b = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = wave_index();
  const int H = p.H, F = p.F;
  const size_t rb = q_row_bytes<BITS>(H);
  const QConsts<BITS> kc = q_consts<BITS>();

  // The lane's groups of x (as halves) and their sums.  x is read from global
  // memory in order (one 16-byte piece per thread), converted and turned through LDS:
  // piece j of group g goes to slot (block, j, lane = g % 64), which each lane
  // then reads back without bank conflicts.  Lanes without a group get zeros.
  extern __shared__ uint4 xs[];
  uint4 x[NBLK][8];
  GroupSums xsum[NBLK];
  const uint4* xg = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(p.x) + (size_t)b * H);
  // The pieces of x are requested first of all, before the expert pointers are fetched, and turned
  // through LDS after the first weight requests, all without conditions.  The weight requests of the
  // whole chip start a microsecond into the launch and keep the queues of the memory system full
  // from then on: a small load issued among them comes back microseconds later, and no wavefront
  // can compute before x is in its registers.  Issued ahead of all of them, x is there within 2 us.
  constexpr int kXRounds = (NBLK * 512 + kI4GateUpThreads - 1) / kI4GateUpThreads;
  struct StageX {
    uint4 v[kXRounds];
  };
  const int pieces = H >> 3;
  auto stage_x_issue = [&]() -> StageX {
    StageX sx;
#pragma unroll
    for (int u = 0; u < kXRounds; ++u) sx.v[u] = xg[min((int)threadIdx.x + u * kI4GateUpThreads, pieces - 1)];
    return sx;
  };
  auto stage_x = [&](const StageX& sx) {
#pragma unroll
    for (int u = 0; u < kXRounds; ++u) {
      const int c = threadIdx.x + u * kI4GateUpThreads;
      const int g = c >> 3, j = c & 7;
      if (c < NBLK * 512) xs[((g >> 6) * 8 + j) * 64 + (g & 63)] = c < pieces ? bf16x8_to_f16x8(sx.v[u]) : make_uint4(0, 0, 0, 0);
    }
    lds_barrier();
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) x[i][j] = xs[(i * 8 + j) * 64 + lane];
      xsum[i] = group_sums<BITS>(x[i]);
    }
  };

  const StageX sxv = stage_x_issue();   // before anything else of this launch asks for memory

  const char* base[2];
  float wj[2];
  // what resolve_experts returns was loaded per lane; told that it is the same in every lane, the
  // compiler keeps everything derived from it (row counts, cursors, branches) on the scalar unit
  const int kk = __builtin_amdgcn_readfirstlane(resolve_experts(p, b, base, wj));
  base[0] = uniform_ptr(base[0]);
  base[1] = uniform_ptr(base[1]);
  // resident activated experts taking part, rank order (written with selects: arrays indexed
  // with run-time values would live in scratch memory)
  const bool windowed = p.j_only >= 0;
  const bool t0 = base[0] != nullptr && (!windowed || p.j_only == 0);
  const bool t1 = kk > 1 && base[1] != nullptr && (!windowed || p.j_only == 1);
  const int nv = (int)t0 + (int)t1;
  const char* rbase[2] = {t0 ? base[0] : base[1], base[1]};
  const float rw[2] = {t0 ? wj[0] : wj[1], wj[1]};
  const int rj[2] = {t0 ? 0 : 1, 1};

  // rows are numbered r = (index among the taking-part experts) * F + f
  const int total = windowed ? (nv ? p.r1 : 0) : nv * F;
  const int stride = gridDim.x * (kI4GateUpThreads / kWave);
  const int first = (windowed ? p.r0 : 0) + blockIdx.x * (kI4GateUpThreads / kWave) + wave;
  const int nrows = first < total ? (total - first + stride - 1) / stride : 0;
  uint16_t* a_out = reinterpret_cast<uint16_t*>(p.a + (size_t)b * 2 * p.a_stride);

  // groups per block and the lane's offsets inside each block
  int nbs[NBLK];
  LaneOff lo[NBLK];
#pragma unroll
  for (int i = 0; i < NBLK; ++i) {
    nbs[i] = min(64, (H >> 6) - i * 64);
    lo[i] = lane_off(lane, nbs[i]);
  }

  auto load_row = [&](I4RowPair<BITS, NBLK>& buf, int r_any) {
    const int r = __builtin_amdgcn_readfirstlane(r_any);   // the same in every lane: address arithmetic on the scalar unit
    const int j = r >= F ? 1 : 0;
    const char* row = pick2(rbase, j) + (size_t)(r - j * F) * 2 * rb;
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      const LaneOff l = fresh(lo[i]);
      q_load_group(row, H, i, nbs[i], l, buf.g1[i]);
      q_load_group(row + rb, H, i, nbs[i], l, buf.g3[i]);
    }
  };
  // The two sums of a row pair come out of one joint reduction (gate sum in lanes 0..31, up sum in
  // lanes 32..63) and are parked in lanes ns and ns + 32 of `parked`; SiLU, the product, the rounding
  // and the store are then done for up to 32 row pairs at once, one per lane, instead of by the whole
  // wavefront for every pair.  Parked pairs are consecutive rows of this wavefront: pair i of a batch
  // is row rpark + i * stride.
  float parked = 0.f;
  int ns = 0, rpark = first;
  const int lane31 = lane & 31;
  auto flush = [&]() {
    const float other = swap_halves(parked);   // lanes < 32: the up sum of their pair
    if (lane < ns) {
      const int rv = rpark + lane * stride;
      const int j = rv >= F ? 1 : 0;
      const int f = rv - j * F;
      a_out[(size_t)pick2(rj, j) * 2 * p.a_stride + i4_a_pos(f)] = (uint16_t)f32_to_f16_bits(pick2(rw, j) * silu_f32(parked) * other);
    }
    rpark += ns * stride;
    ns = 0;
  };
  auto consume_row = [&](const I4RowPair<BITS, NBLK>& buf) {
    float g = q_group_dot(buf.g1[0], x[0], xsum[0], kc), u = q_group_dot(buf.g3[0], x[0], xsum[0], kc);
#pragma unroll
    for (int i = 1; i < NBLK; ++i) {
      g += q_group_dot(buf.g1[i], x[i], xsum[i], kc);
      u += q_group_dot(buf.g3[i], x[i], xsum[i], kc);
    }
    const float s = pair_sum(g, u);
    parked = lane31 == ns ? s : parked;
    if (++ns == 32) flush();
  };

  // Rows are dealt out in advance, row first + i * stride to this wavefront.  (Drawing the last
  // passes from shared counters, as the fp32/bf16 kernel does, was measured slower here in every
  // form tried: a wavefront has only seven row pairs at Mixtral size and each draw costs a round trip.)
  int ra = first;
  auto load_next = [&](I4RowPair<BITS, NBLK>& buf, bool advance) {
    load_row(buf, ra);
    if (advance) ra += stride;
  };
  stream_bufs<I4RowPair<BITS, NBLK>, 1>(nrows, load_next, consume_row, [&, sxv]() { stage_x(sxv); });
  flush();
}

// --------------------------------------------------------------------- down --

// A piece of one W2 row of one expert as a wavefront holds it: lane l owns group l of each of the
// piece's PB blocks of 64 groups.
template <int BITS, int PB>
struct QRow {
  QGroup<BITS> g[PB];
};

// (THREADS = 1024 or 768: 12 wavefronts per workgroup when that deals the rows out evenly and 16 do not.)
// One wavefront per output element y[h]; a wavefront streams its rows through four register
// buffers (the unit in flight is one block of 64 groups of a row: 36 bytes per lane with 4-bit
// codes).  The intermediate vectors a_j of the activated experts (halves, written by the
// gate/up kernel in the order [block][vector][lane]) are staged in LDS once per workgroup together
// with the two sums per group that the dequantisation needs, so that the weight stream is the only
// traffic that grows with the number of rows; a lane reads its group's 64 values back with eight
// conflict-free 16-byte reads per block.
template <int BITS, int NBLK, int THREADS>
__global__ __launch_bounds__(THREADS) void ffn_down_quant_kernel(FfnArgs p) {
  extern __shared__ uint4 smem[];   // a[jj][NBLK*8*64] vectors of 8 halves, then sums[jj][NBLK*64]
  const int b = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
  const int H = p.H, F = p.F;
  const size_t rb = q_row_bytes<BITS>(F);
  const int G = F >> 6;
  const QConsts<BITS> kc = q_consts<BITS>();
  constexpr int kWaves = THREADS / kWave;
  constexpr int kAVecs = NBLK * 8 * 64;          // 16-byte vectors of one expert's a_j
  constexpr int PB = 1;                          // blocks per piece
  constexpr int NP = NBLK / PB;                  // pieces per row

  uint4* as = smem;
  GroupSums* sums = reinterpret_cast<GroupSums*>(smem + 2 * kAVecs);

  // Staging of a_j, both slots of the token whatever its k (an unused slot holds old values that
  // nothing reads).  The loads are issued first of all, before the expert pointers are fetched: the
  // weight loads of the whole chip follow a microsecond later and fill the queues of the memory
  // system for the first 5 us of the launch; a small load issued among them comes back only then,
  // and no wavefront can start computing before a_j is in LDS.  Issued ahead of all of them, a_j
  // arrives within 2 us.  The LDS writes come after the first weight requests.
  const uint4* ag = reinterpret_cast<const uint4*>(p.a + (size_t)b * 2 * p.a_stride);
  const int S4 = (int)(p.a_stride >> 2);      // 16-byte vectors per (token, expert) of the scratch
  constexpr int kStage = (2 * kAVecs + THREADS - 1) / THREADS;
  struct StageA {
    uint4 v[kStage];
  };
  auto stage_issue = [&]() -> StageA {
    StageA st;
#pragma unroll
    for (int u = 0; u < kStage; ++u) {
      const int i = min(tid + u * THREADS, 2 * kAVecs - 1);
      const int jj = i >= kAVecs ? 1 : 0;
      st.v[u] = ag[(size_t)jj * S4 + (i - jj * kAVecs)];
    }
    return st;
  };
  const StageA sta = stage_issue();

  const char* base[2];
  float wj[2];
  // what resolve_experts returns was loaded per lane; told that it is the same in every lane, the
  // compiler keeps everything derived from it (row counts, cursors, branches) on the scalar unit
  const int kk = __builtin_amdgcn_readfirstlane(resolve_experts(p, b, base, wj));
  base[0] = uniform_ptr(base[0]);
  base[1] = uniform_ptr(base[1]);
  const size_t w2_off = (size_t)2 * F * q_row_bytes<BITS>(H);
  const bool windowed = p.j_only >= 0;
  // resident activated experts taking part, rank order (selects, not run-time-indexed arrays)
  const bool t0 = base[0] != nullptr && (!windowed || p.j_only == 0);
  const bool t1 = kk > 1 && base[1] != nullptr && (!windowed || p.j_only == 1);
  const int nv = (int)t0 + (int)t1;
  const char* w2[2] = {(t0 ? base[0] : base[1]) + w2_off, base[1] + w2_off};   // w2[1] is used only when nv == 2
  const int rj[2] = {t0 ? 0 : 1, 1};

  const int hlo = windowed ? p.r0 : 0, hhi = windowed ? p.r1 : H;
  const int first = hlo + blockIdx.x * kWaves + wave;
  const int hstride = gridDim.x * kWaves;
  const int nrows = (nv > 0 && first < hhi) ? (hhi - first + hstride - 1) / hstride : 0;
  float* y = p.y + (size_t)b * H;
  const bool accumulate = p.accumulate != 0;
  // the gate/up kernel's row counters are cleared here, ready for its next launch
  if (blockIdx.x == 0 && tid < kDynQueues && p.dyn_clear && !windowed) p.dyn_clear[((size_t)b * kDynQueues + tid) * kDynStride] = 0u;

  auto stage_finish = [&](const StageA& st) {
#pragma unroll
    for (int u = 0; u < kStage; ++u) {
      // vector i of a slot belongs to group (i / 512) * 64 + i % 64; groups beyond the row's G do not
      // exist (the scratch vector holds old values there) and are staged as zeros
      const int i = min(tid + u * THREADS, 2 * kAVecs - 1);
      const int iv = i >= kAVecs ? i - kAVecs : i;
      const bool real = ((iv >> 9) << 6) + (iv & 63) < G;
      as[i] = real ? st.v[u] : make_uint4(0, 0, 0, 0);
    }
    lds_barrier();
    // two sums per group: thread t takes group t % (NBLK*64) of slot t / (NBLK*64)
    if (tid < 2 * NBLK * 64) {
      const int jj = tid / (NBLK * 64), g = tid - jj * (NBLK * 64);
      const uint4* src = as + jj * kAVecs + (g >> 6) * 512 + (g & 63);
      uint4 v[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) v[c] = src[c * 64];
      sums[jj * (NBLK * 64) + g] = group_sums<BITS>(v);
    }
    lds_barrier();
  };

  // The lane's offsets inside a full block and inside the row's last block (which may hold fewer
  // than 64 groups).
  const int nb_last = G - (NBLK - 1) * 64;
  const LaneOff lo_full = lane_off(lane, 64), lo_last = lane_off(lane, nb_last);

  // The number of pieces per row is hidden from the optimiser: when it equals the four buffers of the
  // streamer the compiler specialises the loop body per piece and runs out of registers (spills).
  int np_rt = NP;
  asm volatile("" : "+s"(np_rt));
  // Cursors are wavefront-uniform; the empty asm statements pin them to scalar registers so that row
  // addresses are computed on the scalar unit and the loads take a scalar base plus the lane's offset.
  int ha = first, ja = 0, pa = 0;   // load cursor
  auto load_next = [&](QRow<BITS, PB>& buf, bool advance) {
    asm volatile("" : "+s"(ha), "+s"(ja), "+s"(pa));
    const char* row = pick2(w2, ja) + (size_t)ha * rb;
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      const int blk = pa * PB + i;
      const bool last = blk == NBLK - 1;
      const LaneOff lo = fresh(LaneOff{last ? lo_last.c16 : lo_full.c16, last ? lo_last.s4 : lo_full.s4});
      q_load_group(row, F, blk, last ? nb_last : 64, lo, buf.g[i]);
    }
    if (advance && ++pa == np_rt) {
      pa = 0;
      if (++ja == nv) { ja = 0; ha += hstride; }
    }
  };
  int hc = first, jc = 0, pc = 0;   // consume cursor
  float acc = 0.f;
  auto consume = [&](const QRow<BITS, PB>& buf) {
    asm volatile("" : "+s"(hc), "+s"(jc), "+s"(pc));
    const int slot = pick2(rj, jc);
    const uint4* aj = as + (slot * kAVecs + pc * (PB * 512)) + lane;
    const GroupSums* sj = sums + (slot * (NBLK * 64) + pc * (PB * 64)) + lane;
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      uint4 a[8];
#pragma unroll
      for (int c = 0; c < 8; ++c) a[c] = aj[(i * 8 + c) * 64];
      acc += q_group_dot(buf.g[i], a, sj[i * 64], kc);
      __builtin_amdgcn_sched_barrier(0);   // one block at a time: hoisting the next block's LDS reads costs 32 registers
    }
    if (++pc == np_rt) {
      pc = 0;
      if (++jc == nv) {
        const float s = wave_sum(acc);
        if (lane == 0) y[hc] = accumulate ? y[hc] + s : s;
        acc = 0.f;
        jc = 0;
        hc += hstride;
      }
    }
  };
  stream_bufs4<QRow<BITS, PB>, 1>(nrows * nv * NP, load_next, consume, [&, sta]() { stage_finish(sta); });
  // no activated expert of this token is resident (flagged by resolve_experts): the output is zero
  if (nv == 0 && !accumulate)
    for (int h = first; h < hhi; h += hstride)
      if (lane == 0) y[h] = 0.f;
}

// ------------------------------------------------------------------ launch ---

template <int BITS, int NBLK>
static constexpr size_t q_down_lds() { return (size_t)2 * NBLK * 8 * 64 * 16 + (size_t)2 * NBLK * 64 * sizeof(GroupSums); }

template <typename K>
static hipError_t allow_lds(K kernel, size_t bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int BITS, int THREADS>
static hipError_t quant_init_bits_t() {
  hipError_t e;
  if ((e = allow_lds(ffn_down_quant_kernel<BITS, 1, THREADS>, q_down_lds<BITS, 1>())) != hipSuccess) return e;
  if ((e = allow_lds(ffn_down_quant_kernel<BITS, 2, THREADS>, q_down_lds<BITS, 2>())) != hipSuccess) return e;
  if ((e = allow_lds(ffn_down_quant_kernel<BITS, 3, THREADS>, q_down_lds<BITS, 3>())) != hipSuccess) return e;
  return allow_lds(ffn_down_quant_kernel<BITS, 4, THREADS>, q_down_lds<BITS, 4>());
}
template <int BITS>
static hipError_t quant_init_bits() {
  const hipError_t e = quant_init_bits_t<BITS, kQDownThreads>();
  return e != hipSuccess ? e : quant_init_bits_t<BITS, 768>();
}

hipError_t quant_kernels_init(int bits) { return bits == 4 ? quant_init_bits<4>() : quant_init_bits<2>(); }

hipError_t launch_ffn_gateup_quant(const FfnArgs& p, int bits, const LaunchCfg& lc, hipStream_t s) {
  const int nblk = ((p.H >> 6) + 63) >> 6;
  const int threads = nblk == 1 ? gateup_threads<1>() : gateup_threads<2>();
  const int waves = threads / kWave;
  // lc.gateup_blocks counts workgroups of 16 wavefronts; smaller workgroups are launched in proportion
  int blocks = lc.gateup_blocks * (1024 / threads);
  if (p.j_only >= 0) blocks = std::max(1, std::min(blocks, (p.r1 - p.r0 + waves - 1) / waves));
  dim3 grid(blocks, p.B), block(threads);
  if (bits == 4) {
    if (nblk == 1) launch_kernel(ffn_gateup_quant_kernel<4, 1>, grid, block, 1 * 8192, s, lc.timing, p);
    else launch_kernel(ffn_gateup_quant_kernel<4, 2>, grid, block, 2 * 8192, s, lc.timing, p);
  } else {
    if (nblk == 1) launch_kernel(ffn_gateup_quant_kernel<2, 1>, grid, block, 1 * 8192, s, lc.timing, p);
    else launch_kernel(ffn_gateup_quant_kernel<2, 2>, grid, block, 2 * 8192, s, lc.timing, p);
  }
  return hipGetLastError();
}

template <int BITS, int THREADS>
static void launch_down_quant_t(const FfnArgs& p, int nblk, dim3 grid, hipStream_t s, const KernelTiming& t) {
  dim3 block(THREADS);
  if (nblk == 1) launch_kernel(ffn_down_quant_kernel<BITS, 1, THREADS>, grid, block, q_down_lds<BITS, 1>(), s, t, p);
  else if (nblk == 2) launch_kernel(ffn_down_quant_kernel<BITS, 2, THREADS>, grid, block, q_down_lds<BITS, 2>(), s, t, p);
  else if (nblk == 3) launch_kernel(ffn_down_quant_kernel<BITS, 3, THREADS>, grid, block, q_down_lds<BITS, 3>(), s, t, p);
  else launch_kernel(ffn_down_quant_kernel<BITS, 4, THREADS>, grid, block, q_down_lds<BITS, 4>(), s, t, p);
}

hipError_t launch_ffn_down_quant(const FfnArgs& p, int bits, const LaunchCfg& lc, hipStream_t s) {
  const int rows = p.j_only >= 0 ? p.r1 - p.r0 : p.H;
  // 16 wavefronts per workgroup, or 12 if that wastes less of the last pass over the rows
  auto blocks_for = [&](int waves) { return std::max(1, std::min(lc.down_blocks, (rows + waves - 1) / waves)); };
  const bool twelve = p.j_only < 0 && blocks_for(12) == blocks_for(16) && down_waves_per_workgroup(rows, blocks_for(16)) == 12;
  const int waves = twelve ? 12 : kQDownThreads / kWave;
  dim3 grid(blocks_for(waves), p.B);
  const int nblk = ((p.F >> 6) + 63) >> 6;     // F <= 16384: at most 4 blocks of 64 groups
  if (bits == 4) {
    if (twelve) launch_down_quant_t<4, 768>(p, nblk, grid, s, lc.timing);
    else launch_down_quant_t<4, kQDownThreads>(p, nblk, grid, s, lc.timing);
  } else {
    if (twelve) launch_down_quant_t<2, 768>(p, nblk, grid, s, lc.timing);
    else launch_down_quant_t<2, kQDownThreads>(p, nblk, grid, s, lc.timing);
  }
  return hipGetLastError();
}

}  // namespace adapmoe
