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
// Arithmetic: a nibble pair masked into two bfloat16 mantissas with exponent
// 2^7 reads as (128+q0, 128+q1); v_dot2_f32_bf16 multiplies it with a packed
// bfloat16 activation pair and accumulates in fp32.  Per group
//   sum (q s + z) x = s * sum (128+q) x + (z - 128 s) * sum x.
// The gate/up kernel writes a_j = w_j silu(g) u rounded to bfloat16 (the down
// kernel multiplies it on the same instruction); see the error budget in the
// design notes.
#include "../../include/adapmoe.h"
#include "stream_parts.h"

namespace adapmoe {

constexpr int kI4GateUpThreads = 256;
constexpr int kI4DownThreads = 256;   // 4 wavefronts = 4 blocks of 64 groups of a W2 row
constexpr int kI4DownRows = 4;        // output rows per workgroup

template <int BITS>
__device__ __forceinline__ size_t q_row_bytes(int n) { return (size_t)n * BITS / 8 + (size_t)n / 16; }

// The mask and the exponent pattern live in registers (fetched through opaque
// moves) so that (v & mask) | pattern is a single v_and_or_b32; as literals the
// compiler has to split it into two instructions (VOP3 takes no literals here).
struct I4Consts {
  uint32_t mask, magic;
};
template <int BITS>
__device__ __forceinline__ I4Consts q_consts() {
  I4Consts k;
  if constexpr (BITS == 4) asm("s_mov_b32 %0, 0x000F000F" : "=s"(k.mask));
  else asm("s_mov_b32 %0, 0x00030003" : "=s"(k.mask));
  asm("v_mov_b32 %0, 0x43004300" : "=v"(k.magic));
  return k;
}

// sum over the 32 codes of one 16-byte vector of (128+q) * x, x given as 4 vectors of packed bf16 pairs.
// Four independent accumulators (one per nibble position) keep the dot2 pipeline busy.
__device__ __forceinline__ void dot_codes16(const uint4& c, const uint4* x, float (&acc)[4], const I4Consts& k) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint4 xv = x[d];
    acc[0] = dot2_bf16((w[d] & k.mask) | k.magic, xv.x, acc[0]);
    acc[1] = dot2_bf16(((w[d] >> 4) & k.mask) | k.magic, xv.y, acc[1]);
    acc[2] = dot2_bf16(((w[d] >> 8) & k.mask) | k.magic, xv.z, acc[2]);
    acc[3] = dot2_bf16(((w[d] >> 12) & k.mask) | k.magic, xv.w, acc[3]);
  }
}

// the same for a 16-byte vector of 64 two-bit codes, x given as 8 vectors
__device__ __forceinline__ void dot_codes16_2bit(const uint4& c, const uint4* x, float (&acc)[4], const I4Consts& k) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
  for (int d = 0; d < 4; ++d) {
    const uint4 xa = x[2 * d], xb = x[2 * d + 1];
    acc[0] = dot2_bf16((w[d] & k.mask) | k.magic, xa.x, acc[0]);
    acc[1] = dot2_bf16(((w[d] >> 2) & k.mask) | k.magic, xa.y, acc[1]);
    acc[2] = dot2_bf16(((w[d] >> 4) & k.mask) | k.magic, xa.z, acc[2]);
    acc[3] = dot2_bf16(((w[d] >> 6) & k.mask) | k.magic, xa.w, acc[3]);
    acc[0] = dot2_bf16(((w[d] >> 8) & k.mask) | k.magic, xb.x, acc[0]);
    acc[1] = dot2_bf16(((w[d] >> 10) & k.mask) | k.magic, xb.y, acc[1]);
    acc[2] = dot2_bf16(((w[d] >> 12) & k.mask) | k.magic, xb.z, acc[2]);
    acc[3] = dot2_bf16(((w[d] >> 14) & k.mask) | k.magic, xb.w, acc[3]);
  }
}

// sum of the 64 bfloat16 values of a group held as 8 vectors of packed pairs
__device__ __forceinline__ float sum_group(const uint4* x) {
  const uint32_t ones = 0x3F803F80u;
  float s[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    s[0] = dot2_bf16(x[j].x, ones, s[0]);
    s[1] = dot2_bf16(x[j].y, ones, s[1]);
    s[2] = dot2_bf16(x[j].z, ones, s[2]);
    s[3] = dot2_bf16(x[j].w, ones, s[3]);
  }
  return (s[0] + s[1]) + (s[2] + s[3]);
}

template <int BITS>
struct QGroup {  // what one lane holds of one row block: its group's codes (BITS/2 vectors) and (scale, zero)
  uint4 c[BITS / 2];
  uint32_t sz;
};

// lane's share of block `blk` (nb groups) of the row starting at `row`.  Lanes
// beyond nb re-read the block's last group (no branch around the loads, so the
// compiler can count outstanding loads exactly); i4_group_dot ignores them.
template <int BITS>
__device__ __forceinline__ void i4_load_group(const char* row, int n, int blk, int lane, QGroup<BITS>& g) {
  const int G = n >> 6;
  const int nb = min(64, G - blk * 64);
  const int l = min(lane, nb - 1);
  const char* cb = row + (size_t)blk * (64 * BITS * 8);
#pragma unroll
  for (int v = 0; v < BITS / 2; ++v) g.c[v] = load_stream16(cb + v * nb * 16 + l * 16);
  g.sz = load_stream4(row + (size_t)n * BITS / 8 + (size_t)(blk * 64 + l) * 4);
}

// value of the lane's group: sum (q s + z) x, with xs = sum of the group's x
template <int BITS>
__device__ __forceinline__ float i4_group_dot(const QGroup<BITS>& g, const uint4* x, float xsum, const I4Consts& k, bool live) {
  float a0[4] = {0.f, 0.f, 0.f, 0.f}, a1[4] = {0.f, 0.f, 0.f, 0.f};
  if constexpr (BITS == 4) {
    dot_codes16(g.c[0], x, a0, k);
    dot_codes16(g.c[1], x + 4, a1, k);
  } else {
    dot_codes16_2bit(g.c[0], x, a0, k);
  }
  const float d = ((a0[0] + a0[1]) + (a0[2] + a0[3])) + ((a1[0] + a1[1]) + (a1[2] + a1[3]));
  const float s = half_bits_to_float(g.sz & 0xffffu), z = half_bits_to_float(g.sz >> 16);
  return live ? fmaf(s, d, (z - 128.f * s) * xsum) : 0.f;
}

// position (in bfloat16 elements) of a_j[f] in the scratch vector the down kernel reads:
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
// both rows, its share of x stays in registers for the whole kernel.
template <int BITS, int NBLK>
__global__ __launch_bounds__(kI4GateUpThreads) void ffn_gateup_quant_kernel(FfnArgs p) {
  const int b = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = wave_index();
  const int H = p.H, F = p.F;
  const size_t rb = q_row_bytes<BITS>(H);
  const I4Consts kc = q_consts<BITS>();

  const char* base[2];
  float wj[2];
  const int kk = resolve_experts(p, b, base, wj);
  // resident activated experts taking part, rank order (written with selects: arrays indexed
  // with run-time values would live in scratch memory)
  const bool windowed = p.j_only >= 0;
  const bool t0 = base[0] != nullptr && (!windowed || p.j_only == 0);
  const bool t1 = kk > 1 && base[1] != nullptr && (!windowed || p.j_only == 1);
  const int nv = (int)t0 + (int)t1;
  const char* rbase[2] = {t0 ? base[0] : base[1], base[1]};
  const float rw[2] = {t0 ? wj[0] : wj[1], wj[1]};
  const int rj[2] = {t0 ? 0 : 1, 1};

  // The lane's groups of x (bfloat16) and their sums.  x is read from global
  // memory in order (one 16-byte piece per thread) and turned through LDS:
  // piece j of group g goes to slot (block, j, lane = g % 64), which each lane
  // then reads back without bank conflicts.  This runs after the first weight
  // loads have been issued.
  extern __shared__ uint4 xs[];
  uint4 x[NBLK][8];
  float xsum[NBLK];
  const uint4* xg = reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(p.x) + (size_t)b * H);
  // 2-bit codes: the pieces of x are requested before the first weight loads (stage_x_issue) and
  // turned through LDS after them (stage_x), all without conditions, so that these small loads
  // neither queue behind the weights nor wait one by one.  4-bit codes: a plain loop after the
  // first weight loads (measured faster there by 0.4 us, while the other form gains 1.2 us with 2 bits).
  constexpr int kXRounds = NBLK * 512 / kI4GateUpThreads;
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
    if constexpr (BITS == 2) {
#pragma unroll
      for (int u = 0; u < kXRounds; ++u) {
        const int c = threadIdx.x + u * kI4GateUpThreads;
        const int g = c >> 3, j = c & 7;
        xs[((g >> 6) * 8 + j) * 64 + (g & 63)] = c < pieces ? sx.v[u] : make_uint4(0, 0, 0, 0);
      }
    } else {
      for (int c = threadIdx.x; c < NBLK * 512; c += kI4GateUpThreads) {
        const int g = c >> 3, j = c & 7;
        xs[((g >> 6) * 8 + j) * 64 + (g & 63)] = c < pieces ? xg[c] : make_uint4(0, 0, 0, 0);
      }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
#pragma unroll
      for (int j = 0; j < 8; ++j) x[i][j] = xs[(i * 8 + j) * 64 + lane];
      xsum[i] = sum_group(x[i]);
    }
  };

  // rows are numbered r = (index among the taking-part experts) * F + f
  const int total = windowed ? (nv ? p.r1 : 0) : nv * F;
  const int stride = gridDim.x * (kI4GateUpThreads / kWave);
  const int first = (windowed ? p.r0 : 0) + blockIdx.x * (kI4GateUpThreads / kWave) + wave;
  const int nrows = first < total ? (total - first + stride - 1) / stride : 0;
  uint16_t* a_out = reinterpret_cast<uint16_t*>(p.a + (size_t)b * 2 * p.a_stride);

  int ra = first;
  auto load_next = [&](I4RowPair<BITS, NBLK>& buf) {
    const int j = ra >= F ? 1 : 0;
    const char* row = pick2(rbase, j) + (size_t)(ra - j * F) * 2 * rb;
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      i4_load_group(row, H, i, lane, buf.g1[i]);
      i4_load_group(row + rb, H, i, lane, buf.g3[i]);
    }
    ra += stride;
  };
  // The two sums of a row pair are parked in lane `ns` of gv / uv; SiLU, the product, the rounding
  // and the store are then done for up to 64 row pairs at once, one per lane, instead of by the
  // whole wavefront for every pair (the kernel is close to the vector-ALU limit).
  float gv = 0.f, uv = 0.f;
  int ns = 0, r_first = first;   // the parked sums belong to row pairs r_first + t * stride, t < ns
  auto flush = [&]() {
    if (lane < ns) {
      const int r = r_first + lane * stride;
      const int j = r >= F ? 1 : 0;
      const int f = r - j * F;
      a_out[(size_t)pick2(rj, j) * 2 * p.a_stride + i4_a_pos(f)] = f32_to_bf16_bits(pick2(rw, j) * silu_f32(gv) * uv);
    }
    r_first += ns * stride;
    ns = 0;
  };
  auto consume = [&](const I4RowPair<BITS, NBLK>& buf) {
    float g = 0.f, u = 0.f;
#pragma unroll
    for (int i = 0; i < NBLK; ++i) {
      g += i4_group_dot(buf.g1[i], x[i], xsum[i], kc, i * 64 + lane < (H >> 6));
      u += i4_group_dot(buf.g3[i], x[i], xsum[i], kc, i * 64 + lane < (H >> 6));
    }
    g = wave_sum(g);
    u = wave_sum(u);
    gv = lane == ns ? g : gv;
    uv = lane == ns ? u : uv;
    if (++ns == kWave) flush();
  };
  if constexpr (BITS == 2) {
    const StageX sxv = stage_x_issue();
    stream_bufs<I4RowPair<BITS, NBLK>>(nrows, load_next, consume, [&, sxv]() { stage_x(sxv); });
  } else {
    stream_bufs<I4RowPair<BITS, NBLK>>(nrows, load_next, consume, [&]() { stage_x(StageX{}); });
  }
  flush();
}

// --------------------------------------------------------------------- down --

template <int BITS>
struct I4DownRows {
  QGroup<BITS> g[kI4DownRows];
};

// One workgroup per kI4DownRows consecutive output rows; wavefront w owns block
// w (64 groups) of every W2 row and keeps its share of a_j in registers.
template <int BITS>
__global__ __launch_bounds__(kI4DownThreads) void ffn_down_quant_kernel(FfnArgs p) {
  __shared__ float part[kI4DownThreads / kWave][kI4DownRows];
  const int b = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = wave_index();
  const int H = p.H, F = p.F;
  const size_t rb = q_row_bytes<BITS>(F);
  const int G = F >> 6;
  const int nblk = (G + 63) >> 6;
  const I4Consts kc = q_consts<BITS>();

  const char* base[2];
  float wj[2];
  const int kk = resolve_experts(p, b, base, wj);
  const char* w2[2];
  int rj[2];
  int nv = 0;
  const size_t w2_off = (size_t)2 * F * q_row_bytes<BITS>(H);
  const bool windowed = p.j_only >= 0;
  for (int j = 0; j < kk; ++j)
    if (base[j] && (!windowed || j == p.j_only)) { w2[nv] = base[j] + w2_off; rj[nv] = j; ++nv; }

  const int h0 = (windowed ? p.r0 : 0) + blockIdx.x * kI4DownRows;
  const int hhi = windowed ? p.r1 : H;
  float acc[kI4DownRows];
#pragma unroll
  for (int r = 0; r < kI4DownRows; ++r) acc[r] = 0.f;

  if (wave < nblk) {
    const bool has_group = wave * 64 + lane < G;
    I4DownRows<BITS> buf[2];
    uint4 a[2][8];
    // all weight loads of the workgroup's rows go out first, then the lane's 64 values of
    // each a_j (written by the gate/up kernel as packed bfloat16 pairs, L2-resident)
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
      if (jj < nv) {
#pragma unroll
        for (int r = 0; r < kI4DownRows; ++r) {
          const int h = min(h0 + r, H - 1);
          i4_load_group(w2[jj] + (size_t)h * rb, F, wave, lane, buf[jj].g[r]);
        }
      }
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
      if (jj < nv) {
        const uint4* ag = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(p.a + (size_t)b * 2 * p.a_stride) +
                                                          (size_t)rj[jj] * 2 * p.a_stride);
#pragma unroll
        for (int c = 0; c < 8; ++c) a[jj][c] = has_group ? ag[(wave * 8 + c) * 64 + lane] : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
      if (jj < nv) {
        const float asum = sum_group(a[jj]);
#pragma unroll
        for (int r = 0; r < kI4DownRows; ++r) acc[r] += i4_group_dot(buf[jj].g[r], a[jj], asum, kc, has_group);
      }
  }
#pragma unroll
  for (int r = 0; r < kI4DownRows; ++r) {
    const float s = wave_sum(acc[r]);
    if (lane == 0) part[wave][r] = s;
  }
  __syncthreads();
  if (threadIdx.x < kI4DownRows && h0 + threadIdx.x < hhi) {
    float y = 0.f;
#pragma unroll
    for (int w = 0; w < kI4DownThreads / kWave; ++w) y += part[w][threadIdx.x];
    float* out = p.y + (size_t)b * H + h0 + threadIdx.x;
    *out = p.accumulate ? *out + y : y;
  }
}

// ------------------------------------------------------------------ launch ---

hipError_t launch_ffn_gateup_quant(const FfnArgs& p, int bits, const LaunchCfg& lc, hipStream_t s) {
  dim3 grid(lc.gateup_blocks, p.B), block(kI4GateUpThreads);
  if (p.j_only >= 0) grid.x = std::max(1, std::min(lc.gateup_blocks, (p.r1 - p.r0 + 3) / (kI4GateUpThreads / kWave)));
  const int nblk = ((p.H >> 6) + 63) >> 6;
  if (bits == 4) {
    if (nblk == 1) launch_kernel(ffn_gateup_quant_kernel<4, 1>, grid, block, 1 * 8192, s, lc.timing, p);
    else launch_kernel(ffn_gateup_quant_kernel<4, 2>, grid, block, 2 * 8192, s, lc.timing, p);
  } else {
    if (nblk == 1) launch_kernel(ffn_gateup_quant_kernel<2, 1>, grid, block, 1 * 8192, s, lc.timing, p);
    else launch_kernel(ffn_gateup_quant_kernel<2, 2>, grid, block, 2 * 8192, s, lc.timing, p);
  }
  return hipGetLastError();
}

hipError_t launch_ffn_down_quant(const FfnArgs& p, int bits, const LaunchCfg& lc, hipStream_t s) {
  const int rows = p.j_only >= 0 ? p.r1 - p.r0 : p.H;
  dim3 grid(std::max(1, (rows + kI4DownRows - 1) / kI4DownRows), p.B), block(kI4DownThreads);
  if (bits == 4) launch_kernel(ffn_down_quant_kernel<4>, grid, block, 0, s, lc.timing, p);
  else launch_kernel(ffn_down_quant_kernel<2>, grid, block, 0, s, lc.timing, p);
  return hipGetLastError();
}

}  // namespace adapmoe
