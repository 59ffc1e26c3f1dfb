// Long token segments (prefill): one product per expert, y_e = x_e (W + Delta~_e)^T  -- Eq. 4 before it is
// decoupled.  With hundreds of tokens on one expert the layer is a dense contraction bound by the matrix cores,
// not by weight bytes, and streaming the weights once per 64 tokens (the decode kernel) wastes both.  Here the
// expert's effective weight is formed in registers, never in memory: per 16 x 32 block, bf16(W + (u - z) s) from
// the tiled base weight and the packed codes, as the A operand of the bf16 matrix instruction.  Salient input
// channels store code 0, so the main product carries (0 - z) s for them; a short second part of the contraction,
// over the gathered salient activations, adds bf16(Delta_S + z s) (Delta_S: the stored fp16 values).
// The rounding of the operands to bf16 adds a relative error of about 2^-9 / sqrt(3) to y, the same size as the
// rounding of y itself.
#include "mes_internal.h"

namespace mes {
namespace {

typedef __attribute__((__vector_size__(16))) uint32_t u32x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;

constexpr int kMaxWorkgroups = 256;  // one workgroup per compute unit; fewer row groups than that split the contraction

constexpr int kMaxSegs = 8;          // long segments (experts) served by one launch

struct PrefillParams {
  const u32x4* base;        // tiled base weight: block (chunk c, row tile jt) = [4 k blocks][64 lanes] x 16 bytes
  // per segment (= per expert with a long segment), n_seg of them:
  const uint32_t* codes[kMaxSegs];   // packed codes: block (c, jt) = 64 * bits words
  const float* step[kMaxSegs];       // [d_out]
  const u32x4* sal[kMaxSegs];        // salient tile: ((jt * n_sb + sb) * 64 + lane) x 8 fp16
  int t_begin[kMaxSegs], t_end[kMaxSegs];   // the segment's rows of x and y
  int tb0[kMaxSegs + 1];             // its first token block (of 256 tokens) in the launch; tb0[n_seg] = all blocks
  int n_seg;
  const u32x4* xt;          // the segments' activations in fragment order: [k block][token tile][64 lanes] x 16 bytes,
                            // k blocks 0 .. 4 n_chunks - 1 the input channels, then 4 n_ssteps blocks of gathered salient ones
  uint16_t* y;              // bf16 [T, d_out]
  f32x4* tiles;             // split contraction only: accumulator tiles, [split][row group][token block][16 tiles][thread]
  int d_out, n_jt, n_chunks, n_sb, n_ssteps, n_tq, steps_per_split, n_split;
  float z;
};

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  const bf16x2 h = __builtin_convertvector(f32x2{a, b}, bf16x2);   // round to nearest even
  return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ f32x4 mfma_bf16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// The barrier between two steps: waits for this wavefront's LDS traffic only.  (__syncthreads() would also wait for
// the memory loads in flight: the weights a builder has just requested for a later step, the activation copies a
// multiplier keeps ahead of itself -- a full memory round trip per step.)
__device__ __forceinline__ void step_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

struct TileParams {
  const uint16_t* x;
  const int32_t* sidx[kMaxSegs];
  int t_begin[kMaxSegs], t_end[kMaxSegs], tb0[kMaxSegs + 1];
  int n_seg, k, d_in, n_kb_main, n_tq;
  int kb_begin;             // this launch writes the k blocks kb_begin .. kb_begin + n_blk / n_tq - 1
  size_t n_blk;
  u32x4* xt;
};

// The segments' rows of x -> fragment order.  Block (kbi, tq), lane l: token 16 tq' + (l & 15) of the segment that
// token tile tq belongs to (tq' counted from the segment's first tile); for kbi < n_kb_main the 8 input channels
// 32 kbi + 8 (l >> 4) .., else the 8 salient channels of that segment's expert with ranks
// 32 (kbi - n_kb_main) + 8 (l >> 4) ..; zero beyond the segment's last token, the last channel or rank.
__global__ void k_prefill_tile_x(const TileParams p) {
  const int lane = threadIdx.x & 63;
  const size_t blk = (size_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (blk >= p.n_blk) return;
  const int tq = (int)(blk % p.n_tq), kbi = p.kb_begin + (int)(blk / p.n_tq);
  int sg = 0;
  while (sg + 1 < p.n_seg && tq >= 16 * p.tb0[sg + 1]) ++sg;
  const int t = p.t_begin[sg] + 16 * (tq - 16 * p.tb0[sg]) + (lane & 15);
  u32x4 v = {0, 0, 0, 0};
  if (t < p.t_end[sg]) {
    const uint16_t* row = p.x + (size_t)t * p.d_in;
    if (kbi < p.n_kb_main) {
      const int c = 32 * kbi + 8 * (lane >> 4);
      if (c < p.d_in) v = *reinterpret_cast<const u32x4*>(row + c);
    } else {
      const int r0 = 32 * (kbi - p.n_kb_main) + 8 * (lane >> 4);
      const int32_t* sidx = p.sidx[sg];
      uint32_t h[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        h[q] = 0;
        if (r0 + q < p.k) {
          const int c = sidx[r0 + q];
          if (c >= 0 && c < p.d_in) h[q] = row[c];   // a corrupt list can never address outside the row
        }
      }
      v = u32x4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
    }
  }
  p.xt[((size_t)kbi * p.n_tq + tq) * 64 + lane] = v;
}

// What a builder keeps in flight for one step (128 input channels, or 128 salient ranks) of its row tile.
template <int BITS>
struct StepData {
  u32x4 w[4];                              // base fragments (main step) or 8 fp16 salient values (salient step), per k block
  uint32_t lo[4], hi[BITS >= 3 ? 4 : 1];   // code words
};

// Grid: (row groups of 16 RT output channels, token blocks of 64 NM tokens, n_split); NM + RT wavefronts in two
// roles, spread evenly over the SIMDs (RT = 8, or 7 where that fills the last round of workgroups: prefill_plan).
// The token blocks of up to 8 long segments (each with its own expert's codes, steps and salient values) share one
// launch, so that the compute units go from one expert's work to the next without a launch in between:
//   builders (the last RT wavefronts): builder r forms the operand of row tile r (16 output channels) for the next
//     step of 128 input channels in the idle LDS buffer, from base weight and codes requested two steps ahead;
//   multipliers (wavefronts 0 .. NM - 1): every one multiplies all RT row tiles of the current step (from LDS) with
//     its own 64 tokens.  With RT = 8 the activations reach it through an LDS ring of its own, filled by
//     asynchronous copies two k blocks ahead; with RT = 7 the 16 registers that leaves free hold a second set of
//     activation fragments, loaded straight from memory one k block ahead (5 % faster: less LDS traffic).
// Every workgroup reads all the activations of its tokens from L2 once per step, so the rows per workgroup set the
// L2 traffic: 128 rows x 256 tokens halve it against 64 rows x 512 tokens, at the price of building every operand
// once per 256 tokens.  Measured with parts of the kernel taken out (3 experts x 512 tokens, 14336 rows; the whole
// kernel 213 us): barriers and LDS traffic alone 88 us, + activation copies 120 us, + the builders' loads and
// arithmetic 165 us, the matrix instructions the rest -- the parts add up rather than overlap, and what they share
// is the LDS pipe (operands for 4 multipliers, the builders' stores, the ring's copies and reads).
// One barrier per step.  The steps are the n_chunks chunks of input channels followed by n_ssteps steps over the
// salient ranks; with n_split > 1 a workgroup covers a share of them and leaves its accumulators to
// k_prefill_reduce.
template <int BITS, int RT, int NM>
__global__ __launch_bounds__(64 * (NM + RT), 1) void k_prefill_fused(const PrefillParams p) {
  constexpr int TT = 4;                                  // token tiles per multiplier
  constexpr int XD = 3;                                  // ring depth in k blocks
  __shared__ __attribute__((aligned(16))) u32x4 afrag[2][RT][4][64];     // [buffer][row tile][k block][lane]
  constexpr bool kXDirect = RT <= 7;                     // activations straight into registers (RT = 8 has none to spare)
  __shared__ __attribute__((aligned(16))) u32x4 xring[kXDirect ? 1 : NM][XD][TT][64];   // [multiplier][slot][token tile][lane]
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = lane & 15, g = lane >> 4;
  const int n_steps = p.n_chunks + p.n_ssteps;
  const int st0 = blockIdx.z * p.steps_per_split;
  const int st1 = st0 + p.steps_per_split < n_steps ? st0 + p.steps_per_split : n_steps;
  int sg = 0;                                            // the segment (expert) this token block belongs to
  while (sg + 1 < p.n_seg && (int)blockIdx.y >= p.tb0[sg + 1]) ++sg;

  if (wave >= NM) {
    // ---- builder
    const int rt = wave - NM;
    int jt = RT * blockIdx.x + rt;                       // stored matrices are padded to whole groups of 4 row tiles:
    jt = jt < p.n_jt ? jt : p.n_jt - 1;                  // a last group of 8 may repeat tiles (its rows are never stored)
    const int row = 16 * jt + n < p.d_out ? 16 * jt + n : p.d_out - 1;
    const float s = p.step[sg][row];
    const float zs = p.z * s;
    StepData<BITS> sd[2];
    // Straight-line on purpose (addresses are selected, not branched on): the compiler then knows exactly which
    // loads are in flight and never waits for the ones just requested.
    auto fetch = [&](int slot, int st) {
      st = st < st1 ? st : st1 - 1;
      StepData<BITS>& d = sd[slot];
      const bool main_step = st < p.n_chunks;
      const size_t blk = (size_t)(main_step ? st : p.n_chunks - 1) * p.n_jt + jt;   // a salient step re-reads code words it never uses
      const uint32_t* cw = p.codes[sg] + blk * (64 * BITS);
      const int ss = main_step ? 0 : st - p.n_chunks;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        int sb = 4 * ss + kb;
        sb = sb < p.n_sb ? sb : p.n_sb - 1;              // past the last salient block: repeated, zeroed in build()
        const u32x4* src = main_step ? p.base + (blk * 4 + kb) * 64 : p.sal[sg] + ((size_t)jt * p.n_sb + sb) * 64;
        d.w[kb] = src[lane];
        const int cl = 16 * kb + n;                      // the code block's lane cl owns columns 32 kb + 8 g + 0..7
        if constexpr (BITS == 1) {
          d.lo[kb] = cw[cl];
        } else {
          d.lo[kb] = cw[2 * cl + (g >> 1)];
          if constexpr (BITS == 3) d.hi[kb] = cw[128 + cl];
          if constexpr (BITS == 4) d.hi[kb] = cw[128 + 2 * cl + (g >> 1)];
        }
      }
    };
    auto build = [&](int slot, int st) {                // sd[slot] (of step st) -> LDS buffer st & 1
      const int buf = st & 1;                           // a step past the end repeats the last one, into the idle buffer
      st = st < st1 ? st : st1 - 1;
      const StepData<BITS>& d = sd[slot];
      if (st < p.n_chunks) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
          uint32_t lo = d.lo[kb], hi = 0;
          constexpr uint32_t lo_mask = BITS == 1 ? 1u : 3u, hi_mask = BITS == 3 ? 1u : (BITS == 4 ? 3u : 0u);
          if constexpr (BITS == 1) lo >>= g; else lo >>= 2 * (g & 1);
          if constexpr (BITS == 3) hi = d.hi[kb] >> g;
          if constexpr (BITS == 4) hi = d.hi[kb] >> (2 * (g & 1));
          float v[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const uint32_t u = ((lo >> (4 * q)) & lo_mask) | (((hi >> (4 * q)) & hi_mask) << 2);
            const uint32_t ww = d.w[kb][q >> 1];
            const float w = (q & 1) ? bf16_hi(ww) : bf16_lo(ww);
            v[q] = w + __builtin_fmaf((float)u, s, -zs);   // W + (u - z) s
          }
          afrag[buf][rt][kb][lane] = u32x4{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
        }
      } else {
        const int ss = st - p.n_chunks;
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) {
          u32x4 out = {0, 0, 0, 0};
          if (4 * ss + kb < p.n_sb) {                    // ranks past k hold 0 and meet activations that are 0
            const f16x8 h = __builtin_bit_cast(f16x8, d.w[kb]);
            float v[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) v[q] = (float)h[q] + zs;
            out = u32x4{pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
          }
          afrag[buf][rt][kb][lane] = out;
        }
      }
    };
    fetch(0, st0);
    fetch(1, st0 + 1);
    build(0, st0);
    fetch(0, st0 + 2);
    __syncthreads();
    // iteration st builds step st + 1 (slot alternates 1, 0, 1, ...) and requests step st + 3 into the same slot
    for (int st = st0; st < st1; st += 2) {
      build(1, st + 1);
      fetch(1, st + 3);
      step_barrier();
      if (st + 1 >= st1) break;
      build(0, st + 2);
      fetch(0, st + 4);
      step_barrier();
    }
    return;
  }

  // ---- multiplier: token tiles TT (NM by + wave) .. + TT - 1 of the segment
  const int tq0 = TT * (NM * blockIdx.y + wave);
  f32x4 acc[RT][TT];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = f32x4{0, 0, 0, 0};
  if constexpr (kXDirect) {
    // two register sets filled by ordinary loads one k block ahead: no LDS traffic for the activations
    const u32x4* xsrc = p.xt + (size_t)tq0 * 64 + lane;
    const size_t x_stride = (size_t)p.n_tq * 64;        // 16-byte units between k blocks
    const int kbg_last = 4 * st1 - 1;
    u32x4 xb[2][TT];
    auto request_x = [&](int kbg, int set) {
      const u32x4* src = xsrc + (size_t)(kbg < kbg_last ? kbg : kbg_last) * x_stride;
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) xb[set][tt] = src[tt * 64];
    };
    request_x(4 * st0, 0);
    __syncthreads();
    for (int st = st0; st < st1; ++st) {
      const int cur = st & 1;
      u32x4 a[2];                                        // operands are read from LDS one row tile ahead of their use
      a[0] = afrag[cur][0][0][lane];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        request_x(4 * st + kb + 1, (kb + 1) & 1);
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          constexpr int kNone = -1;
          const int rn = rt < RT - 1 ? rt + 1 : 0, kn = rt < RT - 1 ? kb : (kb < 3 ? kb + 1 : kNone);
          if (kn != kNone) a[(kb * RT + rt + 1) & 1] = afrag[cur][rn][kn][lane];
          __builtin_amdgcn_sched_barrier(0);             // keep the read above ahead of the matrix instructions below
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = mfma_bf16(a[(kb * RT + rt) & 1], xb[kb & 1][tt], acc[rt][tt]);
        }
      }
      step_barrier();
    }
  } else {
    const char* xbase = reinterpret_cast<const char*>(p.xt + (size_t)tq0 * 64);
    const size_t x_stride = (size_t)p.n_tq * 1024;        // bytes between k blocks
    const int kbg_last = 4 * st1 - 1;
    auto request_x = [&](int kbg, int slot) {             // TT copies of 1 KiB: lane l moves 16 bytes
      const char* src = xbase + (size_t)(kbg < kbg_last ? kbg : kbg_last) * x_stride;
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        const uint32_t l = (uint32_t)(uintptr_t)&xring[wave][slot][tt][0];
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     : : "v"((uint32_t)lane * 16u), "s"(src + tt * 1024), "s"(l) : "memory", "m0");
      }
    };
    // the copies are this wavefront's only memory loads, TT per k block, completed in order: "at most TT (XD - 1)
    // outstanding" means the oldest requested block has arrived
    constexpr int kXAhead = XD - 1;
#pragma unroll
    for (int b = 0; b < kXAhead; ++b) request_x(4 * st0 + b, b);
    int slot = 0;                                          // ring slot of the block multiplied next
    __syncthreads();
    for (int st = st0; st < st1; ++st) {
      const int cur = st & 1;
      u32x4 a[2];                                          // operands are read from LDS one row tile ahead of their use
      a[0] = afrag[cur][0][0][lane];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        const int ahead = slot + kXAhead < XD ? slot + kXAhead : slot + kXAhead - XD;   // the slot multiplied last
        request_x(4 * st + kb + kXAhead, ahead);
        asm volatile("s_waitcnt vmcnt(%0)" : : "n"(TT * kXAhead) : "memory");
        u32x4 xb[TT];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) xb[tt] = xring[wave][slot][tt][lane];
        slot = slot + 1 < XD ? slot + 1 : 0;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          constexpr int kNone = -1;
          const int rn = rt < RT - 1 ? rt + 1 : 0, kn = rt < RT - 1 ? kb : (kb < 3 ? kb + 1 : kNone);
          if (kn != kNone) a[(kb * RT + rt + 1) & 1] = afrag[cur][rn][kn][lane];
          __builtin_amdgcn_sched_barrier(0);               // keep the read above ahead of the matrix instructions below
#pragma unroll
          for (int tt = 0; tt < TT; ++tt) acc[rt][tt] = mfma_bf16(a[(kb * RT + rt) & 1], xb[tt], acc[rt][tt]);
        }
      }
      step_barrier();
    }
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");     // the surplus copies must land before the LDS is given back
  }

  if (p.n_split > 1) {   // this workgroup saw a share of the contraction only: leave the tiles, in thread order
    constexpr int NT = 64 * NM;
    f32x4* t = p.tiles + ((((size_t)blockIdx.z * gridDim.x + blockIdx.x) * gridDim.y + blockIdx.y) * (RT * TT)) * NT + threadIdx.x;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) t[(size_t)(rt * TT + tt) * NT] = acc[rt][tt];
    return;
  }
  // this lane holds, per row tile and token tile, rows 4 g .. 4 g + 3 at token n
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int j = 16 * (RT * blockIdx.x + rt) + 4 * g;
    if (j >= p.d_out) continue;                          // d_out % 4 == 0
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      const int t = p.t_begin[sg] + 16 * (tq0 - 16 * p.tb0[sg] + tt) + n;
      if (t < p.t_end[sg]) {
        const f32x4 o = acc[rt][tt];
        uint2 pk;
        pk.x = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
        pk.y = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
        *reinterpret_cast<uint2*>(p.y + (size_t)t * p.d_out + j) = pk;
      }
    }
  }
}

// Split contraction only: y = sum over splits (in split order) of the accumulator tiles, rounded to bf16.
// Grid (row groups, token blocks, 4 RT tiles), NM wavefronts laid out like the multipliers of the main kernel; one
// tile (row tile rt = z / 4, token tile tt = z % 4) per workgroup.
template <int RT, int NM>
__global__ __launch_bounds__(64 * NM) void k_prefill_reduce(const PrefillParams p) {
  constexpr int NT = 64 * NM, TT = 4;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, g = lane >> 4;
  const int rt = blockIdx.z >> 2, tt = blockIdx.z & 3;
  f32x4 o = {0, 0, 0, 0};
  for (int sp = 0; sp < p.n_split; ++sp)
    o += p.tiles[((((size_t)sp * gridDim.x + blockIdx.x) * gridDim.y + blockIdx.y) * (RT * TT) + blockIdx.z) * NT + threadIdx.x];
  const int j = 16 * (RT * blockIdx.x + rt) + 4 * g;
  int sg = 0;
  while (sg + 1 < p.n_seg && (int)blockIdx.y >= p.tb0[sg + 1]) ++sg;
  const int t = p.t_begin[sg] + 16 * (TT * (NM * ((int)blockIdx.y - p.tb0[sg]) + wave) + tt) + n;
  if (j < p.d_out && t < p.t_end[sg]) {
    uint2 pk;
    pk.x = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
    pk.y = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
    *reinterpret_cast<uint2*>(p.y + (size_t)t * p.d_out + j) = pk;
  }
}

struct PrefillPlan {
  int rt, nm, n_rg, n_tb, n_tq, n_split, steps_per_split, n_chunks, n_ssteps;
  size_t xt_bytes, tiles_at, tiles_bytes;
};

// n_tb: token blocks of all the segments of the launch together
PrefillPlan prefill_plan(int d_in, int d_out, int k, int n_tb) {
  PrefillPlan pl;
  pl.rt = 8;   // 128 rows x 256 tokens per workgroup: measured 6 % faster than 64 x 512 and 14 % faster than 64 x 256
  pl.nm = 4;
  pl.n_tb = n_tb;
  pl.n_tq = pl.n_tb * 4 * pl.nm;
  const int n_jt = ceil_to(d_out, kRowPad) / 16;
  pl.n_rg = (n_jt + pl.rt - 1) / pl.rt;
  // One workgroup per compute unit at a time: the launch takes ceil(workgroups / 256) rounds of one workgroup's
  // time, which grows with its row tiles.  7 row tiles per workgroup win where they fill the last round better
  // (14336 rows x 6 token blocks: 768 workgroups = 3 full rounds of 7 tiles against 2.6 -> 3 rounds of 8; 4096 rows x
  // 6 blocks: one round of 222 workgroups against one of 192); + 1 below: the part of a workgroup's time that does
  // not shrink with its rows.  (Equal tile-rounds -- 14336 rows x 16 token blocks: 8 rounds of 7 or 7 rounds of 8 --
  // measured no better with 7.)  128 workgroups or fewer split the contraction instead and keep 8 tiles.
  {
    const long wg8 = (long)pl.n_rg * n_tb, rg7 = (n_jt + 6) / 7, wg7 = rg7 * n_tb;
    const long rounds8 = (wg8 + kMaxWorkgroups - 1) / kMaxWorkgroups, rounds7 = (wg7 + kMaxWorkgroups - 1) / kMaxWorkgroups;
    if (2 * wg8 > kMaxWorkgroups && rounds7 * (7 + 1) < rounds8 * (8 + 1)) {
      pl.rt = 7;
      pl.n_rg = (int)rg7;
    }
  }
  pl.n_chunks = ceil_to(d_in, kColPad) / 128;
  pl.n_ssteps = (ceil_to(k, kSalPad) / 32 + 3) / 4;
  const int n_steps = pl.n_chunks + pl.n_ssteps;
  const long base = (long)pl.n_rg * pl.n_tb;
  int want = (int)(kMaxWorkgroups / base);
  want = want < 1 ? 1 : (want > 8 ? 8 : want);
  pl.steps_per_split = (n_steps + want - 1) / want;
  if (pl.steps_per_split < 4) pl.steps_per_split = n_steps < 4 ? n_steps : 4;
  pl.n_split = (n_steps + pl.steps_per_split - 1) / pl.steps_per_split;
  pl.xt_bytes = (size_t)(4 * n_steps) * pl.n_tq * 1024;
  pl.tiles_at = (pl.xt_bytes + 255) / 256 * 256;
  pl.tiles_bytes = pl.n_split > 1 ? (size_t)pl.n_split * base * (4 * pl.rt) * (64 * pl.nm) * 16 : 0;
  return pl;
}

template <int BITS>
hipError_t launch_fused(const PrefillParams& p, const PrefillPlan& pl, dim3 grid, hipStream_t s) {
  if (pl.rt == 7) k_prefill_fused<BITS, 7, 4><<<grid, 64 * (4 + 7), 0, s>>>(p);
  else k_prefill_fused<BITS, 8, 4><<<grid, 768, 0, s>>>(p);
  return hipGetLastError();
}

}  // namespace

// Scratch for the long segments of a call of up to max_tokens tokens: their activations in fragment order (input
// channels, then up to d_in gathered salient ones; every segment padded to whole blocks of 256 tokens, at most
// max_tokens / 192 segments) and, for a split contraction, the accumulator tiles: a split happens only while
// splits x row groups x token blocks stays within 256 workgroups, each leaving 128 rows x 256 tokens x 4 bytes.
size_t prefill_scratch_bytes(int d_in, int max_tokens) {
  const size_t tok_pad = (size_t)max_tokens + (size_t)256 * (max_tokens / 192 + 1);
  const size_t xt = tok_pad * (size_t)(ceil_to(d_in, kColPad) + ceil_to(ceil_to(d_in, kSalPad), 128)) * 2;
  const size_t tiles = (size_t)2 * kMaxWorkgroups * 128 * 256 * 4;
  return (xt + 255) / 256 * 256 + tiles;
}

// y rows of the n_seg long segments seg_experts[i] (expert numbers; rows seg[e] .. seg[e + 1]) of the n_linears layers
// of a call (they read the same x and routing), each layer with its own experts' deltas, up to kMaxSegs segments per
// launch.  The segments' activations are re-tiled once for all layers; the gathered salient activations, which
// depend on the layer's salient sets, once per layer into the same place (the launches are stream-ordered).
// scratch: prefill_scratch_bytes(d_in, >= all their tokens).
// ev_start / ev_stop (measurement hook, may be null): recorded immediately before the first fused kernel (only while
// *first_kernel is set, which this clears) and immediately after every fused kernel and its reduction.
hipError_t launch_prefill_segments(const mes_linear* lin, int n_linears, const int* seg_experts, int n_seg,
                                   const int32_t* seg, const void* x, void* scratch, hipEvent_t ev_start,
                                   hipEvent_t ev_stop, bool* first_kernel, hipStream_t s) {
  char* ws = reinterpret_cast<char*>(scratch);
  for (int first = 0; first < n_seg; first += kMaxSegs) {
    const int ns = n_seg - first < kMaxSegs ? n_seg - first : kMaxSegs;
    for (int l = 0; l < n_linears; ++l) {
      const mes_delta* experts = lin[l].experts;
      const mes_delta& d = experts[seg_experts[first]];   // shape, bits, grid and k are the same for all experts of a linear
      PrefillParams p;
      TileParams tp;
      int n_tb = 0;
      for (int i = 0; i < kMaxSegs; ++i) {
        const mes_delta& de = experts[seg_experts[first + (i < ns ? i : 0)]];
        const int e = seg_experts[first + (i < ns ? i : 0)];
        p.codes[i] = reinterpret_cast<const uint32_t*>(de.codes);
        p.step[i] = de.step;
        p.sal[i] = reinterpret_cast<const u32x4*>(de.salient);
        tp.sidx[i] = de.salient_idx;
        p.t_begin[i] = tp.t_begin[i] = seg[e];
        p.t_end[i] = tp.t_end[i] = seg[e + 1];
        p.tb0[i] = tp.tb0[i] = n_tb;
        if (i < ns) n_tb += (seg[e + 1] - seg[e] + 255) / 256;
      }
      p.tb0[kMaxSegs] = tp.tb0[kMaxSegs] = n_tb;
      for (int i = ns; i <= kMaxSegs; ++i) p.tb0[i] = tp.tb0[i] = n_tb;
      p.n_seg = tp.n_seg = ns;
      const PrefillPlan pl = prefill_plan(d.d_in, d.d_out, d.k, n_tb);
      p.base = reinterpret_cast<const u32x4*>(lin[l].w_base_tiled);
      p.xt = reinterpret_cast<const u32x4*>(ws);
      p.y = reinterpret_cast<uint16_t*>(lin[l].y);
      p.tiles = reinterpret_cast<f32x4*>(ws + pl.tiles_at);
      p.d_out = d.d_out;
      p.n_jt = ceil_to(d.d_out, kRowPad) / 16;
      p.n_chunks = pl.n_chunks;
      p.n_sb = ceil_to(d.k, kSalPad) / 32;
      p.n_ssteps = pl.n_ssteps;
      p.n_tq = pl.n_tq;
      p.steps_per_split = pl.steps_per_split;
      p.n_split = pl.n_split;
      p.z = d.grid == MES_GRID_SYM ? (float)(1 << (d.bits - 1)) - 0.5f : (float)(1 << (d.bits - 1));
      tp.x = reinterpret_cast<const uint16_t*>(x);
      tp.k = d.k;
      tp.d_in = d.d_in;
      tp.n_kb_main = 4 * pl.n_chunks;
      tp.n_tq = pl.n_tq;
      tp.xt = reinterpret_cast<u32x4*>(ws);
      hipError_t e = hipSuccess;
      if (l == 0) {   // the input channels: the same for every layer of the call
        tp.kb_begin = 0;
        tp.n_blk = (size_t)tp.n_kb_main * pl.n_tq;
        k_prefill_tile_x<<<(unsigned)((tp.n_blk + 3) / 4), 256, 0, s>>>(tp);
        if ((e = hipGetLastError()) != hipSuccess) return e;
      }
      if (pl.n_ssteps > 0) {   // this layer's gathered salient channels, behind them
        tp.kb_begin = tp.n_kb_main;
        tp.n_blk = (size_t)4 * pl.n_ssteps * pl.n_tq;
        k_prefill_tile_x<<<(unsigned)((tp.n_blk + 3) / 4), 256, 0, s>>>(tp);
        if ((e = hipGetLastError()) != hipSuccess) return e;
      }
      const dim3 grid(pl.n_rg, pl.n_tb, pl.n_split);
      if (ev_start && *first_kernel && (e = hipEventRecord(ev_start, s)) != hipSuccess) return e;
      *first_kernel = false;
      switch (d.bits) {
        case 1: e = launch_fused<1>(p, pl, grid, s); break;
        case 2: e = launch_fused<2>(p, pl, grid, s); break;
        case 3: e = launch_fused<3>(p, pl, grid, s); break;
        default: e = launch_fused<4>(p, pl, grid, s); break;
      }
      if (e != hipSuccess) return e;
      if (pl.n_split > 1) {
        k_prefill_reduce<8, 4><<<dim3(grid.x, grid.y, 32), 256, 0, s>>>(p);
        if ((e = hipGetLastError()) != hipSuccess) return e;
      }
      if (ev_stop && (e = hipEventRecord(ev_stop, s)) != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

}  // namespace mes
