// The serving hot path (Eq. 4, batched across experts):
//   y[t] = x[t] W^T + step_e .* (x_ns[t] (U_e - z)^T) + x_s[t] D_e^T
// for groups of up to 64 tokens.  Per group: one small preparation launch, the main streaming launch
// and, only when the columns had to be split over workgroups, a small reduction launch.
//
// Main kernel mapping.  A workgroup owns 16*R output channels and a range of input columns; its
// wavefronts split that column range step by step (a "step" is the KSTEP columns one packed code
// word per lane covers).  Weights are the A operand of v_mfma_f32_16x16x32_bf16 (16 output channels
// x 32 columns), tokens the B operand (32 columns x 16 tokens), so the 16x16 fp32 result tile is
// [channel][token].  Everything the main kernel streams is stored tile-major: one wavefront load
// instruction reads 1 KiB (base, salient, activations) or 256 B (codes) of contiguous memory and the
// loaded registers are the MFMA operand as they are.  All loads are unconditional and issued one step
// ahead of the arithmetic that uses them.
//
// Preparation kernel.  Re-tiles the activations of the group into B-operand order, gathers the
// activations at every active expert's salient columns (per expert and 16-token tile, zero outside the
// expert's segment), and computes per token the correction that undoes the dequantisation trick below.
//
// Dequantisation.  A packed code is moved into the low mantissa bits of a bf16 whose exponent makes
// one code unit equal 1.0: (word >> s) & mask | magic gives two bf16 weights per 32-bit operation,
// equal to  bias + u  with bias = 128, 32 or 8 (b = 2, 3) or 2^(7-c) (b = 1) depending on the bit
// position.  Biases, zero point z and the codes stored at salient / padding columns (code 0) are
// removed after the reduction:  sum over non-salient i of x_i (u_i - z)
//   = sum_all x_i (bias_i + u_i) - [ sum_all x_i bias_i + z (sum_all x_i - sum_salient x_i) ],
// the bracket being the per-token correction.  The per-output-channel step multiplies the reduced sum
// in the epilogue, so the inner loop has no multiply and no rounding.
//
// Several experts may share a 16-token tile: a lane whose token is not in the expert's segment feeds
// zeros, so every expert accumulates into the same per-token accumulators.
//
// Salient fp16 columns: each fp16 value is split exactly into two bf16 values (fp16 has 11 significant
// bits, two bf16 carry 16), so two bf16 MFMAs reproduce the fp16 product exactly.
//
// Reduction: the wavefronts of a workgroup add their partial tiles through LDS in a fixed order.  With
// split columns each workgroup writes its fp32 tile to the workspace and the reduction launch adds the
// tiles in split order -- deterministic, and no device-wide fence inside the streaming kernel.
#include "mes_internal.h"

namespace mes {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr int kMaxSlots = MES_MAX_EXPERTS;   // experts with tokens in one 64-token group
constexpr int kMaxVisits = kMaxSlots + 3;    // (expert, 16-token tile) pairs in one group
constexpr int kMaxPrefetch = 16;             // slots whose code words are prefetched in registers

// Kernel arguments.  Per-expert arrays are indexed by ACTIVE SLOT: the host lists, for the token group of
// this launch, only the experts that have tokens in it (an expert with an empty segment is never touched).
struct LinearParams {
  const u32x4* w_base;
  const uint16_t* x;
  uint16_t* y;
  u32x4* xt;        // workspace: activations in B-operand order [d_in_pad/32][4 tiles][64 lanes]
  u32x4* xs;        // workspace: salient activations per visit  [visit][k_pad/32][64 lanes]
  float* corr;      // workspace: per-token correction [64]
  float* partial;   // workspace: [nsplit][64 tokens][d_out_pad] fp32 (split columns only)
  const uint32_t* codes[kMaxSlots];
  const float* step[kMaxSlots];
  const u32x4* sal[kMaxSlots];
  const int32_t* sidx[kMaxSlots];
  int16_t lo[kMaxSlots], hi[kMaxSlots];   // tokens [lo, hi) of the group belong to the slot's expert
  uint8_t vis_slot[kMaxVisits + 1], vis_tt[kMaxVisits + 1];   // visits in tile-major order
  uint32_t vis_mask[kMaxVisits + 1];      // bit n: token 16 tt + n of the visit's tile belongs to the visit's expert
  int tile_beg[5];                        // visits tile_beg[tt] .. tile_beg[tt + 1] are the ones of tile tt
  int d_in, d_out, d_out_pad, n_kb, n_chunks, n_sb, k, T, t0, n_act, n_vis, n_vis_all, nsplit, bits;
  float z;
};

__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// acc += A x B with the accumulator updated in place.  Used where the update sits under a (wave-uniform)
// branch: tying source and destination keeps the compiler from copying accumulators around the branch.
__device__ __forceinline__ void mfma16_acc(f32x4& acc, u32x4 a, u32x4 b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}

// (a & mask) | orv in one VALU operation (the mask rides the scalar operand slot).
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t orv) {
  uint32_t d;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(mask), "v"(orv));
  return d;
}

// (mask & a) | (~mask & b) in one VALU operation.
__device__ __forceinline__ uint32_t bit_insert(uint32_t mask, uint32_t a, uint32_t b) {
  uint32_t d;
  asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(d) : "s"(mask), "v"(a), "v"(b));
  return d;
}

constexpr uint32_t dup16(uint32_t h) { return h | (h << 16); }

// bf16 bit pattern of 2^e.
constexpr uint32_t bf16_pow2(int e) { return (uint32_t)(127 + e) << 7; }

template <int BITS> struct Codec;

// b = 2: pair p = 4 m + q sits at bits [2 p, 2 p + 2) of both halves.  Three pairs share one shift.
template <> struct Codec<2> {
  static constexpr int NM = 2, PLANES = 1, KSTEP = 64;
  static constexpr int cls(int m, int q) { return (4 * m + q) % 3; }
  static constexpr int bias_log2(int m, int q) { return 7 - 2 * cls(m, q); }
  static __device__ __forceinline__ void dequant(const uint32_t (&w)[1], u32x4 (&out)[2]) {
    const uint32_t sh[3] = {w[0], w[0] >> 6, w[0] >> 12};
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = 4 * m + q, sg = p / 3, c = p % 3;
        out[m][q] = and_or(sh[sg], 0x00030003u << (2 * c), dup16(bf16_pow2(bias_log2(m, q))));
      }
  }
};

// b = 1: pair p = 4 m + q sits at bit p of both halves.  Seven pairs share one shift.
template <> struct Codec<1> {
  static constexpr int NM = 4, PLANES = 1, KSTEP = 128;
  static constexpr int cls(int m, int q) { return (4 * m + q) % 7; }
  static constexpr int bias_log2(int m, int q) { return 7 - cls(m, q); }
  static __device__ __forceinline__ void dequant(const uint32_t (&w)[1], u32x4 (&out)[4]) {
    const uint32_t sh[3] = {w[0], w[0] >> 7, w[0] >> 14};
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = 4 * m + q, sg = p / 7, c = p % 7;
        out[m][q] = and_or(sh[sg], 0x00010001u << c, dup16(bf16_pow2(bias_log2(m, q))));
      }
  }
};

// b = 3: words 0 / 1 hold the low two bits like b = 2 (for m < 2 / m >= 2), word 2 the high bits,
// placed so that one shift of word 2 serves the three pairs that share a shift of word 0 / 1.
template <> struct Codec<3> {
  static constexpr int NM = 4, PLANES = 3, KSTEP = 128;
  static constexpr int cls(int m, int q) { return (4 * (m & 1) + q) % 3; }
  static constexpr int bias_log2(int m, int q) { return 7 - 2 * cls(m, q); }
  static constexpr int hi_pos(int m, int q) {
    const int p = 4 * (m & 1) + q;
    return m < 2 ? (p <= 6 ? 2 * p + 2 : 0) : 2 * p + 1;
  }
  static __device__ __forceinline__ void dequant(const uint32_t (&w)[3], u32x4 (&out)[4]) {
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = 4 * (m & 1) + q, sg = p / 3, c = p % 3;
        const uint32_t src = w[m < 2 ? 0 : 1];
        const uint32_t lo = and_or(src >> (6 * sg), 0x00030003u << (2 * c), dup16(bf16_pow2(bias_log2(m, q))));
        const int sh = hi_pos(m, q) - (2 * c + 2);
        const uint32_t hs = sh >= 0 ? (w[2] >> (sh >= 0 ? sh : 0)) : (w[2] << (sh < 0 ? -sh : 0));
        out[m][q] = bit_insert(0x00010001u << (2 * c + 2), hs, lo);
      }
  }
};

// Dequantisation bias of column `col` (what Codec<BITS>::dequant adds to the code stored there).
__device__ __forceinline__ float bias_of_column(int bits, int col) {
  const int q = (col >> 1) & 3;
  if (bits == 2) return (float)(1 << Codec<2>::bias_log2((col >> 5) & 1, q));
  if (bits == 1) return (float)(1 << Codec<1>::bias_log2((col >> 5) & 3, q));
  return (float)(1 << Codec<3>::bias_log2((col >> 5) & 3, q));
}

// fp16 pair -> (bf16 hi pair, bf16 lo pair), value = hi + lo exactly.
__device__ __forceinline__ void split_f16_pair(uint32_t w, uint32_t& hi, uint32_t& lo) {
  const float f0 = (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xffffu));
  const float f1 = (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16));
  const uint32_t h0 = __float_as_uint(f0) & 0xffff0000u;
  const uint32_t h1 = __float_as_uint(f1) & 0xffff0000u;
  const float l0 = f0 - __uint_as_float(h0);
  const float l1 = f1 - __uint_as_float(h1);
  hi = (h0 >> 16) | h1;
  lo = (__float_as_uint(l0) >> 16) | (__float_as_uint(l1) & 0xffff0000u);
}

// fp32 -> bf16 bits, round to nearest even.
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// ---- preparation ------------------------------------------------------------------------------------
// Block roles by blockIdx.x: [0, n_kb) re-tile one 32-column block of x for the four token tiles;
// [n_kb, n_kb + n_vis) gather one visit's salient activations; then 64 blocks, one per token, for the
// per-token correction.  256 threads per block.
__global__ __launch_bounds__(256) void k_prepare(const LinearParams p) {
  const int b = blockIdx.x, tid = threadIdx.x;
  if (b < p.n_kb) {
    const int tt = tid >> 6, lane = tid & 63, n = lane & 15, g = lane >> 4;
    const int t = p.t0 + 16 * tt + n, col = 32 * b + 8 * g;
    u32x4 v = {0, 0, 0, 0};
    if (t < p.T && col < p.d_in) v = *reinterpret_cast<const u32x4*>(p.x + (size_t)t * p.d_in + col);
    p.xt[((size_t)b * 4 + tt) * 64 + lane] = v;
    return;
  }
  if (b < p.n_kb + p.n_vis) {
    const int v = b - p.n_kb;
    const int a = p.vis_slot[v], tt = p.vis_tt[v];
    const int32_t* si = p.sidx[a];
    for (int i = tid; i < p.n_sb * 64; i += 256) {
      const int sb = i >> 6, lane = i & 63, n = lane & 15, g = lane >> 4;
      const int tl = 16 * tt + n;
      const bool inm = tl >= p.lo[a] && tl < p.hi[a];
      const uint16_t* xrow = p.x + (size_t)(p.t0 + tl) * p.d_in;
      u32x4 o;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int r0 = 32 * sb + 8 * g + 2 * q;
        uint32_t v0 = 0, v1 = 0;
        // indices are clamped so that a corrupt list can never address outside the row
        if (inm && r0 < p.k) v0 = xrow[min((uint32_t)si[r0], (uint32_t)(p.d_in - 1))];
        if (inm && r0 + 1 < p.k) v1 = xrow[min((uint32_t)si[r0 + 1], (uint32_t)(p.d_in - 1))];
        o[q] = v0 | (v1 << 16);
      }
      p.xs[((size_t)v * p.n_sb + sb) * 64 + lane] = o;
    }
    return;
  }
  // per-token correction  sum_i x_i bias_i + z (sum_i x_i - sum_{salient} x_i)
  const int tl = b - p.n_kb - p.n_vis;
  const int t = p.t0 + tl;
  __shared__ double red[256];
  double acc = 0.0;
  if (t < p.T) {
    const uint16_t* xrow = p.x + (size_t)t * p.d_in;
    for (int c8 = tid; c8 < p.d_in / 8; c8 += 256) {   // eight columns (four bias pairs) per 16-byte load
      const u32x4 v = *reinterpret_cast<const u32x4*>(xrow + 8 * c8);
      float part = 0.0f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float bz = bias_of_column(p.bits, 8 * c8 + 2 * q) + p.z;
        part += (bf16_to_f32((uint16_t)(v[q] & 0xffffu)) + bf16_to_f32((uint16_t)(v[q] >> 16))) * bz;
      }
      acc += (double)part;
    }
    int a = -1;
    for (int s = 0; s < p.n_act; ++s)
      if (tl >= p.lo[s] && tl < p.hi[s]) a = s;
    if (a >= 0)
      for (int r = tid; r < p.k; r += 256)
        acc -= (double)p.z * (double)bf16_to_f32(xrow[min((uint32_t)p.sidx[a][r], (uint32_t)(p.d_in - 1))]);
  }
  red[tid] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if (tid < s) red[tid] += red[tid + s];
    __syncthreads();
  }
  if (tid == 0) p.corr[tl] = (float)red[0];
}

// ---- main kernel ------------------------------------------------------------------------------------

// Loads are written as (wave-uniform pointer) + (32-bit unsigned lane offset): the pointer then lives in
// scalar registers and one vector register per lane serves every stream.
__device__ __forceinline__ u32x4 ld128(const void* uniform_ptr, uint32_t lane_off) {
  return *reinterpret_cast<const u32x4*>(reinterpret_cast<const char*>(uniform_ptr) + lane_off);
}
__device__ __forceinline__ uint32_t ld32(const void* uniform_ptr, uint32_t lane_off) {
  return *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(uniform_ptr) + lane_off);
}

// x where the lane's bit of `lane_mask` is set, else 0 (the mask rides a scalar register pair).
__device__ __forceinline__ uint32_t keep_if(uint32_t x, uint64_t lane_mask) {
  uint32_t d;
  asm("v_cndmask_b32 %0, 0, %1, %2" : "=v"(d) : "v"(x), "s"(lane_mask));
  return d;
}

template <int BITS, int TT>
struct ActBuf {
  u32x4 xb[TT][Codec<BITS>::NM];
};

template <int BITS, int TT>
__device__ __forceinline__ void load_act(const LinearParams& p, int s, int lane, ActBuf<BITS, TT>& b) {
  using C = Codec<BITS>;
  const char* src = reinterpret_cast<const char*>(p.xt) + (size_t)s * (C::NM * 4 * 1024);
#pragma unroll
  for (int m = 0; m < C::NM; ++m)
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) b.xb[tt][m] = ld128(src + (m * 4 + tt) * 1024, (uint32_t)lane * 16u);
}

template <int BITS, int R>
__device__ __forceinline__ void load_base(const LinearParams& p, int s, int lane, int jt0, u32x4 (&base)[R][Codec<BITS>::NM]) {
  using C = Codec<BITS>;
#pragma unroll
  for (int rt = 0; rt < R; ++rt) {
    const char* src = reinterpret_cast<const char*>(p.w_base) + ((size_t)(jt0 + rt) * p.n_kb + (size_t)s * C::NM) * 1024;
#pragma unroll
    for (int m = 0; m < C::NM; ++m) base[rt][m] = ld128(src + m * 1024, (uint32_t)lane * 16u);
  }
}

// Code words of step s for the first NA active slots (slots past n_act alias slot 0; the host fills them in).
template <int BITS, int R, int NA>
__device__ __forceinline__ void load_codes(const LinearParams& p, int s, int lane, int jt0, int n_steps,
                                           uint32_t (&cw)[NA][R][Codec<BITS>::PLANES]) {
  using C = Codec<BITS>;
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
      const char* src = reinterpret_cast<const char*>(p.codes[a]) + ((size_t)(jt0 + rt) * n_steps + s) * (C::PLANES * 256);
#pragma unroll
      for (int pl = 0; pl < C::PLANES; ++pl) cw[a][rt][pl] = ld32(src + pl * 256, (uint32_t)lane * 4u);
    }
}

// One (visit, 32-salient-column block) pair of the fp16 product.
template <int R>
struct SalBuf {
  u32x4 xs;
  u32x4 d[R];
};

template <int R>
__device__ __forceinline__ void load_sal(const LinearParams& p, int pair, int lane, int jt0, SalBuf<R>& b) {
  const int v = pair / p.n_sb, sb = pair - v * p.n_sb;
  const int a = p.vis_slot[v];
  b.xs = ld128(reinterpret_cast<const char*>(p.xs) + ((size_t)v * p.n_sb + sb) * 1024, (uint32_t)lane * 16u);
#pragma unroll
  for (int rt = 0; rt < R; ++rt)
    b.d[rt] = ld128(reinterpret_cast<const char*>(p.sal[a]) + ((size_t)(jt0 + rt) * p.n_sb + sb) * 1024, (uint32_t)lane * 16u);
}

template <int R, int TT>
__device__ __forceinline__ void compute_sal(const LinearParams& p, int pair, const SalBuf<R>& b, f32x4 (&acc_base)[R][TT]) {
  const int tt_dyn = p.vis_tt[pair / p.n_sb];
#pragma unroll
  for (int rt = 0; rt < R; ++rt) {
    u32x4 dh, dl;
#pragma unroll
    for (int q = 0; q < 4; ++q) { uint32_t h, l; split_f16_pair(b.d[rt][q], h, l); dh[q] = h; dl[q] = l; }
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
      if (tt == tt_dyn) {
        acc_base[rt][tt] = mfma16(dh, b.xs, acc_base[rt][tt]);
        acc_base[rt][tt] = mfma16(dl, b.xs, acc_base[rt][tt]);
      }
  }
}

// Per-wavefront LDS: the code words of the current step, [slot][row tile][plane][lane], so that the loop
// over the experts of a token tile can index experts at run time (registers cannot be indexed that way).
template <int BITS, int R, int NA>
struct CodeStore {
  uint32_t w[NA][R][Codec<BITS>::PLANES][64];
};

// Code words of `slot` for this lane: from the wavefront's LDS store, or straight from memory when the group
// has more active experts than prefetch slots (> 16 experts inside one 64-token group).
template <int BITS, int R, int NA>
__device__ __forceinline__ void fetch_codes(const LinearParams& p, uint32_t slot, int s, int lane, int jt0, int n_steps,
                                            const CodeStore<BITS, R, NA>& cs, uint32_t (&cw)[R][Codec<BITS>::PLANES]) {
  using C = Codec<BITS>;
  if (slot < (uint32_t)NA) {
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
#pragma unroll
      for (int pl = 0; pl < C::PLANES; ++pl) cw[rt][pl] = cs.w[slot][rt][pl][lane];
  } else {
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
      const char* src = reinterpret_cast<const char*>(p.codes[slot]) + ((size_t)(jt0 + rt) * n_steps + s) * (C::PLANES * 256);
#pragma unroll
      for (int pl = 0; pl < C::PLANES; ++pl) cw[rt][pl] = ld32(src + pl * 256, (uint32_t)lane * 4u);
    }
  }
}

// Arithmetic of one step.  Token tiles are walked in a fixed (unrolled) order; the experts that have tokens
// in a tile are walked by a plain loop over the host-built visit table, whose body has no branch around an
// accumulator: dequantise the expert's code words, zero the lanes of other experts' tokens, accumulate.
// The visit table lives in two vector registers (lane v = visit v: slot, token mask) and is read with
// v_readlane; the code words of the next visit are fetched from LDS while the current visit is multiplied.
template <int BITS, int R, int TT, int NA>
__device__ __forceinline__ void compute_step(const LinearParams& p, int s, int s_next, int lane, int jt0, int n_steps,
                                             u32x4 (&base)[R][Codec<BITS>::NM], const ActBuf<BITS, TT>& x,
                                             const CodeStore<BITS, R, NA>& cs, const uint32_t (&vslot)[2],
                                             const uint32_t (&vmask)[2], f32x4 (&acc_base)[R][TT], f32x4 (&acc_raw)[R][TT]) {
  using C = Codec<BITS>;
#pragma unroll
  for (int m = 0; m < C::NM; ++m)
#pragma unroll
    for (int rt = 0; rt < R; ++rt)
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) acc_base[rt][tt] = mfma16(base[rt][m], x.xb[tt][m], acc_base[rt][tt]);
  load_base<BITS, R>(p, s_next, lane, jt0, base);   // reloaded in place for the next step, a full step ahead
  auto desc = [&](const uint32_t (&tab)[2], int v) {
    return v < 64 ? __builtin_amdgcn_readlane(tab[0], v) : __builtin_amdgcn_readlane(tab[1], v - 64);
  };
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    const int v_beg = p.tile_beg[tt], v_end = p.tile_beg[tt + 1];
    if (v_beg < v_end) {
      uint32_t cw[R][C::PLANES];
      fetch_codes<BITS, R, NA>(p, desc(vslot, v_beg), s, lane, jt0, n_steps, cs, cw);
      for (int v = v_beg; v < v_end; ++v) {
        const uint32_t m16 = desc(vmask, v);
        const uint64_t lane_mask = ((uint64_t)m16 << 32) | m16;
        u32x4 dq[R][C::NM];
#pragma unroll
        for (int rt = 0; rt < R; ++rt) C::dequant(cw[rt], dq[rt]);
        const int vn = v + 1 < v_end ? v + 1 : v;
        fetch_codes<BITS, R, NA>(p, desc(vslot, vn), s, lane, jt0, n_steps, cs, cw);   // next visit's words
#pragma unroll
        for (int m = 0; m < C::NM; ++m) {
          u32x4 xm;
#pragma unroll
          for (int q = 0; q < 4; ++q) xm[q] = keep_if(x.xb[tt][m][q], lane_mask);
#pragma unroll
          for (int rt = 0; rt < R; ++rt) acc_raw[rt][tt] = mfma16(dq[rt][m], xm, acc_raw[rt][tt]);
        }
      }
    }
  }
}

template <int BITS, int R, int TT, int NA, int NW>
__global__ __launch_bounds__(64 * NW) void k_delta_linear(const LinearParams p) {
  using C = Codec<BITS>;
  constexpr int SPC = 128 / C::KSTEP;  // steps per 128-column chunk
  constexpr bool XDB = C::NM * TT <= 8;   // double-buffer the activation operands when they fit in registers
  const int lane = threadIdx.x & 63;
  // The wavefront index is the same in all 64 lanes; saying so keeps every value derived from it (step
  // numbers, addresses, which token tile a salient pair belongs to) in scalar registers and every branch on
  // them a scalar branch.  That matters for correctness too: MFMA ignores the EXEC mask, so an MFMA must
  // never sit in a region the compiler predicates with EXEC instead of branching around.
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int n = lane & 15, g = lane >> 4;
  const int rg = blockIdx.x, sp = blockIdx.y;
  const int jt0 = rg * R;
  const int n_steps = p.n_chunks * SPC;
  const int s_begin = (int)((long)sp * p.n_chunks / p.nsplit) * SPC;
  const int s_end = (int)((long)(sp + 1) * p.n_chunks / p.nsplit) * SPC;

  constexpr int kCodeBytes = (int)sizeof(CodeStore<BITS, R, NA>) * NW;
  constexpr int kRedBytes = NW * R * TT * 4 * 64 * 4;
  __shared__ __attribute__((aligned(16))) char smem[kCodeBytes > kRedBytes ? kCodeBytes : kRedBytes];
  CodeStore<BITS, R, NA>& cs = reinterpret_cast<CodeStore<BITS, R, NA>*>(smem)[wave];
  // visit table in registers: lane v (and lane v - 64 of the second register) holds visit v
  uint32_t vslot[2], vmask[2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int v = 64 * h + lane;
    vslot[h] = v <= kMaxVisits ? p.vis_slot[v] : 0;
    vmask[h] = v <= kMaxVisits ? p.vis_mask[v] : 0;
  }

  f32x4 acc_base[R][TT], acc_raw[R][TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt)
#pragma unroll
    for (int rt = 0; rt < R; ++rt) { acc_base[rt][tt] = f32x4{0, 0, 0, 0}; acc_raw[rt][tt] = f32x4{0, 0, 0, 0}; }

  // This wavefront's steps are s_begin + wave + NW j, j < cnt, visited from a start that differs from row
  // group to row group, so that workgroups running side by side stream from different places of their rows
  // instead of marching through addresses a large power of two apart in lockstep.  The step after the last
  // is prefetched again from the last (a harmless reload).  All loads are unconditional and in a fixed
  // order, so the compiler can wait for exactly the ones a computation needs while younger ones fly.
  {
    const int len = s_end - s_begin;
    const int cnt = len > wave ? (len - wave + NW - 1) / NW : 0;
    if (cnt > 0) {
      const int rot = (int)(((uint32_t)rg * 2654435761u) >> 8) % cnt;
      auto step_of = [&](int j) { j = j < cnt ? j : cnt - 1; int r = j + rot; r = r >= cnt ? r - cnt : r; return s_begin + wave + NW * r; };
      u32x4 base[R][C::NM];
      uint32_t cw[NA][R][C::PLANES];
      ActBuf<BITS, TT> xa, xb;
      load_act<BITS, TT>(p, step_of(0), lane, xa);
      load_base<BITS, R>(p, step_of(0), lane, jt0, base);
      load_codes<BITS, R, NA>(p, step_of(0), lane, jt0, n_steps, cw);
      auto one_step = [&](int j, ActBuf<BITS, TT>& xcur, ActBuf<BITS, TT>& xnext) {
        // park this step's code words in LDS, then put the next step's loads in flight
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
          for (int rt = 0; rt < R; ++rt)
#pragma unroll
            for (int pl = 0; pl < C::PLANES; ++pl) cs.w[a][rt][pl][lane] = cw[a][rt][pl];
        const int s = step_of(j), sn = step_of(j + 1);
        if (XDB) load_act<BITS, TT>(p, sn, lane, xnext);
        load_codes<BITS, R, NA>(p, sn, lane, jt0, n_steps, cw);
        compute_step<BITS, R, TT, NA>(p, s, sn, lane, jt0, n_steps, base, xcur, cs, vslot, vmask, acc_base, acc_raw);
        if (!XDB) load_act<BITS, TT>(p, sn, lane, xcur);
      };
      for (int j = 0; j < cnt; j += 2) {
        one_step(j, xa, XDB ? xb : xa);
        if (j + 1 >= cnt) break;
        one_step(j + 1, XDB ? xb : xa, xa);
      }
    }
  }

  // salient fp16 columns: (visit, 32-column block) pairs are dealt round-robin to all wavefronts of the
  // row group, each wavefront prefetching its next pair while it multiplies the current one
  if (p.k > 0) {
    const int n_pairs = p.n_vis * p.n_sb;
    const int stride = p.nsplit * NW;
    int pair = sp * NW + wave;
    if (pair < n_pairs) {
      SalBuf<R> sa, sb;
      load_sal<R>(p, pair, lane, jt0, sa);
      while (true) {
        const int nx = pair + stride;
        load_sal<R>(p, nx < n_pairs ? nx : pair, lane, jt0, sb);
        compute_sal<R, TT>(p, pair, sa, acc_base);
        if (nx >= n_pairs) break;
        pair = nx;
        const int nx2 = pair + stride;
        load_sal<R>(p, nx2 < n_pairs ? nx2 : pair, lane, jt0, sa);
        compute_sal<R, TT>(p, pair, sb, acc_base);
        if (nx2 >= n_pairs) break;
        pair = nx2;
      }
    }
  }

  // epilogue: remove biases / zero point, apply the expert's step, add across wavefronts
  __syncthreads();   // the reduction buffer reuses the code-word storage
  float (*red)[R * TT * 4][64] = reinterpret_cast<float (*)[R * TT * 4][64]>(smem);
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    const int tl = 16 * tt + n;
    int at = -1;
    for (int a = 0; a < p.n_act; ++a)
      if (tl >= p.lo[a] && tl < p.hi[a]) at = a;
    // the correction belongs to the whole column range: only the first wavefront of the first split applies it
    const float cr = (sp == 0 && wave == 0) ? p.corr[tl] : 0.0f;
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
      const int j = 16 * (jt0 + rt) + 4 * g;
      f32x4 st = {0, 0, 0, 0};
      if (at >= 0 && j < p.d_out) st = *reinterpret_cast<const f32x4*>(p.step[at] + j);
#pragma unroll
      for (int v = 0; v < 4; ++v)
        red[wave][(rt * TT + tt) * 4 + v][lane] = acc_base[rt][tt][v] + st[v] * (acc_raw[rt][tt][v] - cr);
    }
  }
  __syncthreads();

  for (int pi = wave; pi < R * TT; pi += NW) {
    const int rt = pi / TT, tt = pi % TT;
    f32x4 o;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      float s = red[0][pi * 4 + v][lane];
#pragma unroll
      for (int w = 1; w < NW; ++w) s += red[w][pi * 4 + v][lane];
      o[v] = s;
    }
    const int tl = 16 * tt + n, t = p.t0 + tl;
    const int j = 16 * (jt0 + rt) + 4 * g;
    if (p.nsplit == 1) {
      if (t < p.T && j < p.d_out) {
        uint2 pk;
        pk.x = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
        pk.y = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
        *reinterpret_cast<uint2*>(p.y + (size_t)t * p.d_out + j) = pk;
      }
    } else {
      *reinterpret_cast<f32x4*>(p.partial + ((size_t)(sp * kTokGroup + tl) * p.d_out_pad + j)) = o;
    }
  }
}

// Split columns only: y = sum over splits (in split order) of the fp32 partial tiles, rounded to bf16.
__global__ __launch_bounds__(256) void k_reduce_splits(const LinearParams p, int n_tok) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int quads = p.d_out / 4;
  if (idx >= n_tok * quads) return;
  const int tl = idx / quads, j = (idx - tl * quads) * 4;
  f32x4 o = {0, 0, 0, 0};
  for (int s = 0; s < p.nsplit; ++s)
    o += *reinterpret_cast<const f32x4*>(p.partial + ((size_t)(s * kTokGroup + tl) * p.d_out_pad + j));
  uint2 pk;
  pk.x = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
  pk.y = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
  *reinterpret_cast<uint2*>(p.y + (size_t)(p.t0 + tl) * p.d_out + j) = pk;
}

constexpr int kRowsPerGroup = 32;   // two 16-row tiles per wavefront
constexpr int kWaves = 4;           // wavefronts per workgroup; they split the workgroup's columns

struct Plan {
  int nsplit;  // workgroups that share one row group's columns
};

// Pure function of the layer shape (not of bits or T), so the workspace size is known up front.  Two
// workgroups fit a compute unit; columns are split over workgroups until there are about two per unit.
Plan plan_for(int d_in, int d_out) {
  const int po = ceil_to(d_out, kRowPad), pi = ceil_to(d_in, kColPad);
  const int n_chunks = pi / 128;
  const int row_groups = po / kRowsPerGroup;
  int ns = (512 + row_groups - 1) / row_groups;
  const int max_split = n_chunks / 8 > 0 ? n_chunks / 8 : 1;   // at least eight 128-column chunks per workgroup
  if (ns > max_split) ns = max_split;
  if (ns < 1) ns = 1;
  Plan pl;
  pl.nsplit = ns;
  return pl;
}

struct WorkspaceLayout {
  size_t xt, xs, corr, partial, total;
};

WorkspaceLayout workspace_layout(int d_in, int d_out) {
  const Plan pl = plan_for(d_in, d_out);
  const int po = ceil_to(d_out, kRowPad), pi = ceil_to(d_in, kColPad);
  WorkspaceLayout w;
  size_t off = 0;
  w.xt = off;      off += (size_t)(pi / 32) * 4 * 1024;
  w.xs = off;      off += (size_t)kMaxVisits * (ceil_to(d_in, kSalPad) / 32) * 1024;   // k <= d_in
  w.corr = off;    off += 256;
  w.partial = off; off += pl.nsplit > 1 ? (size_t)pl.nsplit * kTokGroup * po * sizeof(float) : 0;
  w.total = off;
  return w;
}

template <int BITS, int TT, int NA>
hipError_t launch_main(const LinearParams& p, dim3 grid, hipStream_t s) {
  k_delta_linear<BITS, kRowsPerGroup / 16, TT, NA, kWaves><<<grid, 64 * kWaves, 0, s>>>(p);
  return hipGetLastError();
}

template <int BITS, int NA>
hipError_t launch_tt(const LinearParams& p, int tt, dim3 grid, hipStream_t s) {
  switch (tt) {
    case 1: return launch_main<BITS, 1, NA>(p, grid, s);
    case 2: return launch_main<BITS, 2, NA>(p, grid, s);
    case 3: return launch_main<BITS, 3, NA>(p, grid, s);
    default: return launch_main<BITS, 4, NA>(p, grid, s);
  }
}

template <int BITS>
hipError_t launch_na(const LinearParams& p, int tt, dim3 grid, hipStream_t s) {
  if (p.n_act <= 4) return launch_tt<BITS, 4>(p, tt, grid, s);
  if (p.n_act <= 8) return launch_tt<BITS, 8>(p, tt, grid, s);
  return launch_tt<BITS, kMaxPrefetch>(p, tt, grid, s);
}

}  // namespace

size_t linear_workspace_bytes(int d_in, int d_out, int max_tokens) {
  (void)max_tokens;  // one 64-token group is in flight at a time
  return workspace_layout(d_in, d_out).total;
}

hipError_t launch_delta_linear(const LinearCall& c, hipStream_t s) {
  const mes_delta& d0 = c.experts[0];
  const Plan pl = plan_for(d0.d_in, d0.d_out);
  const WorkspaceLayout wl = workspace_layout(d0.d_in, d0.d_out);
  char* ws = reinterpret_cast<char*>(c.ws);
  LinearParams p;
  p.w_base = reinterpret_cast<const u32x4*>(c.w_base);
  p.x = reinterpret_cast<const uint16_t*>(c.x);
  p.y = reinterpret_cast<uint16_t*>(c.y);
  p.xt = reinterpret_cast<u32x4*>(ws + wl.xt);
  p.xs = reinterpret_cast<u32x4*>(ws + wl.xs);
  p.corr = reinterpret_cast<float*>(ws + wl.corr);
  p.partial = reinterpret_cast<float*>(ws + wl.partial);
  const int po = ceil_to(d0.d_out, kRowPad), pi = ceil_to(d0.d_in, kColPad);
  p.d_in = d0.d_in;
  p.d_out = d0.d_out;
  p.d_out_pad = po;
  p.n_kb = pi / 32;
  p.n_chunks = pi / 128;
  p.n_sb = ceil_to(d0.k, kSalPad) / 32;
  p.k = d0.k;
  p.T = c.T;
  p.nsplit = pl.nsplit;
  p.bits = d0.bits;
  p.z = d0.grid == MES_GRID_SYM ? (float)(1 << (d0.bits - 1)) - 0.5f : (float)(1 << (d0.bits - 1));
  const dim3 grid(po / kRowsPerGroup, pl.nsplit);
  for (int t0 = 0; t0 < c.T; t0 += kTokGroup) {
    p.t0 = t0;
    const int nt = c.T - t0 < kTokGroup ? c.T - t0 : kTokGroup;
    const int tt = (nt + 15) / 16;
    // active slots: the experts that own tokens of this group, in expert order
    int na = 0;
    for (int e = 0; e < c.n_experts; ++e) {
      const int lo = (c.seg[e] > t0 ? c.seg[e] : t0) - t0;
      const int hi = (c.seg[e + 1] < t0 + nt ? c.seg[e + 1] : t0 + nt) - t0;
      if (hi <= lo) continue;
      p.codes[na] = reinterpret_cast<const uint32_t*>(c.experts[e].codes);
      p.step[na] = c.experts[e].step;
      p.sal[na] = reinterpret_cast<const u32x4*>(c.experts[e].salient);
      p.sidx[na] = c.experts[e].salient_idx;
      p.lo[na] = (int16_t)lo;
      p.hi[na] = (int16_t)hi;
      ++na;
    }
    for (int a = na; a < kMaxSlots; ++a) {   // unused slots alias slot 0 so that unconditional prefetches stay valid
      p.codes[a] = p.codes[0]; p.step[a] = p.step[0]; p.sal[a] = p.sal[0]; p.sidx[a] = p.sidx[0];
      p.lo[a] = 0; p.hi[a] = 0;
    }
    // visits, tile-major: for every 16-token tile the slots that own tokens in it, with the tile's token mask
    int nv = 0;
    for (int t = 0; t < 4; ++t) {
      p.tile_beg[t] = nv;
      for (int a = 0; a < na; ++a) {
        const int l = p.lo[a] > 16 * t ? p.lo[a] : 16 * t;
        const int h = p.hi[a] < 16 * t + 16 ? p.hi[a] : 16 * t + 16;
        if (h <= l) continue;
        uint32_t m16 = 0;
        for (int n = l - 16 * t; n < h - 16 * t; ++n) m16 |= 1u << n;
        p.vis_slot[nv] = (uint8_t)a;
        p.vis_tt[nv] = (uint8_t)t;
        p.vis_mask[nv] = m16 | (m16 << 16);
        ++nv;
      }
    }
    p.tile_beg[4] = nv;
    for (int v = nv; v <= kMaxVisits; ++v) { p.vis_slot[v] = 0; p.vis_tt[v] = 0; p.vis_mask[v] = 0; }
    p.n_vis_all = nv;
    p.n_act = na;
    p.n_vis = d0.k > 0 ? nv : 0;
    k_prepare<<<p.n_kb + p.n_vis + kTokGroup, 256, 0, s>>>(p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    switch (d0.bits) {
      case 1: e = launch_na<1>(p, tt, grid, s); break;
      case 2: e = launch_na<2>(p, tt, grid, s); break;
      default: e = launch_na<3>(p, tt, grid, s); break;
    }
    if (e != hipSuccess) return e;
    if (pl.nsplit > 1) {
      const int total = nt * (d0.d_out / 4);
      k_reduce_splits<<<(total + 255) / 256, 256, 0, s>>>(p, nt);
      if ((e = hipGetLastError()) != hipSuccess) return e;
    }
  }
  return hipSuccess;
}

}  // namespace mes
