// The serving hot path (Eq. 4, batched across experts):
//   y[t] = x[t] W^T + step_e .* (x_ns[t] (U_e - z)^T) + x_s[t] D_e^T
// as one fused gfx950 kernel per group of up to 64 tokens.
//
// Mapping.  A workgroup owns 16*R output channels and a range of input columns; its four
// wavefronts split that column range step by step (a "step" is the KSTEP columns one packed
// code word per lane covers).  Weights are the A operand of v_mfma_f32_16x16x32_bf16 (16 output
// channels x 32 columns), tokens the B operand (32 columns x 16 tokens), so the 16x16 fp32
// result tile is [channel][token].  All streamed matrices are stored tile-major: one wavefront
// load instruction reads 1 KiB (base, salient) or 256 B (codes) of contiguous memory and the
// loaded registers are the MFMA operand as they are.
//
// Dequantisation.  A packed code is moved into the low mantissa bits of a bf16 whose exponent
// makes one code unit equal 1.0: (word >> s) & mask | magic gives two bf16 weights per 32-bit
// operation, equal to  bias + u  with bias = 128, 32 or 8 (b = 2, 3) or 2^(7-c) (b = 1) depending
// on the bit position.  The biases, the zero point z and the codes stored at salient / padding
// columns are removed after the reduction with per-token sums that one extra MFMA per column
// block produces:  sum_i x_i (u_i - z) over non-salient i
//   = sum_all x_i (bias_i + u_i) - sum_all x_i bias_i - z (sum_all x_i - sum_salient x_i),
// salient and padding columns holding code 0.  The per-output-channel step multiplies the
// reduced sum in the epilogue, so the inner loop has no multiply and no rounding.
//
// Several experts may share a 16-token tile: a lane whose token is not in the expert's segment
// feeds zeros, so every expert accumulates into the same per-token accumulators.
//
// Salient fp16 columns: each fp16 value is split exactly into two bf16 values (fp16 has 11
// significant bits, two bf16 carry 16), so two bf16 MFMAs reproduce the fp16 product exactly.
//
// Reduction: the four wavefronts add their partial tiles through LDS in a fixed order; when the
// columns are split over several workgroups each writes its fp32 tile to the workspace and the
// last one to arrive (a counter per row group) adds them in split order -- deterministic.
#include "mes_internal.h"

namespace mes {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

struct LinearParams {
  const u32x4* w_base;
  const uint16_t* x;
  uint16_t* y;
  float* partial;
  int* counters;
  const uint32_t* codes[MES_MAX_EXPERTS];
  const float* step[MES_MAX_EXPERTS];
  const u32x4* sal[MES_MAX_EXPERTS];
  const int32_t* sidx[MES_MAX_EXPERTS];
  int32_t off[MES_MAX_EXPERTS + 1];
  int d_in, d_out, d_out_pad, n_kb, n_chunks, n_sb, k, T, t0, n_experts, nsplit;
  float z;
};

__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

constexpr uint32_t dup16(uint32_t h) { return h | (h << 16); }

// bf16 bit pattern of 2^e.
constexpr uint32_t bf16_pow2(int e) { return (uint32_t)(127 + e) << 7; }

template <int BITS> struct Codec;

// b = 2: pair p = 4 m + q sits at bits [2 p, 2 p + 2) of both halves.  Three pairs share one shift.
template <> struct Codec<2> {
  static constexpr int NM = 2, PLANES = 1, KSTEP = 64;
  static constexpr int cls(int m, int q) { return (4 * m + q) % 3; }
  static constexpr uint32_t bias_pair(int m, int q) { return dup16(bf16_pow2(7 - 2 * cls(m, q))); }
  static __device__ __forceinline__ void dequant(const uint32_t (&w)[1], u32x4 (&out)[2]) {
#pragma unroll
    for (int m = 0; m < 2; ++m)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = 4 * m + q, sg = p / 3, c = p % 3;
        out[m][q] = ((w[0] >> (6 * sg)) & (0x00030003u << (2 * c))) | bias_pair(m, q);
      }
  }
};

// b = 1: pair p = 4 m + q sits at bit p of both halves.  Seven pairs share one shift.
template <> struct Codec<1> {
  static constexpr int NM = 4, PLANES = 1, KSTEP = 128;
  static constexpr int cls(int m, int q) { return (4 * m + q) % 7; }
  static constexpr uint32_t bias_pair(int m, int q) { return dup16(bf16_pow2(7 - cls(m, q))); }
  static __device__ __forceinline__ void dequant(const uint32_t (&w)[1], u32x4 (&out)[4]) {
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int p = 4 * m + q, sg = p / 7, c = p % 7;
        out[m][q] = ((w[0] >> (7 * sg)) & (0x00010001u << c)) | bias_pair(m, q);
      }
  }
};

// b = 3: words 0 / 1 hold the low two bits like b = 2 (for m < 2 / m >= 2), word 2 the high bits,
// placed so that one shift of word 2 serves the three pairs that share a shift of word 0 / 1.
template <> struct Codec<3> {
  static constexpr int NM = 4, PLANES = 3, KSTEP = 128;
  static constexpr int cls(int m, int q) { return (4 * (m & 1) + q) % 3; }
  static constexpr uint32_t bias_pair(int m, int q) { return dup16(bf16_pow2(7 - 2 * cls(m, q))); }
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
        const uint32_t lo = (src >> (6 * sg)) & (0x00030003u << (2 * c));
        const int sh = hi_pos(m, q) - (2 * c + 2);
        const uint32_t hs = sh >= 0 ? (w[2] >> (sh >= 0 ? sh : 0)) : (w[2] << (sh < 0 ? -sh : 0));
        out[m][q] = lo | (hs & (0x00010001u << (2 * c + 2))) | bias_pair(m, q);
      }
  }
};

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

template <int BITS, int R, int TT>
__global__ __launch_bounds__(256) void k_delta_linear(const LinearParams p) {
  using C = Codec<BITS>;
  constexpr int NM = C::NM;
  constexpr int PL = C::PLANES;
  constexpr int SPC = 128 / C::KSTEP;  // steps per 128-column chunk
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n = lane & 15, g = lane >> 4;
  const int rg = blockIdx.x, sp = blockIdx.y;
  const int jt0 = rg * R;
  const int n_steps = p.n_chunks * SPC;
  const int s_begin = (int)((long)sp * p.n_chunks / p.nsplit) * SPC;
  const int s_end = (int)((long)(sp + 1) * p.n_chunks / p.nsplit) * SPC;
  const int t_hi = p.t0 + 16 * TT;

  f32x4 acc_base[R][TT], acc_raw[R][TT], acc_c[TT], acc_cs[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    acc_c[tt] = f32x4{0, 0, 0, 0};
    acc_cs[tt] = f32x4{0, 0, 0, 0};
#pragma unroll
    for (int rt = 0; rt < R; ++rt) { acc_base[rt][tt] = f32x4{0, 0, 0, 0}; acc_raw[rt][tt] = f32x4{0, 0, 0, 0}; }
  }

  // Constant A operand: rows = 0 (mod 4) carry the dequantisation biases, rows = 1 (mod 4) carry 1.0,
  // so result register 0 is sum_i x_i bias_i and register 1 is sum_i x_i for the lane's token.
  u32x4 ca[NM];
  const int rsel = n & 3;
#pragma unroll
  for (int m = 0; m < NM; ++m)
#pragma unroll
    for (int q = 0; q < 4; ++q) ca[m][q] = rsel == 0 ? C::bias_pair(m, q) : (rsel == 1 ? 0x3f803f80u : 0u);
  const uint32_t one_sel = rsel == 0 ? 0x3f803f80u : 0u;
  const u32x4 ones_a = {one_sel, one_sel, one_sel, one_sel};

  for (int s = s_begin + wave; s < s_end; s += 4) {
    // activations of this step, already in B-operand form
    u32x4 xb[TT][NM];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        const int t = p.t0 + 16 * tt + n;
        const int col = C::KSTEP * s + 32 * m + 8 * g;
        u32x4 v = {0, 0, 0, 0};
        if (t < p.T && col < p.d_in) v = *reinterpret_cast<const u32x4*>(p.x + (size_t)t * p.d_in + col);
        xb[tt][m] = v;
      }
    // shared base product and the per-token sums
#pragma unroll
    for (int m = 0; m < NM; ++m) {
#pragma unroll
      for (int rt = 0; rt < R; ++rt) {
        const u32x4 a = p.w_base[((size_t)(jt0 + rt) * p.n_kb + (s * NM + m)) * 64 + lane];
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) acc_base[rt][tt] = mfma16(a, xb[tt][m], acc_base[rt][tt]);
      }
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) acc_c[tt] = mfma16(ca[m], xb[tt][m], acc_c[tt]);
    }
    // every expert that has tokens in this group
    for (int e = 0; e < p.n_experts; ++e) {
      const int lo = max(p.off[e], p.t0) - p.t0;
      const int hi = min(p.off[e + 1], t_hi) - p.t0;
      if (hi <= lo) continue;
      u32x4 dq[R][NM];
#pragma unroll
      for (int rt = 0; rt < R; ++rt) {
        uint32_t cw[PL];
        const uint32_t* src = p.codes[e] + ((size_t)(jt0 + rt) * n_steps + s) * (PL * 64) + lane;
#pragma unroll
        for (int pl = 0; pl < PL; ++pl) cw[pl] = src[pl * 64];
        C::dequant(cw, dq[rt]);
      }
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        if (16 * tt < hi && 16 * tt + 16 > lo) {
          const int tl = 16 * tt + n;
          const bool inm = tl >= lo && tl < hi;
#pragma unroll
          for (int m = 0; m < NM; ++m) {
            u32x4 xm;
#pragma unroll
            for (int q = 0; q < 4; ++q) xm[q] = inm ? xb[tt][m][q] : 0u;
#pragma unroll
            for (int rt = 0; rt < R; ++rt) acc_raw[rt][tt] = mfma16(dq[rt][m], xm, acc_raw[rt][tt]);
          }
        }
      }
    }
  }

  // salient fp16 columns: (expert, token tile) pairs are dealt round-robin to all wavefronts of the row group
  if (p.k > 0) {
    const int n_workers = p.nsplit * 4, me = sp * 4 + wave;
    int vis = 0;
    for (int e = 0; e < p.n_experts; ++e) {
      const int lo = max(p.off[e], p.t0) - p.t0;
      const int hi = min(p.off[e + 1], t_hi) - p.t0;
      if (hi <= lo) continue;
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        if (16 * tt < hi && 16 * tt + 16 > lo) {
          if (vis % n_workers == me) {
            const int tl = 16 * tt + n;
            const bool inm = tl >= lo && tl < hi;
            const uint16_t* xrow = p.x + (size_t)(p.t0 + tl) * p.d_in;
            const int32_t* si = p.sidx[e];
            for (int sb = 0; sb < p.n_sb; ++sb) {
              u32x4 xs;
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const int r0 = 32 * sb + 8 * g + 2 * q;
                uint32_t v0 = 0, v1 = 0;
                // indices are clamped so that a corrupt list can never address outside the row
                if (inm && r0 < p.k) v0 = xrow[min((uint32_t)si[r0], (uint32_t)(p.d_in - 1))];
                if (inm && r0 + 1 < p.k) v1 = xrow[min((uint32_t)si[r0 + 1], (uint32_t)(p.d_in - 1))];
                xs[q] = v0 | (v1 << 16);
              }
              acc_cs[tt] = mfma16(ones_a, xs, acc_cs[tt]);
#pragma unroll
              for (int rt = 0; rt < R; ++rt) {
                const u32x4 d = p.sal[e][((size_t)(jt0 + rt) * p.n_sb + sb) * 64 + lane];
                u32x4 dh, dl;
#pragma unroll
                for (int q = 0; q < 4; ++q) { uint32_t h, l; split_f16_pair(d[q], h, l); dh[q] = h; dl[q] = l; }
                acc_base[rt][tt] = mfma16(dh, xs, acc_base[rt][tt]);
                acc_base[rt][tt] = mfma16(dl, xs, acc_base[rt][tt]);
              }
            }
          }
          ++vis;
        }
      }
    }
  }

  // epilogue: remove biases / zero point, apply the expert's step, add across wavefronts
  __shared__ float red[4][R * TT * 4][64];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    const int t = p.t0 + 16 * tt + n;
    int et = -1;
    for (int e = 0; e < p.n_experts; ++e)
      if (t >= p.off[e] && t < p.off[e + 1]) et = e;
    const float corr = acc_c[tt][0] + p.z * (acc_c[tt][1] - acc_cs[tt][0]);
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
      const int j = 16 * (jt0 + rt) + 4 * g;
      f32x4 st = {0, 0, 0, 0};
      if (et >= 0 && j < p.d_out) st = *reinterpret_cast<const f32x4*>(p.step[et] + j);
#pragma unroll
      for (int v = 0; v < 4; ++v)
        red[wave][(rt * TT + tt) * 4 + v][lane] = acc_base[rt][tt][v] + st[v] * (acc_raw[rt][tt][v] - corr);
    }
  }
  __syncthreads();

  for (int pi = wave; pi < R * TT; pi += 4) {
    const int rt = pi / TT, tt = pi % TT;
    f32x4 o;
#pragma unroll
    for (int v = 0; v < 4; ++v)
      o[v] = ((red[0][pi * 4 + v][lane] + red[1][pi * 4 + v][lane]) + red[2][pi * 4 + v][lane]) + red[3][pi * 4 + v][lane];
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
  if (p.nsplit == 1) return;

  // split columns: the last workgroup of this row group adds the partial tiles in split order
  __shared__ int s_last;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) s_last = atomicAdd(p.counters + rg, 1) == p.nsplit - 1;
  __syncthreads();
  if (!s_last) return;
  __threadfence();
  for (int pi = wave; pi < R * TT; pi += 4) {
    const int rt = pi / TT, tt = pi % TT;
    const int tl = 16 * tt + n, t = p.t0 + tl;
    const int j = 16 * (jt0 + rt) + 4 * g;
    if (t < p.T && j < p.d_out) {
      f32x4 o = {0, 0, 0, 0};
      for (int s2 = 0; s2 < p.nsplit; ++s2) {
        const f32x4 v = *reinterpret_cast<const f32x4*>(p.partial + ((size_t)(s2 * kTokGroup + tl) * p.d_out_pad + j));
        o += v;
      }
      uint2 pk;
      pk.x = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
      pk.y = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
      *reinterpret_cast<uint2*>(p.y + (size_t)t * p.d_out + j) = pk;
    }
  }
  if (threadIdx.x == 0) p.counters[rg] = 0;
}

struct Plan {
  int R;       // 16-row tiles per workgroup
  int nsplit;  // workgroups that share one row group's columns
};

// Pure function of the layer shape (not of bits or T), so the workspace size is known up front.
Plan plan_for(int d_in, int d_out) {
  const int po = ceil_to(d_out, kRowPad), pi = ceil_to(d_in, kColPad);
  const int n_chunks = pi / 128;
  Plan pl;
  pl.R = 2;
  const int row_groups = po / (16 * pl.R);
  int ns = (512 + row_groups - 1) / row_groups;
  const int max_split = n_chunks / 4 > 0 ? n_chunks / 4 : 1;   // at least four chunks per workgroup
  if (ns > max_split) ns = max_split;
  if (ns > 16) ns = 16;
  if (ns < 1) ns = 1;
  pl.nsplit = ns;
  return pl;
}

template <int BITS, int R>
hipError_t launch_tt(const LinearParams& p, int tt, dim3 grid, hipStream_t s) {
  switch (tt) {
    case 1: k_delta_linear<BITS, R, 1><<<grid, 256, 0, s>>>(p); break;
    case 2: k_delta_linear<BITS, R, 2><<<grid, 256, 0, s>>>(p); break;
    case 3: k_delta_linear<BITS, R, 3><<<grid, 256, 0, s>>>(p); break;
    default: k_delta_linear<BITS, R, 4><<<grid, 256, 0, s>>>(p); break;
  }
  return hipGetLastError();
}

template <int R>
hipError_t launch_bits(const LinearParams& p, int bits, int tt, dim3 grid, hipStream_t s) {
  switch (bits) {
    case 1: return launch_tt<1, R>(p, tt, grid, s);
    case 2: return launch_tt<2, R>(p, tt, grid, s);
    default: return launch_tt<3, R>(p, tt, grid, s);
  }
}

}  // namespace

size_t linear_workspace_bytes(int d_in, int d_out, int max_tokens) {
  (void)max_tokens;  // one 64-token group is in flight at a time
  const Plan pl = plan_for(d_in, d_out);
  const int po = ceil_to(d_out, kRowPad);
  size_t counters = (size_t)ceil_to(po / 16, 64) * sizeof(int);
  size_t partial = pl.nsplit > 1 ? (size_t)pl.nsplit * kTokGroup * po * sizeof(float) : 0;
  return counters + partial;
}

hipError_t launch_delta_linear(const LinearCall& c, hipStream_t s) {
  const mes_delta& d0 = c.experts[0];
  const Plan pl = plan_for(d0.d_in, d0.d_out);
  LinearParams p;
  p.w_base = reinterpret_cast<const u32x4*>(c.w_base);
  p.x = reinterpret_cast<const uint16_t*>(c.x);
  p.y = reinterpret_cast<uint16_t*>(c.y);
  const int po = ceil_to(d0.d_out, kRowPad), pi = ceil_to(d0.d_in, kColPad);
  p.counters = reinterpret_cast<int*>(c.ws);
  p.partial = reinterpret_cast<float*>(reinterpret_cast<char*>(c.ws) + (size_t)ceil_to(po / 16, 64) * sizeof(int));
  for (int e = 0; e < MES_MAX_EXPERTS; ++e) {
    const bool in = e < c.n_experts;
    p.codes[e] = in ? reinterpret_cast<const uint32_t*>(c.experts[e].codes) : nullptr;
    p.step[e] = in ? c.experts[e].step : nullptr;
    p.sal[e] = in ? reinterpret_cast<const u32x4*>(c.experts[e].salient) : nullptr;
    p.sidx[e] = in ? c.experts[e].salient_idx : nullptr;
  }
  for (int e = 0; e <= MES_MAX_EXPERTS; ++e) p.off[e] = e <= c.n_experts ? c.seg[e] : c.T;
  p.d_in = d0.d_in;
  p.d_out = d0.d_out;
  p.d_out_pad = po;
  p.n_kb = pi / 32;
  p.n_chunks = pi / 128;
  p.n_sb = ceil_to(d0.k, kSalPad) / 32;
  p.k = d0.k;
  p.T = c.T;
  p.n_experts = c.n_experts;
  p.nsplit = pl.nsplit;
  p.z = d0.grid == MES_GRID_SYM ? (float)(1 << (d0.bits - 1)) - 0.5f : (float)(1 << (d0.bits - 1));
  const dim3 grid(po / (16 * pl.R), pl.nsplit);
  for (int t0 = 0; t0 < c.T; t0 += kTokGroup) {
    p.t0 = t0;
    const int nt = c.T - t0 < kTokGroup ? c.T - t0 : kTokGroup;
    const int tt = (nt + 15) / 16;
    hipError_t e;
    switch (pl.R) {
      case 1: e = launch_bits<1>(p, d0.bits, tt, grid, s); break;
      case 2: e = launch_bits<2>(p, d0.bits, tt, grid, s); break;
      default: e = launch_bits<4>(p, d0.bits, tt, grid, s); break;
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace mes
