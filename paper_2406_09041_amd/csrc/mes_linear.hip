// The serving hot path (Eq. 4, batched across experts):
//   y[t] = x[t] W^T + step_e .* (x_ns[t] (U_e - z)^T) + x_s[t] D_e^T
// for token groups of up to 64 tokens, up to four groups per launch.  Per launch: one small preparation launch, the
// main streaming launch and, only when the columns had to be split over workgroups, a small reduction launch.
// (Letting the last workgroup of a row group do that reduction inside the main kernel was measured and is slower:
// the device-wide hand-over costs more than the extra launch.  Likewise the preparation folded into the main kernel.)
//
// Main kernel.  A workgroup of eight wavefronts (two per SIMD: while one waits for memory or for the
// matrix core the other issues) owns 128 output channels, one 16-row tile per wavefront, and a range of
// 128-column chunks.  The activations of a chunk are shared by all wavefronts through LDS (double
// buffered, copied memory -> LDS one chunk ahead); every weight byte is read once, by the one wavefront
// that needs it, at least one chunk ahead.
//
// Three products accumulate per wavefront, all on the matrix cores, weights as the A operand (16 output
// channels), tokens as the B operand (16 tokens), so a result tile is [channel][token]:
//   base     v_mfma_f32_16x16x32_bf16: bf16 W tile x bf16 x tile.
//   low-bit  v_mfma_scale_f32_16x16x128_f8f6f4 with A in fp4 (E2M1) and B in fp8 (E4M3).  An fp4 nibble
//            00uu is the number u / 2 and 0h00 is 2 h, so the packed codes become the A operand with one
//            AND (plus one shift for every second register): no conversion, no multiply.  The activations
//            are split by the preparation kernel into two fp8 pieces, x * 2^-s = hi + lo with s a power of
//            two per (token, chunk); hi is the value rounded to four significant bits and lo the remainder
//            (four bits at most), so the two products together are the exact bf16 x code product whenever
//            the value is within 2^-10 of the largest of its token in the chunk (below that lo is rounded at
//            2^-17 of that largest value).  The instruction's per-lane block scale (a power of two applied
//            to a token's products) carries 2^(s+1) for tokens of the expert being multiplied and 2^-127
//            for every other token of the tile -- that is how several experts share a 16-token tile.
//   salient  v_mfma_f32_16x16x32_bf16, twice: the activations at the expert's salient columns as gathered (bf16,
//            nothing converted) x the expert's fp16 values D, each written as the sum of two bf16 numbers
//            (8 + 8 significant bits hold the 11 of an fp16 value, and then some).
// Zero point and per-output-channel step are applied after the reduction:
//   sum over non-salient i of x_i (u_i - z) = sum_all x_i u_i - z sum_all x_i + z sum_salient x_i
// (codes stored at salient and padding columns are 0).  The middle term is a per-token number (the preparation
// leaves per-chunk sums, the loop adds them up); the last one, times the step, is folded into the salient product:
// its weights are D + z step instead of D.
//
// Slots.  The host lists the experts that own tokens of the group ("slots", in expert order; an expert
// with an empty segment is never touched).  Tokens are sorted by expert, so the slots with tokens in one
// 16-token tile are a contiguous range, walked by a plain loop; the code words of the chunk wait in LDS,
// where a run-time slot number can index them.
#include "mes_internal.h"


namespace mes {
namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;
typedef int v8i __attribute__((ext_vector_type(8)));
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;

constexpr int kChunk = 128;                     // columns per chunk (one fp4 x fp8 MFMA deep)
constexpr int kStageVec = 2048;                 // 16-byte slots of activations per chunk
constexpr int kStageBytes = kStageVec * 16 + 1024;  // + a block of per-token numbers (block scales, sums)
constexpr int kStageFp8 = 16384;                // byte offset of the fp8 pieces inside a stage
constexpr int kStageScale = 32768;              // byte offset of the scales inside a stage
constexpr int kStageSum = 32768 + 256;          // byte offset of the tokens' sums over the chunk's columns
constexpr int kStageBlocks = 33;                // 1 KiB blocks the main kernel copies to LDS per chunk
constexpr int kStageLds = 32 * 1024;            // LDS bytes of a stage's operand images; its 33rd block sits apart (see k_delta_linear)
constexpr int kMaxSlots = 16;                   // experts with tokens in one token group (the host cuts groups accordingly)
constexpr int kMaxVisits = kMaxSlots + 3;       // (expert, 16-token tile) pairs in one group

constexpr int kMaxSplits = 32;                  // workgroups that may share one row group's columns

constexpr int kMaxLinears = MES_MAX_FUSED;    // linear layers one launch serves (they read the same activations)

// Per linear layer: where its weights, outputs and its share of the workspace are.  Per-expert arrays are indexed by slot.
struct PerLinear {
  const char* w_base;
  uint16_t* y;
  u32x4* xs;        // workspace: salient activations per visit, bf16 as gathered  [visit][k_pad/32][64 lanes]
  const char* codes[kMaxSlots];
  const float* step[kMaxSlots];
  const char* sal[kMaxSlots];
  const int32_t* sidx[kMaxSlots];
  int d_out, n_jt;
  int rg_begin, rg_end;   // its row groups among the launch's
};

// Kernel arguments.
struct LinearParams {
  const uint16_t* x;
  char* xt;         // workspace: one stage per chunk (see prepare_item), shared by the linears
  f32x4* partial;   // workspace: [row group][nsplit][4 tiles][threads of a workgroup] partial result tiles (split columns only)
  PerLinear lin[kMaxLinears];
  int16_t lo[kMaxSlots], hi[kMaxSlots];   // tokens [lo, hi) of the group belong to the slot's expert
  uint8_t tok_slot[kTokGroup];            // slot of every token of the group, 0xFF past the last token
  int vis_info[kMaxVisits + 1];           // visits (slot, tile) in tile-major order: slot | tile << 8
  int tile_first[4], tile_last[4];        // slots that own tokens of 16-token tile tt: tile_first[tt] .. tile_last[tt]
  int d_in, n_linears, n_chunks, n_sb, k, T, t0, n_act, n_vis, nsplit, bits;
  int16_t c_split[kMaxSplits + 1];        // workgroup sp of a row group covers the chunks c_split[sp] .. c_split[sp + 1]
  int tiles;                              // 16-token tiles of the group that hold tokens
  int n_stage_items, n_items;             // preparation items: tiles * n_chunks stage items, then n_linears * n_vis gathers
  float z;
  // Gated pair (see launch_delta_linear): lin[0] is the gate, lin[1] the up projection of an MLP block.  The first
  // half of a workgroup's wavefronts owns row tiles of the gate, the second half the same row tiles of the up
  // projection, and the workgroup writes SiLU(gate) * up to lin[0].y instead of the two results.
  int pair;
};

// One launch serves up to kMaxGroups token groups (256 tokens), in two classes: the groups with many experts (their
// workgroups take about half as long again as the others') come first in g[] and in the workgroup ids, so that the
// long workgroups start first and the short ones fill the compute units behind them -- in the order of the token
// groups the last workgroups to start would be long ones, with most of the chip idle while they finish.
// Within a class the ids are laid out so that the workgroups of one row group -- one per token group -- are
// neighbours on one XCD: they start together, stream the same base weights at about the same time, and all but the
// first find them in that XCD's L2.  Memory sees the base weights once per class rather than once per token group.
constexpr int kMaxGroups = 4;
struct LaunchParams {
  LinearParams g[kMaxGroups];
  int n_groups;
  int n_first;  // groups of the first class (g[0 .. n_first)), at least 1
  int rgs;      // row groups of the launch (all linears)
  int rg8;      // ... in eights, rounded up
  int wg_per_group;   // rg8 * 8 * nsplit.  Flat workgroup id within a class of m groups:
                      // ((split * rg8 + rg / 8) * m + group) * 8 + rg % 8
};

// The linear a row group belongs to.
__device__ __forceinline__ int linear_of(const LinearParams& p, int rg) {
  int l = 0;
#pragma unroll
  for (int i = 0; i + 1 < kMaxLinears; ++i) l += (i + 1 < p.n_linears && rg >= p.lin[i].rg_end) ? 1 : 0;
  return l;
}


__device__ __forceinline__ f32x4 mfma_bf16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// acc += A x (Bhi + Blo) [+ Ah x (Bhi + Blo)], fp4 (A, four registers) x fp8 E4M3 (B, eight registers each),
// B scaled per lane by 2^(scale_b - 127).  Written as instructions with the accumulator tied to itself: these
// updates sit in loops and wave-uniform branches, and only a tied operand keeps the compiler from copying
// whole accumulator sets from block to block.  The compiler does not know what the block contains, so the
// block itself provides the two wait states the hardware needs between a vector-ALU write of an operand
// register and a matrix instruction reading it.  (Same opcode, same register as source C and destination:
// back-to-back issue needs no further wait states.)
// scale_a is A's block scale byte: 127 for 2^0; the high plane of 4-bit codes takes 129 (its codes count four times).
__device__ __forceinline__ void mfma_fp4_fp8_pair(f32x4& acc, u32x4 a, v8i bhi, v8i blo, int scale_b, int scale_a = 127) {
  asm volatile("s_nop 1\n\t"
               "v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %2, %0, %4, %5 op_sel_hi:[0,0,0] cbsz:4\n\t"
               "v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %3, %0, %4, %5 op_sel_hi:[0,0,0] cbsz:4"
               : "+v"(acc) : "v"(a), "v"(bhi), "v"(blo), "v"(scale_a), "v"(scale_b));
}

// Code words of one slot for one (chunk, row tile): LW low words per lane and HW words of high bits (b = 3: one
// word, the third bit; b = 4: two words, the high two bits laid out like the low two).
template <int BITS> struct Codec;
template <> struct Codec<2> { static constexpr int LW = 2, HW = 0; };
template <> struct Codec<1> { static constexpr int LW = 1, HW = 0; };
template <> struct Codec<3> { static constexpr int LW = 2, HW = 1; };
template <> struct Codec<4> { static constexpr int LW = 2, HW = 2; };

template <int BITS>
struct CodeRegs {
  uint32_t lo[Codec<BITS>::LW];
  uint32_t hi[Codec<BITS>::HW > 0 ? Codec<BITS>::HW : 1];
};

// Bytes of one (chunk, row tile) block of a slot's codes.
__host__ __device__ constexpr int code_block_bytes(int bits) { return 256 * bits; }

template <int BITS>
// `blk` is the same in all lanes and the lane offset an unsigned 32-bit number: the load then takes its
// address as (scalar base) + (vector offset) and needs no 64-bit vector arithmetic.
__device__ __forceinline__ void load_codes(const char* blk, int lane, CodeRegs<BITS>& r) {
  if constexpr (BITS == 1) {
    r.lo[0] = *reinterpret_cast<const uint32_t*>(blk + (uint32_t)lane * 4u);
  } else {
    const u32x2 v = *reinterpret_cast<const u32x2*>(blk + (uint32_t)lane * 8u);
    r.lo[0] = v[0]; r.lo[1] = v[1];
    if constexpr (BITS == 3) r.hi[0] = *reinterpret_cast<const uint32_t*>(blk + 512 + (uint32_t)lane * 4u);
    if constexpr (BITS == 4) {
      const u32x2 h = *reinterpret_cast<const u32x2*>(blk + 512 + (uint32_t)lane * 8u);
      r.hi[0] = h[0]; r.hi[1] = h[1];
    }
  }
}

// Low code bits as an fp4 A operand (values u / 2, or (u mod 4) / 2 for b = 3).
template <int BITS>
__device__ __forceinline__ u32x4 dequant_lo(const CodeRegs<BITS>& r) {
  u32x4 a;
  if constexpr (BITS == 1) {
    const uint32_t w = r.lo[0];
    a[0] = w & 0x11111111u; a[1] = (w >> 1) & 0x11111111u; a[2] = (w >> 2) & 0x11111111u; a[3] = (w >> 3) & 0x11111111u;
  } else {
    const uint32_t w0 = r.lo[0], w1 = r.lo[1];
    a[0] = w0 & 0x33333333u; a[1] = (w0 >> 2) & 0x33333333u; a[2] = w1 & 0x33333333u; a[3] = (w1 >> 2) & 0x33333333u;
  }
  return a;
}

// High code bit (b = 3) as an fp4 A operand: nibble 0h00 = 2 h = (4 h) / 2.
__device__ __forceinline__ u32x4 dequant_hi(const CodeRegs<3>& r) {
  const uint32_t w = r.hi[0];
  u32x4 a;
  a[0] = (w << 2) & 0x44444444u; a[1] = (w << 1) & 0x44444444u; a[2] = w & 0x44444444u; a[3] = (w >> 1) & 0x44444444u;
  return a;
}

// High two code bits (b = 4) as an fp4 A operand: values h / 2; the matrix instruction scales them by four.
__device__ __forceinline__ u32x4 dequant_hi(const CodeRegs<4>& r) {
  const uint32_t w0 = r.hi[0], w1 = r.hi[1];
  return u32x4{w0 & 0x33333333u, (w0 >> 2) & 0x33333333u, w1 & 0x33333333u, (w1 >> 2) & 0x33333333u};
}

// fp32 -> bf16 bits, round to nearest even.
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// SiLU(gate) * up, element by element, in fp32: SiLU(v) = v / (1 + e^-v).
__device__ __forceinline__ f32x4 gated(f32x4 gate, f32x4 up) {
  f32x4 h;
#pragma unroll
  for (int v = 0; v < 4; ++v) h[v] = gate[v] / (1.0f + expf(-gate[v])) * up[v];
  return h;
}

// ---- preparation ------------------------------------------------------------------------------------
// The preparation launch: one item per block of 256 threads.  Items [0, n_stage_items) build one token tile of one
// chunk's stage (item = chunk * tiles + tile) and that tile's per-token sums over the chunk's columns; the items after
// them gather, per linear and visit, the visit's salient activations.
//
// Stage of chunk c (what the main loop copies to LDS), columns counted from 128 c, lane = 16 g + n:
//   bytes [0, 16384)      bf16, [kb][tt][lane][8]: x[16 tt + n][32 kb + 8 g + 0..7]
//   bytes [16384, 32768)  fp8,  [tt][piece][half][lane][16]: piece (0 = hi, 1 = lo) of
//                         x[16 tt + n][64 half + 16 g + 0..15] * 2^-s   (the B operand's own column order)
//   bytes [32768, 33024)  int32 [64]: 128 + s of token 16 tt + n, i.e. the scale byte 2^(s+1) (the extra
//                         factor two undoes the fp4 codes' u / 2)
//   bytes [33024, 33280)  float [64]: sum of the token's activations over the chunk's columns; the rest of the
//                         33rd KiB is padding
__global__ __launch_bounds__(256) void k_prepare(const LaunchParams mp) {
  const LinearParams& p = mp.g[blockIdx.y];
  const int tid = threadIdx.x, item = blockIdx.x;
  if (item >= p.n_items) return;   // the grid is as wide as the group with the most items
  if (item < p.n_stage_items) {
    // (chunk c, token tile tt): thread = (token n of the tile, 8 columns `part` of the chunk's 128)
    const int c = item / p.tiles, tt = item - c * p.tiles;
    char* stage = p.xt + (size_t)c * kStageBytes;
    const int n = tid >> 4, part = tid & 15, q = part >> 2, i = part & 3;
    const int t = p.t0 + 16 * tt + n, col = kChunk * c + 8 * part;
    u32x4 v = {0, 0, 0, 0};
    if (t < p.T && col < p.d_in) v = *reinterpret_cast<const u32x4*>(p.x + (size_t)t * p.d_in + col);
    // bf16 image: these eight columns are lane 16 i + n of block (kb = q, tt)
    *reinterpret_cast<u32x4*>(stage + ((q * 4 + tt) * 64 + 16 * i + n) * 16) = v;
    float xv[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      xv[2 * e] = bf16_to_f32((uint16_t)(v[e] & 0xffffu));
      xv[2 * e + 1] = bf16_to_f32((uint16_t)(v[e] >> 16));
    }
    float amax = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) amax = fmaxf(amax, fabsf(xv[e]));
    // the token's sum over this chunk (what the zero point is multiplied with), in a fixed order
    float rs = ((xv[0] + xv[1]) + (xv[2] + xv[3])) + ((xv[4] + xv[5]) + (xv[6] + xv[7]));
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) {   // the token's 16 threads
      amax = fmaxf(amax, __shfl_xor(amax, off));
      rs += __shfl_xor(rs, off);
    }
    // s = exponent(amax) - 7 puts the largest scaled value in [128, 256); clamped so that 128 + s is a
    // valid scale byte.  Non-finite activations give non-finite outputs either way.
    int s = (int)((__float_as_uint(amax) >> 23) & 0xffu) - 127 - 7;
    if (amax == 0.0f) s = 0;
    s = s < -126 ? -126 : (s > 120 ? 120 : s);
    const float inv = __uint_as_float((uint32_t)(127 - s) << 23);   // 2^-s
    // hi = x 2^-s rounded to the E4M3 grid (to nearest: the hardware conversion), lo = what is left, on the same grid
    int hw[2] = {0, 0}, lw[2] = {0, 0};
    // (the half of the word a conversion writes or reads is part of the instruction: spelled out, not looped)
#define MES_SPLIT_PAIR(E, W, UPPER)                                                                     \
    {                                                                                                   \
      const float s0 = xv[E] * inv, s1 = xv[E + 1] * inv;                                               \
      hw[W] = __builtin_amdgcn_cvt_pk_fp8_f32(s0, s1, hw[W], UPPER);                                    \
      const auto back = __builtin_amdgcn_cvt_pk_f32_fp8(hw[W], UPPER);                                  \
      lw[W] = __builtin_amdgcn_cvt_pk_fp8_f32(s0 - back[0], s1 - back[1], lw[W], UPPER);                \
    }
    MES_SPLIT_PAIR(0, 0, false)
    MES_SPLIT_PAIR(2, 0, true)
    MES_SPLIT_PAIR(4, 1, false)
    MES_SPLIT_PAIR(6, 1, true)
#undef MES_SPLIT_PAIR
    // columns 32 q + 8 i + e  ->  half = q / 2, lane group g = 2 (q % 2) + i / 2, bytes 8 (i % 2) + e
    const int lane = 16 * (2 * (q & 1) + (i >> 1)) + n;
    char* dst = stage + kStageFp8 + ((tt * 2 + 0) * 2 + (q >> 1)) * 1024 + lane * 16 + 8 * (i & 1);
    *reinterpret_cast<u32x2*>(dst) = u32x2{(uint32_t)hw[0], (uint32_t)hw[1]};
    *reinterpret_cast<u32x2*>(dst + 2048) = u32x2{(uint32_t)lw[0], (uint32_t)lw[1]};
    if (part == 0) {
      *reinterpret_cast<int*>(stage + kStageScale + (16 * tt + n) * 4) = 128 + s;
      *reinterpret_cast<float*>(stage + kStageSum + (16 * tt + n) * 4) = rs;
    }
    return;
  }
  // Salient activations of one visit as B operands: block sb, lane 16 g + n holds x[token n of the tile][S[32 sb + 8 g + 0..7]]
  // for the tokens of the tile that belong to the visit's expert, zero for the others and for ranks past k.
  const int gi = item - p.n_stage_items;
  const int li = gi / p.n_vis, v = gi - li * p.n_vis;
  const PerLinear& L = p.lin[li];
  const int a = p.vis_info[v] & 0xff, tt = p.vis_info[v] >> 8;
  const int32_t* si = L.sidx[a];
  for (int i = tid; i < p.n_sb * 64; i += 256) {
    const int sb = i >> 6, lane = i & 63, n = lane & 15, gg = lane >> 4;
    const int tl = 16 * tt + n;
    const bool inm = tl >= p.lo[a] && tl < p.hi[a];
    const uint16_t* xrow = p.x + (size_t)(p.t0 + tl) * p.d_in;
    u32x4 o;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r0 = 32 * sb + 8 * gg + 2 * q;   // indices are clamped so that a corrupt list can never address outside the row
      uint32_t v0 = 0, v1 = 0;
      if (inm && r0 < p.k) v0 = xrow[min((uint32_t)si[r0], (uint32_t)(p.d_in - 1))];
      if (inm && r0 + 1 < p.k) v1 = xrow[min((uint32_t)si[r0 + 1], (uint32_t)(p.d_in - 1))];
      o[q] = v0 | (v1 << 16);
    }
    L.xs[((size_t)v * p.n_sb + sb) * 64 + lane] = o;
  }
}

// ---- main kernel ------------------------------------------------------------------------------------

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_void;
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// Loads are written as (wave-uniform pointer) + (32-bit unsigned lane offset): the pointer then lives in
// scalar registers and one vector register per lane serves every stream.
// The pointers are declared to be device (global) memory: one that has been through keep() has lost the
// compiler's knowledge of that, and a generic load would also count as an LDS access.
typedef __attribute__((address_space(1))) const char global_char;
__device__ __forceinline__ global_char* gptr(const void* q) { return reinterpret_cast<global_char*>(reinterpret_cast<uintptr_t>(q)); }
__device__ __forceinline__ u32x4 ld128(const void* uniform_ptr, uint32_t lane_off) {
  return *reinterpret_cast<__attribute__((address_space(1))) const u32x4*>(gptr(uniform_ptr) + lane_off);
}


__device__ __forceinline__ u32x4 lds128(const char* stage, int off) { return *reinterpret_cast<const u32x4*>(stage + off); }

__device__ __forceinline__ v8i lds_fp8(const char* stage, int tt, int piece, int lane) {
  const char* s = stage + kStageFp8 + (tt * 2 + piece) * 2048 + lane * 16;
  const u32x4 h0 = *reinterpret_cast<const u32x4*>(s), h1 = *reinterpret_cast<const u32x4*>(s + 1024);
  return v8i{(int)h0[0], (int)h0[1], (int)h0[2], (int)h0[3], (int)h1[0], (int)h1[1], (int)h1[2], (int)h1[3]};
}

// Copies one chunk's stage from memory straight into LDS (no registers in between): wavefront `wave` of NW
// copies the 1 KiB blocks wave, wave + NW, ... of the 32.  The number of copy instructions per wavefront is a
// compile-time constant, so the wait below can name exactly how many younger loads may still be in flight.
// Written as instructions rather than through the compiler's builtin: the compiler would make every later
// LDS access of the wavefront wait for these copies, i.e. stall each chunk for a full memory round trip,
// because it cannot tell that they go to the stage nobody reads yet.  stage_barrier() does the waiting.
template <int NW>
__device__ __forceinline__ void stage_copy(const char* src, char* dst_lds, char* dst_extra, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < (kStageBlocks + NW - 1) / NW; ++i) {
    const int blk = wave + NW * i;
    if (kStageBlocks % NW != 0 && blk >= kStageBlocks) break;   // 33 blocks dealt round-robin: some wavefronts carry one more
    const char* g = src + blk * 1024;                                 // scalar base; the lanes add 16 * lane
    // LDS byte address (the hardware adds 16 * lane): the operand images, or the block of per-token numbers
    const uint32_t l = (uint32_t)(uintptr_t)(blk < 32 ? dst_lds + blk * 1024 : dst_extra);
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"((uint32_t)lane * 16u), "s"(g), "s"(l) : "memory", "m0");
  }
}

// vmcnt(n) lgkmcnt(0) (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 left at its maximum).
constexpr int waitcnt_vm_lgkm0(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0070; }

// Waits until at most `younger` of this wavefront's loads are in flight (loads complete in order, so the
// stage copy issued before them has landed), for its LDS accesses, and then for the whole workgroup.
// Deliberately not __syncthreads(): that would also wait for the weight loads of the next chunk.
template <int YOUNGER>
__device__ __forceinline__ void stage_barrier() {
  __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(YOUNGER));
  asm volatile("s_barrier" ::: "memory");
}

// A value read from the kernel's argument block is kept in a register from here on.  Left alone the compiler treats
// such a value as free to fetch again (it is constant memory) wherever scalar registers run short, i.e. all over
// the streaming loop; every such fetch is a scalar memory load, and while one is in flight every wait for an LDS
// read of the wavefront has to be a wait for everything, which takes the pipelining out of the operand reads.
template <class V>
__device__ __forceinline__ V keep(V v) {
  asm volatile("" : "+s"(v));
  return v;
}

// 16 bytes from a device address held in a lane's registers (a global load, not a generic one: a generic load
// would also count as an LDS access and make every wait for an operand read wait for memory as well).
typedef __attribute__((address_space(1))) const u32x4 global_u32x4;
__device__ __forceinline__ u32x4 ld128_at(uint64_t addr) { return *reinterpret_cast<global_u32x4*>(addr); }

// Per-wavefront state of the streaming loop.
//  - Base weights are double buffered in registers: while chunk c is multiplied out of buffer c % 2, the
//    4 KiB of chunk c + 1 are in flight into the other buffer.
//  - Code words travel memory -> registers -> LDS.  Two register buffers hold the next two chunks' words;
//    at the top of a chunk the buffer that has arrived is parked in the wavefront's private LDS area and
//    reloaded at once with the chunk after next.  LDS can be indexed at run time, registers cannot: that
//    is what lets the loop over the experts of a token tile be a plain loop with a run-time trip count.
//    The words of all slots of a (chunk, row tile) are fetched 1 KiB per load instruction, 16 bytes per lane,
//    whatever slot they belong to: the lanes carry their own addresses (the slots' buffers are separate
//    allocations), worked out once per sweep, and the LDS area is the plain concatenation of the slots' blocks.
//  - Everything the loop needs of the argument block sits in registers or in two small LDS tables (see keep()).
template <int BITS, int TT, int NA, int NW>
struct Stream {
  static constexpr int kSlotLds = code_block_bytes(BITS);       // LDS bytes of one parked slot
  static constexpr int kParkWave = NA * kSlotLds;               // ... of all slots of a sweep
  static constexpr int NL = (kParkWave + 1023) / 1024;          // loads of 1 KiB that bring them in

  const LinearParams& p;
  const PerLinear& L;
  int lane, n, jt;
  // The wavefront's tile tt (a compile-time index: it names accumulators) is token tile pt(tt) of the launch:
  // the same, or the mirror image for the second wavefront of each SIMD.  The two then run through the tiles
  // in opposite orders, so that the tile with many visits (long runs of matrix instructions) of one falls on
  // the tiles with few of the other instead of both queueing for the matrix pipeline at the same time.
  int rev;
  __device__ __forceinline__ int pt(int tt) const { return rev ? TT - 1 - tt : tt; }
  char* parkp;                // this wavefront's LDS area: [NA][kSlotLds]
  // A launch holds up to kMaxSlots experts but only NA of them fit the registers and the LDS area at a time:
  // the chunks are swept once per group of NA slots, the first sweep also doing the base product.
  // a0 = first slot of the current sweep.
  int a0 = 0;
  // launch constants (see keep())
  const char* xt;             // the activation stages
  const char* xs;             // this linear's gathered salient activations
  const char* base_at;        // this row tile's base block of chunk 0
  uint32_t base_stride, code_stride;   // bytes from one chunk's block of this row tile to the next chunk's
  int n_sb, nsplit;
  int tfirst[TT], tlast[TT];  // the tile's visits among the slots of the current sweep (slot numbers relative to a0)
  uint64_t code_at[NL];       // per lane: where its 16 bytes of load i are for chunk 0
  const int* vis_lds;         // LDS copy of the visit table
  const uint64_t* sal_lds;    // LDS: per slot, this linear's salient tile of that expert
  uint32_t slot_tok[TT];
  float rs_acc = 0.0f;        // lane = token: sum of its activations over the chunks done so far
  u32x4 base[2][4];
  u32x4 code[2][NL];
  f32x4 acc_base[TT], acc_raw[TT];

  // Salient fp16 columns ride along with the stream: the (visit, 32-column block) pairs of this workgroup
  // (pairs sp, sp + nsplit, ... of n_vis * n_sb) are dealt kSalPerChunk to a chunk, requested one chunk before
  // they are multiplied.  A = the expert's fp16 tile (turned into D + z step, as two bf16 numbers), B = the visit's gathered activations, bf16.
  static constexpr int kSalPerChunk = 1;
  const float* step_w;   // LDS: this wavefront's steps, [slot][16 rows]
  float z;
  u32x4 sal_x[kSalPerChunk], sal_d[kSalPerChunk];
  int sal_tt[kSalPerChunk], sal_slot[kSalPerChunk];
  int sal_v, sal_sb, sal_left;   // (visit, block) of the next pair to request; pairs not yet requested
  bool nx_more;                  // the request being prepared: is there a pair, its visit entry, its addresses
  int nx_info_v;                 // (as read from LDS: the same in every lane)
  int nx_tt, nx_slot;
  uint64_t nx_sal_v;
  uint32_t nx_xoff, nx_doff;

  __device__ __forceinline__ Stream(const LinearParams& p_, const PerLinear& L_, int lane_, int jt_, char* park_,
                                    const float* step_w_, const int* vis_lds_, const uint64_t* sal_lds_, int rev_)
      : p(p_), L(L_), lane(lane_), n(lane_ & 15), jt(jt_), rev(rev_), parkp(park_), vis_lds(vis_lds_), sal_lds(sal_lds_), step_w(step_w_) {
    z = keep(p.z);
    xt = keep(p.xt);
    xs = keep(reinterpret_cast<const char*>(L.xs));
    base_at = keep(L.w_base + (size_t)jt * 4096);
    base_stride = keep((uint32_t)L.n_jt * 4096u);
    code_stride = keep((uint32_t)L.n_jt * (uint32_t)kSlotLds);
    n_sb = keep(p.n_sb);
    nsplit = keep(p.nsplit);
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      slot_tok[tt] = p.tok_slot[16 * pt(tt) + n];
      acc_base[tt] = f32x4{0, 0, 0, 0};
      acc_raw[tt] = f32x4{0, 0, 0, 0};
    }
  }

  // The slots a0_ .. a0_ + NA - 1 are the ones multiplied from now on.
  __device__ __forceinline__ void begin_sweep(int a0_) {
    a0 = a0_;
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      // a tile with no visit among these slots runs slot 0 of the sweep once with every token's scale 0, like an
      // empty tile: no branch around the visit loop, no second copy of the accumulator
      int first = p.tile_first[pt(tt)] - a0, last = p.tile_last[pt(tt)] - a0;
      first = first < 0 ? 0 : first;
      last = last > NA - 1 ? NA - 1 : last;
      if (first > last) first = last = 0;
      tfirst[tt] = keep(first);
      tlast[tt] = keep(last);
    }
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int byte = i * 1024 + lane * 16;
      int s = byte / kSlotLds;
      const int o = byte - s * kSlotLds;
      s = s < NA ? s : NA - 1;                        // past the last slot (3-bit planes: 7.5 KiB): re-read, never parked
      s = a0 + s < kMaxSlots ? a0 + s : kMaxSlots - 1;
      code_at[i] = reinterpret_cast<uint64_t>(L.codes[s]) + (uint32_t)o + (uint64_t)jt * kSlotLds;
    }
  }

  __device__ __forceinline__ void sal_begin(int sp) {
    const int n_pairs = p.n_vis * n_sb;
    sal_left = n_pairs > sp ? (n_pairs - sp + nsplit - 1) / nsplit : 0;
    sal_v = 0;
    sal_sb = sp;
    while (sal_left > 0 && sal_sb >= n_sb) { sal_sb -= n_sb; ++sal_v; }
  }

  // A request is made in three steps spread over a chunk, because its addresses sit behind two dependent
  // look-ups (visit -> slot -> that expert's salient tile; both tables are in LDS) and a wavefront that issues
  // in order would otherwise sit out both:  look up the visit;  later look up the tile and move on to the next
  // pair;  later still form the addresses and issue the loads.
  __device__ __forceinline__ void sal_lookup() {
    nx_more = sal_left > 0;
    nx_info_v = vis_lds[nx_more ? sal_v : 0];
  }
  __device__ __forceinline__ void sal_address() {
    const int info = __builtin_amdgcn_readfirstlane(nx_info_v);
    nx_tt = nx_more ? info >> 8 : -1;
    nx_slot = info & 0xff;
    nx_sal_v = sal_lds[info & 0xff];
    nx_xoff = ((uint32_t)sal_v * (uint32_t)n_sb + (uint32_t)sal_sb) * 1024u;
    nx_doff = ((uint32_t)jt * (uint32_t)n_sb + (uint32_t)sal_sb) * 1024u;
    if (nx_more) {
      --sal_left;
      sal_sb += nsplit;
      while (sal_left > 0 && sal_sb >= n_sb) { sal_sb -= n_sb; ++sal_v; }
    }
  }
  // Always two loads, so that the number of loads in flight does not depend on the data: once the pairs are
  // used up both read the start of the activation stages and tt_out = -1.
  __device__ __forceinline__ void sal_issue(u32x4& x, u32x4& d, int& tt_out, int& slot_out) {
    tt_out = nx_tt;
    slot_out = nx_slot;
    const bool more = nx_tt >= 0;
    // the tile pointer was read from LDS a good while ago and is the same in every lane: into scalar registers with it
    const uint64_t tile = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(nx_sal_v >> 32)) << 32) |
                          (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)nx_sal_v);
    x = ld128(more ? xs + nx_xoff : xt, (uint32_t)lane * 16u);
    d = ld128(more ? reinterpret_cast<const char*>(tile) + nx_doff : xt, (uint32_t)lane * 16u);
  }

  // The pair's 16 x 16 product goes to the base accumulators of its token tile.  Its weights are D + z step (see the
  // top of the file), formed in fp32 from the fp16 values and the row's step and written as the sum of two bf16
  // numbers.  Which tile the product belongs to is known only at run time; rather than branch around the matrix
  // instructions (which makes the compiler keep two copies of every accumulator), the product is formed once and
  // added to the tile it belongs to through a select.
  __device__ __forceinline__ void sal_multiply(int i) {
    const f16x8 dh = __builtin_bit_cast(f16x8, sal_d[i]);
    const float zs = z * step_w[sal_slot[i] * 16 + (lane & 15)];
    u32x4 hi, lo;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float f0 = (float)dh[2 * q] + zs, f1 = (float)dh[2 * q + 1] + zs;
      const uint32_t h = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{f0, f1}, bf16x2));   // round to nearest even
      const float r0 = f0 - __uint_as_float(h << 16), r1 = f1 - __uint_as_float(h & 0xffff0000u);
      hi[q] = h;
      lo[q] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{r0, r1}, bf16x2));
    }
    f32x4 t = mfma_bf16(hi, sal_x[i], f32x4{0, 0, 0, 0});
    t = mfma_bf16(lo, sal_x[i], t);
    const int stt = sal_tt[i];
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      const bool mine = pt(tt) == stt;
#pragma unroll
      for (int v = 0; v < 4; ++v) acc_base[tt][v] += mine ? t[v] : 0.0f;
    }
  }

  template <int BUF>
  __device__ __forceinline__ void load_base(int c) {
    const char* src = base_at + (size_t)((uint32_t)c * base_stride);
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) base[BUF][kb] = ld128(src + kb * 1024, (uint32_t)lane * 16u);
  }

  template <int BUF>
  __device__ __forceinline__ void load_code_regs(int c) {
    const uint32_t off = (uint32_t)c * code_stride;
#pragma unroll
    for (int i = 0; i < NL; ++i) code[BUF][i] = ld128_at(code_at[i] + off);
  }

  // Register buffer BUF (the chunk that starts now) -> this wavefront's LDS area.
  template <int BUF>
  __device__ __forceinline__ void park() {
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      if (NL * 1024 == kParkWave || i * 1024 + lane * 16 < kParkWave)
        *reinterpret_cast<u32x4*>(parkp + i * 1024 + lane * 16) = code[BUF][i];
    }
  }

  // Tile tt's share of the requests of one chunk: code words of chunk c2 (two ahead) into the register buffer
  // that was just parked, base weights of chunk cn (one ahead) into the other base buffer.
  template <int BUF, bool NOBASE>
  __device__ __forceinline__ void request_share(int tt, int cn, int c2) {
    const uint32_t off = (uint32_t)c2 * code_stride;
#pragma unroll
    for (int i = 0; i < NL; ++i)
      if (i * TT / NL == tt) code[BUF][i] = ld128_at(code_at[i] + off);
    if constexpr (!NOBASE) {
      const char* src = base_at + (size_t)((uint32_t)cn * base_stride);
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
        if (kb * TT / 4 == tt) base[BUF ^ 1][kb] = ld128(src + kb * 1024, (uint32_t)lane * 16u);
    }
  }

  __device__ __forceinline__ CodeRegs<BITS> parked(int a) const {
    CodeRegs<BITS> r;
    load_codes<BITS>(parkp + a * kSlotLds, lane, r);
    return r;
  }

  // Loads of one chunk() call that are younger than its stage copy: all of its weight and scale requests.
  template <bool NOBASE> static constexpr int younger() { return NL + (NOBASE ? 0 : 4) + 2 * kSalPerChunk; }

  // One chunk out of base buffer BUF and stage `cur` (its per-token numbers: cur_x); the next chunks' data are
  // requested first.  NOBASE: a sweep after the first -- the base product is done, only the slots of this sweep are multiplied.
  template <int BUF, bool NOBASE>
  __device__ __forceinline__ void chunk(int cn, int c2, const char* cur, const char* cur_x, char* nxt, char* nxt_x, int wave) {
    stage_copy<NW>(xt + (size_t)cn * kStageBytes, nxt, nxt_x, wave, lane);
    sal_lookup();
    if constexpr (!NOBASE) rs_acc += *reinterpret_cast<const float*>(cur_x + 256 + lane * 4);   // this chunk's share of the tokens' sums
    // Order inside a tile: the low-bit visits first (operands bhi / blo, read from LDS during the previous
    // tile's base product), then the base product (operands xb, read while the visits ran).  Every LDS read is
    // thereby issued a good stretch of arithmetic before its data are needed.
    v8i bhi = lds_fp8(cur, pt(0), 0, lane), blo = lds_fp8(cur, pt(0), 1, lane);
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      // this tile's share of the next chunks' requests: spreading them over the chunk keeps the memory
      // pipeline fed without ever asking it to take a whole chunk's loads at once (which blocks the
      // wavefront, and with it the arithmetic it could be doing, until the pipeline has room)
      request_share<BUF, NOBASE>(tt, cn, c2);
      const int last = tlast[tt];
      int a = tfirst[tt];
      const int scale = *reinterpret_cast<const int*>(cur_x + 64 * pt(tt) + n * 4);   // the tokens' block scales for this chunk
      CodeRegs<BITS> cr = parked(a);
      u32x4 xb[4];
      if constexpr (!NOBASE) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) xb[kb] = lds128(cur, (kb * 4 + pt(tt)) * 1024 + lane * 16);
      }
      do {
        const int sc = slot_tok[tt] == (uint32_t)(a + a0) ? scale : 0;
        const u32x4 d = dequant_lo<BITS>(cr);
        u32x4 h;
        if constexpr (BITS >= 3) h = dequant_hi(cr);
        cr = parked(a < last ? a + 1 : a);   // the next visit's words, fetched while this one multiplies
        mfma_fp4_fp8_pair(acc_raw[tt], d, bhi, blo, sc);
        if constexpr (BITS >= 3) mfma_fp4_fp8_pair(acc_raw[tt], h, bhi, blo, sc, BITS == 4 ? 129 : 127);
      } while (++a <= last);
      if (tt + 1 < TT) { bhi = lds_fp8(cur, pt(tt + 1), 0, lane); blo = lds_fp8(cur, pt(tt + 1), 1, lane); }
      if constexpr (!NOBASE) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb) acc_base[tt] = mfma_bf16(base[BUF][kb], xb[kb], acc_base[tt]);
      }
      if (tt == 0) sal_address();
    }
    static_assert(kSalPerChunk == 1, "one pair per chunk: the request steps above prepare exactly one");
    sal_multiply(0);
    sal_issue(sal_x[0], sal_d[0], sal_tt[0], sal_slot[0]);
    // The next chunk's code words (requested during the previous chunk) go to this wavefront's LDS area now:
    // its visits of this chunk are over, the area is its own, and the wavefronts get here at slightly
    // different times -- the 64 KiB of LDS writes spread out and fill what would be waiting at the barrier.
    park<BUF ^ 1>();
    stage_barrier<younger<NOBASE>()>();
  }
};

// Active experts one sweep handles: their code words for one chunk are parked in LDS (8 wavefronts x slots x
// 256 b bytes next to the two activation stages must fit the 160 KiB of a compute unit).
constexpr int max_pass_slots(int bits) { return bits >= 3 ? 8 : 16; }

// LDS of a workgroup, carved up by hand, the two activation stages first: below 64 KiB their addresses fit the
// offset field of the LDS instructions, so one lane-offset register serves every operand read.
//   [0, 32 KiB) stage 0 | [32, 64 KiB) stage 1 | the stages' blocks of per-token numbers, 1 KiB each |
//   parked code words, one private area per wavefront |
//   per wavefront and slot the 16 steps | visit table | salient tile table | 256 bytes nobody reads
template <int BITS, int NA, int NW>
struct LdsPlan {
  static constexpr int kParkBytes = NW * NA * code_block_bytes(BITS);
  static constexpr int kLaunchSlots = NA == 4 ? 4 : kMaxSlots;   // experts of one group; NA of them per sweep
  static constexpr int kStepBytes = NW * kLaunchSlots * 16 * 4;
  static constexpr int kVisBytes = (kMaxVisits + 1 + 3) / 4 * 16;
  static constexpr int kStages = 2 * kStageLds + 2048;
  static constexpr int kSalBytes = 2 * kMaxSlots * 8;   // two tables: a gated pair's workgroup serves two layers
  static constexpr int kTotal = kStages + kParkBytes + kStepBytes + kVisBytes + kSalBytes + 256;
};

// One workgroup's work: row group rg, column split sp of token group p, with NA expert slots per sweep.
template <int BITS, int TT, int NA, int NW>
__device__ __forceinline__ void stream_rows(const LinearParams& p, char* lds, int rg, int sp) {
  const int tid = threadIdx.x, lane = tid & 63;
  // The wavefront index is the same in all 64 lanes; saying so keeps every value derived from it in scalar
  // registers and every branch on them a scalar branch.  MFMA ignores the EXEC mask, so an MFMA must never
  // sit in a region the compiler predicates with EXEC instead of branching around.
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 15, g = lane >> 4;
  constexpr int kHalf = NW / 2;             // gated pair: wavefront w < kHalf and wavefront w + kHalf own the same row tile
  const bool upper = p.pair && wave >= kHalf;
  const PerLinear& L = p.pair ? p.lin[upper ? 1 : 0] : p.lin[linear_of(p, rg)];
  int jt = p.pair ? rg * kHalf + (upper ? wave - kHalf : wave) : (rg - L.rg_begin) * NW + wave;
  const bool live = jt < L.n_jt && !(p.pair && wave >= 2 * kHalf);   // wavefronts past the last row tile recompute the last one and store nothing
  jt = jt < L.n_jt ? jt : L.n_jt - 1;
  const int c_begin = p.c_split[sp], c_end = p.c_split[sp + 1];

  using Plan = LdsPlan<BITS, NA, NW>;
  constexpr int kParkBytes = Plan::kParkBytes, kLaunchSlots = Plan::kLaunchSlots, kStepBytes = Plan::kStepBytes;
  constexpr int kVisBytes = Plan::kVisBytes, kStages = Plan::kStages;
  char* const stage0 = lds;
  char* const stage1 = lds + kStageLds;
  char* const extra0 = lds + 2 * kStageLds;
  char* const extra1 = lds + 2 * kStageLds + 1024;
  char* const park_all = lds + kStages;
  float (*step_lds)[kLaunchSlots][16] = reinterpret_cast<float (*)[kLaunchSlots][16]>(lds + kStages + kParkBytes);
  int* const vis_lds = reinterpret_cast<int*>(lds + kStages + kParkBytes + kStepBytes);
  uint64_t* const sal_lds = reinterpret_cast<uint64_t*>(lds + kStages + kParkBytes + kStepBytes + kVisBytes);
  char* const warm_lds = lds + kStages + kParkBytes + kStepBytes + kVisBytes + Plan::kSalBytes;

  using S = Stream<BITS, TT, NA, NW>;
  S ws(p, L, lane, jt, park_all + wave * (NA * code_block_bytes(BITS)), &step_lds[wave][0][0], vis_lds, sal_lds + (upper ? kMaxSlots : 0), wave >= 4);   // wavefronts w and w + 4 share a SIMD
  f32x4 (&acc_base)[TT] = ws.acc_base;
  f32x4 (&acc_raw)[TT] = ws.acc_raw;
  const uint32_t (&slot_tok)[TT] = ws.slot_tok;

  // The chunks of the range are visited from a start that differs from XCD to XCD (the sum does not care
  // about the order; workgroups go round-robin to the 8 XCDs, so rg & 7 names the XCD): the XCDs do not
  // march in lockstep through the same columns, while the workgroups that share one XCD's L2 read the same
  // activation stage at about the same time and fetch it from memory once.
  const int len = c_end - c_begin;
  const int rot = ((rg & 7) * len) >> 3;
  auto chunk_at = [&](int i) { i = i < len ? i : len - 1; int r = i + rot; r = r >= len ? r - len : r; return c_begin + r; };
  ws.begin_sweep(0);
  // Address translation warm-up.  The first loads of a workgroup go to as many pages as there are experts; one
  // 4-byte LDS-DMA load (no destination register to keep track of) touches the first two chunks' pages of every
  // slot at once, lanes 0 .. 15 those of the first chunk and lanes 16 .. 31 those of the second.
  {
    const int a = lane & 15;
    const uint64_t g = reinterpret_cast<uint64_t>(L.codes[a < p.n_act ? a : 0]) +
                       ((uint64_t)chunk_at((lane >> 4) & 1) * L.n_jt + jt) * code_block_bytes(BITS);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
                 : : "v"(g), "s"((uint32_t)(uintptr_t)warm_lds) : "memory", "m0");
  }
  // first chunks' weights and activations: requested now
  stage_copy<NW>(ws.xt + (size_t)chunk_at(0) * kStageBytes, stage0, extra0, wave, lane);
  ws.template load_base<0>(chunk_at(0));
  ws.template load_code_regs<0>(chunk_at(0));
  ws.template load_code_regs<1>(chunk_at(1));
  // Every slot's step for this wavefront's 16 output channels (for the salient weights and the epilogue) is fetched
  // now and kept in LDS: in registers it would be live across the whole stream.  Likewise the two tables of the
  // salient requests.
  const int st_a = lane >> 2, st_j = 16 * jt + 4 * (lane & 3);
  f32x4 st_v = {0, 0, 0, 0};
  if (st_a < kLaunchSlots && st_a < p.n_act && st_j < L.d_out) st_v = *reinterpret_cast<const f32x4*>(L.step[st_a] + st_j);
  int vis_v = 0;
  uint64_t sal_v = 0;
  if (tid <= kMaxVisits) vis_v = p.vis_info[tid];
  // (the salient tile table is per layer: wavefront 0 writes its layer's, and in a gated pair the first wavefront of
  // the upper half writes the other layer's behind it)
  const bool fills_sal = lane < kMaxSlots && (wave == 0 || (p.pair && wave == kHalf));
  if (fills_sal) sal_v = reinterpret_cast<uint64_t>(L.sal[lane]);
  ws.sal_begin(sp);
  if (st_a < kLaunchSlots) *reinterpret_cast<f32x4*>(&step_lds[wave][st_a][4 * (lane & 3)]) = st_v;
  if (tid <= kMaxVisits) vis_lds[tid] = vis_v;
  if (fills_sal) sal_lds[(wave == 0 ? 0 : kMaxSlots) + lane] = sal_v;

  ws.template park<0>();
  stage_barrier<0>();
  // Salient pairs beyond what the chunks of this workgroup can carry (short column ranges with many visits)
  // are multiplied here, one at a time; then the first chunk's pairs are requested.
  const int n_sweeps = p.n_act > NA ? (p.n_act + NA - 1) / NA : 1;
  while (ws.sal_left > S::kSalPerChunk * len * n_sweeps) {
    ws.sal_lookup();
    ws.sal_address();
    ws.sal_issue(ws.sal_x[0], ws.sal_d[0], ws.sal_tt[0], ws.sal_slot[0]);
    ws.sal_multiply(0);
  }
  ws.sal_lookup();
  ws.sal_address();
  ws.sal_issue(ws.sal_x[0], ws.sal_d[0], ws.sal_tt[0], ws.sal_slot[0]);
  for (int i = 0; i < len; i += 2) {
    ws.template chunk<0, false>(chunk_at(i + 1), chunk_at(i + 2), stage0, extra0, stage1, extra1, wave);
    if (i + 1 >= len) break;
    ws.template chunk<1, false>(chunk_at(i + 2), chunk_at(i + 3), stage1, extra1, stage0, extra0, wave);
  }
  // Further sweeps over the same chunks for the slots beyond the first NA: activations again (from L2), these
  // slots' code words, no base weights.  The last barrier of the sweep before has every wavefront done with
  // both stages.
  for (int sweep = 1; sweep < n_sweeps; ++sweep) {
    ws.begin_sweep(sweep * NA);
    stage_copy<NW>(ws.xt + (size_t)chunk_at(0) * kStageBytes, stage0, extra0, wave, lane);
    ws.template load_code_regs<0>(chunk_at(0));
    ws.template load_code_regs<1>(chunk_at(1));
    ws.template park<0>();
    stage_barrier<0>();
    for (int i = 0; i < len; i += 2) {
      ws.template chunk<0, true>(chunk_at(i + 1), chunk_at(i + 2), stage0, extra0, stage1, extra1, wave);
      if (i + 1 >= len) break;
      ws.template chunk<1, true>(chunk_at(i + 2), chunk_at(i + 3), stage1, extra1, stage0, extra0, wave);
    }
  }

  // epilogue: remove the zero point, apply the expert's step (the salient product is already in acc_base).
  // The last matrix instructions above were issued from an assembly block: give them the wait states a
  // matrix result needs before vector instructions may read it.
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
  f32x4 o[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) {
    f32x4 stepv = {0, 0, 0, 0};
    if (slot_tok[tt] != 0xffu) stepv = *reinterpret_cast<const f32x4*>(&step_lds[wave][slot_tok[tt]][4 * g]);
    // zero point: z times the token's sum over this workgroup's columns (lane = token in rs_acc)
    const float corr = p.z * __shfl(ws.rs_acc, 16 * ws.pt(tt) + n);
#pragma unroll
    for (int v = 0; v < 4; ++v)
      o[tt][v] = acc_base[tt][v] + stepv[v] * (acc_raw[tt][v] - corr);
  }

  if (p.nsplit > 1) {
    // Split columns: the partial tile goes to the workspace in this kernel's own thread order (fully
    // coalesced); the reduction launch adds the tiles of a row group in split order.
    constexpr int NT = 64 * NW;
    f32x4* part = p.partial + ((size_t)rg * p.nsplit + sp) * (4 * NT);
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) part[ws.pt(tt) * NT + tid] = o[tt];
  } else {
    if (p.pair) {
      // The up projection's tiles cross over to the wavefronts that hold the gate's through LDS.  The activation
      // stages are free: the loop's last barrier had every wavefront done with them.
      f32x4* xch = reinterpret_cast<f32x4*>(lds);
      if (upper && wave < 2 * kHalf) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) xch[((wave - kHalf) * 4 + ws.pt(tt)) * 64 + lane] = o[tt];
      }
      __syncthreads();
      if (!upper) {
#pragma unroll
        for (int tt = 0; tt < TT; ++tt) o[tt] = gated(o[tt], xch[(wave * 4 + ws.pt(tt)) * 64 + lane]);
      }
    }
    if (live && !upper) {
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        const int t = p.t0 + 16 * ws.pt(tt) + n, j = 16 * jt + 4 * g;
        if (t < p.T && j < L.d_out) {
          uint2 pk;
          pk.x = f32_to_bf16(o[tt][0]) | (f32_to_bf16(o[tt][1]) << 16);
          pk.y = f32_to_bf16(o[tt][2]) | (f32_to_bf16(o[tt][3]) << 16);
          *reinterpret_cast<uint2*>(L.y + (size_t)t * L.d_out + j) = pk;
        }
      }
    }
  }
}

// The kernel: finds its (row group, column split, token group) and runs it with as few expert slots per sweep as
// the group needs -- a group whose tokens belong to four experts or fewer (most groups of a batch that is sorted by
// expert) moves a quarter of the code words of a full one through registers and LDS.
// CLASSES: 0 = every group of the launch is such a short one, 1 = none is, 2 = both kinds (the workgroup looks).
template <int BITS, int TT, int NW, int CLASSES>
__global__ __launch_bounds__(64 * NW) void k_delta_linear(const LaunchParams mp) {
  constexpr int NA = max_pass_slots(BITS);
  __shared__ __attribute__((aligned(16))) char lds[LdsPlan<BITS, CLASSES == 0 ? 4 : NA, NW>::kTotal];
  // flat workgroup id -> (class, split, row group, token group), see LaunchParams; ids go round-robin to the XCDs
  const int first_wgs = mp.n_first * mp.wg_per_group;
  const bool second = (int)blockIdx.x >= first_wgs;
  const int b = second ? blockIdx.x - first_wgs : blockIdx.x, m = second ? mp.n_groups - mp.n_first : mp.n_first;
  const int bq = b >> 3, bq2 = bq / m;
  const int rg = (bq2 % mp.rg8) * 8 + (b & 7), sp = bq2 / mp.rg8;
  if (rg >= mp.rgs) return;   // padding of the row groups to a multiple of eight
  const LinearParams& p = mp.g[(second ? mp.n_first : 0) + bq - bq2 * m];
  if constexpr (CLASSES == 0) stream_rows<BITS, TT, 4, NW>(p, lds, rg, sp);
  else if constexpr (CLASSES == 1) stream_rows<BITS, TT, NA, NW>(p, lds, rg, sp);
  else if (p.n_act <= 4) stream_rows<BITS, TT, 4, NW>(p, lds, rg, sp);
  else stream_rows<BITS, TT, NA, NW>(p, lds, rg, sp);
}

// Split columns only: y = sum over splits (in split order) of the fp32 partial tiles, rounded to bf16.  One
// workgroup per (row group, token tile), threads laid out as in the main kernel.
template <int NW>
__global__ __launch_bounds__(64 * NW) void k_reduce_splits(const LaunchParams mp) {
  const LinearParams& p = mp.g[blockIdx.z];
  constexpr int NT = 64 * NW;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 15, g = lane >> 4;
  const int rg = blockIdx.x, tt = blockIdx.y;
  const f32x4* part = p.partial + (size_t)rg * p.nsplit * (4 * NT) + tt * NT + tid;
  f32x4 o = {0, 0, 0, 0};
  for (int s = 0; s < p.nsplit; ++s) o += part[(size_t)s * (4 * NT)];
  constexpr int kHalf = NW / 2;
  const bool upper = p.pair && wave >= kHalf;
  if (p.pair) {   // gated pair: the up projection's sums cross over to the threads that hold the gate's
    __shared__ f32x4 xch[kHalf * 64];
    if (upper && wave < 2 * kHalf) xch[(wave - kHalf) * 64 + lane] = o;
    __syncthreads();
    if (!upper) o = gated(o, xch[wave * 64 + lane]);
  }
  const PerLinear& L = p.pair ? p.lin[0] : p.lin[linear_of(p, rg)];
  const int jt = p.pair ? rg * kHalf + wave : (rg - L.rg_begin) * NW + wave;
  const int t = p.t0 + 16 * tt + n, j = 16 * jt + 4 * g;
  if (!upper && jt < L.n_jt && t < p.T && j < L.d_out) {
    uint2 pk;
    pk.x = f32_to_bf16(o[0]) | (f32_to_bf16(o[1]) << 16);
    pk.y = f32_to_bf16(o[2]) | (f32_to_bf16(o[3]) << 16);
    *reinterpret_cast<uint2*>(L.y + (size_t)t * L.d_out + j) = pk;
  }
}

// Wavefronts per workgroup (each owns 16 output channels): 8 fill a compute unit's four SIMDs two deep; 7 or 6
// are chosen when that makes the number of workgroups fit the 256 compute units better.
constexpr int kMaxWaves = 8;

struct Plan {
  int nsplit;  // workgroups that share one row group's columns
  int nw;      // wavefronts (row tiles) per workgroup
};

inline int row_groups_of(int d_out, int nw) { return (ceil_to(d_out, kRowPad) / 16 + nw - 1) / nw; }

// Row groups of a launch.  A gated pair's workgroups hold nw / 2 row tiles of each of the two layers.
inline int row_groups_total(const int* d_out, int n_linears, int nw, bool pair) {
  if (pair) return row_groups_of(d_out[0], nw / 2);
  int rgs = 0;
  for (int l = 0; l < n_linears; ++l) rgs += row_groups_of(d_out[l], nw);
  return rgs;
}

// Pure function of the shapes (not of bits or T), so the workspace size is known up front.
// One workgroup runs per compute unit (256 of them).  The chunks are split over `nsplit` workgroups so that
// the grid fills the largest part of the last round of 256, with at least four chunks per workgroup and,
// among equals, few splits (every split writes and re-reads a partial output tile).
Plan plan_for(int d_in, const int* d_out, int n_linears, bool pair) {
  const int n_chunks = ceil_to(d_in, kColPad) / kChunk;
  Plan best{1, kMaxWaves};
  double best_cost = 1e30;
  for (int nw = kMaxWaves; nw >= 6; --nw) {
    if (pair && nw % 2) continue;   // a gated pair splits the wavefronts evenly between its two layers
    const int rgs = row_groups_total(d_out, n_linears, nw, pair);
    for (int ns = 1; ns <= kMaxSplits && (ns == 1 || ns * 4 <= n_chunks); ++ns) {
      const long wgs = (long)rgs * ns;
      const long rounds = (wgs + 255) / 256;
      const int chunks_wg = (n_chunks + ns - 1) / ns;
      // time ~ rounds x (chunks per workgroup, each a little shorter with fewer wavefronts, + a fixed start and
      // finish cost of about three chunks) + the partial tiles
      const double cost = (double)rounds * (chunks_wg * (nw + 2) / 10.0 + 3.0) + (ns > 1 ? 0.25 * ns : 0.0);
      if (cost < best_cost - 1e-9) { best_cost = cost; best = Plan{ns, nw}; }
    }
  }
  return best;
}

// The workspace of one token group; a launch of n groups uses n of these, one after the other.
struct WorkspaceLayout {
  size_t xt, per_linear[kMaxLinears], partial, total;   // per linear: xs; total is a multiple of 256
  size_t xs_bytes;
};

WorkspaceLayout workspace_layout(int d_in, const int* d_out, int n_linears, bool pair) {
  const Plan pl = plan_for(d_in, d_out, n_linears, pair);
  const int rgs = row_groups_total(d_out, n_linears, pl.nw, pair);
  const int pi = ceil_to(d_in, kColPad);
  WorkspaceLayout w;
  size_t off = 0;
  w.xt = off;      off += (size_t)(pi / kChunk) * kStageBytes;
  w.xs_bytes = (size_t)kMaxVisits * (ceil_to(d_in, kSalPad) / 32) * 1024;   // k <= d_in
  for (int l = 0; l < kMaxLinears; ++l) {
    w.per_linear[l] = off;
    if (l < n_linears) off += w.xs_bytes;
  }
  w.partial = off; off += pl.nsplit > 1 ? (size_t)rgs * pl.nsplit * 4 * (64 * pl.nw) * 16 : 0;
  w.total = (off + 255) / 256 * 256;
  return w;
}

// Token groups a workspace sized for `max_tokens` holds.
inline int groups_for(int max_tokens) { return max_tokens <= kTokGroup ? 1 : max_tokens <= 2 * kTokGroup ? 2 : kMaxGroups; }

template <int BITS, int NW>
hipError_t launch_tt(const LaunchParams& mp, int tt, int classes, int grid, hipStream_t s) {
  if (classes == 2) {   // both kinds of groups: built for four token tiles only (fewer tiles are a special case of it)
    k_delta_linear<BITS, 4, NW, 2><<<grid, 64 * NW, 0, s>>>(mp);
    return hipGetLastError();
  }
  switch (tt * 2 + classes) {
    case 2: k_delta_linear<BITS, 1, NW, 0><<<grid, 64 * NW, 0, s>>>(mp); break;
    case 3: k_delta_linear<BITS, 1, NW, 1><<<grid, 64 * NW, 0, s>>>(mp); break;
    case 4: k_delta_linear<BITS, 2, NW, 0><<<grid, 64 * NW, 0, s>>>(mp); break;
    case 5: k_delta_linear<BITS, 2, NW, 1><<<grid, 64 * NW, 0, s>>>(mp); break;
    case 8: k_delta_linear<BITS, 4, NW, 0><<<grid, 64 * NW, 0, s>>>(mp); break;
    default: k_delta_linear<BITS, 4, NW, 1><<<grid, 64 * NW, 0, s>>>(mp); break;
  }
  return hipGetLastError();
}

template <int BITS>
hipError_t launch_nw(const LaunchParams& mp, int tt, int classes, int nw, int grid, hipStream_t s) {
  switch (nw) {
    case 6: return launch_tt<BITS, 6>(mp, tt, classes, grid, s);
    case 7: return launch_tt<BITS, 7>(mp, tt, classes, grid, s);
    default: return launch_tt<BITS, 8>(mp, tt, classes, grid, s);
  }
}

hipError_t launch_reduce(const LaunchParams& mp, int tt, int nw, hipStream_t s) {
  const dim3 grid(mp.rgs, tt, mp.n_groups);
  switch (nw) {
    case 6: k_reduce_splits<6><<<grid, 64 * 6, 0, s>>>(mp); break;
    case 7: k_reduce_splits<7><<<grid, 64 * 7, 0, s>>>(mp); break;
    default: k_reduce_splits<8><<<grid, 64 * 8, 0, s>>>(mp); break;
  }
  return hipGetLastError();
}

}  // namespace


// Expert segments at least this long take the one-product path of mes_prefill.hip (W + Delta~ formed in registers,
// one dense contraction) when the workspace has room for it: from here on it is cheaper than streaming the weights
// once per 64 tokens.
constexpr int kPrefillMin = 192;
int long_segment_tokens() { return kPrefillMin; }

size_t gated_workspace_bytes(int d_in, int d_out, int max_tokens) {
  const int d[2] = {d_out, d_out};
  return groups_for(max_tokens) * workspace_layout(d_in, d, 2, true).total;   // the gated pair always streams
}

size_t linear_workspace_bytes(int d_in, const int* d_out, int n_linears, int max_tokens) {
  const size_t per_group = workspace_layout(d_in, d_out, n_linears, false).total;
  // the one-product scratch always sits behind kMaxGroups groups' worth (a workspace that has it was sized for
  // at least kPrefillMin tokens, i.e. for all the groups)
  if (max_tokens >= kPrefillMin) return kMaxGroups * per_group + prefill_scratch_bytes(d_in, max_tokens);
  return groups_for(max_tokens) * per_group;
}

hipError_t launch_delta_linear(const LinearCall& c, hipStream_t s) {
  const mes_delta& d0 = c.lin[0].experts[0];
  int d_outs[kMaxLinears];
  for (int l = 0; l < c.n_linears; ++l) d_outs[l] = c.lin[l].experts[0].d_out;
  const bool pair = c.gated != 0;   // lin[0] = gate, lin[1] = up, one output SiLU(gate) * up at lin[0].y
  const WorkspaceLayout wl = workspace_layout(d0.d_in, d_outs, c.n_linears, pair);
  char* ws = reinterpret_cast<char*>(c.ws);
  // token groups one launch may hold: as many as the workspace has room for
  const int max_groups = (int)(c.ws_bytes / wl.total < (size_t)kMaxGroups ? c.ws_bytes / wl.total : (size_t)kMaxGroups);
  // what all groups of all launches have in common
  LinearParams p0;
  p0.x = reinterpret_cast<const uint16_t*>(c.x);
  const int pi = ceil_to(d0.d_in, kColPad);
  p0.d_in = d0.d_in;
  p0.n_linears = c.n_linears;
  p0.n_chunks = pi / kChunk;
  p0.n_sb = ceil_to(d0.k, kSalPad) / 32;
  p0.k = d0.k;
  p0.bits = d0.bits;
  p0.z = d0.grid == MES_GRID_SYM ? (float)(1 << (d0.bits - 1)) - 0.5f : (float)(1 << (d0.bits - 1));
  p0.pair = pair ? 1 : 0;
  const Plan pl = plan_for(d0.d_in, d_outs, c.n_linears, pair);
  int rgs = 0;
  for (int l = 0; l < kMaxLinears; ++l) {
    PerLinear& L = p0.lin[l];
    const int ll = l < c.n_linears ? l : 0;   // unused entries repeat the first (never selected)
    L.w_base = reinterpret_cast<const char*>(c.lin[ll].w_base_tiled);
    L.y = reinterpret_cast<uint16_t*>(c.lin[ll].y);
    L.d_out = d_outs[ll];
    L.n_jt = ceil_to(d_outs[ll], kRowPad) / 16;
    L.rg_begin = rgs;
    if (l < c.n_linears) rgs += row_groups_of(d_outs[l], pl.nw);
    L.rg_end = rgs;
  }
  if (pair) rgs = row_groups_total(d_outs, 2, pl.nw, true);
  p0.nsplit = pl.nsplit;
  for (int sp = 0; sp <= pl.nsplit; ++sp) p0.c_split[sp] = (int16_t)((long)sp * p0.n_chunks / pl.nsplit);
  LaunchParams mp;
  mp.rgs = rgs;
  mp.rg8 = (rgs + 7) / 8;
  // Token groups: up to 64 consecutive tokens that belong to at most kMaxSlots experts (the kernel sweeps the
  // chunks once per max_pass_slots of them).
  const int max_slots = kMaxSlots;
  bool first_kernel = true;   // measurement hook: the start event goes before the first streaming kernel / GEMM
  // The streaming (decode) path.  Token groups are collected from all the token ranges it covers (the stretches
  // between long segments) and launched kMaxGroups at a time.
  int ng = 0, tt_max = 1, items_max = 0;
  auto flush = [&]() -> hipError_t {
    if (ng == 0) return hipSuccess;
    // the groups with more experts than the short variant of the kernel holds go first (stable otherwise)
    int n_first = 0;
    for (int g = 0; g < ng; ++g)
      if (mp.g[g].n_act > 4) {
        const LinearParams heavy = mp.g[g];
        for (int h = g; h > n_first; --h) mp.g[h] = mp.g[h - 1];
        mp.g[n_first++] = heavy;
      }
    for (int g = ng; g < kMaxGroups; ++g) mp.g[g] = mp.g[0];   // never selected
    mp.n_groups = ng;
    const int classes = n_first == 0 ? 0 : n_first == ng ? 1 : 2;
    mp.n_first = n_first > 0 ? n_first : ng;
    mp.wg_per_group = mp.rg8 * 8 * pl.nsplit;
    k_prepare<<<dim3(items_max, ng), 256, 0, s>>>(mp);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (c.ev_start && first_kernel && (e = hipEventRecord(c.ev_start, s)) != hipSuccess) return e;
    first_kernel = false;
    const int grid = mp.rg8 * 8 * pl.nsplit * ng;
    switch (d0.bits) {
      case 1: e = launch_nw<1>(mp, tt_max, classes, pl.nw, grid, s); break;
      case 2: e = launch_nw<2>(mp, tt_max, classes, pl.nw, grid, s); break;
      case 4: e = launch_nw<4>(mp, tt_max, classes, pl.nw, grid, s); break;
      default: e = launch_nw<3>(mp, tt_max, classes, pl.nw, grid, s); break;
    }
    if (e != hipSuccess) return e;
    if (c.ev_stop && (e = hipEventRecord(c.ev_stop, s)) != hipSuccess) return e;   // re-recorded by every later one
    if (pl.nsplit > 1) {
      if ((e = launch_reduce(mp, tt_max, pl.nw, s)) != hipSuccess) return e;
    }
    ng = 0; tt_max = 1; items_max = 0;
    return hipSuccess;
  };
  auto run_range = [&](int t_lo, int t_hi) -> hipError_t {
    int e_cur = 0;   // first expert that may own token t0
    for (int t0 = t_lo; t0 < t_hi;) {
      {
        LinearParams& p = mp.g[ng];
        p = p0;
        char* wsg = ws + (size_t)ng * wl.total;
        p.xt = wsg + wl.xt;
        p.partial = reinterpret_cast<f32x4*>(wsg + wl.partial);
        for (int l = 0; l < kMaxLinears; ++l) p.lin[l].xs = reinterpret_cast<u32x4*>(wsg + wl.per_linear[l < c.n_linears ? l : 0]);
        while (c.seg[e_cur + 1] <= t0) ++e_cur;
        int nt = t_hi - t0 < kTokGroup ? t_hi - t0 : kTokGroup;
        {   // cut the group where one expert too many would start
          int act = 0;
          for (int e = e_cur; e < c.n_experts && c.seg[e] < t0 + nt; ++e) {
            if (c.seg[e + 1] <= c.seg[e]) continue;
            if (++act > max_slots) { nt = c.seg[e] - t0; break; }
          }
        }
        p.t0 = t0;
        const int tt = nt <= 16 ? 1 : nt <= 32 ? 2 : 4;
        // active slots: the experts that own tokens of this group, in expert order
        int na = 0;
        for (int tl = 0; tl < kTokGroup; ++tl) p.tok_slot[tl] = 0xff;
        for (int e = e_cur; e < c.n_experts && c.seg[e] < t0 + nt; ++e) {
          const int lo = (c.seg[e] > t0 ? c.seg[e] : t0) - t0;
          const int hi = (c.seg[e + 1] < t0 + nt ? c.seg[e + 1] : t0 + nt) - t0;
          if (hi <= lo) continue;
          for (int l = 0; l < kMaxLinears; ++l) {
            const mes_delta& d = c.lin[l < c.n_linears ? l : 0].experts[e];
            p.lin[l].codes[na] = reinterpret_cast<const char*>(d.codes);
            p.lin[l].step[na] = d.step;
            p.lin[l].sal[na] = reinterpret_cast<const char*>(d.salient);
            p.lin[l].sidx[na] = d.salient_idx;
          }
          p.lo[na] = (int16_t)lo;
          p.hi[na] = (int16_t)hi;
          for (int tl = lo; tl < hi; ++tl) p.tok_slot[tl] = (uint8_t)na;
          ++na;
        }
        for (int a = na; a < kMaxSlots; ++a) {   // unused slots alias slot 0 so that unconditional loads stay valid
          for (int l = 0; l < kMaxLinears; ++l) {
            PerLinear& L = p.lin[l];
            L.codes[a] = L.codes[0]; L.step[a] = L.step[0]; L.sal[a] = L.sal[0]; L.sidx[a] = L.sidx[0];
          }
          p.lo[a] = 0; p.hi[a] = 0;
        }
        // visits, tile-major: for every 16-token tile the slots that own tokens in it
        int nv = 0;
        for (int t = 0; t < 4; ++t)
          for (int a = 0; a < na; ++a) {
            const int l = p.lo[a] > 16 * t ? p.lo[a] : 16 * t;
            const int h = p.hi[a] < 16 * t + 16 ? p.hi[a] : 16 * t + 16;
            if (h <= l) continue;
            p.vis_info[nv] = a | (t << 8);
            ++nv;
          }
        for (int v = nv; v <= kMaxVisits; ++v) p.vis_info[v] = 0;
        for (int t = 0; t < 4; ++t) {
          p.tile_first[t] = 0; p.tile_last[t] = 0;
          const int tl0 = 16 * t, tl1 = 16 * t + 15 < nt - 1 ? 16 * t + 15 : nt - 1;
          if (tl0 < nt) { p.tile_first[t] = p.tok_slot[tl0]; p.tile_last[t] = p.tok_slot[tl1]; }
        }
        p.n_act = na;
        p.n_vis = d0.k > 0 ? nv : 0;
        p.T = t0 + nt;   // rows past the group are not this group's: the kernels treat them as padding
        p.tiles = (nt + 15) / 16;
        p.n_stage_items = p.tiles * p.n_chunks;
        p.n_items = p.n_stage_items + c.n_linears * p.n_vis;
        tt_max = tt > tt_max ? tt : tt_max;
        items_max = p.n_items > items_max ? p.n_items : items_max;
        t0 += nt;
      }
      ++ng;
      if (ng == max_groups) {
        hipError_t e = flush();
        if (e != hipSuccess) return e;
      }
    }
    return hipSuccess;
  };   // run_range

  // Long expert segments go to the one-product path, everything between them to the streaming path.
  // (their activations are re-tiled into the scratch together: it must hold all the long segments' tokens)
  int long_tokens = 0;
  for (int e = 0; e < c.n_experts; ++e)
    if (c.seg[e + 1] - c.seg[e] >= kPrefillMin) long_tokens += c.seg[e + 1] - c.seg[e];
  const size_t scratch_at = kMaxGroups * wl.total;
  // (a gated pair always streams: the one-product path has no gated epilogue)
  const bool can_prefill = !pair && long_tokens > 0 && c.ws_bytes >= scratch_at + prefill_scratch_bytes(d0.d_in, long_tokens);
  // the long segments of every linear in one go (up to 8 experts per launch), then the streaming ranges between them
  int cursor = 0;
  if (can_prefill) {
    int long_experts[MES_MAX_EXPERTS], n_long = 0;
    for (int e = 0; e < c.n_experts; ++e)
      if (c.seg[e + 1] - c.seg[e] >= kPrefillMin) long_experts[n_long++] = e;
    hipError_t perr = launch_prefill_segments(c.lin, c.n_linears, long_experts, n_long, c.seg, c.x, ws + scratch_at,
                                              c.ev_start, c.ev_stop, &first_kernel, s);
    if (perr != hipSuccess) return perr;
    for (int i = 0; i < n_long; ++i) {
      const int e = long_experts[i];
      hipError_t err = run_range(cursor, c.seg[e]);
      if (err != hipSuccess) return err;
      cursor = c.seg[e + 1];
    }
  }
  if (hipError_t err = run_range(cursor, c.T)) return err;
  return flush();
}

}  // namespace mes
