// Offline kernels: re-tiling of the base weight, compression of one expert's delta
// (Eq. 1 per output channel, fp16 salient columns -- Section 4.1), its inverse for tests,
// and the salient-channel selection of Eq. 2.  None of these is on the serving path;
// they are written for clarity and exact (fp64) arithmetic, not for speed.
#include "mes_internal.h"

#include <hip/hip_fp16.h>

namespace mes {
namespace {

__device__ __forceinline__ bool is_salient(const int32_t* sidx, int k, int col, int* pos) {
  int lo = 0, hi = k;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    int v = sidx[mid];
    if (v < col) lo = mid + 1; else hi = mid;
  }
  if (lo < k && sidx[lo] == col) { if (pos) *pos = lo; return true; }
  return false;
}

__device__ __forceinline__ double zero_point(int bits, int grid) {
  return grid == MES_GRID_SYM ? (double)(1 << (bits - 1)) - 0.5 : (double)(1 << (bits - 1));
}

// Eq. 1 with an unsigned code: SYM takes the cell index floor(t), EQ1 rounds half to even.
__device__ __forceinline__ uint32_t quant_code(float w, float step, int bits, int grid) {
  const int half = 1 << (bits - 1);
  if (!(step > 0.0f)) return (uint32_t)half;
  double t = (double)w / (double)step;
  double u;
  if (grid == MES_GRID_SYM) {
    u = floor(t) + (double)half;
    u = fmin(fmax(u, 0.0), (double)(2 * half - 1));
  } else {
    u = fmin(fmax(rint(t), (double)-half), (double)(half - 1)) + (double)half;
  }
  return (uint32_t)(int)u;
}

// ---- base weight tiling --------------------------------------------------------------------------

__global__ void k_pack_base(const uint16_t* __restrict__ w, int d_in, int d_out, int n_kb, size_t n_slots,
                            uint4* __restrict__ out) {
  size_t slot = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (slot >= n_slots) return;
  // slot = ((c * n_jt + jt) * 4 + kb) * 64 + lane: chunk-major
  int lane = (int)(slot & 63);
  size_t blk = slot >> 6;
  int kb = (int)(blk & 3);
  blk >>= 2;
  const int n_jt = (d_out + 63) / 64 * 4;
  int jt = (int)(blk % n_jt);
  int c = (int)(blk / n_jt);
  int row = 16 * jt + (lane & 15);
  int col = 128 * c + 32 * kb + 8 * (lane >> 4);
  uint4 v = make_uint4(0, 0, 0, 0);
  if (row < d_out && col < d_in) v = *reinterpret_cast<const uint4*>(w + (size_t)row * d_in + col);
  out[slot] = v;
}

__global__ void k_unpack_base(const uint4* __restrict__ t, int d_in, int d_out, int n_kb, size_t n_slots,
                              uint16_t* __restrict__ w) {
  size_t slot = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (slot >= n_slots) return;
  int lane = (int)(slot & 63);
  size_t blk = slot >> 6;
  int kb = (int)(blk & 3);
  blk >>= 2;
  const int n_jt = (d_out + 63) / 64 * 4;
  int jt = (int)(blk % n_jt);
  int c = (int)(blk / n_jt);
  int row = 16 * jt + (lane & 15);
  int col = 128 * c + 32 * kb + 8 * (lane >> 4);
  if (row < d_out && col < d_in) *reinterpret_cast<uint4*>(w + (size_t)row * d_in + col) = t[slot];
}

// ---- delta compression -----------------------------------------------------------------------------

__global__ void k_check_salient(const int32_t* __restrict__ sidx, int k, int d_in, int* flag) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= k) return;
  int v = sidx[i];
  bool bad = v < 0 || v >= d_in || (i > 0 && sidx[i - 1] >= v);
  if (bad) atomicOr(flag, 1);
}

// One block per output channel.  MAXABS: exact max over the non-salient columns, then one fp64
// division.  MEANABS: ascending sequential fp64 sum (thread 0), so the order is defined.
__global__ void k_row_step(const float* __restrict__ delta, int d_in, const int32_t* __restrict__ sidx, int k,
                           int bits, int grid, int policy, const float* __restrict__ step_in,
                           float* __restrict__ step_out) {
  const int row = blockIdx.x;
  const float* r = delta + (size_t)row * d_in;
  if (policy == MES_STEP_GIVEN) {
    if (threadIdx.x == 0) { float s = step_in[row]; step_out[row] = s > 0.0f ? s : 0.0f; }
    return;
  }
  if (policy == MES_STEP_MEANABS) {
    if (threadIdx.x == 0) {
      double tot = 0.0; int cnt = 0;
      for (int c = 0; c < d_in; ++c)
        if (!is_salient(sidx, k, c, nullptr)) { tot += (double)fabsf(r[c]); ++cnt; }
      step_out[row] = cnt ? (float)(2.0 * (tot / (double)cnt)) : 0.0f;
    }
    return;
  }
  __shared__ float red[256];
  float m = 0.0f;
  for (int c = threadIdx.x; c < d_in; c += blockDim.x)
    if (!is_salient(sidx, k, c, nullptr)) m = fmaxf(m, fabsf(r[c]));
  red[threadIdx.x] = m;
  __syncthreads();
  for (int s = blockDim.x / 2; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    double div = grid == MES_GRID_SYM ? (double)(1 << (bits - 1)) - 0.5 : (double)(1 << (bits - 1)) - 1.0;
    step_out[row] = (float)((double)red[0] / div);
  }
}

// Where the code of (row, col) is stored (see mes.h, "codes").  Blocks of 16 rows x 128 columns, chunk-major;
// inside a block lane = 16 g + r owns the 32 columns 32 g + e, e = 8 q + pp.
struct CodeLoc {
  size_t lo_word;   // index of the 32-bit word holding the low bits (all bits for b = 1, 2)
  int lo_shift;
  size_t hi_word;   // b = 3: word holding the high bit; b = 4: word holding the high two bits
  int hi_shift;
};

__device__ __forceinline__ CodeLoc code_location(int bits, int n_jt, int row, int col) {
  const int jt = row >> 4, r = row & 15;
  const int c = col >> 7, g = (col >> 5) & 3, e = col & 31, q = e >> 3, pp = e & 7;
  const int lane = 16 * g + r;
  const size_t blk = ((size_t)c * n_jt + jt) * (64 * bits);
  CodeLoc L;
  if (bits == 1) {
    L.lo_word = blk + lane;
    L.lo_shift = 4 * pp + q;
    L.hi_word = 0; L.hi_shift = 0;
  } else {
    L.lo_word = blk + lane * 2 + (q >> 1);
    L.lo_shift = 4 * pp + 2 * (q & 1);
    if (bits == 4) {   // a second 2-bit block
      L.hi_word = blk + 128 + lane * 2 + (q >> 1);
      L.hi_shift = 4 * pp + 2 * (q & 1);
    } else {
      L.hi_word = blk + 128 + lane;
      L.hi_shift = 4 * pp + q;
    }
  }
  return L;
}

// One thread per (row, 8 consecutive columns): quantise and OR the codes into their words (the buffer was
// zeroed before; words are shared by threads, hence atomicOr).
__global__ void k_pack_codes(const float* __restrict__ delta, int d_in, int d_out, const int32_t* __restrict__ sidx,
                             int k, int bits, int grid, const float* __restrict__ step, int n_jt,
                             uint32_t* __restrict__ out) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int groups = d_in / 8;
  if (idx >= (size_t)d_out * groups) return;
  const int row = (int)(idx / groups), col0 = (int)(idx % groups) * 8;
  const float s = step[row];
  const float* r = delta + (size_t)row * d_in;
  uint32_t lo_bits = 0, hi_bits = 0;
  const CodeLoc L0 = code_location(bits, n_jt, row, col0);   // the 8 columns share both words
  for (int pp = 0; pp < 8; ++pp) {
    const int col = col0 + pp;
    if (is_salient(sidx, k, col, nullptr)) continue;
    const uint32_t u = quant_code(r[col], s, bits, grid);
    const CodeLoc L = code_location(bits, n_jt, row, col);
    lo_bits |= (bits >= 3 ? (u & 3u) : u) << L.lo_shift;
    if (bits >= 3) hi_bits |= (u >> 2) << L.hi_shift;
  }
  if (lo_bits) atomicOr(out + L0.lo_word, lo_bits);
  if (bits >= 3 && hi_bits) atomicOr(out + L0.hi_word, hi_bits);
}

// `flag` was written by k_check_salient earlier on the same stream: with indices that failed the check
// nothing is gathered (an index is never used as an address unless the whole list is valid).
__global__ void k_pack_salient(const float* __restrict__ delta, int d_in, int d_out, const int32_t* __restrict__ sidx,
                               int k, int n_sb, size_t n_elems, const int* __restrict__ flag,
                               uint16_t* __restrict__ out) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_elems) return;
  if (*flag) { out[idx] = 0; return; }
  int e = (int)(idx & 7);
  int lane = (int)((idx >> 3) & 63);
  size_t blk = idx >> 9;
  int sb = (int)(blk % n_sb);
  int jt = (int)(blk / n_sb);
  int row = 16 * jt + (lane & 15);
  int rc = 32 * sb + 8 * (lane >> 4) + e;
  uint16_t v = 0;
  if (row < d_out && rc < k) {
    const int col = min(max(sidx[rc], 0), d_in - 1);
    __half h = __float2half_rn(delta[(size_t)row * d_in + col]);
    v = __half_as_ushort(h);
  }
  out[idx] = v;
}

__device__ __forceinline__ uint32_t load_code(const uint32_t* codes, int bits, int n_jt, int row, int col) {
  const CodeLoc L = code_location(bits, n_jt, row, col);
  if (bits == 1) return (codes[L.lo_word] >> L.lo_shift) & 1u;
  const uint32_t lo = (codes[L.lo_word] >> L.lo_shift) & 3u;
  if (bits == 2) return lo;
  return lo | (((codes[L.hi_word] >> L.hi_shift) & (bits == 4 ? 3u : 1u)) << 2);
}

__global__ void k_unpack_delta(const uint32_t* __restrict__ codes, const float* __restrict__ step,
                               const uint16_t* __restrict__ sal, const int32_t* __restrict__ sidx, int d_in,
                               int d_out, int k, int bits, int grid, int n_ks, int n_sb,
                               float* __restrict__ delta_hat, uint8_t* __restrict__ codes_out) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)d_in * d_out) return;
  int row = (int)(idx / d_in), col = (int)(idx % d_in);
  int pos = 0;
  if (is_salient(sidx, k, col, &pos)) {
    int jt = row >> 4, r = row & 15, sb = pos >> 5, g = (pos >> 3) & 3, e = pos & 7;
    uint16_t hb = sal[(((size_t)(jt * n_sb + sb) * 64) + 16 * g + r) * 8 + e];
    if (delta_hat) delta_hat[idx] = __half2float(__ushort_as_half(hb));
    if (codes_out) codes_out[idx] = 0xFF;
    return;
  }
  uint32_t u = load_code(codes, bits, n_ks, row, col);
  if (codes_out) codes_out[idx] = (uint8_t)u;
  if (delta_hat) delta_hat[idx] = (float)(((double)u - zero_point(bits, grid)) * (double)step[row]);
}

// ---- salient selection (Eq. 2) ------------------------------------------------------------------------
// score_i = (sum_t x_ti^2) * (sum_j (D_ji - Dhat_ji)^2): the same number as the double sum of Eq. 2,
// since x_ti factors out of each squared term.  One thread per input channel, ascending fp64 sums.
__global__ void k_scores(const float* __restrict__ delta, const float* __restrict__ xc, int n, int d_in, int d_out,
                         int bits, int grid, const float* __restrict__ step, double* __restrict__ score) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d_in) return;
  const double z = zero_point(bits, grid);
  double err = 0.0;
  for (int j = 0; j < d_out; ++j) {
    float w = delta[(size_t)j * d_in + i];
    float s = step[j];
    double wh = ((double)quant_code(w, s, bits, grid) - z) * (double)s;
    double d = (double)w - wh;
    err += d * d;
  }
  double xs = 0.0;
  for (int t = 0; t < n; ++t) { double v = (double)xc[(size_t)t * d_in + i]; xs += v * v; }
  score[i] = xs * err;
}

__global__ void k_rank(const double* __restrict__ score, int d_in, int k, int* __restrict__ chosen) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d_in) return;
  double s = score[i];
  int rank = 0;
  for (int o = 0; o < d_in; ++o) {
    double so = score[o];
    rank += (so > s) || (so == s && o < i);
  }
  chosen[i] = rank < k;
}

__global__ void k_compact(const int* __restrict__ chosen, int d_in, int k, int32_t* __restrict__ idx_out) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= d_in || !chosen[i]) return;
  int pos = 0;
  for (int o = 0; o < i; ++o) pos += chosen[o];
  if (pos < k) idx_out[pos] = i;   // more than k can only be chosen when scores are NaN
}

__global__ void k_fill_zero(uint32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

inline unsigned blocks_for(size_t n, int bs) { return (unsigned)((n + bs - 1) / bs); }

}  // namespace

hipError_t launch_pack_base(const uint16_t* w, int d_in, int d_out, uint16_t* out, hipStream_t s) {
  int n_kb = ceil_to(d_in, kColPad) / 32;
  size_t n_slots = (size_t)(ceil_to(d_out, kRowPad) / 16) * n_kb * 64;
  k_pack_base<<<blocks_for(n_slots, 256), 256, 0, s>>>(w, d_in, d_out, n_kb, n_slots, reinterpret_cast<uint4*>(out));
  return hipGetLastError();
}

hipError_t launch_unpack_base(const uint16_t* t, int d_in, int d_out, uint16_t* out, hipStream_t s) {
  int n_kb = ceil_to(d_in, kColPad) / 32;
  size_t n_slots = (size_t)(ceil_to(d_out, kRowPad) / 16) * n_kb * 64;
  k_unpack_base<<<blocks_for(n_slots, 256), 256, 0, s>>>(reinterpret_cast<const uint4*>(t), d_in, d_out, n_kb, n_slots, out);
  return hipGetLastError();
}

// Plain streaming copy, 16 bytes per thread and iteration: the yardstick the HBM byte counters are scaled by.
__global__ __launch_bounds__(256) void k_copy_probe(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy_probe(void* dst, const void* src, size_t bytes, hipStream_t s) {
  const size_t n = bytes / 16;
  if (n == 0) return hipSuccess;
  k_copy_probe<<<(unsigned)(blocks_for(n, 256) < 8192 ? blocks_for(n, 256) : 8192), 256, 0, s>>>(
      reinterpret_cast<const uint4*>(src), reinterpret_cast<uint4*>(dst), n);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  size_t n = bytes / 4;
  if (n == 0) return hipSuccess;
  k_fill_zero<<<blocks_for(n, 256), 256, 0, s>>>(reinterpret_cast<uint32_t*>(p), n);
  return hipGetLastError();
}

hipError_t launch_pack_delta(const float* delta, int d_in, int d_out, const int32_t* sidx, int k, int bits,
                             int grid, int policy, const float* step_in, uint32_t* codes, float* step_out,
                             uint16_t* sal, int* flag, hipStream_t s) {
  hipError_t e;
  k_fill_zero<<<1, 64, 0, s>>>(reinterpret_cast<uint32_t*>(flag), 1);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (k > 0) {
    k_check_salient<<<blocks_for(k, 256), 256, 0, s>>>(sidx, k, d_in, flag);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  k_row_step<<<d_out, 256, 0, s>>>(delta, d_in, sidx, k, bits, grid, policy, step_in, step_out);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  int po = ceil_to(d_out, kRowPad), pi = ceil_to(d_in, kColPad);
  const int n_jt = po / 16;
  if ((e = launch_fill_zero(codes, (size_t)po * pi * bits / 8, s)) != hipSuccess) return e;
  k_pack_codes<<<blocks_for((size_t)d_out * (d_in / 8), 256), 256, 0, s>>>(delta, d_in, d_out, sidx, k, bits, grid, step_out, n_jt, codes);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (k > 0) {
    int n_sb = ceil_to(k, kSalPad) / 32;
    size_t n_el = (size_t)(po / 16) * n_sb * 512;
    k_pack_salient<<<blocks_for(n_el, 256), 256, 0, s>>>(delta, d_in, d_out, sidx, k, n_sb, n_el, flag, sal);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_unpack_delta(const mes_delta& d, float* delta_hat, uint8_t* codes_out, hipStream_t s) {
  int pi = ceil_to(d.d_in, kColPad);
  int n_ks = ceil_to(d.d_out, kRowPad) / 16;   // row tiles
  int n_sb = ceil_to(d.k, kSalPad) / 32;
  size_t n = (size_t)d.d_in * d.d_out;
  k_unpack_delta<<<blocks_for(n, 256), 256, 0, s>>>(reinterpret_cast<const uint32_t*>(d.codes), d.step,
                                                    reinterpret_cast<const uint16_t*>(d.salient), d.salient_idx, d.d_in,
                                                    d.d_out, d.k, d.bits, d.grid, n_ks, n_sb, delta_hat, codes_out);
  return hipGetLastError();
}

hipError_t launch_select(const float* delta, const float* xc, int n, int d_in, int d_out, int bits, int grid,
                         int policy, int k, int32_t* idx_out, double* score_out, void* ws, hipStream_t s) {
  // workspace: double score[d_in] | float step[d_out] | int chosen[d_in]
  char* p = reinterpret_cast<char*>(ws);
  double* score = reinterpret_cast<double*>(p);
  p += (size_t)ceil_to(d_in, 32) * sizeof(double);
  float* step = reinterpret_cast<float*>(p);
  p += (size_t)ceil_to(d_out, 64) * sizeof(float);
  int* chosen = reinterpret_cast<int*>(p);
  hipError_t e;
  k_row_step<<<d_out, 256, 0, s>>>(delta, d_in, nullptr, 0, bits, grid, policy, nullptr, step);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  k_scores<<<blocks_for(d_in, 64), 64, 0, s>>>(delta, xc, n, d_in, d_out, bits, grid, step, score);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  k_rank<<<blocks_for(d_in, 256), 256, 0, s>>>(score, d_in, k, chosen);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (k > 0) {
    k_compact<<<blocks_for(d_in, 256), 256, 0, s>>>(chosen, d_in, k, idx_out);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if (score_out) e = hipMemcpyAsync(score_out, score, (size_t)d_in * sizeof(double), hipMemcpyDeviceToDevice, s);
  return e;
}

}  // namespace mes
