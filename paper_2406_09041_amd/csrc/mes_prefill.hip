// Long token segments (prefill): one product per expert, y_e = x_e (W + Delta~_e)^T  -- Eq. 4 before it is
// decoupled.  With hundreds of tokens on one expert the layer is a dense contraction bound by the matrix cores,
// not by weight bytes, and streaming the weights once per 64 tokens (the decode kernel) wastes both.  Here the
// expert's effective weight W + Delta~_e is written out once as bf16 (k_materialize: base tile + dequantised
// codes, fp16 salient columns in their places) and multiplied with the segment's activations by the vendor's
// plain bf16 GEMM (rocBLAS, loaded on first use).  The rounding of W + Delta~ to bf16 adds a relative error of
// about 2^-9 / sqrt(3) to y, the same size as the rounding of y itself.
#include "mes_internal.h"

#include <dlfcn.h>
#include <mutex>

#include <rocblas/rocblas.h>

namespace mes {
namespace {

typedef __attribute__((__vector_size__(16))) uint32_t u32x4;

__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// rank[col] = position of input channel `col` in the expert's salient list, or -1.
__global__ void k_rank_fill(int16_t* rank, int d_in) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < d_in) rank[i] = -1;
}
__global__ void k_rank_scatter(int16_t* rank, const int32_t* __restrict__ sidx, int k, int d_in) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < k) {
    const int c = sidx[r];
    if (c >= 0 && c < d_in) rank[c] = (int16_t)r;   // a corrupt list can never address outside the table
  }
}

// One wavefront per (chunk c, row tile jt) block of 16 output channels x 128 input channels, in the order the tiled
// buffers are stored: lane 16 g + r reads, for kb = 0..3, the 16-byte base slot of row 16 jt + r, columns
// 128 c + 32 kb + 8 g + 0..7 (1 KiB per wavefront and kb, contiguous) and the matching code word(s), and writes
// the eight bf16 sums to the row-major output (four lanes fill 64 contiguous bytes of a row).
__global__ __launch_bounds__(256) void k_materialize(const u32x4* __restrict__ base, const uint32_t* __restrict__ codes,
                                                     const float* __restrict__ step, const uint16_t* __restrict__ sal,
                                                     const int16_t* __restrict__ rank, int d_in, int d_out, int k,
                                                     int bits, float z, int n_jt, int n_sb, int n_blocks,
                                                     uint16_t* __restrict__ w_eff) {
  const int blk_id = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (blk_id >= n_blocks) return;
  const int c = blk_id / n_jt, jt = blk_id - c * n_jt;
  const int lane = threadIdx.x & 63, g = lane >> 4, r = lane & 15;
  const int row = 16 * jt + r < d_out ? 16 * jt + r : d_out - 1;   // padding rows repeat the last one; never stored
  constexpr int kTileRow = 256 + 16;
  __shared__ __attribute__((aligned(16))) char tiles[4][16 * kTileRow];
  char* tile = tiles[threadIdx.x >> 6];
  const uint32_t* blk = codes + (size_t)blk_id * (64 * bits);
  const float s = step[row];
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
    const int col0 = 128 * c + 32 * kb + 8 * g;
    if (col0 >= d_in) continue;                          // padding columns of the last chunk: never stored
    const u32x4 b = base[((size_t)blk_id * 4 + kb) * 64 + lane];
    const int cl = 16 * kb + r, q = g;                    // the code block's lane cl owns columns 32 kb + 8 q + p
    uint32_t lo, hi = 0;
    int lo_shift, lo_mask, hi_shift = 0, hi_mask = 0;
    if (bits == 1) {
      lo = blk[cl]; lo_shift = q; lo_mask = 1;
    } else {
      lo = blk[2 * cl + (q >> 1)]; lo_shift = 2 * (q & 1); lo_mask = 3;
      if (bits == 3) { hi = blk[128 + cl]; hi_shift = q; hi_mask = 1; }
      if (bits == 4) { hi = blk[128 + 2 * cl + (q >> 1)]; hi_shift = 2 * (q & 1); hi_mask = 3; }
    }
    u32x4 rk4 = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu};   // eight int16 ranks, -1 = not salient
    if (k > 0) rk4 = *reinterpret_cast<const u32x4*>(rank + col0);
    uint32_t out[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const float w = bf16_to_f32((b[p >> 1] >> (16 * (p & 1))) & 0xffffu);
      const int u = (int)((lo >> (4 * p + lo_shift)) & lo_mask) | ((int)((hi >> (4 * p + hi_shift)) & hi_mask) << 2);
      float delta = ((float)u - z) * s;
      const int rk = (int)(int16_t)((rk4[p >> 1] >> (16 * (p & 1))) & 0xffffu);
      if (rk >= 0) {
        const uint16_t h = sal[(((size_t)jt * n_sb + (rk >> 5)) * 64 + 16 * ((rk & 31) >> 3) + r) * 8 + (rk & 7)];
        delta = (float)__builtin_bit_cast(_Float16, h);
      }
      out[p] = f32_to_bf16(w + delta);
    }
    // through the wavefront's 16 x 128 LDS tile (rows padded by 16 bytes against bank conflicts), so that the
    // global writes below are whole 256-byte row segments
    *reinterpret_cast<u32x4*>(tile + r * kTileRow + (32 * kb + 8 * g) * 2) =
        u32x4{out[0] | (out[1] << 16), out[2] | (out[3] << 16), out[4] | (out[5] << 16), out[6] | (out[7] << 16)};
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int rr = 4 * i + (lane >> 4), cc = 128 * c + 8 * (lane & 15);   // 16 lanes cover one row's 128 columns
    const u32x4 v = *reinterpret_cast<const u32x4*>(tile + rr * kTileRow + (lane & 15) * 16);
    if (16 * jt + rr < d_out && cc < d_in) *reinterpret_cast<u32x4*>(w_eff + (size_t)(16 * jt + rr) * d_in + cc) = v;
  }
}

// ---- the vendor GEMM, loaded on first use ---------------------------------------------------------------
struct Blas {
  void* lib = nullptr;
  rocblas_handle handle = nullptr;
  decltype(&rocblas_create_handle) create = nullptr;
  decltype(&rocblas_set_stream) set_stream = nullptr;
  decltype(&rocblas_gemm_ex) gemm_ex = nullptr;
  bool tried = false;
};
Blas g_blas;
std::mutex g_blas_mutex;

// Returns nullptr (and leaves a message) when the library or one of its entry points is not there.
Blas* blas() {
  if (g_blas.tried) return g_blas.handle ? &g_blas : nullptr;
  g_blas.tried = true;
  g_blas.lib = dlopen("librocblas.so", RTLD_NOW | RTLD_LOCAL);
  if (!g_blas.lib) g_blas.lib = dlopen("/opt/rocm/lib/librocblas.so", RTLD_NOW | RTLD_LOCAL);
  if (!g_blas.lib) return nullptr;
  g_blas.create = reinterpret_cast<decltype(g_blas.create)>(dlsym(g_blas.lib, "rocblas_create_handle"));
  g_blas.set_stream = reinterpret_cast<decltype(g_blas.set_stream)>(dlsym(g_blas.lib, "rocblas_set_stream"));
  g_blas.gemm_ex = reinterpret_cast<decltype(g_blas.gemm_ex)>(dlsym(g_blas.lib, "rocblas_gemm_ex"));
  if (!g_blas.create || !g_blas.set_stream || !g_blas.gemm_ex) return nullptr;
  if (g_blas.create(&g_blas.handle) != rocblas_status_success) { g_blas.handle = nullptr; return nullptr; }
  return &g_blas;
}

}  // namespace

// False when the vendor GEMM cannot be loaded: long segments then stay on the streaming kernel.
bool prefill_available() {
  std::lock_guard<std::mutex> lock(g_blas_mutex);
  return blas() != nullptr;
}

size_t prefill_scratch_bytes(int d_in, int max_d_out) {
  return (size_t)max_d_out * d_in * 2 + (((size_t)d_in * 2 + 255) / 256) * 256;
}

// y[rows t_begin .. t_end) of one linear for ONE expert.  scratch: prefill_scratch_bytes(d_in, d_out) bytes.
hipError_t launch_prefill_segment(const void* w_base_tiled, const mes_delta& d, const void* x, int t_begin, int t_end,
                                  void* y, void* scratch, hipStream_t s) {
  const int n_tok = t_end - t_begin;
  if (n_tok <= 0) return hipSuccess;
  std::lock_guard<std::mutex> lock(g_blas_mutex);   // one handle, one stream setting at a time
  Blas* bl = blas();
  if (!bl) return hipErrorSharedObjectInitFailed;
  char* w_eff = reinterpret_cast<char*>(scratch);
  int16_t* rank = reinterpret_cast<int16_t*>(w_eff + (size_t)d.d_out * d.d_in * 2);
  const int n_jt = ceil_to(d.d_out, kRowPad) / 16, n_sb = ceil_to(d.k, kSalPad) / 32;
  if (d.k > 0) {
    k_rank_fill<<<(d.d_in + 255) / 256, 256, 0, s>>>(rank, d.d_in);
    k_rank_scatter<<<(d.k + 255) / 256, 256, 0, s>>>(rank, d.salient_idx, d.k, d.d_in);
  }
  const float z = d.grid == MES_GRID_SYM ? (float)(1 << (d.bits - 1)) - 0.5f : (float)(1 << (d.bits - 1));
  const int n_blocks = ceil_to(d.d_in, kColPad) / 128 * n_jt;
  k_materialize<<<(n_blocks + 3) / 4, 256, 0, s>>>(
      reinterpret_cast<const u32x4*>(w_base_tiled), reinterpret_cast<const uint32_t*>(d.codes), d.step,
      reinterpret_cast<const uint16_t*>(d.salient), rank, d.d_in, d.d_out, d.k, d.bits, z, n_jt, n_sb, n_blocks,
      reinterpret_cast<uint16_t*>(w_eff));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // Row-major y[n_tok, d_out] = x[n_tok, d_in] W_eff^T, i.e. column-major  Y (d_out x n_tok) = A^T B  with
  // A = W_eff seen column-major (d_in x d_out) and B = x seen column-major (d_in x n_tok).
  if (bl->set_stream(bl->handle, s) != rocblas_status_success) return hipErrorUnknown;
  const float alpha = 1.0f, beta = 0.0f;
  const char* xb = reinterpret_cast<const char*>(x) + (size_t)t_begin * d.d_in * 2;
  char* yb = reinterpret_cast<char*>(y) + (size_t)t_begin * d.d_out * 2;
  const rocblas_status st = bl->gemm_ex(bl->handle, rocblas_operation_transpose, rocblas_operation_none, d.d_out, n_tok, d.d_in,
                                        &alpha, w_eff, rocblas_datatype_bf16_r, d.d_in, xb, rocblas_datatype_bf16_r, d.d_in,
                                        &beta, yb, rocblas_datatype_bf16_r, d.d_out, yb, rocblas_datatype_bf16_r, d.d_out,
                                        rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
  return st == rocblas_status_success ? hipSuccess : hipErrorUnknown;
}

}  // namespace mes
