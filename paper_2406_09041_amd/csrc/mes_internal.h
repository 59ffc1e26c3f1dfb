// Internal declarations shared by the translation units of libmes (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mes.h"

namespace mes {

constexpr int kRowPad = 64;    // stored rows are padded to a multiple of this
constexpr int kColPad = 128;   // stored columns are padded to a multiple of this (one chunk)
constexpr int kSalPad = 32;    // stored salient columns are padded to a multiple of this
constexpr int kTokGroup = 64;  // tokens one decode launch covers

inline int ceil_to(int n, int m) { return (n + m - 1) / m * m; }

// Error plumbing (thread-local message, see mes_last_error()).
mes_status fail(mes_status st, const char* fmt, ...);
mes_status check_hip(hipError_t e, const char* what);

// ---- launchers implemented in mes_pack.hip ------------------------------------------------------
hipError_t launch_pack_base(const uint16_t* w, int d_in, int d_out, uint16_t* out, hipStream_t s);
hipError_t launch_unpack_base(const uint16_t* t, int d_in, int d_out, uint16_t* out, hipStream_t s);
hipError_t launch_pack_delta(const float* delta, int d_in, int d_out, const int32_t* sidx, int k, int bits,
                             int grid, int policy, const float* step_in, uint32_t* codes, float* step_out,
                             uint16_t* sal, int* flag, hipStream_t s);
hipError_t launch_unpack_delta(const mes_delta& d, float* delta_hat, uint8_t* codes_out, hipStream_t s);
hipError_t launch_select(const float* delta, const float* xc, int n, int d_in, int d_out, int bits, int grid,
                         int policy, int k, int32_t* idx_out, double* score_out, void* ws, hipStream_t s);
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t launch_copy_probe(void* dst, const void* src, size_t bytes, hipStream_t s);

// ---- launcher implemented in mes_linear.hip -----------------------------------------------------
struct LinearCall {
  const mes_linear* lin;   // n_linears entries
  int n_linears;
  int n_experts;
  const void* x;
  int T;
  const int32_t* seg;
  void* ws;
  size_t ws_bytes;
  hipEvent_t ev_start, ev_stop;   // measurement hook (nullptr: none)
  int gated;               // 1: lin[0] = gate, lin[1] = up projection; the one output SiLU(gate) * up goes to lin[0].y
};
size_t linear_workspace_bytes(int d_in, const int* d_out, int n_linears, int max_tokens);
size_t gated_workspace_bytes(int d_in, int d_out, int max_tokens);
int long_segment_tokens();
hipError_t launch_delta_linear(const LinearCall& c, hipStream_t s);

// ---- implemented in mes_step.hip ---------------------------------------------------------------
size_t step_grad_workspace_bytes(int d_in, int d_out, int n_tokens);
hipError_t launch_step_grad(const float* delta, int d_in, int d_out, const int32_t* sidx, int k, int bits, int grid,
                            const float* step, const void* x, int n_tokens, float* loss, float* grad, void* ws,
                            hipEvent_t ev_start, hipEvent_t ev_stop, hipStream_t s);
hipError_t launch_adamw(float* step, const float* grad, float* m, float* v, int n, int t, float lr, float beta1,
                        float beta2, float eps, float weight_decay, hipStream_t s);

// ---- implemented in mes_prefill.hip ------------------------------------------------------------
size_t prefill_scratch_bytes(int d_in, int max_tokens);
hipError_t launch_prefill_segments(const mes_linear* lin, int n_linears, const int* seg_experts, int n_seg,
                                   const int32_t* seg, const void* x, void* scratch, hipEvent_t ev_start,
                                   hipEvent_t ev_stop, bool* first_kernel, hipStream_t s);

}  // namespace mes
