// extern "C" entry points: argument validation on the host (before any HIP call), then launch.
#include "mes_internal.h"
#include "mes_bench.h"

#include <cstdarg>
#include <cstdio>

namespace mes {

static thread_local char g_err[512] = "";
static thread_local hipEvent_t g_ev_start = nullptr, g_ev_stop = nullptr;

mes_status fail(mes_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

mes_status check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return MES_OK;
  return fail(MES_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static mes_status check_dims(int d_in, int d_out) {
  if (d_in <= 0 || d_out <= 0) return fail(MES_ERR_SHAPE, "d_in and d_out must be positive (got %d, %d)", d_in, d_out);
  if (d_in % 8 != 0) return fail(MES_ERR_SHAPE, "d_in must be a multiple of 8 (got %d)", d_in);
  if (d_out % 4 != 0) return fail(MES_ERR_SHAPE, "d_out must be a multiple of 4 (got %d)", d_out);
  return MES_OK;
}

static mes_status check_quant(int bits, int grid, int policy, bool allow_given) {
  if (bits < 1 || bits > 4) return fail(MES_ERR_BITS, "bits must be 1, 2, 3 or 4 (got %d)", bits);
  if (grid != MES_GRID_SYM && grid != MES_GRID_EQ1) return fail(MES_ERR_BITS, "unknown grid %d", grid);
  if (grid == MES_GRID_EQ1 && bits == 1) return fail(MES_ERR_BITS, "the Eq. 1 grid is undefined for bits = 1");
  if (policy < MES_STEP_GIVEN || policy > MES_STEP_MEANABS) return fail(MES_ERR_BITS, "unknown step policy %d", policy);
  if (policy == MES_STEP_GIVEN && !allow_given) return fail(MES_ERR_BITS, "step policy GIVEN is not valid here");
  if (policy == MES_STEP_MEANABS && bits != 1) return fail(MES_ERR_BITS, "step policy MEANABS needs bits = 1");
  return MES_OK;
}

}  // namespace mes

using namespace mes;

extern "C" {

const char* mes_last_error(void) { return g_err; }
int mes_layout_version(void) { return MES_LAYOUT_VERSION; }
int mes_long_segment_tokens(void) { return long_segment_tokens(); }

size_t mes_base_bytes(int d_in, int d_out) {
  if (d_in <= 0 || d_out <= 0) return 0;
  return (size_t)ceil_to(d_out, kRowPad) * ceil_to(d_in, kColPad) * 2;
}

size_t mes_codes_bytes(int d_in, int d_out, int bits) {
  if (d_in <= 0 || d_out <= 0 || bits < 1 || bits > 4) return 0;
  return (size_t)ceil_to(d_out, kRowPad) * ceil_to(d_in, kColPad) * bits / 8;
}

size_t mes_salient_bytes(int d_out, int k) {
  if (d_out <= 0 || k < 0) return 0;
  return (size_t)ceil_to(d_out, kRowPad) * ceil_to(k, kSalPad) * 2;
}

size_t mes_pack_workspace_bytes(void) { return 256; }

size_t mes_select_workspace_bytes(int n, int d_in, int d_out) {
  if (n <= 0 || d_in <= 0 || d_out <= 0) return 0;
  return (size_t)ceil_to(d_in, 32) * 8 + (size_t)ceil_to(d_out, 64) * 4 + (size_t)ceil_to(d_in, 32) * 4;
}

size_t mes_linear_multi_workspace_bytes(int d_in, const int32_t* d_out, int n_linears, int max_tokens) {
  if (d_in <= 0 || !d_out || n_linears < 1 || n_linears > MES_MAX_FUSED || max_tokens < 0) return 0;
  int d[MES_MAX_FUSED];
  for (int l = 0; l < n_linears; ++l) {
    if (d_out[l] <= 0) return 0;
    d[l] = d_out[l];
  }
  return linear_workspace_bytes(d_in, d, n_linears, max_tokens);
}

size_t mes_linear_workspace_bytes(int d_in, int d_out, int max_tokens) {
  const int32_t d = d_out;
  return mes_linear_multi_workspace_bytes(d_in, &d, 1, max_tokens);
}

mes_status mes_pack_base(const void* w, int d_in, int d_out, void* w_tiled_out, void* stream) {
  if (!w || !w_tiled_out) return fail(MES_ERR_NULL, "mes_pack_base: null pointer");
  if (mes_status st = check_dims(d_in, d_out)) return st;
  if (!aligned16(w) || !aligned16(w_tiled_out)) return fail(MES_ERR_ALIGN, "mes_pack_base: pointers must be 16-byte aligned");
  return check_hip(launch_pack_base((const uint16_t*)w, d_in, d_out, (uint16_t*)w_tiled_out, (hipStream_t)stream), "mes_pack_base");
}

mes_status mes_unpack_base(const void* w_tiled, int d_in, int d_out, void* w_out, void* stream) {
  if (!w_tiled || !w_out) return fail(MES_ERR_NULL, "mes_unpack_base: null pointer");
  if (mes_status st = check_dims(d_in, d_out)) return st;
  if (!aligned16(w_tiled) || !aligned16(w_out)) return fail(MES_ERR_ALIGN, "mes_unpack_base: pointers must be 16-byte aligned");
  return check_hip(launch_unpack_base((const uint16_t*)w_tiled, d_in, d_out, (uint16_t*)w_out, (hipStream_t)stream), "mes_unpack_base");
}

mes_status mes_select_salient(const float* delta, const float* x_calib, int n, int d_in, int d_out, int bits,
                              int grid, int step_policy, int k, int32_t* idx_out, double* score_out,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!delta || !x_calib) return fail(MES_ERR_NULL, "mes_select_salient: null input");
  if (mes_status st = check_dims(d_in, d_out)) return st;
  if (n <= 0) return fail(MES_ERR_SHAPE, "mes_select_salient: n must be positive (got %d)", n);
  if (mes_status st = check_quant(bits, grid, step_policy, false)) return st;
  if (k < 0 || k > d_in) return fail(MES_ERR_SALIENT, "mes_select_salient: k = %d outside [0, %d]", k, d_in);
  if (k > 0 && !idx_out) return fail(MES_ERR_NULL, "mes_select_salient: idx_out is null");
  if (!workspace || workspace_bytes < mes_select_workspace_bytes(n, d_in, d_out))
    return fail(MES_ERR_WORKSPACE, "mes_select_salient: workspace needs %zu bytes", mes_select_workspace_bytes(n, d_in, d_out));
  if (!aligned16(workspace)) return fail(MES_ERR_ALIGN, "mes_select_salient: workspace must be 16-byte aligned");
  return check_hip(launch_select(delta, x_calib, n, d_in, d_out, bits, grid, step_policy, k, idx_out, score_out,
                                 workspace, (hipStream_t)stream), "mes_select_salient");
}

mes_status mes_pack_delta(const float* delta, int d_in, int d_out, const int32_t* salient_idx, int k, int bits,
                          int grid, int step_policy, const float* step_in, void* codes_out, float* step_out,
                          void* salient_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!delta || !codes_out || !step_out) return fail(MES_ERR_NULL, "mes_pack_delta: null pointer");
  if (mes_status st = check_dims(d_in, d_out)) return st;
  if (mes_status st = check_quant(bits, grid, step_policy, true)) return st;
  if (k < 0 || k > d_in) return fail(MES_ERR_SALIENT, "mes_pack_delta: k = %d outside [0, %d]", k, d_in);
  if (k > 0 && (!salient_idx || !salient_out)) return fail(MES_ERR_NULL, "mes_pack_delta: k > 0 needs salient_idx and salient_out");
  if (step_policy == MES_STEP_GIVEN && !step_in) return fail(MES_ERR_NULL, "mes_pack_delta: step policy GIVEN needs step_in");
  if (!aligned16(codes_out) || !aligned16(step_out) || (k > 0 && !aligned16(salient_out)))
    return fail(MES_ERR_ALIGN, "mes_pack_delta: outputs must be 16-byte aligned");
  if (!workspace || workspace_bytes < mes_pack_workspace_bytes())
    return fail(MES_ERR_WORKSPACE, "mes_pack_delta: workspace needs %zu bytes", mes_pack_workspace_bytes());
  hipStream_t s = (hipStream_t)stream;
  int* flag = reinterpret_cast<int*>(workspace);
  if (mes_status st = check_hip(launch_pack_delta(delta, d_in, d_out, salient_idx, k, bits, grid, step_policy, step_in,
                                                  (uint32_t*)codes_out, step_out, (uint16_t*)salient_out, flag, s),
                                "mes_pack_delta"))
    return st;
  int host_flag = 0;
  if (mes_status st = check_hip(hipMemcpyAsync(&host_flag, flag, sizeof(int), hipMemcpyDeviceToHost, s), "mes_pack_delta: flag copy"))
    return st;
  if (mes_status st = check_hip(hipStreamSynchronize(s), "mes_pack_delta: synchronize")) return st;
  if (host_flag) return fail(MES_ERR_SALIENT, "mes_pack_delta: salient_idx must be strictly ascending and inside [0, d_in)");
  return MES_OK;
}

static mes_status check_delta(const mes_delta* d, const char* who) {
  if (!d) return fail(MES_ERR_NULL, "%s: null descriptor", who);
  if (mes_status st = check_dims(d->d_in, d->d_out)) return st;
  if (mes_status st = check_quant(d->bits, d->grid, MES_STEP_GIVEN, true)) return st;
  if (d->layout_version != MES_LAYOUT_VERSION) return fail(MES_ERR_SHAPE, "%s: layout_version %d, library has %d", who, d->layout_version, MES_LAYOUT_VERSION);
  if (d->k < 0 || d->k > d->d_in) return fail(MES_ERR_SALIENT, "%s: k = %d outside [0, %d]", who, d->k, d->d_in);
  if (!d->codes || !d->step) return fail(MES_ERR_NULL, "%s: codes / step pointer is null", who);
  if (d->k > 0 && (!d->salient || !d->salient_idx)) return fail(MES_ERR_NULL, "%s: k > 0 needs salient and salient_idx", who);
  if (!aligned16(d->codes) || !aligned16(d->step) || (d->k > 0 && !aligned16(d->salient)))
    return fail(MES_ERR_ALIGN, "%s: codes, step and salient must be 16-byte aligned", who);
  return MES_OK;
}

mes_status mes_unpack_delta(const mes_delta* d, float* delta_hat_out, uint8_t* codes_out, void* stream) {
  if (mes_status st = check_delta(d, "mes_unpack_delta")) return st;
  if (!delta_hat_out && !codes_out) return fail(MES_ERR_NULL, "mes_unpack_delta: both outputs are null");
  return check_hip(launch_unpack_delta(*d, delta_hat_out, codes_out, (hipStream_t)stream), "mes_unpack_delta");
}

// mes_delta_linear_multi and, with gated != 0 (two layers: gate, up; one output at linears[0].y), mes_delta_linear_gated.
static mes_status run_linears(const char* who, const mes_linear* linears, int n_linears, int n_experts, const void* x, int T,
                              const int32_t* seg_offsets, void* workspace, size_t workspace_bytes, void* stream, int gated) {
  // the measurement hook is one-shot: this call consumes the events whichever way it returns
  const hipEvent_t ev_start = g_ev_start, ev_stop = g_ev_stop;
  g_ev_start = g_ev_stop = nullptr;
  if (n_linears < 1 || n_linears > MES_MAX_FUSED)
    return fail(MES_ERR_SHAPE, "%s: n_linears = %d outside [1, %d]", who, n_linears, MES_MAX_FUSED);
  if (n_experts < 1 || n_experts > MES_MAX_EXPERTS)
    return fail(MES_ERR_SHAPE, "%s: n_experts = %d outside [1, %d]", who, n_experts, MES_MAX_EXPERTS);
  if (T < 0) return fail(MES_ERR_SHAPE, "%s: T = %d is negative", who, T);
  if (!linears || !seg_offsets) return fail(MES_ERR_NULL, "%s: linears / seg_offsets is null", who);
  int32_t d_outs[MES_MAX_FUSED];
  for (int l = 0; l < n_linears; ++l) {
    if (!linears[l].experts) return fail(MES_ERR_NULL, "%s: experts is null", who);
    for (int e = 0; e < n_experts; ++e) {
      if (mes_status st = check_delta(&linears[l].experts[e], who)) return st;
      const mes_delta &a = linears[0].experts[0], &b = linears[l].experts[e];
      if (a.d_in != b.d_in || a.k != b.k || a.bits != b.bits || a.grid != b.grid || b.d_out != linears[l].experts[0].d_out)
        return fail(MES_ERR_SHAPE, "%s: expert %d of layer %d differs in d_in/d_out/k/bits/grid", who, e, l);
    }
    d_outs[l] = linears[l].experts[0].d_out;
  }
  if (seg_offsets[0] != 0) return fail(MES_ERR_SEGMENTS, "%s: seg_offsets[0] must be 0 (got %d)", who, seg_offsets[0]);
  for (int e = 0; e < n_experts; ++e)
    if (seg_offsets[e + 1] < seg_offsets[e]) return fail(MES_ERR_SEGMENTS, "%s: seg_offsets decreases at %d", who, e + 1);
  if (seg_offsets[n_experts] != T)
    return fail(MES_ERR_SEGMENTS, "%s: seg_offsets[%d] = %d, expected T = %d", who, n_experts, seg_offsets[n_experts], T);
  if (T == 0) return MES_OK;
  if (!x) return fail(MES_ERR_NULL, "%s: w_base / x / y is null", who);
  for (int l = 0; l < n_linears; ++l) {
    const bool has_y = !(gated && l > 0);   // the gated pair has one output
    if (!linears[l].w_base_tiled || (has_y && !linears[l].y)) return fail(MES_ERR_NULL, "%s: w_base / x / y is null", who);
    if (!aligned16(linears[l].w_base_tiled) || (has_y && !aligned16(linears[l].y)))
      return fail(MES_ERR_ALIGN, "%s: w_base, x and y must be 16-byte aligned", who);
  }
  if (!aligned16(x)) return fail(MES_ERR_ALIGN, "%s: w_base, x and y must be 16-byte aligned", who);
  if (gated && d_outs[0] != d_outs[1]) return fail(MES_ERR_SHAPE, "%s: gate and up projection differ in d_out (%d, %d)", who, d_outs[0], d_outs[1]);
  // the streaming path's share is what a call needs; the one-product scratch (sizes asked for with max_tokens >= 192)
  // is used when it is there
  const size_t need = gated ? gated_workspace_bytes(linears[0].experts[0].d_in, d_outs[0], 1)
                            : mes_linear_multi_workspace_bytes(linears[0].experts[0].d_in, d_outs, n_linears, 1);
  if (!workspace || workspace_bytes < need) return fail(MES_ERR_WORKSPACE, "%s: workspace needs %zu bytes", who, need);
  if (!aligned16(workspace)) return fail(MES_ERR_ALIGN, "%s: workspace must be 16-byte aligned", who);
  LinearCall c{linears, n_linears, n_experts, x, T, seg_offsets, workspace, workspace_bytes, ev_start, ev_stop, gated};
  return check_hip(launch_delta_linear(c, (hipStream_t)stream), who);
}

mes_status mes_delta_linear_multi(const mes_linear* linears, int n_linears, int n_experts, const void* x, int T,
                                  const int32_t* seg_offsets, void* workspace, size_t workspace_bytes, void* stream) {
  return run_linears("mes_delta_linear", linears, n_linears, n_experts, x, T, seg_offsets, workspace, workspace_bytes, stream, 0);
}

size_t mes_gated_workspace_bytes(int d_in, int d_out, int max_tokens) {
  if (d_in <= 0 || d_out <= 0 || max_tokens < 0) return 0;
  return gated_workspace_bytes(d_in, d_out, max_tokens);
}

mes_status mes_delta_linear_gated(const void* w_gate_tiled, const mes_delta* gate_experts, const void* w_up_tiled,
                                  const mes_delta* up_experts, int n_experts, const void* x, int T,
                                  const int32_t* seg_offsets, void* h, void* workspace, size_t workspace_bytes, void* stream) {
  const mes_linear pair[2] = {{w_gate_tiled, gate_experts, h}, {w_up_tiled, up_experts, nullptr}};
  return run_linears("mes_delta_linear_gated", pair, 2, n_experts, x, T, seg_offsets, workspace, workspace_bytes, stream, 1);
}

mes_status mes_delta_linear(const void* w_base_tiled, const mes_delta* experts, int n_experts, const void* x, int T,
                            const int32_t* seg_offsets, void* y, void* workspace, size_t workspace_bytes,
                            void* stream) {
  const mes_linear one{w_base_tiled, experts, y};
  return mes_delta_linear_multi(&one, 1, n_experts, x, T, seg_offsets, workspace, workspace_bytes, stream);
}

mes_status mes_time_next_call(void* start_event, void* stop_event) {
  if ((start_event == nullptr) != (stop_event == nullptr)) return fail(MES_ERR_NULL, "mes_time_next_call: give both events or neither");
  g_ev_start = (hipEvent_t)start_event;
  g_ev_stop = (hipEvent_t)stop_event;
  return MES_OK;
}

size_t mes_step_grad_workspace_bytes(int d_in, int d_out, int n_tokens) {
  if (d_in <= 0 || d_out <= 0 || n_tokens < 0) return 0;
  return step_grad_workspace_bytes(d_in, d_out, n_tokens);
}

mes_status mes_step_grad(const float* delta, int d_in, int d_out, const int32_t* salient_idx, int k, int bits, int grid,
                         const float* step, const void* x, int n_tokens, float* loss_out, float* grad_out,
                         void* workspace, size_t workspace_bytes, void* stream) {
  const hipEvent_t e0 = g_ev_start, e1 = g_ev_stop;   // one-shot measurement hook, consumed on every exit path
  g_ev_start = g_ev_stop = nullptr;
  if (!delta || !step || !loss_out || !grad_out) return fail(MES_ERR_NULL, "mes_step_grad: null pointer");
  if (mes_status st = check_dims(d_in, d_out)) return st;
  if (mes_status st = check_quant(bits, grid, MES_STEP_GIVEN, true)) return st;
  if (k < 0 || k > d_in) return fail(MES_ERR_SALIENT, "mes_step_grad: k = %d outside [0, %d]", k, d_in);
  if (k > 0 && !salient_idx) return fail(MES_ERR_NULL, "mes_step_grad: k > 0 needs salient_idx");
  if (n_tokens < 0) return fail(MES_ERR_SHAPE, "mes_step_grad: n_tokens must not be negative (got %d)", n_tokens);
  if (n_tokens > 0 && !x) return fail(MES_ERR_NULL, "mes_step_grad: x is null");
  if (!aligned16(delta) || !aligned16(step) || !aligned16(x))
    return fail(MES_ERR_ALIGN, "mes_step_grad: delta, step and x must be 16-byte aligned");
  if (!workspace || workspace_bytes < mes_step_grad_workspace_bytes(d_in, d_out, n_tokens))
    return fail(MES_ERR_WORKSPACE, "mes_step_grad: workspace needs %zu bytes", mes_step_grad_workspace_bytes(d_in, d_out, n_tokens));
  if (!aligned16(workspace)) return fail(MES_ERR_ALIGN, "mes_step_grad: workspace must be 16-byte aligned");
  return check_hip(launch_step_grad(delta, d_in, d_out, salient_idx, k, bits, grid, step, x, n_tokens, loss_out, grad_out,
                                    workspace, e0, e1, (hipStream_t)stream), "mes_step_grad");
}

mes_status mes_step_adamw(float* step, const float* grad, float* m, float* v, int n, int t, float lr, float beta1,
                          float beta2, float eps, float weight_decay, void* stream) {
  if (!step || !grad || !m || !v) return fail(MES_ERR_NULL, "mes_step_adamw: null pointer");
  if (n <= 0) return fail(MES_ERR_SHAPE, "mes_step_adamw: n must be positive (got %d)", n);
  if (t < 1) return fail(MES_ERR_SHAPE, "mes_step_adamw: t counts updates from 1 (got %d)", t);
  if (!(beta1 >= 0.0f && beta1 < 1.0f) || !(beta2 >= 0.0f && beta2 < 1.0f))
    return fail(MES_ERR_SHAPE, "mes_step_adamw: beta1 and beta2 must lie in [0, 1)");
  return check_hip(launch_adamw(step, grad, m, v, n, t, lr, beta1, beta2, eps, weight_decay, (hipStream_t)stream), "mes_step_adamw");
}

mes_status mes_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
  if (!dst || !src) return fail(MES_ERR_NULL, "mes_copy_probe: null buffer");
  if (bytes % 16 || ((uintptr_t)dst | (uintptr_t)src) % 16) return fail(MES_ERR_ALIGN, "mes_copy_probe: buffers and size must be multiples of 16 bytes");
  return check_hip(launch_copy_probe(dst, src, bytes, (hipStream_t)stream), "mes_copy_probe");
}

}  // extern "C"
