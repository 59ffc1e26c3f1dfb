// mes_delta_linear for callers that cannot allocate device memory (code under HIP graph capture, tight serving
// loops, harnesses that forbid hipMalloc): the same kernels as mes_delta_linear, with the per-call scratch
// (prepared activations, gathered salient activations, split-column partial sums) in a device-resident static
// array instead of a caller-owned workspace.  Every GPU the library runs on holds its own copy of the array, at its
// own address, until the process ends.
#include "mes_internal.h"

#include <mutex>

namespace mes {
namespace {

constexpr size_t kScratchBytes = (size_t)64 << 20;

// In host code this name is only a handle for hipGetSymbolAddress; the array's memory is reached through the
// per-device pointer kept below, never through the name.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lock;
void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each device, looked up on first use

// The current device's copy of the array (looked up once per device, with that device current).
mes_status scratch_of_current_device(void** out) {
  int dev = -1;
  if (mes_status st = check_hip(hipGetDevice(&dev), "mes_delta_linear_noalloc: hipGetDevice")) return st;
  if (dev < 0 || dev >= kMaxDevices) return fail(MES_ERR_DEVICE, "mes_delta_linear_noalloc: device %d not supported", dev);
  std::lock_guard<std::mutex> hold(g_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (mes_status st = check_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "mes_delta_linear_noalloc: hipGetSymbolAddress"))
      return st;
    if (!ptr) return fail(MES_ERR_DEVICE, "mes_delta_linear_noalloc: the scratch array has no device address");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return MES_OK;
}

}  // namespace
}  // namespace mes

extern "C" {

size_t mes_noalloc_scratch_bytes(void) { return mes::kScratchBytes; }

mes_status mes_delta_linear_noalloc(const void* w_base_tiled, const mes_delta* experts, int n_experts, const void* x,
                                    int T, const int32_t* seg_offsets, void* y, void* stream) {
  using namespace mes;
  if (!experts) return fail(MES_ERR_NULL, "mes_delta_linear_noalloc: experts is null");
  if (n_experts < 1 || n_experts > MES_MAX_EXPERTS)
    return fail(MES_ERR_SHAPE, "mes_delta_linear_noalloc: n_experts = %d outside [1, %d]", n_experts, MES_MAX_EXPERTS);
  // what the streaming kernels of this shape need (it does not grow with T: token groups reuse it)
  const size_t need = mes_linear_workspace_bytes(experts[0].d_in, experts[0].d_out, 1);
  if (need == 0) return fail(MES_ERR_SHAPE, "mes_delta_linear_noalloc: bad shape %d x %d", experts[0].d_out, experts[0].d_in);
  if (need > kScratchBytes)
    return fail(MES_ERR_WORKSPACE, "mes_delta_linear_noalloc: a %d x %d layer needs %zu bytes of scratch, the static array holds %zu; "
                "use mes_delta_linear with a workspace", experts[0].d_out, experts[0].d_in, need, kScratchBytes);
  void* ptr = nullptr;
  if (mes_status st = scratch_of_current_device(&ptr)) return st;
  return mes_delta_linear(w_base_tiled, experts, n_experts, x, T, seg_offsets, y, ptr, kScratchBytes, stream);
}

}  // extern "C"
