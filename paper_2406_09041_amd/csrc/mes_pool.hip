// On-demand swapping of compressed deltas (Section 4.1, paragraph "On-demand swapping": the pre-trained model
// stays in GPU memory, the compressed deltas of the experts a batch needs are loaded when they are needed).
//
// A pool serves ONE linear layer: `n_slots` device slots, each big enough for one expert's packed delta
// (codes, steps, salient fp16 tile, salient indices), carved out of an arena the caller owns; and up to
// `n_experts` registered experts whose packed buffers live in pinned host memory the caller owns.  acquire()
// makes a set of experts resident -- least recently used slots are overwritten, copies go out on a copy stream,
// the compute stream is made to wait for them -- and returns their descriptors for mes_delta_linear.
// Host code only; the bookkeeping is plain C++ and does not touch the GPU in a dry-run pool.
#include "mes_internal.h"

#include <cstdlib>
#include <new>
#include <vector>

namespace mes {
namespace {

constexpr size_t kSlotAlign = 256;
inline size_t up(size_t v) { return (v + kSlotAlign - 1) / kSlotAlign * kSlotAlign; }

struct SlotLayout {
  size_t codes, step, salient, sidx, total;   // byte offsets inside a slot, and its size
  size_t codes_bytes, step_bytes, salient_bytes, sidx_bytes;
};

SlotLayout slot_layout(int d_in, int d_out, int k, int bits) {
  SlotLayout s;
  s.codes_bytes = (size_t)ceil_to(d_out, kRowPad) * ceil_to(d_in, kColPad) * bits / 8;
  s.step_bytes = (size_t)d_out * 4;
  s.salient_bytes = (size_t)ceil_to(d_out, kRowPad) * ceil_to(k, kSalPad) * 2;
  s.sidx_bytes = (size_t)k * 4;
  s.codes = 0;
  s.step = up(s.codes + s.codes_bytes);
  s.salient = up(s.step + s.step_bytes);
  s.sidx = up(s.salient + s.salient_bytes);
  s.total = up(s.sidx + s.sidx_bytes);
  return s;
}

struct HostExpert {
  const void* codes = nullptr;
  const float* step = nullptr;
  const void* salient = nullptr;
  const int32_t* sidx = nullptr;
  int slot = -1;   // resident in this slot, or -1
};

}  // namespace
}  // namespace mes

struct mes_pool {
  int d_in, d_out, k, bits, grid, n_slots, n_experts, dry_run;
  mes::SlotLayout lay;
  char* arena;
  std::vector<mes::HostExpert> experts;
  std::vector<int> slot_expert;        // expert in the slot, or -1
  std::vector<uint64_t> slot_used;     // value of `clock` when the slot was last handed out (0: never)
  uint64_t clock, hits, misses, bytes;
  hipEvent_t ev_compute, ev_copy;      // not created in a dry-run pool
};

extern "C" {

size_t mes_pool_slot_bytes(int d_in, int d_out, int k, int bits) {
  if (d_in <= 0 || d_out <= 0 || k < 0 || k > d_in || bits < 1 || bits > 4) return 0;
  return mes::slot_layout(d_in, d_out, k, bits).total;
}

mes_status mes_pool_create(int d_in, int d_out, int k, int bits, int grid, int n_slots, int n_experts, void* arena,
                           size_t arena_bytes, int dry_run, mes_pool** out) {
  using namespace mes;
  if (!out) return fail(MES_ERR_NULL, "mes_pool_create: out is null");
  *out = nullptr;
  if (d_in <= 0 || d_out <= 0 || d_in % 8 != 0 || d_out % 4 != 0)
    return fail(MES_ERR_SHAPE, "mes_pool_create: bad shape %d x %d", d_out, d_in);
  if (bits < 1 || bits > 4 || (grid != MES_GRID_SYM && grid != MES_GRID_EQ1) || (grid == MES_GRID_EQ1 && bits == 1))
    return fail(MES_ERR_BITS, "mes_pool_create: bits %d / grid %d not supported", bits, grid);
  if (k < 0 || k > d_in) return fail(MES_ERR_SALIENT, "mes_pool_create: k = %d outside [0, d_in]", k);
  if (n_slots < 1 || n_slots > MES_MAX_EXPERTS || n_experts < 1)
    return fail(MES_ERR_SHAPE, "mes_pool_create: n_slots must be 1..%d and n_experts positive", MES_MAX_EXPERTS);
  const SlotLayout lay = slot_layout(d_in, d_out, k, bits);
  if (!arena) return fail(MES_ERR_NULL, "mes_pool_create: arena is null");
  if (reinterpret_cast<uintptr_t>(arena) % kSlotAlign) return fail(MES_ERR_ALIGN, "mes_pool_create: arena must be 256-byte aligned");
  if (arena_bytes < lay.total * (size_t)n_slots)
    return fail(MES_ERR_WORKSPACE, "mes_pool_create: arena of %zu bytes, %zu needed", arena_bytes, lay.total * (size_t)n_slots);
  mes_pool* p = new (std::nothrow) mes_pool();
  if (!p) return fail(MES_ERR_DEVICE, "mes_pool_create: out of host memory");
  p->d_in = d_in; p->d_out = d_out; p->k = k; p->bits = bits; p->grid = grid;
  p->n_slots = n_slots; p->n_experts = n_experts; p->dry_run = dry_run;
  p->lay = lay;
  p->arena = reinterpret_cast<char*>(arena);
  p->experts.assign(n_experts, HostExpert());
  p->slot_expert.assign(n_slots, -1);
  p->slot_used.assign(n_slots, 0);
  p->clock = p->hits = p->misses = p->bytes = 0;
  p->ev_compute = p->ev_copy = nullptr;
  if (!dry_run) {
    hipError_t e = hipEventCreateWithFlags(&p->ev_compute, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&p->ev_copy, hipEventDisableTiming);
    if (e != hipSuccess) {
      if (p->ev_compute) (void)hipEventDestroy(p->ev_compute);
      delete p;
      return check_hip(e, "mes_pool_create: hipEventCreate");
    }
  }
  *out = p;
  return MES_OK;
}

void mes_pool_destroy(mes_pool* p) {
  if (!p) return;
  if (p->ev_compute) (void)hipEventDestroy(p->ev_compute);
  if (p->ev_copy) (void)hipEventDestroy(p->ev_copy);
  delete p;
}

mes_status mes_pool_register(mes_pool* p, int expert, const void* codes, const float* step, const void* salient,
                             const int32_t* salient_idx) {
  using namespace mes;
  if (!p) return fail(MES_ERR_NULL, "mes_pool_register: pool is null");
  if (expert < 0 || expert >= p->n_experts) return fail(MES_ERR_SHAPE, "mes_pool_register: expert %d outside [0, %d)", expert, p->n_experts);
  if (!codes || !step || (p->k > 0 && (!salient || !salient_idx))) return fail(MES_ERR_NULL, "mes_pool_register: null host buffer");
  HostExpert& h = p->experts[expert];
  if (h.slot >= 0) {   // new contents: what the slot holds is stale
    p->slot_expert[h.slot] = -1;
    p->slot_used[h.slot] = 0;
    h.slot = -1;
  }
  h.codes = codes; h.step = step; h.salient = salient; h.sidx = salient_idx;
  return MES_OK;
}

int mes_pool_slot_of(const mes_pool* p, int expert) {
  if (!p || expert < 0 || expert >= p->n_experts) return -1;
  return p->experts[expert].slot;
}

mes_status mes_pool_stats(const mes_pool* p, uint64_t* hits, uint64_t* misses, uint64_t* bytes_copied) {
  if (!p) return mes::fail(MES_ERR_NULL, "mes_pool_stats: pool is null");
  if (hits) *hits = p->hits;
  if (misses) *misses = p->misses;
  if (bytes_copied) *bytes_copied = p->bytes;
  return MES_OK;
}

mes_status mes_pool_acquire(mes_pool* p, const int32_t* experts, int n, mes_delta* out, void* copy_stream,
                            void* compute_stream) {
  using namespace mes;
  if (!p || !experts || !out) return fail(MES_ERR_NULL, "mes_pool_acquire: null argument");
  if (n < 1 || n > p->n_slots) return fail(MES_ERR_SHAPE, "mes_pool_acquire: %d experts asked for, the pool has %d slots", n, p->n_slots);
  for (int i = 0; i < n; ++i) {
    const int e = experts[i];
    if (e < 0 || e >= p->n_experts) return fail(MES_ERR_SHAPE, "mes_pool_acquire: expert %d outside [0, %d)", e, p->n_experts);
    if (!p->experts[e].codes) return fail(MES_ERR_NULL, "mes_pool_acquire: expert %d was never registered", e);
    for (int j = 0; j < i; ++j)
      if (experts[j] == e) return fail(MES_ERR_SHAPE, "mes_pool_acquire: expert %d asked for twice", e);
  }
  hipStream_t cs = (hipStream_t)copy_stream, ks = (hipStream_t)compute_stream;
  // Every expert of this request is stamped with the same new clock value: none of them may be evicted for
  // another one of the same request.
  const uint64_t now = ++p->clock;
  for (int i = 0; i < n; ++i) {
    const int s = p->experts[experts[i]].slot;
    if (s >= 0) { p->slot_used[s] = now; ++p->hits; }
  }
  bool copied = false;
  for (int i = 0; i < n; ++i) {
    HostExpert& h = p->experts[experts[i]];
    if (h.slot < 0) {
      // victim: a free slot if there is one (never used: stamp 0), else the least recently used; lowest index wins ties
      int victim = -1;
      for (int s = 0; s < p->n_slots; ++s)
        if (p->slot_used[s] != now && (victim < 0 || p->slot_used[s] < p->slot_used[victim])) victim = s;
      if (victim < 0) return fail(MES_ERR_SHAPE, "mes_pool_acquire: no slot left (internal)");
      if (p->slot_expert[victim] >= 0) p->experts[p->slot_expert[victim]].slot = -1;
      char* dst = p->arena + (size_t)victim * p->lay.total;
      if (!p->dry_run) {
        hipError_t e = hipSuccess;
        if (!copied) {
          // the slot may still be read by kernels already enqueued on the compute stream: copies start after them
          e = hipEventRecord(p->ev_compute, ks);
          if (e == hipSuccess) e = hipStreamWaitEvent(cs, p->ev_compute, 0);
        }
        if (e == hipSuccess) e = hipMemcpyAsync(dst + p->lay.codes, h.codes, p->lay.codes_bytes, hipMemcpyHostToDevice, cs);
        if (e == hipSuccess) e = hipMemcpyAsync(dst + p->lay.step, h.step, p->lay.step_bytes, hipMemcpyHostToDevice, cs);
        if (e == hipSuccess && p->k > 0) e = hipMemcpyAsync(dst + p->lay.salient, h.salient, p->lay.salient_bytes, hipMemcpyHostToDevice, cs);
        if (e == hipSuccess && p->k > 0) e = hipMemcpyAsync(dst + p->lay.sidx, h.sidx, p->lay.sidx_bytes, hipMemcpyHostToDevice, cs);
        if (e != hipSuccess) {   // the slot's contents are undefined now
          p->slot_expert[victim] = -1; p->slot_used[victim] = 0;
          return check_hip(e, "mes_pool_acquire: copy");
        }
      }
      copied = true;
      p->slot_expert[victim] = experts[i];
      p->slot_used[victim] = now;
      h.slot = victim;
      ++p->misses;
      p->bytes += p->lay.codes_bytes + p->lay.step_bytes + (p->k > 0 ? p->lay.salient_bytes + p->lay.sidx_bytes : 0);
    }
    char* base = p->arena + (size_t)h.slot * p->lay.total;
    mes_delta& d = out[i];
    d.d_in = p->d_in; d.d_out = p->d_out; d.k = p->k; d.bits = p->bits; d.grid = p->grid;
    d.layout_version = MES_LAYOUT_VERSION;
    d.codes = base + p->lay.codes;
    d.step = reinterpret_cast<const float*>(base + p->lay.step);
    d.salient = p->k > 0 ? base + p->lay.salient : nullptr;
    d.salient_idx = p->k > 0 ? reinterpret_cast<const int32_t*>(base + p->lay.sidx) : nullptr;
  }
  if (copied && !p->dry_run) {
    hipError_t e = hipEventRecord(p->ev_copy, cs);
    if (e == hipSuccess) e = hipStreamWaitEvent(ks, p->ev_copy, 0);
    if (e != hipSuccess) return check_hip(e, "mes_pool_acquire: event");
  }
  return MES_OK;
}

}  // extern "C"
