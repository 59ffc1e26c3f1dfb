// On-demand swapping of compressed deltas (Section 4.1, paragraph "On-demand swapping": the pre-trained model
// stays in GPU memory, the compressed deltas of the experts a batch needs are loaded when they are needed).
//
// A pool serves one or several linear layers (up to a whole transformer block): `n_slots` device slots, each big
// enough for one expert's packed deltas of all of them (codes, steps, salient fp16 tile, salient indices per
// linear), carved out of an arena the caller owns; and up to `n_experts` registered experts whose packed buffers
// live in pinned host memory the caller owns -- best as one blob in the slot's own layout, so that a miss is a
// single copy.  acquire() makes a set of experts resident -- least recently used slots are overwritten, copies go
// out on a copy stream, the compute stream is made to wait for them -- and returns their descriptors for
// mes_delta_linear.  prefetch() starts such copies without making the compute stream wait, into slots the latest
// acquire did not hand out, so that they run under the kernels of the current batch.
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
  // either four separate pinned buffers per linear (four copies per linear and miss) ...
  std::vector<const void*> codes, salient;
  std::vector<const float*> step;
  std::vector<const int32_t*> sidx;
  // ... or one pinned blob in the slot's own layout (one copy per miss)
  const void* blob = nullptr;
  bool registered = false;
  int slot = -1;   // resident in this slot, or -1
};

}  // namespace
}  // namespace mes

struct mes_pool {
  int n_linears, bits, grid, n_slots, n_experts, dry_run;
  std::vector<int> d_in, d_out, k;
  std::vector<mes::SlotLayout> lay;    // per linear, offsets relative to the linear's part of the slot
  std::vector<size_t> lin_at;          // where each linear's part starts inside a slot
  size_t slot_bytes;
  char* arena;
  std::vector<mes::HostExpert> experts;
  std::vector<int> slot_expert;        // expert in the slot, or -1
  std::vector<uint64_t> slot_used;     // value of `clock` when the slot was last handed out or prefetched into (0: never)
  std::vector<char> slot_pending;      // a prefetch copy into the slot may still be in flight as far as the compute stream knows
  uint64_t clock, last_acquire, hits, misses, prefetched, bytes;
  hipEvent_t ev_compute, ev_copy;      // not created in a dry-run pool
  bool ev_compute_valid, ev_copy_valid;
};

namespace mes {
namespace {

size_t payload_bytes(const mes_pool* p) {
  size_t n = 0;
  for (int l = 0; l < p->n_linears; ++l)
    n += p->lay[l].codes_bytes + p->lay[l].step_bytes + (p->k[l] > 0 ? p->lay[l].salient_bytes + p->lay[l].sidx_bytes : 0);
  return n;
}

// Host -> slot copies of one expert, on `cs`.
hipError_t copy_in(const mes_pool* p, const HostExpert& h, int slot, hipStream_t cs) {
  char* dst = p->arena + (size_t)slot * p->slot_bytes;
  if (h.blob) return hipMemcpyAsync(dst, h.blob, p->slot_bytes, hipMemcpyHostToDevice, cs);
  hipError_t e = hipSuccess;
  for (int l = 0; l < p->n_linears && e == hipSuccess; ++l) {
    const SlotLayout& y = p->lay[l];
    char* d = dst + p->lin_at[l];
    e = hipMemcpyAsync(d + y.codes, h.codes[l], y.codes_bytes, hipMemcpyHostToDevice, cs);
    if (e == hipSuccess) e = hipMemcpyAsync(d + y.step, h.step[l], y.step_bytes, hipMemcpyHostToDevice, cs);
    if (e == hipSuccess && p->k[l] > 0) e = hipMemcpyAsync(d + y.salient, h.salient[l], y.salient_bytes, hipMemcpyHostToDevice, cs);
    if (e == hipSuccess && p->k[l] > 0) e = hipMemcpyAsync(d + y.sidx, h.sidx[l], y.sidx_bytes, hipMemcpyHostToDevice, cs);
  }
  return e;
}

void describe(const mes_pool* p, int slot, int l, mes_delta& d) {
  char* base = p->arena + (size_t)slot * p->slot_bytes + p->lin_at[l];
  const SlotLayout& y = p->lay[l];
  d.d_in = p->d_in[l]; d.d_out = p->d_out[l]; d.k = p->k[l]; d.bits = p->bits; d.grid = p->grid;
  d.layout_version = MES_LAYOUT_VERSION;
  d.codes = base + y.codes;
  d.step = reinterpret_cast<const float*>(base + y.step);
  d.salient = p->k[l] > 0 ? base + y.salient : nullptr;
  d.salient_idx = p->k[l] > 0 ? reinterpret_cast<const int32_t*>(base + y.sidx) : nullptr;
}

mes_status check_request(const mes_pool* p, const int32_t* experts, int n, const char* who) {
  if (n < 1 || n > p->n_slots) return fail(MES_ERR_SHAPE, "%s: %d experts asked for, the pool has %d slots", who, n, p->n_slots);
  for (int i = 0; i < n; ++i) {
    const int e = experts[i];
    if (e < 0 || e >= p->n_experts) return fail(MES_ERR_SHAPE, "%s: expert %d outside [0, %d)", who, e, p->n_experts);
    if (!p->experts[e].registered) return fail(MES_ERR_NULL, "%s: expert %d was never registered", who, e);
    for (int j = 0; j < i; ++j)
      if (experts[j] == e) return fail(MES_ERR_SHAPE, "%s: expert %d asked for twice", who, e);
  }
  return MES_OK;
}

void forget(mes_pool* p, int slot) {
  if (p->slot_expert[slot] >= 0) p->experts[p->slot_expert[slot]].slot = -1;
  p->slot_expert[slot] = -1;
  p->slot_used[slot] = 0;
  p->slot_pending[slot] = 0;
}

}  // namespace
}  // namespace mes

extern "C" {

size_t mes_pool_slot_layout(int d_in, int d_out, int k, int bits, size_t offsets_out[4]) {
  if (d_in <= 0 || d_out <= 0 || k < 0 || k > d_in || bits < 1 || bits > 4) return 0;
  const mes::SlotLayout y = mes::slot_layout(d_in, d_out, k, bits);
  if (offsets_out) { offsets_out[0] = y.codes; offsets_out[1] = y.step; offsets_out[2] = y.salient; offsets_out[3] = y.sidx; }
  return y.total;
}

size_t mes_pool_slot_bytes(int d_in, int d_out, int k, int bits) { return mes_pool_slot_layout(d_in, d_out, k, bits, nullptr); }

size_t mes_pool_multi_slot_bytes(int n_linears, const int32_t* d_in, const int32_t* d_out, const int32_t* k, int bits) {
  if (n_linears < 1 || n_linears > MES_POOL_MAX_LINEARS || !d_in || !d_out || !k) return 0;
  size_t n = 0;
  for (int l = 0; l < n_linears; ++l) {
    const size_t b = mes_pool_slot_bytes(d_in[l], d_out[l], k[l], bits);
    if (b == 0) return 0;
    n += b;
  }
  return n;
}

mes_status mes_pool_create_multi(int n_linears, const int32_t* d_in, const int32_t* d_out, const int32_t* k, int bits, int grid,
                                 int n_slots, int n_experts, void* arena, size_t arena_bytes, int dry_run, mes_pool** out) {
  using namespace mes;
  if (!out) return fail(MES_ERR_NULL, "mes_pool_create: out is null");
  *out = nullptr;
  if (n_linears < 1 || n_linears > MES_POOL_MAX_LINEARS)
    return fail(MES_ERR_SHAPE, "mes_pool_create: n_linears = %d outside [1, %d]", n_linears, MES_POOL_MAX_LINEARS);
  if (!d_in || !d_out || !k) return fail(MES_ERR_NULL, "mes_pool_create: shape array is null");
  if (bits < 1 || bits > 4 || (grid != MES_GRID_SYM && grid != MES_GRID_EQ1) || (grid == MES_GRID_EQ1 && bits == 1))
    return fail(MES_ERR_BITS, "mes_pool_create: bits %d / grid %d not supported", bits, grid);
  for (int l = 0; l < n_linears; ++l) {
    if (d_in[l] <= 0 || d_out[l] <= 0 || d_in[l] % 8 != 0 || d_out[l] % 4 != 0)
      return fail(MES_ERR_SHAPE, "mes_pool_create: bad shape %d x %d", d_out[l], d_in[l]);
    if (k[l] < 0 || k[l] > d_in[l]) return fail(MES_ERR_SALIENT, "mes_pool_create: k = %d outside [0, d_in]", k[l]);
  }
  if (n_slots < 1 || n_slots > MES_MAX_EXPERTS || n_experts < 1)
    return fail(MES_ERR_SHAPE, "mes_pool_create: n_slots must be 1..%d and n_experts positive", MES_MAX_EXPERTS);
  const size_t slot_bytes = mes_pool_multi_slot_bytes(n_linears, d_in, d_out, k, bits);
  if (!arena) return fail(MES_ERR_NULL, "mes_pool_create: arena is null");
  if (reinterpret_cast<uintptr_t>(arena) % kSlotAlign) return fail(MES_ERR_ALIGN, "mes_pool_create: arena must be 256-byte aligned");
  if (arena_bytes < slot_bytes * (size_t)n_slots)
    return fail(MES_ERR_WORKSPACE, "mes_pool_create: arena of %zu bytes, %zu needed", arena_bytes, slot_bytes * (size_t)n_slots);
  mes_pool* p = new (std::nothrow) mes_pool();
  if (!p) return fail(MES_ERR_DEVICE, "mes_pool_create: out of host memory");
  p->n_linears = n_linears; p->bits = bits; p->grid = grid;
  p->n_slots = n_slots; p->n_experts = n_experts; p->dry_run = dry_run;
  size_t at = 0;
  for (int l = 0; l < n_linears; ++l) {
    p->d_in.push_back(d_in[l]); p->d_out.push_back(d_out[l]); p->k.push_back(k[l]);
    p->lay.push_back(slot_layout(d_in[l], d_out[l], k[l], bits));
    p->lin_at.push_back(at);
    at += p->lay.back().total;
  }
  p->slot_bytes = slot_bytes;
  p->arena = reinterpret_cast<char*>(arena);
  p->experts.assign(n_experts, HostExpert());
  p->slot_expert.assign(n_slots, -1);
  p->slot_used.assign(n_slots, 0);
  p->slot_pending.assign(n_slots, 0);
  p->clock = p->last_acquire = p->hits = p->misses = p->prefetched = p->bytes = 0;
  p->ev_compute = p->ev_copy = nullptr;
  p->ev_compute_valid = p->ev_copy_valid = false;
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

mes_status mes_pool_create(int d_in, int d_out, int k, int bits, int grid, int n_slots, int n_experts, void* arena,
                           size_t arena_bytes, int dry_run, mes_pool** out) {
  const int32_t di = d_in, dn = d_out, kk = k;
  return mes_pool_create_multi(1, &di, &dn, &kk, bits, grid, n_slots, n_experts, arena, arena_bytes, dry_run, out);
}

void mes_pool_destroy(mes_pool* p) {
  if (!p) return;
  if (p->ev_compute) (void)hipEventDestroy(p->ev_compute);
  if (p->ev_copy) (void)hipEventDestroy(p->ev_copy);
  delete p;
}

size_t mes_pool_linear_offset(const mes_pool* p, int linear) {
  if (!p || linear < 0 || linear >= p->n_linears) return 0;
  return p->lin_at[linear];
}

static mes_status register_common(mes_pool* p, int expert, const char* who) {
  using namespace mes;
  if (!p) return fail(MES_ERR_NULL, "%s: pool is null", who);
  if (expert < 0 || expert >= p->n_experts) return fail(MES_ERR_SHAPE, "%s: expert %d outside [0, %d)", who, expert, p->n_experts);
  return MES_OK;
}

mes_status mes_pool_register(mes_pool* p, int expert, const void* codes, const float* step, const void* salient,
                             const int32_t* salient_idx) {
  using namespace mes;
  if (mes_status st = register_common(p, expert, "mes_pool_register")) return st;
  if (p->n_linears != 1) return fail(MES_ERR_SHAPE, "mes_pool_register: the pool spans %d linear layers; register a blob", p->n_linears);
  if (!codes || !step || (p->k[0] > 0 && (!salient || !salient_idx))) return fail(MES_ERR_NULL, "mes_pool_register: null host buffer");
  HostExpert& h = p->experts[expert];
  if (h.slot >= 0) forget(p, h.slot);   // new contents: what the slot holds is stale
  h.codes.assign(1, codes); h.step.assign(1, step); h.salient.assign(1, salient); h.sidx.assign(1, salient_idx);
  h.blob = nullptr;
  h.registered = true;
  return MES_OK;
}

mes_status mes_pool_register_blob(mes_pool* p, int expert, const void* host_blob) {
  using namespace mes;
  if (mes_status st = register_common(p, expert, "mes_pool_register_blob")) return st;
  if (!host_blob) return fail(MES_ERR_NULL, "mes_pool_register_blob: null host buffer");
  if (reinterpret_cast<uintptr_t>(host_blob) % 16) return fail(MES_ERR_ALIGN, "mes_pool_register_blob: the blob must be 16-byte aligned");
  HostExpert& h = p->experts[expert];
  if (h.slot >= 0) forget(p, h.slot);
  h.codes.clear(); h.step.clear(); h.salient.clear(); h.sidx.clear();
  h.blob = host_blob;
  h.registered = true;
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

uint64_t mes_pool_prefetched(const mes_pool* p) { return p ? p->prefetched : 0; }

mes_status mes_pool_acquire_multi(mes_pool* p, const int32_t* experts, int n, mes_delta* out, void* copy_stream,
                                  void* compute_stream) {
  using namespace mes;
  if (!p || !experts || !out) return fail(MES_ERR_NULL, "mes_pool_acquire: null argument");
  if (mes_status st = check_request(p, experts, n, "mes_pool_acquire")) return st;
  hipStream_t cs = (hipStream_t)copy_stream, ks = (hipStream_t)compute_stream;
  // Every expert of this request is stamped with the same new clock value: none of them may be evicted for
  // another one of the same request.
  const uint64_t now = ++p->clock;
  p->last_acquire = now;
  if (!p->dry_run) {
    // Everything enqueued on the compute stream so far may still read any slot handed out earlier: copies into
    // such slots (this call's misses, later prefetches) start after this point of the compute stream.
    if (mes_status st = check_hip(hipEventRecord(p->ev_compute, ks), "mes_pool_acquire: event")) return st;
    p->ev_compute_valid = true;
  }
  bool must_wait = false;   // does the compute stream have to wait for the copy stream?
  for (int i = 0; i < n; ++i) {
    const int s = p->experts[experts[i]].slot;
    if (s >= 0) {
      p->slot_used[s] = now;
      ++p->hits;
      must_wait = must_wait || p->slot_pending[s];
    }
  }
  bool copied = false;
  std::vector<int> loaded;   // slots this call copied into (forgotten again if a copy fails)
  for (int i = 0; i < n; ++i) {
    HostExpert& h = p->experts[experts[i]];
    if (h.slot < 0) {
      // victim: a free slot if there is one (never used: stamp 0), else the least recently used; lowest index wins ties
      int victim = -1;
      for (int s = 0; s < p->n_slots; ++s)
        if (p->slot_used[s] != now && (victim < 0 || p->slot_used[s] < p->slot_used[victim])) victim = s;
      if (victim < 0) return fail(MES_ERR_SHAPE, "mes_pool_acquire: no slot left (internal)");
      forget(p, victim);
      if (!p->dry_run) {
        hipError_t e = hipSuccess;
        if (!copied) e = hipStreamWaitEvent(cs, p->ev_compute, 0);
        if (e == hipSuccess) e = copy_in(p, h, victim, cs);
        if (e != hipSuccess) {
          // Nothing of this call may be taken for resident: the failed slot is undefined and the compute stream
          // has not been told to wait for the copies that did go out.
          for (int s : loaded) forget(p, s);
          return check_hip(e, "mes_pool_acquire: copy");
        }
      }
      copied = true;
      loaded.push_back(victim);
      p->slot_expert[victim] = experts[i];
      p->slot_used[victim] = now;
      h.slot = victim;
      ++p->misses;
      p->bytes += payload_bytes(p);
    }
    for (int l = 0; l < p->n_linears; ++l) describe(p, h.slot, l, out[(size_t)l * n + i]);
  }
  if (!p->dry_run && (copied || must_wait)) {
    hipError_t e = hipSuccess;
    if (copied) {
      e = hipEventRecord(p->ev_copy, cs);
      p->ev_copy_valid = p->ev_copy_valid || e == hipSuccess;
    }
    // the latest event of the copy stream covers every copy issued before it, prefetches included
    if (e == hipSuccess && p->ev_copy_valid) e = hipStreamWaitEvent(ks, p->ev_copy, 0);
    if (e != hipSuccess) {
      for (int s : loaded) forget(p, s);
      return check_hip(e, "mes_pool_acquire: event");
    }
    for (int s = 0; s < p->n_slots; ++s) p->slot_pending[s] = 0;
  } else if (p->dry_run) {
    for (int s = 0; s < p->n_slots; ++s) p->slot_pending[s] = 0;
  }
  return MES_OK;
}

mes_status mes_pool_acquire(mes_pool* p, const int32_t* experts, int n, mes_delta* out, void* copy_stream,
                            void* compute_stream) {
  if (p && p->n_linears != 1)
    return mes::fail(MES_ERR_SHAPE, "mes_pool_acquire: the pool spans %d linear layers; use mes_pool_acquire_multi", p->n_linears);
  return mes_pool_acquire_multi(p, experts, n, out, copy_stream, compute_stream);
}

mes_status mes_pool_prefetch(mes_pool* p, const int32_t* experts, int n, int* n_loaded, void* copy_stream) {
  using namespace mes;
  if (n_loaded) *n_loaded = 0;
  if (!p || !experts) return fail(MES_ERR_NULL, "mes_pool_prefetch: null argument");
  if (mes_status st = check_request(p, experts, n, "mes_pool_prefetch")) return st;
  hipStream_t cs = (hipStream_t)copy_stream;
  const uint64_t now = ++p->clock;
  for (int i = 0; i < n; ++i) {   // resident ones first: they must not be the victims of the others
    const int s = p->experts[experts[i]].slot;
    if (s >= 0) p->slot_used[s] = now;
  }
  bool copied = false;
  int loaded = 0;
  hipError_t e = hipSuccess;
  for (int i = 0; i < n && e == hipSuccess; ++i) {
    HostExpert& h = p->experts[experts[i]];
    if (h.slot >= 0) continue;
    // Only slots that the latest acquire did not hand out (and no prefetch since has filled) may go: the kernels
    // that read them were enqueued before that acquire, and its event on the compute stream covers them.
    int victim = -1;
    for (int s = 0; s < p->n_slots; ++s)
      if ((p->slot_used[s] == 0 || p->slot_used[s] < p->last_acquire) && (victim < 0 || p->slot_used[s] < p->slot_used[victim])) victim = s;
    if (victim < 0) continue;   // best effort: this expert will be a miss of its acquire
    forget(p, victim);
    if (!p->dry_run) {
      if (!copied && p->ev_compute_valid) e = hipStreamWaitEvent(cs, p->ev_compute, 0);
      if (e == hipSuccess) e = copy_in(p, h, victim, cs);
      if (e != hipSuccess) break;
    }
    copied = true;
    p->slot_expert[victim] = experts[i];
    p->slot_used[victim] = now;
    p->slot_pending[victim] = 1;
    h.slot = victim;
    ++loaded;
    ++p->prefetched;
    p->bytes += payload_bytes(p);
  }
  if (!p->dry_run && copied && e == hipSuccess) {
    e = hipEventRecord(p->ev_copy, cs);
    p->ev_copy_valid = p->ev_copy_valid || e == hipSuccess;
  }
  if (e != hipSuccess) {
    // the copies that went out cannot be waited for by event: nothing this call touched counts as resident
    for (int s = 0; s < p->n_slots; ++s)
      if (p->slot_used[s] == now && p->slot_pending[s]) forget(p, s);
    return check_hip(e, "mes_pool_prefetch: copy");
  }
  if (n_loaded) *n_loaded = loaded;
  return MES_OK;
}

}  // extern "C"
