/*
 * mes_bench.h -- measurement helpers of libmes.  NOT part of the product ABI (include/mes.h): nothing that
 * serves requests needs them.  They exist so that a benchmark can time the library's dominant kernel on the
 * kernel's own stream and scale a profiler's memory-traffic counters; both are exported by the same shared
 * library because the timing hook has to sit between the kernels of one call.
 */
#ifndef MES_BENCH_H
#define MES_BENCH_H

#include <stddef.h>

#include "mes.h"

#ifdef __cplusplus
extern "C" {
#endif

/* The NEXT mes_delta_linear / mes_delta_linear_multi / mes_step_grad call of the calling thread records
 * `start_event` on its stream immediately before its first streaming (or contraction) kernel and `stop_event`
 * immediately after its last one (hipEvent_t passed as void*, HOST handles owned by the caller).  A decode call of
 * at most 256 tokens has exactly one streaming kernel between the two; a larger batch also has the helper
 * kernels of its later token groups in between.  One-shot: the call consumes the events on every exit path, also
 * when it fails its argument checks or has no tokens.  Two NULLs cancel. */
mes_status mes_time_next_call(void* start_event, void* stop_event);

/* A plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers DEVICE, 16-byte aligned, not
 * overlapping) done by one kernel, k_copy_probe.  It reads and writes exactly `bytes` of HBM, which is what a
 * profiler's memory-traffic counters are scaled by before they are compared with a kernel's algorithmic bytes. */
mes_status mes_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MES_BENCH_H */
