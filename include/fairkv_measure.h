/* fairkv_measure.h: measurement aids of libfairkv.  Nothing here is part of the method: these entry points exist so
 * that the benchmark can say where the time of a launch goes and what the data path reaches with nothing to do.
 * Same conventions as fairkv.h (plain pointers and sizes, status codes, nothing allocated, nothing synchronised). */
#ifndef FAIRKV_MEASURE_H
#define FAIRKV_MEASURE_H

#include "fairkv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid, not part of the method: fairkv_decode_attn (bf16 in, fp32 out, D = 128, G = 4 or 8; else
 * FAIRKV_EUNSUPPORTED) through an instantiation of the same kernel
 * that also stamps the phases of every workgroup with the GPU's 100 MHz wall clock.
 * trace: device, FAIRKV_TRACE_STAMPS uint64 per workgroup (trace_bytes >= n_slots * FAIRKV_TRACE_STAMPS * 8, else
 * FAIRKV_EINVAL), zero-filled by the caller; stamp k of workgroup j is trace[j * FAIRKV_TRACE_STAMPS + k]:
 * 0 first instruction, 1 item list landed and checked, 2 first K/V tile landed, 3 first item streamed (wave 0),
 * 4 first item folded and written, 5 last item streamed (wave 0), 6 hand-over begins, 7 partial results' stores
 * issued, 8 counted in, 9 merges done, 10 hand-over ends (6-10: the workgroup's last hand-over; 0 if it had none),
 * 11 last instruction.  bench.py --phases turns one launch's stamps into the phase table under profiles/. */
enum { FAIRKV_TRACE_STAMPS = 16 };
int fairkv_decode_attn_trace(const void *q, const void *k, const void *v, int64_t n_rows,
                             const fairkv_item *items, const fairkv_item *items_host, int32_t n_items,
                             const int32_t *slot_ptr, int32_t n_slots, int32_t n_parts, void *workspace,
                             size_t workspace_bytes, void *out, float *lse, int32_t B, int32_t Hq, int32_t Hkv, int32_t D,
                             float scale, uint64_t *trace, size_t trace_bytes, void *hip_stream);

/* Measurement aid, not part of the method: n_workgroups workgroups stream the first bytes_each
 * bytes (rounded down to a multiple of 4096 * n_workgroups) of the device buffers k and v from HBM
 * into LDS through the decode kernel's data path and discard them.  The time of this launch is what
 * a reader without any work achieves for that many bytes; bench.py reports the decode kernel
 * against it.  sink: any device buffer of n_workgroups words (never written).  No synchronisation. */
int fairkv_stream_probe(const void *k, const void *v, int64_t bytes_each, int32_t n_workgroups, void *sink,
                        void *hip_stream);

/* The same reader in another launch shape, for sweeping what the data path can reach: `waves` waves per workgroup
 * (4, 8 or 16), each with a ring of `stages` stages (2, 3 or 4) of tile_kib KiB of K plus tile_kib KiB of V (2, 4 or
 * 8); fairkv_stream_probe is (4, 2, 4), the decode kernel's shape.  bytes_each is rounded down to a multiple of
 * tile_kib * 1024 * n_workgroups.  FAIRKV_EUNSUPPORTED for other values or when the rings exceed the 160 KB of LDS
 * of a compute unit.  More workgroups than compute units share a compute unit when their rings fit side by side. */
int fairkv_stream_probe_shape(const void *k, const void *v, int64_t bytes_each, int32_t n_workgroups, int32_t waves,
                              int32_t stages, int32_t tile_kib, void *sink, void *hip_stream);

#ifdef __cplusplus
}
#endif

#endif /* FAIRKV_MEASURE_H */
