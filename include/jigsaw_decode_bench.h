/*
 * jigsaw_decode_bench.h -- inspection and measurement entry points of libjigsaw_decode.
 *
 * Nothing here is needed to run a decode step: these calls let tests look at the work partition
 * the decode kernel computes, give benchmarks plain streaming kernels of known traffic, and keep the
 * vector-ALU kernels that the matrix-core kernel was measured against runnable beside it.  They
 * synchronise, copy to the host or allocate where the comments say so; the product calls in
 * jigsaw_decode.h never do.
 */
#ifndef JIGSAW_DECODE_BENCH_H
#define JIGSAW_DECODE_BENCH_H

#include "jigsaw_decode.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Run only the work partitioner of the decode kernel for seq_lens (device, int32 [B]) and copy its
 * tables to the host (synchronises `stream`).  The partition answers, inside one GPU, the imbalance
 * the paper describes for rollout (Motivation, "Varied Decoding Lengths"): the step's work is cut,
 * not its requests.  Waves work in groups of `group_waves`: member i of a group serves the kv heads
 * i, i + group_waves, ...; the work of a step is the line of group-units (request, kv-head group,
 * page), request-major, then kv-head group, then page, and a group of waves owns one span of it.
 *   header_host      int32 [8]: {units, span, active_groups, wave_slots, group_waves, 0, 0, 0}
 *                    units = sum over requests of ceil(L/16) * Hkv / group_waves;
 *                    group g < active_groups owns units [g*span, min((g+1)*span, units)) and consists of
 *                    waves g*group_waves .. (g+1)*group_waves - 1
 *   wave_start_host  int32 [wave_slots * 4]: {request, kv_head, page, 0} of the first page each wave of an
 *                    active group works on (zeros for the others)
 *   cum_pages_host   int32 [B + 1]: pages of all requests before b (exclusive prefix of ceil(L/16))
 * Any of the three host pointers may be NULL.
 */
jd_status jd_debug_partition(jd_handle *h, const int32_t *seq_lens, int32_t *header_host,
                             int32_t *wave_start_host, int32_t *cum_pages_host, void *stream);

/*
 * The schedule for a work line of `units` group-units and `groups` groups of waves, as the kernel
 * computes it: out = {span, active_groups} (see jd_debug_partition).  Pure host function.
 */
jd_status jd_debug_schedule(int32_t units, int32_t groups, int32_t out[2]);

/* Number of wave slots the decode kernel of this handle is launched with (grid waves). */
int32_t jd_wave_slots(const jd_handle *h);

/*
 * Plain streaming kernels of known HBM traffic, for benchmarks and for scaling profiler byte
 * counters: a read-only sweep of `bytes` bytes at src (sink: 4 writable device bytes, practically
 * never written) and a copy of `bytes` bytes.  Device pointers, 16-byte aligned; bytes is rounded
 * down to a multiple of 16.  They only enqueue on `stream`.
 */
jd_status jd_debug_stream_read(const void *src, size_t bytes, void *sink, void *stream);
jd_status jd_debug_stream_copy(void *dst, const void *src, size_t bytes, void *stream);

/*
 * A stream whose kernels may only use `num_cus` of the device's compute units (a multiple of 64, at
 * most all: the units are taken evenly from the 8 dies), at the default priority: the
 * stand-in for the SM partitions the paper runs co-located sub-stages in (Sub-stage Multiplexing,
 * "Dynamic Resource Allocation").  A handle created with cu_budget = num_cus launches one workgroup
 * per unit of such a stream.  JD_ERR_INVALID_ARG for a count outside that set, JD_ERR_HIP if the
 * runtime refuses the stream.  Destroy it with jd_bench_stream_destroy once its work has completed.
 */
jd_status jd_bench_stream_create_cu_masked(int32_t num_cus, void **stream_out);
jd_status jd_bench_stream_destroy(void *stream);

/*
 * The decode step of jd_decode_attention, with the same arguments, layouts and result, computed by the
 * vector-ALU kernels the matrix-core kernel was measured against: a single-block partition kernel, a
 * split-KV partial pass with bf16-pair dot products and cross-lane adds, and a separate combine
 * kernel (three launches).  Group sizes 1, 2, 4, 7 and 8 only (JD_ERR_UNSUPPORTED otherwise).  The
 * first call on a handle allocates a second workspace with hipMalloc and synchronises the device;
 * it is freed by jd_destroy.  Not part of the product path.
 */
jd_status jd_bench_decode_attention_vector(jd_handle *h, const void *q, const void *k_pages, const void *v_pages,
                                           const int32_t *block_table, const int32_t *seq_lens, float *out,
                                           void *stream);

#ifdef __cplusplus
}
#endif
#endif /* JIGSAW_DECODE_BENCH_H */
