/*
 * jigsaw_decode.h -- C ABI of libjigsaw_decode: paged decode attention for rollout
 * batches with ragged, long-tailed sequence lengths, on one MI355X (gfx950).
 *
 * The operation is the attention part of one rollout decode forward step.  The paper
 * delegates rollout to an inference engine and prints no attention formula; what it
 * fixes is the setting this library is built for: every forward step processes the
 * active decoding requests (System Design, "Sub-Stage Graph Abstraction"), the KV cache
 * is the memory object that bounds them (Sub-stage Multiplexing, "GPU Memory
 * Utilization"), decoding is memory-bound (Motivation, "Multi-turn Rollout Idling";
 * Sub-stage Multiplexing, "Compute Resource Utilization") and a few long sequences
 * dominate the step while the effective batch shrinks (Motivation, "Varied Decoding
 * Lengths").  For request b with L = seq_lens[b] tokens, query head h and kv head
 * kv = h / (num_q_heads / num_kv_heads):
 *
 *     s_j   = softmax_scale * <q[b][h], K_j>           j = 0 .. L-1
 *     out[b][h] = sum_j softmax(s)_j * V_j
 *
 * where token j of request b is row (j % 16) of kv head `kv` in physical page
 * block_table[b][j / 16].  K/V are bf16, products and sums are fp32, out is fp32.
 *
 * All pointers passed to jd_decode_attention are DEVICE pointers owned by the caller
 * (for example PyTorch tensors); the library reads q/k_pages/v_pages/block_table/
 * seq_lens and writes out.  The handle and a private device workspace are owned by the
 * library.  No function throws or aborts; every failure is a status code plus a message
 * retrievable with jd_last_error_string.
 */
#ifndef JIGSAW_DECODE_H
#define JIGSAW_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct jd_handle jd_handle;

typedef enum {
    JD_OK = 0,
    JD_ERR_INVALID_ARG = 1, /* null pointer, misaligned buffer, non-positive size, heads not divisible */
    JD_ERR_UNSUPPORTED = 2, /* head_dim not in {64,128}, page_size != 16, group size > 16, batch > 8192 */
    JD_ERR_HIP = 3,         /* a HIP runtime call or kernel launch failed */
    JD_ERR_BAD_INPUT = 4    /* device-side check: a page id, sequence length or query offset outside the declared bounds */
} jd_status;

typedef struct {
    int32_t batch;             /* B: rows of q/out/block_table/seq_lens, at most 8192 (the work partition keeps its
                                  tables in LDS; more is JD_ERR_UNSUPPORTED); requests with seq_len 0 are skipped */
    int32_t num_q_heads;       /* Hq */
    int32_t num_kv_heads;      /* Hkv; must divide Hq; query head h reads kv head h / (Hq / Hkv) */
    int32_t head_dim;          /* D: 64 or 128 */
    int32_t page_size;         /* tokens per page: 16 */
    int32_t max_pages_per_seq; /* MAXP: row stride (in entries) of block_table */
    int32_t num_pages;         /* NP: pages in k_pages / v_pages; page ids are checked against it */
    float softmax_scale;       /* 0 means 1 / sqrt(D) */
    int32_t cu_budget;         /* 0: the library's choice (three quarters of the compute units with head_dim 128,
                                  13/16 of them with head_dim 64: that already saturates HBM); otherwise the number of
                                  one-per-compute-unit workgroups the decode kernel is launched with (spatial
                                  sharing with a co-located job; Sub-stage Multiplexing, "Dynamic Resource
                                  Allocation") */
} jd_config;

/*
 * Pure host check of a configuration; touches no GPU.  Returns JD_OK, JD_ERR_INVALID_ARG
 * or JD_ERR_UNSUPPORTED.
 */
jd_status jd_validate_config(const jd_config *cfg);

/*
 * Bytes of device workspace a handle for `cfg` holds on a 256-compute-unit device (work-partition
 * tables and split-KV partial states; a device with fewer units needs less).  Pure host function;
 * 0 if cfg is invalid.
 */
size_t jd_workspace_bytes(const jd_config *cfg);

/*
 * Create a handle on the current HIP device.  Validates cfg (no GPU touched on failure),
 * then allocates the workspace once with hipMalloc.  *out is set only on JD_OK.  Every later
 * call that takes the handle must be made with that device current (JD_ERR_INVALID_ARG
 * otherwise).  A handle is not thread-safe: calls on one handle come from one thread at a time.
 */
jd_status jd_create(const jd_config *cfg, jd_handle **out);

/*
 * One decode step's attention for the whole batch (one transformer layer).
 *   q           bf16 [B, Hq, D]            device, 16-byte aligned, read
 *   k_pages     bf16 [NP, Hkv, 16, D]      device, 16-byte aligned, read
 *   v_pages     bf16 [NP, Hkv, 16, D]      device, 16-byte aligned, read
 *   block_table int32 [B, MAXP]            device, read; entry j of row b is the physical page of tokens
 *                                          16j..16j+15; entries at or beyond ceil(L/16) are never read
 *   seq_lens    int32 [B]                  device, read; tokens per request INCLUDING the one being decoded
 *                                          (its K/V are already in the cache); <= 0 gives a zero output row
 *   out         fp32 [B, Hq, D]            device, 16-byte aligned, written (every row)
 *   stream      a hipStream_t (NULL = the default stream)
 * Slots beyond L in a last page, pages no request owns and unused block-table entries never
 * influence the result, whatever bits they hold.  The call only enqueues work (work partition,
 * split-KV partial pass, log-sum-exp combine) on `stream`; it performs no allocation, no host
 * synchronisation and no device-to-host copy, so it may be captured into a HIP graph.  Calls on
 * one handle share its workspace: they must be ordered on one stream (or otherwise serialised), and
 * seq_lens must not change while a call that reads it is running.
 * Page ids outside [0, NP) and lengths beyond 16*MAXP are never dereferenced: the offending page is
 * replaced by page 0 / the length clamped (the affected rows are then meaningless) and a sticky flag
 * is raised that jd_check_device_flags reports.
 */
jd_status jd_decode_attention(jd_handle *h, const void *q, const void *k_pages, const void *v_pages,
                              const int32_t *block_table, const int32_t *seq_lens, float *out,
                              void *stream);

/*
 * jd_decode_attention for callers that cannot allocate device memory or hold a handle: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, arguments,
 * layouts and result as jd_decode_attention on a handle created with `cfg` (the kernels are the same);
 * what the handle keeps in its allocated workspace (work-partition tables, arrival counters, split-KV
 * partial records) lives in a 12 MiB array in the library's device image instead, of which every GPU
 * the process uses holds its own copy until the process ends.  The call allocates nothing and frees
 * nothing, on the device or through any library, and only enqueues on `stream` (a small kernel that
 * clears the counters the array kept from the previous call, then the decode kernel).
 *   JD_ERR_UNSUPPORTED   cfg needs more workspace than the array holds (the message says how much; all
 *                        benchmark shapes fit; a group size of 16 with head_dim 128 on all compute units
 *                        does not), or any reason jd_create would give
 *   JD_ERR_INVALID_ARG   as for jd_decode_attention; also when the first call on a device comes inside a
 *                        stream capture (that call resolves the array's address, which cannot be captured)
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race; order them.  Device-side input checks keep every access in bounds as in
 * jd_decode_attention, but their sticky flag is cleared by the next call and reported nowhere.
 */
jd_status jd_decode_attention_static(const jd_config *cfg, const void *q, const void *k_pages, const void *v_pages,
                                     const int32_t *block_table, const int32_t *seq_lens, float *out,
                                     void *stream);

/*
 * The write half of a decode step: append one token per active request to the paged cache and
 * bump its length, so that the jd_decode_attention call that follows attends over it (a decode
 * forward step processes the active decoding requests and grows their KV cache by one token:
 * System Design, "Sub-Stage Graph Abstraction"; Sub-stage Multiplexing, "GPU Memory Utilization").
 *   k_new, v_new  bf16 [B, Hkv, D]        device, 16-byte aligned, read: the new token's rows
 *   k_pages, v_pages  bf16 [NP, Hkv, 16, D]   device, 16-byte aligned, written in place
 *   block_table   int32 [B, MAXP]          device, read; the page of slot L must already be assigned
 *   seq_lens      int32 [B]                device, read and written: L -> L + 1 for active requests
 *   active        int32 [B] or NULL        device, read; non-zero = append.  NULL: every request
 *                                          with L > 0 appends (rows with L = 0 are finished slots)
 * For an active request with L tokens the rows go to slot L % 16 of page block_table[b][L / 16].
 * A request whose next slot lies beyond 16*MAXP, or whose page id is outside [0, NP), is left
 * unchanged and raises the sticky flag reported by jd_check_device_flags.  Only enqueues on
 * `stream`; may be captured into a HIP graph together with jd_decode_attention.
 */
jd_status jd_append_kv(jd_handle *h, const void *k_new, const void *v_new, void *k_pages, void *v_pages,
                       const int32_t *block_table, int32_t *seq_lens, const int32_t *active, void *stream);

/*
 * Causal attention of a chunk of new tokens over the paged cache: prefill of a prompt or of a new
 * turn, and the KV recomputation a migrated request pays (Sub-stage Merging: the migration overhead
 * is dominated by KV cache recomputation; Motivation, "Multi-turn Rollout Idling": new turns trigger
 * additional prefill).  Request b has L = seq_lens[b] tokens in the cache, the last n = q_lens[b]
 * of which are the new ones (their K/V are already in place); new token t sits at position
 * L - n + t and attends to positions 0 .. L - n + t.
 *   q           bf16 [TQ, Hq, D]           device, 16-byte aligned, read; request b's new tokens are rows
 *                                          q_offsets[b] .. q_offsets[b] + n - 1
 *   k_pages, v_pages, block_table, seq_lens   as for jd_decode_attention
 *   q_lens      int32 [B]                  device, read; 0 = nothing to do for the request; values above L
 *                                          are clamped to L
 *   q_offsets   int32 [B]                  device, read; the rows of different requests must not overlap
 *   total_q_rows  host value: TQ, the rows q and out hold.  A request whose rows q_offsets[b] .. q_offsets[b]+n-1
 *                                          do not lie inside [0, TQ) is skipped (nothing of it is read or written)
 *                                          and raises the sticky flag reported by jd_check_device_flags
 *   max_q_len   host value: an upper bound of q_lens (it sizes the launch; tokens beyond it are not computed)
 *   out         fp32 [TQ, Hq, D]           device, 16-byte aligned; the rows of the new tokens are written,
 *                                          all others are left untouched
 * With n = 1 for every request the result is that of jd_decode_attention.  Only enqueues on `stream`
 * (no allocation, no host synchronisation), so it may be captured into a HIP graph; a captured launch is
 * sized by the max_q_len given at capture time.  Uses the handle's workspace like the other calls.
 * Bound by the matrix cores rather than by HBM; same input checks and flags as jd_decode_attention.
 */
jd_status jd_prefill_attention(jd_handle *h, const void *q, const void *k_pages, const void *v_pages,
                               const int32_t *block_table, const int32_t *seq_lens, const int32_t *q_lens,
                               const int32_t *q_offsets, int32_t total_q_rows, int32_t max_q_len, float *out,
                               void *stream);

/*
 * Synchronise `stream` and report device-side input checks of the calls completed so far:
 * JD_OK, JD_ERR_BAD_INPUT (and clears the flag) or JD_ERR_HIP.  The message names what was seen: a
 * sequence length beyond 16*MAXP (clamped), a page id outside [0, NP) (page 0 read or the append
 * skipped), seq_lens changed while a decode kernel was running (rows meaningless), prefill rows
 * outside [0, TQ) (request skipped).
 */
jd_status jd_check_device_flags(jd_handle *h, void *stream);

/* Free the workspace and the handle.  NULL is accepted. */
jd_status jd_destroy(jd_handle *h);

/*
 * Message of the last failure on this handle; with NULL, of the last failed jd_create /
 * jd_validate_config on the calling thread.  Never NULL; valid until the next call.
 */
const char *jd_last_error_string(const jd_handle *h);

#ifdef __cplusplus
}
#endif
#endif /* JIGSAW_DECODE_H */
