/*
 * gqa_decode.h -- C ABI of the MI355X (gfx950) grouped-query decode-attention library.
 *
 * One call = the attention of ONE decode step of ONE transformer layer: every
 * sequence b of a batch contributes one new query token that attends over all
 * kv_lens[b] cached key/value rows of that sequence (the newest token's K/V
 * are already in the cache, so no mask is applied).
 *
 * Why this operator: the method of the paper spends its run time letting a 32B
 * grouped-query reasoning model write traces of thousands of tokens, several
 * samples per task (Section 3.3; Table 3 gives average trace lengths of
 * 6-7 thousand tokens, Section 4.1 a maximum of 32,768).  Every generated
 * token re-reads the whole KV cache of its sequence in every layer, which makes
 * this HBM-bound operator the hot loop.  The paper defines no attention
 * variant of its own; what is computed is standard softmax attention:
 *
 *     g        = h / (num_q_heads / num_kv_heads)          (contiguous head groups)
 *     s_j      = scale * sum_d Q[b,h,d] * K[b,j,g,d]        j in [0, kv_lens[b])
 *     p_j      = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j)
 *     out[b,h,d] = sum_j p_j * V[b,j,g,d]
 *     lse[b,h]   = ln sum_j exp(s_j)                        (natural log, scaled scores)
 *
 * Precision: Q, K, V are bf16; scores, softmax and accumulation are fp32;
 * out and lse are fp32.  The probabilities that multiply V are rounded to
 * bf16 when the matrix-core path is used (the normaliser is summed from the
 * same rounded values, so the rounding cancels to first order).
 *
 * Pointers: every pointer is a DEVICE pointer unless its name starts with
 * host_.  The caller owns all buffers, including the workspace; the library
 * allocates nothing, frees nothing and never synchronises in gqa_decode_attn.
 * Inputs are never written.  Work is enqueued on the given HIP stream and the
 * call returns at once.  No exception or abort crosses this boundary: every
 * failure is a negative status and, for argument errors, nothing is launched.
 */
#ifndef GQA_DECODE_H
#define GQA_DECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum gqa_status {
    GQA_OK = 0,
    GQA_ERR_INVALID_ARG = -1,          /* null pointer, non-positive size, bad stride or alignment */
    GQA_ERR_UNSUPPORTED = -2,          /* head_dim != 128, group size > 16, page size not a power of two >= 16 */
    GQA_ERR_WORKSPACE_TOO_SMALL = -3,  /* workspace_bytes < gqa_decode_workspace_bytes(params) */
    GQA_ERR_LAUNCH = -4,               /* the HIP runtime refused a launch or an event call */
    GQA_ERR_SCRATCH_LIMIT = -5         /* gqa_decode_attn_static: the call needs more than the built-in scratch buffer */
} gqa_status;

/*
 * Shapes and strides of one call.  Strides count bf16 ELEMENTS; the head_dim
 * elements of one row are adjacent (stride 1) and every row must start on a
 * 16-byte boundary (base pointers 16-byte aligned, strides multiples of 8).
 *
 * Contiguous cache (page_size == 0): row (b, g, t) of K starts at
 *     k + b*k_stride_b + g*k_stride_h + t*k_stride_t,
 * which covers both the head-major [B, Hkv, T, D] and the token-major
 * [B, T, Hkv, D] layouts.
 * Paged cache (page_size > 0, a power of two >= 16): token t of sequence b lives
 * in physical block  blk = block_table[b*block_table_stride + t / page_size]
 * at slot t % page_size, i.e. at
 *     k + blk*k_stride_b + g*k_stride_h + (t % page_size)*k_stride_t.
 * Block-table entries beyond ceil(kv_lens[b] / page_size) are never read.
 */
typedef struct gqa_decode_params {
    int32_t batch;               /* B >= 1                                                     */
    int32_t num_q_heads;         /* Hq, a multiple of num_kv_heads; Hq / Hkv <= 16 (<= 8 for variant 1) */
    int32_t num_kv_heads;        /* Hkv                                                        */
    int32_t head_dim;            /* D, must be 128                                             */
    int32_t max_kv_len;          /* host-known upper bound of kv_lens[]; sizes grid + workspace */
    int32_t page_size;           /* 0 = contiguous cache, else tokens per block                 */
    int32_t block_table_stride;  /* int32 entries per block-table row (paged only)              */
    int32_t chunk_tokens;        /* KV tokens per share; 0 = one share per worker; else multiple of 32 */
    float   scale;               /* multiplies q.k before the softmax                           */
    int32_t kernel_variant;      /* 0 = default (matrix-core path); 1 = plain vector-ALU path   */
    int64_t q_stride_b, q_stride_h;
    int64_t k_stride_b, k_stride_h, k_stride_t;
    int64_t v_stride_b, v_stride_h, v_stride_t;
} gqa_decode_params;

/* Library version, major*10000 + minor*100 + patch. */
int gqa_decode_version(void);

/* Static, never-null description of a status code. */
const char* gqa_decode_strerror(int status);

/*
 * Per-device set-up, for the device that is current in the calling thread: looks up
 * the device's compute-unit count and the kernels' occupancy (the persistent launch
 * size), raises the prefill kernel's LDS limit and resolves the built-in scratch
 * buffer of gqa_decode_attn_static.  Optional: every entry point does the part it
 * needs on its first call on a device.  Those first calls query the runtime and
 * must not happen while a stream of the process is being captured into a HIP graph,
 * so a caller that captures calls gqa_decode_init() once per device beforehand
 * (idempotent, thread-safe, cheap after the first time).  Returns GQA_OK, or
 * GQA_ERR_LAUNCH if no usable device is current.
 */
int gqa_decode_init(void);

/*
 * Bytes of device workspace gqa_decode_attn needs for these parameters (a
 * pure host function of batch, head counts, max_kv_len and chunk_tokens; it
 * touches no device).
 * Returns 0 if the parameters are invalid or unsupported.  The workspace must
 * be 256-byte aligned; its contents before the call do not matter and are
 * undefined after it.
 */
size_t gqa_decode_workspace_bytes(const gqa_decode_params* params);

/*
 * How the work is split.  The library lays the (sequence, kv head) rows end to
 * end into one stream of 32-token tiles and cuts it into equal shares; each
 * share is processed by one persistent worker (a wavefront of the default
 * kernel, a workgroup of variant 1) and yields one partial result per row it
 * touches.  chunk_tokens == 0 gives one share per worker (never shorter than 64
 * tokens, so short batches use fewer workers); chunk_tokens > 0 fixes the share
 * length and the workers take shares in turn.
 *   *share_tokens   tokens per share: chunk_tokens if given; else, when
 *                   host_kv_lens (HOST pointer, may be NULL) is given and a
 *                   device is present, the length the device will compute; else 0
 *   *workgroups     persistent workgroups of the partial kernel on the current
 *                   device (0 when no device is present)
 *   *partial_slots  partial results the workspace holds
 * Any output pointer may be NULL.
 */
int gqa_decode_plan_info(const gqa_decode_params* params, const int32_t* host_kv_lens,
                         int32_t* share_tokens, int32_t* workgroups, int64_t* partial_slots);

/*
 * Enqueue one decode-attention call.
 *
 *   q            [B, Hq, D] bf16 via q_stride_b / q_stride_h
 *   k, v         bf16 cache or block pools, see gqa_decode_params
 *   kv_lens      [B] int32 (device).  Values are clamped to [0, max_kv_len] on
 *                the device, so a stale length never reads past the bound
 *   block_table  [B, block_table_stride] int32 (device); NULL iff page_size == 0
 *   host_kv_lens optional HOST copy of kv_lens (may be NULL).  Not needed: the
 *                launch size does not depend on the lengths.  Accepted so that
 *                callers that have it can pass it; results never depend on it.
 *   out          [B, Hq, D] fp32, dense; every row b < B is fully overwritten;
 *                kv_lens[b] == 0 gives a zero row
 *   lse          [B, Hq] fp32, dense, may be NULL; -inf where kv_lens[b] == 0
 *   workspace    >= gqa_decode_workspace_bytes(params) bytes, 256-byte aligned
 *   stream       a hipStream_t passed as void*; NULL = the default stream
 *
 * Calls on different streams with different workspaces are independent.
 * Results are deterministic for fixed parameters (no atomics on the data
 * path).  Returns GQA_OK or a negative gqa_status.
 */
int gqa_decode_attn(const gqa_decode_params* params,
                    const void* q, const void* k, const void* v,
                    const int32_t* kv_lens, const int32_t* block_table,
                    const int32_t* host_kv_lens,
                    float* out, float* lse,
                    void* workspace, size_t workspace_bytes,
                    void* stream);

/*
 * gqa_decode_attn for callers that cannot hand over a workspace because they cannot
 * allocate one: code under HIP-graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, kernels and results as gqa_decode_attn (bit for
 * bit), but the partial results go to a scratch buffer built into the library: a
 * file-scope device array of GQA_DECODE_STATIC_SCRATCH_BYTES that every device the
 * library runs on holds from the first use until the process ends.  The call
 * allocates nothing, frees nothing and does not synchronise.
 *
 * Limit: the call needs  256 + 4 (B + 1) + (W + B Hkv) (Hq / Hkv) 520  bytes (each
 * term rounded up to 256), W = the persistent wavefronts the device runs (1,024 on
 * MI355X; max_kv_len / chunk_tokens shares per row instead when chunk_tokens > 0).
 * Beyond GQA_DECODE_STATIC_SCRATCH_BYTES it returns GQA_ERR_SCRATCH_LIMIT and
 * launches nothing; all five benchmark shapes fit (the largest, B = 128 with 32 / 8
 * heads, needs 4.3 MB).
 *
 * All calls on one device share that device's buffer: it keeps the previous call's
 * contents (nothing in it has to start at zero: every word a call reads it has
 * written first), calls on the same stream are ordered and safe, and calls that
 * overlap on one device (different streams, different threads) race.  The first
 * call on a device resolves the buffer's address (see gqa_decode_init).
 */
#define GQA_DECODE_STATIC_SCRATCH_BYTES (32u << 20)

size_t gqa_decode_static_scratch_bytes(void);     /* = GQA_DECODE_STATIC_SCRATCH_BYTES */

int gqa_decode_attn_static(const gqa_decode_params* params,
                           const void* q, const void* k, const void* v,
                           const int32_t* kv_lens, const int32_t* block_table,
                           float* out, float* lse, void* stream);

/*
 * Per-kernel timing without synchronising inside the measured region.
 *
 * A gqa_timer owns HIP events for up to max_calls calls.  gqa_decode_attn_timed
 * is gqa_decode_attn plus three event records on `stream` (before the split-KV
 * partial kernel, between the kernels, after the combine kernel); it does not wait.
 * gqa_timer_read waits for the last recorded event and returns, summed over
 * the calls recorded since the last reset, the elapsed milliseconds of
 * {split-KV partial, combine} in host_kernel_ms[2] and the number of calls in
 * *host_calls; it then resets the timer.  gqa_timer_read_calls does the same but
 * returns the elapsed milliseconds of every recorded call, in call order, in
 * host_partial_ms[capacity] and host_combine_ms[capacity] (either may be NULL);
 * more recorded calls than `capacity` is an invalid-argument error and leaves the
 * timer untouched.  Creating, reading and destroying a timer are not for hot
 * loops; recording is.
 * A timer serves one stream at a time and is not thread-safe.
 */
typedef struct gqa_timer gqa_timer;

int  gqa_timer_create(int32_t max_calls, gqa_timer** host_out);
void gqa_timer_destroy(gqa_timer* timer);
int  gqa_timer_read(gqa_timer* timer, int32_t* host_calls, float host_kernel_ms[2]);
int  gqa_timer_read_calls(gqa_timer* timer, int32_t capacity, int32_t* host_calls,
                          float* host_partial_ms, float* host_combine_ms);

int gqa_decode_attn_timed(const gqa_decode_params* params,
                          const void* q, const void* k, const void* v,
                          const int32_t* kv_lens, const int32_t* block_table,
                          const int32_t* host_kv_lens,
                          float* out, float* lse,
                          void* workspace, size_t workspace_bytes,
                          void* stream, gqa_timer* timer);

/*
 * Shared-prefix ("cascade") decode attention.  The paper's workload samples
 * every prompt several times (5 generations per task when the data are
 * collected, Section 3.3; 10 per task at evaluation, Section 4.2), so the
 * sequences of a batch come in groups that share the prompt's keys and values.
 * Here the shared prefix of a group is stored once, and one read of it serves 32
 * of the group's samples x heads-per-KV-head query rows (it is read
 * ceil(M * G / 32) times instead of M times: once for 5 samples of the 40 / 8 head
 * shape, twice for 10); each sequence attends over
 *     [ prefix of its group (prefix_lens[j] tokens) ; its own suffix (kv_lens[b] tokens) ]
 * and the result is exactly the attention defined at the top of this header
 * over that concatenation.
 *
 *   params->decode  shapes of q and of the per-sequence SUFFIX caches (contiguous
 *                   or paged, as in gqa_decode_attn); max_kv_len bounds kv_lens
 *   k_prefix, v_prefix  bf16, row (j, g, t) at  j*kp_stride_g + g*kp_stride_h + t*kp_stride_t
 *   prefix_lens     [num_groups] int32 (device), clamped to [0, max_prefix_len]
 *   group_start     [num_groups + 1] int32 (device): group j holds sequences
 *                   group_start[j] .. group_start[j+1]-1; group_start[0] = 0,
 *                   group_start[num_groups] = batch, non-decreasing
 *   host_group_start  the same array in HOST memory (required): the library checks
 *                   it before launching.  A group may hold at most
 *                   64 / (num_q_heads / num_kv_heads) sequences (GQA_ERR_UNSUPPORTED beyond)
 *   kv_lens, block_table, out, lse, workspace, stream  as in gqa_decode_attn;
 *                   workspace >= gqa_cascade_workspace_bytes(params)
 * Only the matrix-core kernel exists for this entry point (kernel_variant must be 0).
 */
typedef struct gqa_cascade_params {
    gqa_decode_params decode;
    int32_t num_groups;          /* >= 1                                   */
    int32_t max_prefix_len;      /* host-known bound of prefix_lens[]      */
    int64_t kp_stride_g, kp_stride_h, kp_stride_t;
    int64_t vp_stride_g, vp_stride_h, vp_stride_t;
} gqa_cascade_params;

size_t gqa_cascade_workspace_bytes(const gqa_cascade_params* params);

int gqa_decode_attn_shared_prefix(const gqa_cascade_params* params,
                                  const void* q,
                                  const void* k_prefix, const void* v_prefix,
                                  const int32_t* prefix_lens, const int32_t* group_start,
                                  const int32_t* host_group_start,
                                  const void* k, const void* v,
                                  const int32_t* kv_lens, const int32_t* block_table,
                                  float* out, float* lse,
                                  void* workspace, size_t workspace_bytes,
                                  void* stream);

/*
 * Causal prefill attention (forward): the compute-bound companion of the decode
 * path.  The prompt of every trace is prefilled once, and fine-tuning on the
 * curated traces runs whole sequences of up to 32,768 tokens through the same
 * attention (Section 4.1).  For every sequence b, token t and query head h
 *     out[b, t, h, :] = attention of q[b, t, h, :] over keys/values 0 .. t of kv head h / group
 * i.e. row t equals gqa_decode_attn of that query over the first t + 1 cached tokens.
 *
 *   q        [B, T, Hq, 128]  bf16, element strides q_stride_b / _t / _h
 *   k, v     [B, T, Hkv, 128] bf16, strides likewise (16-byte aligned rows)
 *   out      [B, T, Hq, 128]  fp32, strides o_stride_b / _t / _h (in floats, multiples of 4)
 *   lse      [B, T, Hq] fp32 dense, may be NULL
 * bf16 inputs, fp32 accumulation, probabilities rounded to bf16 for the second
 * matrix product (as in the decode kernel).  No workspace.  Argument errors as
 * in gqa_decode_attn; nothing is launched on error.
 */
typedef struct gqa_prefill_params {
    int32_t batch, seq_len, num_q_heads, num_kv_heads, head_dim;   /* head_dim must be 128; group <= 16 */
    float   scale;
    int64_t q_stride_b, q_stride_t, q_stride_h;
    int64_t k_stride_b, k_stride_t, k_stride_h;
    int64_t v_stride_b, v_stride_t, v_stride_h;
    int64_t o_stride_b, o_stride_t, o_stride_h;
} gqa_prefill_params;

int gqa_prefill_attn(const gqa_prefill_params* params, const void* q, const void* k, const void* v,
                     float* out, float* lse, void* stream);

/*
 * The same over a batch of prompts of different lengths (the prompts of the paper's tasks differ in
 * length; Section 3.3 samples each of them several times).  seq_lens[b] (device, int32, clamped to
 * [0, seq_len]) is the number of tokens of sequence b; tensors keep the padded [B, T = seq_len, ...]
 * layout.  Rows t >= seq_lens[b] of out / lse are not written and their q / k / v are not read.
 * seq_lens == NULL means every sequence has seq_len tokens (= gqa_prefill_attn).
 */
int gqa_prefill_attn_varlen(const gqa_prefill_params* params, const void* q, const void* k, const void* v,
                            const int32_t* seq_lens, float* out, float* lse, void* stream);

/*
 * The step before attention in a decode layer: append the new token's key and
 * value rows to the cache and, optionally, apply the rotary position embedding
 * to the new key and to the query (the 32B model family whose traces the paper
 * collects, Section 3.3, uses the rotate-half form).
 *
 * For every sequence b with L = kv_lens[b] (clamped to max_kv_len) > 0 the new
 * token sits at position L - 1:
 *     K[b, L-1, g, :] = rot(k_new[b, g, :]),  V[b, L-1, g, :] = v_new[b, g, :],
 *     q_out[b, h, :]  = rot(q_in[b, h, :])
 * with rot the identity if cos_sin is NULL and otherwise, for d < 64,
 *     x'[d] = x[d] cos[L-1][d] - x[d+64] sin[L-1][d],
 *     x'[d+64] = x[d+64] cos[L-1][d] + x[d] sin[L-1][d],
 * evaluated in fp64 (both products are exact there; their difference or sum is
 * rounded to fp64) and then rounded to bf16, nearest even, over the whole bf16
 * range: results below 2^-126 are rounded on the sub-normal grid of spacing 2^-133
 * (never flushed or truncated), zeros keep their sign, results at or beyond
 * 2^128 - 2^119 become infinity, and a NaN result is stored as 0x7FC0.  A sequence
 * with kv_lens[b] <= 0 gets its query copied unchanged and writes nothing.
 *
 *   q_in, q_out  [B, Hq, 128] bf16, both with q_stride_b / q_stride_h; may alias
 *   k_new, v_new [B, Hkv, 128] bf16, dense
 *   k_cache, v_cache  as in gqa_decode_attn (contiguous or paged, same strides)
 *   cos_sin      [rope_positions, 128] fp32: cos in columns [0, 64), sin in
 *                [64, 128); NULL = no rotation; rope_positions >= max_kv_len
 * Argument errors as in gqa_decode_attn; nothing is launched on error.
 */
typedef struct gqa_append_params {
    int32_t batch, num_q_heads, num_kv_heads, head_dim;   /* head_dim must be 128 */
    int32_t max_kv_len;
    int32_t page_size, block_table_stride;
    int32_t rope_positions;
    int64_t q_stride_b, q_stride_h;
    int64_t k_stride_b, k_stride_h, k_stride_t;
    int64_t v_stride_b, v_stride_h, v_stride_t;
} gqa_append_params;

int gqa_decode_kv_append(const gqa_append_params* params,
                         const void* q_in, void* q_out,
                         const void* k_new, const void* v_new,
                         void* k_cache, void* v_cache,
                         const int32_t* kv_lens, const int32_t* block_table,
                         const float* cos_sin, void* stream);

/*
 * Streaming-read probe for the HBM roofline: reads `bytes` (a multiple of 16)
 * from `src` with 128-bit loads, folds them into one 32-bit word per
 * workgroup written to `sink` (at least 4*workgroups bytes).  Used by the
 * benchmark to report the achievable read bandwidth next to the attention
 * kernels; not part of the attention path.
 */
int gqa_decode_stream_read(const void* src, size_t bytes, void* sink, int32_t workgroups, void* stream);

/*
 * Access-pattern probe behind the design choices of the split-KV kernel: persistent
 * wavefronts (4 per workgroup, `workgroups` <= 4096 of them) stream floor(bytes / 16384)
 * tiles of 16 KB from `src`, each wavefront an equal contiguous run, folding the data
 * into one word per wavefront in `sink` (at least 16 * workgroups bytes).  mode:
 *   0  non-temporal loads, 1 KB contiguous per load instruction (how V is read), one tile in flight
 *   1  non-temporal, matrix-operand-shaped: 16 rows x 64 bytes per load instruction (how K is read)
 *   2  as 0, then through LDS (ds_write_b128, operand-shaped ds_read_b128): an LDS-staged tile
 *   3  as 1 with ordinary (temporal) loads
 *   4  as 1 with two tiles in flight per wavefront (double-buffered)
 *   5  as 0 with two tiles in flight
 *   6  the attention kernel's own mix: half of each tile as 1, half as 0
 *   7  as 6 with ordinary loads
 *   8  as 6, but a workgroup owns a contiguous run and its 4 wavefronts take the tiles in turn
 *   9  as 6, but all wavefronts take tiles in turn (the whole chip sweeps through memory together)
 * Not part of the attention path; the benchmark's --probe mode times it.
 */
int gqa_decode_stream_probe(const void* src, size_t bytes, void* sink, int32_t workgroups, int32_t mode, void* stream);

/*
 * Plain device-to-device copy of `bytes` (a multiple of 16; src and dst
 * 16-byte aligned, not overlapping) by a grid-stride kernel.  It reads and
 * writes exactly `bytes` each, which makes it the known-size reference that
 * hardware byte counters of a profile are scaled by; not part of the
 * attention path.
 */
int gqa_decode_stream_copy(const void* src, void* dst, size_t bytes, int32_t workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GQA_DECODE_H */
