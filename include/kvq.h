/*
 * kvq.h -- C ABI of the MI355X (gfx950) mixed-precision KV-cache library.
 *
 * The library implements the inference-side hot path of layer-wise mixed-precision
 * KV-cache quantization (KVTuner, arXiv 2502.04420): every transformer layer l owns a
 * precision pair (key bits, value bits) (Section 5.1); cached keys and values are stored
 * with the round-to-nearest asymmetric quantizer of Section 3.2, Eq. 2,
 *     z = min(X),  s = (max(X) - min(X)) / (2^B - 1),  Q(X) = round((X - z) / s),
 * keys grouped per channel over `group` consecutive tokens and values per token over
 * `group` consecutive channels (the KIVI mode of the experimental-settings appendix:
 * group 32, residual length 32), while the newest tokens stay in fp16; a decode step
 * evaluates Section 3.1, Eq. 1,
 *     a = softmax(q K^T / sqrt(D)),  o = a V,
 * over the dequantized tokens X^ = Q(X) s + z and the fp16 tail without ever writing X^
 * back to memory.
 *
 * Conventions
 *   - Every pointer named *device* points to GPU memory of the current HIP device; every
 *     other pointer is host memory.  The caller owns all device memory, including the
 *     workspace; the library only keeps a small host-side context.
 *   - All GPU work is enqueued on the HIP stream given to kvq_configure (a hipStream_t
 *     passed as void*, NULL = the default stream).  No call synchronises the device.
 *   - Calls on one context are not thread-safe; serialise them.
 *   - fp16 means IEEE binary16.  All sequences of the batch have the same length.
 *   - Functions returning int return KVQ_OK (0) or a negative kvq_status.  Argument, state and
 *     capacity errors are found before anything is enqueued.  KVQ_ELAUNCH means the HIP runtime
 *     refused one of a call's launches; launches before it may have been enqueued (each call says
 *     what state that leaves).
 *   - This build supports head_dim = 128 and group = 32 only (kvq_workspace_bytes returns 0 and
 *     kvq_configure KVQ_EINVAL for anything else): the packed layout is built on 32 x 128 blocks.
 */
#ifndef KVQ_H
#define KVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum kvq_status {
    KVQ_OK = 0,
    KVQ_EINVAL = -1,      /* NULL pointer, bad layer index, unsupported bits / shape / group      */
    KVQ_ECAPACITY = -2,   /* append would exceed max_tokens                                       */
    KVQ_ESTATE = -3,      /* decode on a layer that holds no token                                */
    KVQ_EWORKSPACE = -4,  /* workspace NULL, misaligned (needs 256 B) or smaller than required    */
    KVQ_ELAUNCH = -5,     /* the HIP runtime refused a launch (message via kvq_last_error)        */
    KVQ_ESCRATCH = -6     /* kvq_decode_attention_noalloc: the call needs more scratch than the   */
                          /* built-in array holds (sizes via kvq_last_error)                      */
} kvq_status;

typedef struct kvq_ctx kvq_ctx;

/*
 * Precision in which a group's scale s of Eq. 2 is stored and used (the paper leaves it open;
 * its equivalent-precision figure of Section 5.1 does not count metadata).  The zero-point z
 * is the minimum of fp16 inputs and is always kept exactly.
 *   KVQ_META_FP32: s is the fp32 quotient (max - min) / (2^B - 1).  The default.
 *   KVQ_META_FP16: s is that quotient rounded once to fp16 (round half to even); encoder and
 *     decoder both use the rounded value, codes are clamped to [0, 2^B - 1], and a scale that
 *     rounds to zero encodes its group as all-zero codes.  Saves 8 bytes per token and tensor.
 * kvq_debug_export returns fp32 scales in both cases (exactly the values in use).
 */
/*
 * Axis along which the keys are grouped for Eq. 2 (values are always grouped per token over G
 * channels).  The paper evaluates both (Section 3.2 and its table of per-channel vs per-token
 * errors):
 *   KVQ_KEYS_PER_CHANNEL: one (s, z) per channel over G consecutive tokens -- the KIVI mode
 *     of the paper's experiments.  The default.
 *   KVQ_KEYS_PER_TOKEN: one (s, z) per token over each group of G channels, exactly like the
 *     values -- the paper's "per-token-asym" mode (same group size and window rule here).
 */
typedef enum kvq_key_mode {
    KVQ_KEYS_PER_CHANNEL = 0,
    KVQ_KEYS_PER_TOKEN = 1
} kvq_key_mode;

typedef enum kvq_meta_dtype {
    KVQ_META_FP32 = 0,
    KVQ_META_FP16 = 1
} kvq_meta_dtype;

/*
 * Shapes and the layer-wise precision table P (Section 5.1: one (P_k, P_v) per layer,
 * each in {2, 4, 8}; 16 keeps that tensor in fp16, the paper's half-precision baseline).
 */
typedef struct kvq_config {
    int32_t n_layers;      /* L >= 1                                                             */
    int32_t batch;         /* sequences, >= 1; batch * n_kv_heads <= 65535                       */
    int32_t n_q_heads;     /* multiple of n_kv_heads (grouped-query attention)                   */
    int32_t n_kv_heads;    /* >= 1                                                               */
    int32_t head_dim;      /* D of Eq. 1 (per head); this build supports 128                     */
    int32_t max_tokens;    /* capacity per sequence, >= 1                                        */
    int32_t group;         /* G: tokens per key group = channels per value group; must be 32     */
    int32_t residual;      /* R >= 0: at least this many newest tokens stay fp16 once T >= R     */
    const uint8_t *kbits;  /* host, [n_layers], each in {2, 4, 8, 16}                            */
    const uint8_t *vbits;  /* host, [n_layers], each in {2, 4, 8, 16}                            */
    int32_t meta_dtype;    /* a kvq_meta_dtype: precision of the stored scales (see there)       */
    int32_t key_mode;      /* a kvq_key_mode: axis along which keys are grouped (see there)      */
} kvq_config;

/* Bytes of device workspace kvq_configure needs for this configuration; 0 if it is invalid. */
size_t kvq_workspace_bytes(const kvq_config *cfg);

/*
 * Create a context (Section 5.1: the offline-searched table is loaded once, no online
 * decision remains).  `workspace_device` must be 256-byte aligned, at least
 * kvq_workspace_bytes(cfg) long and stay valid and untouched by the caller until
 * kvq_destroy.  The kbits / vbits arrays are copied.  All layers start empty.
 */
int kvq_configure(kvq_ctx **out, const kvq_config *cfg, void *workspace_device, size_t workspace_bytes,
                  void *hip_stream);

/*
 * Append n_tokens >= 1 new tokens to one layer's cache (Eq. 1: K = concat(K_past, k_i)).
 *   k_device, v_device : fp16 [batch, n_kv_heads, n_tokens, head_dim], contiguous, device.
 * With T tokens appended in total, the oldest N_p = G * floor(max(T - R, 0) / G) are held
 * quantized (Eq. 2 at the layer's bits, keys per channel over the G tokens of a group,
 * values per token over each G channels) and the newest T - N_p stay in fp16.  The result
 * depends only on the concatenated token sequence, not on how it was split into calls.
 * The inputs may be reused once the enqueued work has run.  Inputs must be finite.
 * A zero minimum or maximum of a group counts as +0 whatever the signs of the zeros it holds
 * (z and s have one bit pattern per group).  On any error the layer holds the same tokens as
 * before the call.
 */
int kvq_quantize_append(kvq_ctx *ctx, int32_t layer, const void *k_device, const void *v_device,
                        int32_t n_tokens);

/*
 * One decode step of Eq. 1 for one layer over every token appended so far (no mask).
 *   q_device   : fp16 [batch, n_q_heads, head_dim], device.
 *   out_device : fp16 [batch, n_q_heads, head_dim], device, written.
 * Query head h attends kv head h / (n_q_heads / n_kv_heads).  Quantized tokens enter as
 * X^ = Q(X) s + z (Section 3.2), fp16 tokens as they are; accumulation is fp32.
 */
int kvq_decode_attention(kvq_ctx *ctx, int32_t layer, const void *q_device, void *out_device);

/*
 * kvq_decode_attention for callers that cannot allocate and cannot hand scratch memory along
 * per call: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels, same result as kvq_decode_attention (bit for bit:
 * the token-range splits are planned the same way).  The difference is where the splits'
 * partial results live: not in the caller's workspace but in an array built into the library's
 * device image, 16384 records of (128 outputs, maximum, sum) = 8.1 MiB, which every GPU the
 * library runs on holds from its first use until the process ends.  The call allocates and frees
 * nothing on host or device; on its first use on a GPU (with that GPU current) it looks up the
 * array's address there (make that first call outside a stream capture; every later call only
 * launches kernels and can be recorded into a graph and replayed).
 *   Limit: batch * n_q_heads * splits <= 16384 records, else KVQ_ESCRATCH and nothing is
 *   enqueued (kvq_last_error has the numbers).  With automatic splits (at most 2048 token
 *   ranges over all (batch, kv head) caches) every shape with at most 8 query heads per kv head
 *   fits; splits forced through kvq_set_decode_options may not.
 *   All contexts and streams on one GPU share that GPU's array.  Nothing in it has to start at
 *   zero (each call writes every record it later reads), but two such calls that overlap in time
 *   on one GPU race on it: keep them on one stream or order them yourself.
 */
int kvq_decode_attention_noalloc(kvq_ctx *ctx, int32_t layer, const void *q_device, void *out_device);

/*
 * One decode step of a layer in a single call: append exactly one new token per sequence
 * (k_device, v_device: fp16 [batch, n_kv_heads, 1, head_dim]) and then attend over all tokens,
 * the new one included (Eq. 1: K is the concatenation of the cached keys and the current one).
 * Same result and same cache state as kvq_quantize_append(.., 1) followed by
 * kvq_decode_attention; the difference is that the decode kernel itself takes the new rows
 * from k_device / v_device and stores them into the fp16 window, which saves the separate
 * window-copy launch.  k_device / v_device must stay unchanged until the enqueued work has
 * run (as for every other call).  Errors as for the two calls it replaces.  Whatever error is
 * returned, the layer holds the same tokens as before the call (on KVQ_ELAUNCH the token is
 * not appended even if the refused launch was the second one; kernels enqueued before the
 * refusal only write what a repeat of the call writes again, identically).
 */
int kvq_append_decode_attention(kvq_ctx *ctx, int32_t layer, const void *k_device, const void *v_device,
                                const void *q_device, void *out_device);

/*
 * Prefill-stage attention of one layer over the cache as it stands: the prompt's own causal
 * attention reading the dequantized cache (the paper quantizes the cache in the prefill stage
 * as well as in decoding; calibration design of Section 5.3).  The queries are the last n_q
 * tokens appended; the query at absolute position p attends to positions 0..p (Eq. 1 under
 * the causal mask).  A token enters as X^ = Q(X) s + z (Section 3.2) if the layer holds it
 * quantized now, else as its fp16 value.
 *   q_device   : fp16 [batch, n_q_heads, n_q, head_dim], contiguous, device.
 *   out_device : fp16 [batch, n_q_heads, n_q, head_dim], device, written.
 *   n_q        : 1 .. tokens held by the layer (else KVQ_EINVAL; KVQ_ESTATE for an empty layer).
 * Query head h attends kv head h / (n_q_heads / n_kv_heads).  The dequantized operands and the
 * softmax weights are rounded to fp16 for the matrix cores (keys as the sum of two fp16
 * numbers); accumulation is fp32.  The cache is not modified.  With n_q = 1 the result is that
 * of kvq_decode_attention up to rounding.  The call enqueues two kernels per pass over a group
 * of (batch, kv head) caches: one dequantizes their packed tokens once into a scratch area
 * inside the workspace (16 * floor(max_tokens / 32) * 27 KiB, counted by kvq_workspace_bytes:
 * 16 caches per pass at full length, more when the layer holds fewer tokens), one attends.  For
 * keys quantized per channel, one kernel in front of the passes finds, per cache and from the
 * stored scales and zero-points, the centre of every channel's keys, which is taken off the
 * dequantized keys before they are rounded (a constant per channel moves all scores of a query
 * alike, so the softmax is unchanged; the fp16 window's scores are lowered to match), and decides
 * which channels keep the second fp16 number of their keys: all, or (when one fp16 rounding of
 * the others moves a logit by less than the fp16 softmax weights are rounded by anyway, judged
 * from the same metadata and a sample of the queries) only the 32 channels where it matters
 * most, which shortens the call by a seventh (kvq_set_prefill_options switches both off).  With kernel events set (kvq_set_kernel_events) they receive the start of the
 * first and the end of the last of these kernels.
 */
int kvq_prefill_attention(kvq_ctx *ctx, int32_t layer, const void *q_device, int32_t n_q, void *out_device);

/* Tokens currently held quantized / in fp16 by a layer (host-side bookkeeping, no GPU work). */
int kvq_layer_tokens(const kvq_ctx *ctx, int32_t layer, int32_t *n_packed, int32_t *n_residual);

/* Forget every token of one layer (layer >= 0) or of all layers (layer == -1). */
int kvq_reset(kvq_ctx *ctx, int32_t layer);

/*
 * Write a layer's cache in a layout-independent canonical form into caller-provided
 * DEVICE buffers (any pointer may be NULL to skip that part).  With N_p, N_r from
 * kvq_layer_tokens, B = batch, H = n_kv_heads, D = head_dim, G = group:
 *   k_codes : kbits < 16: uint8 [B, H, N_p/G, D, G*kbits/8] -- per channel, the G codes of
 *             a token group packed little-endian (token i at bits [i*kbits, (i+1)*kbits));
 *             kbits = 16: fp16 [B, H, N_p, D].
 *   k_scale, k_zero : fp32 [B, H, N_p/G, D]   (s and z of Eq. 2; untouched when kbits = 16)
 *             With KVQ_KEYS_PER_TOKEN the three key arrays take the value arrays' form:
 *             k_codes uint8 [B, H, N_p, D*kbits/8], k_scale, k_zero fp32 [B, H, N_p, D/G].
 *   v_codes : vbits < 16: uint8 [B, H, N_p, D*vbits/8] -- per token, the D codes packed
 *             little-endian; vbits = 16: fp16 [B, H, N_p, D].
 *   v_scale, v_zero : fp32 [B, H, N_p, D/G]   (untouched when vbits = 16)
 *   k_res, v_res    : fp16 [B, H, N_r, D], oldest token first.
 */
int kvq_debug_export(kvq_ctx *ctx, int32_t layer, void *k_codes, void *k_scale, void *k_zero,
                     void *v_codes, void *v_scale, void *v_zero, void *k_res, void *v_res);

/*
 * The split plan a decode call would use (host only, no GPU work): with n_tokens tokens in
 * `layer` of a cache configured as *cfg, kernel `variant` and `forced_splits` as in
 * kvq_set_decode_options, each (batch, kv head) cache is divided among *splits groups.  Work
 * units are the packed blocks (N_p / 32, in order) followed by a few virtual units that stand
 * for the fp16 window; group s takes *units_per_split consecutive units, one more if
 * s >= *splits - *split_rem, cut off at the last block; the last group also owns the window.  No group is
 * empty.  For tests and tuning; KVQ_EINVAL on invalid arguments.
 */
int kvq_debug_split_plan(const kvq_config *cfg, int32_t layer, int32_t n_tokens, int32_t variant, int32_t forced_splits,
                         int32_t *splits, int32_t *units_per_split, int32_t *split_rem);

/*
 * Tuning knobs (optional).  variant: 0 = choose automatically, 1 = vector-ALU kernel,
 * 2 = matrix-core kernel.  splits: 0 = automatic, else the number of token-range splits
 * per (batch, kv head) used to fill the GPU (at most 128).  Returns KVQ_EINVAL for unknown
 * values.
 */
int kvq_set_decode_options(kvq_ctx *ctx, int32_t variant, int32_t splits);

/*
 * Tuning knob of kvq_prefill_attention (optional).  low_parts: 0 = per cache, centre the
 * dequantized keys and keep their second fp16 number for all channels or for the 32 that need
 * it (default, see kvq_prefill_attention); 1 = keys as dequantized, second number for all
 * channels of every cache.  Returns KVQ_EINVAL for other values.
 */
int kvq_set_prefill_options(kvq_ctx *ctx, int32_t low_parts);

/*
 * Measurement hook (optional).  begin_event / end_event: two hipEvent_t handles owned by the
 * caller (created with timing enabled), or both NULL to switch the hook off.  While set,
 * every decode call makes its main kernel (the fused dequantize-and-attend kernel) stamp
 * begin_event with the start and end_event with the end of that kernel's own execution on the
 * context's stream (the small kernel that merges the token-range splits runs after end_event);
 * a kvq_prefill_attention call stamps them with the start of its first and the end of its last
 * kernel; the caller synchronises and reads hipEventElapsedTime.  The events must outlive the hook.
 * Returns KVQ_EINVAL when exactly one of the two is NULL.
 */
int kvq_set_kernel_events(kvq_ctx *ctx, void *begin_event, void *end_event);

/* Release the host-side context.  The workspace stays with the caller. */
void kvq_destroy(kvq_ctx *ctx);

/* Static description of a status code. */
const char *kvq_strerror(int status);

/* Detail of the last KVQ_ELAUNCH or KVQ_ESCRATCH on this thread (empty string if none). */
const char *kvq_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KVQ_H */
