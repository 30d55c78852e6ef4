/*
 * rstitch.h - C ABI of the MI355X (gfx950) hot path of entropy-routed stitched
 * decoding between a small and a large autoregressive decoder.
 *
 * What the paper defines and this library computes:
 *   - the active model maps the tokens it has not processed yet to a next-token
 *     distribution and a token (Section "Preliminary"; Algorithm 1, the
 *     "Prefill" and "Decode" branches);
 *   - the uncertainty of a step is the normalised entropy of that distribution
 *     (Eq. 1) and the switching rule compares it with a threshold tau (Eq. 2);
 *   - each model keeps its own KV cache and, when switched to, prefills only
 *     the tokens produced since it last ran (Section "KV Cache management").
 * The decoder layer itself (RMSNorm, rotary embedding, grouped-query attention
 * over a KV cache, SwiGLU MLP, LM head; bf16 weights, fp32 accumulation) is the
 * public Qwen2-style block; the paper does not describe it (Section
 * "Preliminary" only states that every token costs one pass of the active model).
 *
 * General rules of this ABI
 *   - Every pointer argument says whether it is HOST or DEVICE memory.  The
 *     library never allocates or frees device memory: weights, KV caches,
 *     workspace and outputs are owned by the caller and are only borrowed, for
 *     the life time of the rs_model handle (weights, KV, workspace) or of the
 *     call (everything else; "of the call" includes the asynchronous execution
 *     on the stream).
 *   - Calls that take a stream only enqueue work on it and return; results are
 *     valid once the caller has synchronised that stream.  `stream` is a
 *     hipStream_t passed as void* (NULL = the default stream).  Two calls that
 *     use the same rs_model must not run concurrently.
 *   - A forward call is a sequence of ~170 small kernels.  When a call repeats
 *     an earlier call's argument VALUES (same pointers, counts, tau, role and a
 *     non-default stream), the library replays a cached HIP graph of that
 *     sequence; the kernels read tokens, positions and scales from the caller's
 *     buffers when they run, so a serving loop that keeps its buffers at fixed
 *     addresses pays one graph launch per step.  RSTITCH_GRAPHS=0 in the
 *     environment (read by rs_create_model) disables this.
 *   - No call throws.  Every call returns an rs_status; on failure
 *     rs_last_error() describes the most recent failure on the calling thread.
 *   - Arguments the host can see (sizes, counts, null pointers) are checked
 *     before anything is launched.  Values that live in device memory
 *     (positions, token ids, slots) are checked by the kernels themselves: a
 *     row whose position, token or slot is out of range is skipped without any
 *     out-of-bounds access and RS_FLAG_BADARG is set in the output record of
 *     its sequence.
 *   - Layouts: all matrices are row-major [out_features, in_features], bf16.
 */
#ifndef RSTITCH_H
#define RSTITCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int32_t rs_status;
#define RS_OK          0
#define RS_EINVAL     (-1)  /* malformed argument (null pointer, bad count, a shape rule of
                               rs_config violated: see there)                               */
#define RS_ECAPACITY  (-2)  /* request exceeds what the model was created for               */
#define RS_EHIP       (-3)  /* the HIP runtime reported an error (see rs_last_error)        */
#define RS_ENOTIMPL   (-4)  /* valid request that this build does not support               */

/* Which model of the stitched pair a call is made for (Algorithm 1's "active"). */
#define RS_SLM 0
#define RS_LLM 1

/* rs_route_out.flags */
#define RS_FLAG_HI         1u  /* normalised entropy > tau (strictly; Eq. 2)                         */
#define RS_FLAG_ACCEPT     2u  /* the token is kept: always for the LLM, for the SLM only if !HI      */
#define RS_FLAG_NEXT_LLM   4u  /* the model to run next is the LLM (== HI)                            */
#define RS_FLAG_NONFINITE  8u  /* a logit was NaN/Inf; HI is forced, entropy fields are NaN           */
#define RS_FLAG_BADARG    16u  /* a device-side position/token/slot was out of range; record invalid */
#define RS_FLAG_ABORTED   32u  /* a bounded wait inside a kernel ran out: the step did not complete,
                                  the record is invalid and the model refuses further steps          */
#define RS_FLAG_ROUTER_STAY 64u /* R-Stitch+: HI on the small model, but the learned router chose to
                                  stay: ACCEPT is set and NEXT_LLM cleared (rs_route_plus)            */

/* Shape rules (rs_workspace_bytes / rs_kv_bytes return 0 and rs_create_model returns
 * RS_EINVAL when one is violated; rs_last_error names it):
 *   d_model, d_ffn and n_q_heads*head_dim are multiples of 128; d_model and
 *   n_q_heads*head_dim are at most 12288; d_ffn >= 128; head_dim is 32, 64 or 128;
 *   n_kv_heads divides n_q_heads with at most 8 query heads per KV head; vocab >= 2;
 *   max_ctx is a multiple of 8, at least 8; 1 <= max_seqs <= 128; 1 <= max_rows <= 128;
 *   rms_eps > 0; rope_theta > 1. */
typedef struct rs_config {
    int32_t n_layers;      /* >= 1                                                            */
    int32_t d_model;       /* multiple of 128, <= 12288                                      */
    int32_t n_q_heads;     /* n_q_heads * head_dim: multiple of 128, <= 12288                */
    int32_t n_kv_heads;    /* divides n_q_heads; n_q_heads / n_kv_heads <= 8                 */
    int32_t head_dim;      /* 32, 64 or 128                                                  */
    int32_t d_ffn;         /* multiple of 128                                                */
    int32_t vocab;         /* >= 2                                                           */
    int32_t tied_lm_head;  /* informational; lm_head may simply alias embed                  */
    int32_t max_ctx;       /* positions per sequence slot in the KV cache; multiple of 8, >= 8 */
    int32_t max_seqs;      /* sequence slots in the KV cache (1..128)                        */
    int32_t max_rows;      /* most token rows one call may carry (1..128)                    */
    float   rms_eps;       /* > 0                                                            */
    float   rope_theta;    /* > 1                                                            */
} rs_config;

typedef struct rs_weights {
    const void *embed;        /* DEVICE bf16 [vocab, d_model]                                 */
    const void *lm_head;      /* DEVICE bf16 [vocab, d_model]                                 */
    const void *final_norm;   /* DEVICE bf16 [d_model]                                        */
    /* HOST arrays of n_layers DEVICE pointers each: */
    const void *const *attn_norm;   /* bf16 [d_model]                                          */
    const void *const *w_qkv;       /* bf16 [(n_q+2 n_kv) head_dim, d_model]: q heads, k heads, v heads */
    const void *const *w_o;         /* bf16 [d_model, n_q head_dim]                            */
    const void *const *mlp_norm;    /* bf16 [d_model]                                          */
    const void *const *w_gate_up;   /* bf16 [2 d_ffn, d_model]: gate rows then up rows         */
    const void *const *w_down;      /* bf16 [d_model, d_ffn]                                   */
} rs_weights;

/* Router record of one sequence for one call (24 bytes). */
typedef struct rs_route_out {
    int32_t  token;      /* argmax of the logits, lowest index among equals                  */
    uint32_t flags;      /* RS_FLAG_*                                                        */
    float    h_nats;     /* entropy of softmax(scaled logits), natural log                   */
    float    h_norm;     /* h_nats / ln(vocab)  (Eq. 1)                                      */
    float    max_logit;  /* largest scaled logit                                             */
    float    log_z;      /* ln sum exp(scaled logits)                                        */
} rs_route_out;

typedef struct rs_model rs_model;   /* opaque host-side handle */

/* Human-readable description of the last failure on this thread ("" if none). */
const char *rs_last_error(void);

/* ABI version of the loaded library (bumped on incompatible change). */
int32_t rs_abi_version(void);

/* Bytes of DEVICE workspace rs_create_model needs for this configuration
 * (rotary table, activations of max_rows rows, attention and router partials).
 * Returns 0 if the configuration is invalid. */
size_t rs_workspace_bytes(const rs_config *cfg);

/* Bytes of one KV buffer (K or V): n_layers * max_seqs * n_kv_heads * max_ctx *
 * head_dim * 2, bf16.  K is laid out [layer][slot][kv_head][position][head_dim];
 * V is laid out [layer][slot][kv_head][head_dim][position] (transposed, so that
 * the attention kernel can feed consecutive positions of one channel to the
 * matrix cores without a shuffle). */
size_t rs_kv_bytes(const rs_config *cfg);

/* Bind weights, KV caches and workspace into a handle.  Builds the rotary
 * cos/sin table (computed in double on the host) inside the workspace with a
 * synchronous copy; clears the workspace's counters.  kv_k, kv_v, workspace:
 * DEVICE, 256-byte aligned, of at least rs_kv_bytes / rs_workspace_bytes.
 * The KV contents are not touched.
 * Errors: RS_EINVAL (null pointer, shape rule violated, workspace too small or
 * misaligned), RS_EHIP. */
rs_status rs_create_model(const rs_config *cfg, const rs_weights *weights,
                          void *kv_k, void *kv_v,
                          void *workspace, size_t workspace_bytes,
                          rs_model **out);

/* Frees the host handle and the launch graphs cached for it (after draining the
 * device, since a replay may still be running); no device memory is touched. */
rs_status rs_destroy_model(rs_model *model);

/* Algorithm 1, "Decode": one new token for each of n_seqs sequences
 * (1 <= n_seqs <= min(max_seqs, max_rows)).
 *   d_seq_slot    DEVICE int32[n_seqs]  KV slot of each sequence (distinct)
 *   d_token       DEVICE int32[n_seqs]  the token to feed (the last accepted one)
 *   d_pos         DEVICE int32[n_seqs]  its position; its K/V rows are written
 *                                       there and attention covers 0..pos
 *   d_logit_scale DEVICE fp32[n_seqs] or NULL (= 1): the logits are multiplied
 *                                       by it before the softmax
 *   tau, active   threshold of Eq. 2 (in normalised-entropy units) and which
 *                 model this handle plays (RS_SLM / RS_LLM), for the flags
 *   d_out         DEVICE (or pinned host) rs_route_out[n_seqs]
 *   d_logits      DEVICE fp32[n_seqs, vocab] or NULL: scaled logits dump
 * Errors: RS_EINVAL, RS_ECAPACITY (n_seqs too large), RS_EHIP. */
rs_status rs_decode_step(rs_model *model, int32_t n_seqs,
                         const int32_t *d_seq_slot, const int32_t *d_token,
                         const int32_t *d_pos, const float *d_logit_scale,
                         float tau, int32_t active,
                         rs_route_out *d_out, float *d_logits, void *stream);

/* Algorithm 1, "Prefill" of the unseen suffix (Section "KV Cache management"):
 * for each sequence b, feed the span d_tokens[off[b] .. off[b+1]) at positions
 * pos0[b], pos0[b]+1, ...; write the K/V rows of every span token; row i
 * attends to cache positions 0 .. pos0[b]+i (causal); the router record is
 * produced from the LAST row of each span.
 *   n_rows        HOST value: total number of span tokens = off[n_seqs]
 *                 (1 <= n_rows <= max_rows; every span has at least 1 token)
 *   d_tokens      DEVICE int32[n_rows], spans packed back to back
 *   d_span_offset DEVICE int32[n_seqs+1], off[0] = 0, non-decreasing
 *   d_pos0        DEVICE int32[n_seqs]
 *   d_logit_scale DEVICE fp32[n_seqs] or NULL
 * A kernel that finds off[n_seqs] != n_rows, an empty span or a span running
 * past max_ctx flags RS_FLAG_BADARG for that sequence and skips its rows.
 * Errors: RS_EINVAL, RS_ECAPACITY (n_rows > max_rows, n_seqs > max_seqs), RS_EHIP. */
rs_status rs_catchup_prefill(rs_model *model, int32_t n_seqs, int32_t n_rows,
                             const int32_t *d_seq_slot, const int32_t *d_tokens,
                             const int32_t *d_span_offset, const int32_t *d_pos0,
                             const float *d_logit_scale,
                             float tau, int32_t active,
                             rs_route_out *d_out, float *d_logits, void *stream);

/* Eq. 1 and Eq. 2 on caller-provided logits: for each of n rows of
 * d_logits (DEVICE fp32 [n, vocab], row-major) compute, in one pass, the
 * entropy of softmax(scale * logits), its normalised value, the argmax and the
 * routing flags.  Same reduction code as the epilogue fused behind the LM head.
 *   d_scratch / scratch_bytes  DEVICE scratch of at least
 *                              rs_route_scratch_bytes(n, vocab), 256-byte aligned
 * Errors: RS_EINVAL (n < 1, vocab < 2, null pointer, scratch too small). */
size_t    rs_route_scratch_bytes(int32_t n, int32_t vocab);
rs_status rs_route(const float *d_logits, int32_t n, int32_t vocab,
                   const float *d_logit_scale, float tau, int32_t active,
                   rs_route_out *d_out, void *d_scratch, size_t scratch_bytes,
                   void *stream);

/* Sampling instead of greedy decoding (Section "Preliminary": the next token is
 * sampled from the distribution the active model outputs).  While enabled, the
 * `token` of every record this model produces is a draw from softmax(scaled
 * logits) instead of their arg max; entropy and flags are unchanged.  The draw
 * is the arg max of logit_i - ln(-ln u_i) (Gumbel-max), u_i = (n + 0.5) 2^-23
 * with n the top 23 bits of a 64-bit hash of the counter p * vocab + i under
 * `key`, p the position of the token being predicted (the last row's position
 * + 1): x = counter * 0x9E3779B97F4A7C15 + key; x = (x ^ x >> 30) *
 * 0xBF58476D1CE4E5B9; x = (x ^ x >> 27) * 0x94D049BB133111EB; x ^= x >> 31.  The
 * draw therefore depends on (key, position) only, not on which call, model or
 * batch slot produces it.  Changing the setting drains the device and drops the
 * model's cached launch graphs.  rs_route / rs_route_static (no positions) and
 * the experimental single-kernel step do not sample.
 * Errors: RS_EINVAL (null model). */
rs_status rs_set_sampling(rs_model *model, int32_t enabled, uint64_t key);

/* The learned router of R-Stitch+ (Section "RL-based Routing with Latency-aware
 * Reward"; Algorithm 1, R-Stitch+ branch; Section "Architecture and Overhead of
 * Router"): when a small-model step is above tau, the hidden state of that step
 * goes through six residual feed-forward blocks x <- x + W2 gelu(W1 x + b1) + b2
 * (GELU in its erf form), a LayerNorm and a linear layer with two outputs, and
 * the hand-over happens only if output 1 ("large model") exceeds output 0.
 * All tensors DEVICE bf16; the pointer arrays are HOST arrays of 6 DEVICE pointers. */
typedef struct rs_router_weights {
    int32_t d;                 /* input width = d_model of the model whose state is routed; multiple of 8 */
    int32_t r;                 /* bottleneck width of a block: multiple of 8, at most 64                  */
    float   ln_eps;            /* > 0                                                                     */
    const void *const *w1;     /* [r, d]  */
    const void *const *b1;     /* [r]     */
    const void *const *w2;     /* [d, r]  */
    const void *const *b2;     /* [d]     */
    const void *ln_gain;       /* [d]     */
    const void *ln_bias;       /* [d]     */
    const void *w_head;        /* [2, d]: row 0 = stay on the small model, row 1 = switch to the large one */
    const void *b_head;        /* [2]     */
} rs_router_weights;

/* Apply the router to the records a forward call has just produced.
 *   model     the model that made the call (its workspace still holds the final
 *             hidden state, before the final RMSNorm, of the last row of every
 *             sequence of that call), or NULL when d_hidden is given
 *   d_hidden  DEVICE fp32 [n_seqs, w->d] hidden states, or NULL to take the model's
 *   active    RS_SLM / RS_LLM as in the forward call; records of the large model
 *             are never changed (Algorithm 1 consults the router on the small model only)
 *   d_out     DEVICE (or pinned host) rs_route_out[n_seqs] of that call, updated in
 *             place: a record with RS_FLAG_HI whose router output prefers "stay"
 *             gets RS_FLAG_ACCEPT | RS_FLAG_ROUTER_STAY and loses RS_FLAG_NEXT_LLM
 *   d_router_logits  DEVICE fp32 [n_seqs, 2] or NULL: the two outputs
 * Enqueue it on the stream of the forward call, before the next call on that model.
 * Errors: RS_EINVAL (null pointer, both or neither of model / d_hidden, d != the
 * model's d_model, r not a multiple of 8 or above 64), RS_ECAPACITY (n_seqs). */
rs_status rs_route_plus(rs_model *model, const float *d_hidden, int32_t n_seqs,
                        const rs_router_weights *w, int32_t active,
                        rs_route_out *d_out, float *d_router_logits, void *stream);

/* Algorithm 1 ("Inference procedure") with the loop itself on the device: one
 * cooperative kernel runs invocation after invocation, applies the routing flags
 * of Eq. 2 to a loop state in device memory (a rejected small-model token is
 * dropped and the large model redoes the position; the large model hands back
 * at or below tau) and appends the accepted tokens to d_seq.  The host reads
 * nothing between invocations.  The active model's unseen suffix (Section "KV
 * Cache management") is fed one token row at a time inside the kernel; a caller
 * that wants a long prompt prefilled on the matrix cores does that first with
 * rs_catchup_prefill and passes how many rows each model already holds.
 * Greedy decoding with the entropy rule only (no sampling, no R-Stitch+ router).
 * On this machine a software barrier across all compute units costs more than a
 * kernel boundary, so this call is SLOWER than a host loop over rs_decode_step /
 * rs_catchup_prefill; it is here for callers that cannot put the host in the loop. */
#define RS_STITCH_RUNNING     0  /* only seen while the kernel runs                        */
#define RS_STITCH_DONE        1  /* n_new tokens accepted, or the eos token accepted       */
#define RS_STITCH_TRACE_FULL  2  /* max_records invocations made before that               */
#define RS_STITCH_FLAGGED     3  /* a record carried BADARG / NONFINITE (it is the last
                                    record), or the loop state was inconsistent            */
#define RS_STITCH_ABORTED     4  /* a bounded wait inside the kernel ran out               */

typedef struct rs_stitch_record {    /* one invocation (40 bytes) */
    int32_t model;       /* RS_SLM / RS_LLM                                               */
    int32_t pos0;        /* position of the first token row it was fed                    */
    int32_t n_rows;      /* rows fed: the suffix it had not seen                          */
    int32_t reserved;
    rs_route_out out;    /* record of its last row; RS_FLAG_ACCEPT says the token was kept */
} rs_stitch_record;

typedef struct rs_stitch_result {    /* 32 bytes */
    int32_t status;      /* RS_STITCH_*                                                   */
    int32_t n_tokens;    /* tokens in d_seq: prompt + accepted                            */
    int32_t n_records;   /* invocations made = records written                            */
    int32_t seen_slm;    /* rows of d_seq the small model's cache holds                   */
    int32_t seen_llm;    /* same for the large model                                      */
    int32_t active;      /* the model that would run next                                 */
    int32_t n_target;    /* n_prompt + n_new                                              */
    int32_t reserved;
} rs_stitch_result;

/*   slm, llm      two models on the same device with the same head_dim; both use
 *                 KV slot seq_slot; neither may have sampling enabled
 *   d_seq         DEVICE int32[n_prompt + n_new]: the prompt on entry, prompt +
 *                 accepted tokens on return (read and written by the kernel)
 *   n_prompt      >= 1;  n_new >= 1;  n_prompt + n_new - 1 <= max_ctx of both
 *   seen_slm/llm  rows of the prompt already in each model's cache, 0 .. n_prompt - 1
 *   d_logit_scale DEVICE fp32[n_prompt + n_new] or NULL (= 1): entry p scales
 *                 the logits that predict position p
 *   eos           token that ends the run when accepted, or -1
 *   d_trace       DEVICE rs_stitch_record[max_records], 1 <= max_records <= 2^20;
 *                 2 * n_new records always suffice
 *   d_result      DEVICE rs_stitch_result, written when the kernel ends
 * Asynchronous on `stream`; synchronise it before reading d_seq, d_trace, d_result.
 * Calls on one pair must not overlap.
 * Errors: RS_EINVAL (null pointer, counts out of range, different devices or
 * head_dim), RS_ECAPACITY (the sequence does not fit a cache), RS_ENOTIMPL
 * (sampling enabled, or the device cannot launch cooperative kernels), RS_EHIP. */
rs_status rs_stitch_generate(rs_model *slm, rs_model *llm, int32_t seq_slot,
                             int32_t *d_seq, int32_t n_prompt, int32_t n_new,
                             int32_t seen_slm, int32_t seen_llm,
                             const float *d_logit_scale, float tau, int32_t eos,
                             rs_stitch_record *d_trace, int32_t max_records,
                             rs_stitch_result *d_result, void *stream);

/* rs_route for callers that cannot allocate device memory or hand over a
 * scratch buffer (code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation).  Same arguments, kernels and results as rs_route, but
 * the partial states go to a 256 KB array that lives inside the library's code
 * object on every GPU it runs on (held until the process ends).  The call never
 * allocates or frees; the first call on a device looks the array's device
 * address up once (make that first call outside a graph capture).
 *   n             1..64 rows; n * ceil(vocab / 1024, at most 128) partial
 *                 states of 32 bytes must fit the array
 * All calls on one GPU share the array: calls that overlap on one GPU (two
 * streams, two threads) race; calls on one stream are ordered.  Nothing has to
 * be cleared between calls (every state the merge reads is written by the same
 * call).
 * Errors: RS_EINVAL as rs_route; RS_ECAPACITY (n > 64, state count beyond the
 * array, device ordinal >= 64); RS_EHIP. */
rs_status rs_route_static(const float *d_logits, int32_t n, int32_t vocab,
                          const float *d_logit_scale, float tau, int32_t active,
                          rs_route_out *d_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RSTITCH_H */
