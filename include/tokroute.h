/*
 * tokroute — token-level routing decode path for AMD MI355X (gfx950), C ABI.
 *
 * The library runs the on-device small model of a token-level routing system
 * (arxiv 2504.07878, Section 3: "on-device small model inference module" + "token routing
 * selection module") as a batched decode step with a key/value cache, followed by the
 * routing tail: final RMSNorm, LM head over the full vocabulary, softmax confidence and greedy
 * argmax, the MLP router on the exposed last-layer hidden state (Section 3.3, Figure 4) and the
 * rule "route the token to the large model when its score falls below the threshold"
 * (Section 3.1). A context without a router runs the same step for the large model that
 * generates the routed tokens (Section 3.3, Section 4).
 *
 * General conventions
 *  - Every function returns a status: TR_OK (0) or a negative TR_ERR_* code; nothing throws,
 *    aborts or prints. tr_last_error() gives the text of the last failure on a context.
 *  - Errors of the caller (TR_ERR_INVALID_ARG, TR_ERR_SHAPE, TR_ERR_STATE, TR_ERR_CAPACITY) are detected
 *    before anything is enqueued or changed: the context state (cache, page tables, sequence lengths,
 *    counters) is exactly as before the call. TR_ERR_HIP (a failed launch or copy; the code may also
 *    surface an earlier asynchronous failure of the HIP runtime) can occur after part of the call's work
 *    has been enqueued: the sequence lengths are not advanced, but cache contents, page tables and
 *    counters of the slots named in the call are undefined afterwards; reset those slots (tr_prefill)
 *    or destroy the context.
 *  - "device" pointers are HIP device memory of the current device; "host" pointers are
 *    ordinary host memory. The library allocates no device memory and creates no stream: the
 *    caller hands in a workspace and a hipStream_t (as void*; NULL = the default stream).
 *  - tr_prefill / tr_decode_step / tr_tail / tr_seq_load_kv only enqueue work on the stream and
 *    return; outputs are valid once the caller has synchronised that stream. Calls on one
 *    context must be issued from one thread at a time and on streams that are ordered with
 *    respect to each other.
 *  - Positions and token indices are 0-based (Figure 5, "token_index"): the token at cache
 *    index i is rotated with RoPE position i; a sequence's length is the number of tokens whose
 *    keys/values are cached; the token emitted by a step has index equal to that length.
 */
#ifndef TOKROUTE_H
#define TOKROUTE_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { TR_OK = 0, TR_ERR_INVALID_ARG = -1, TR_ERR_SHAPE = -2, TR_ERR_CAPACITY = -3, TR_ERR_STATE = -4, TR_ERR_HIP = -5 };
enum { TR_F32 = 0, TR_BF16 = 1 };
enum { TR_JOINT = 0, TR_SMALL_ONLY = 1 };                 /* inference modes of Section 3.1 */
enum { TR_ROUTE_IF_BELOW = 0, TR_ROUTE_IF_ABOVE = 1 };    /* Section 3.1 rule | the deferral rule of Section 2.2 */
enum { TR_POST_FINAL_NORM = 0, TR_PRE_FINAL_NORM = 1 };   /* which tensor is the "last-layer hidden state" */
/* What the routing score is. TR_POLICY_MLP: the MLP router on the hidden state (Section 3.1). TR_POLICY_CONFIDENCE:
 * the small model's own confidence, i.e. the maximum softmax probability (Figure 1: tokens of low confidence are
 * routed); needs no router weights. TR_POLICY_LINEAR: sigmoid(r_w2 . hidden + r_b2) with r_w2 of length d_model, the
 * shape of a learned deferral probability, normally used with TR_ROUTE_IF_ABOVE (Section 2.2). The comparison with
 * the threshold is route_dir in every case. */
enum { TR_POLICY_MLP = 0, TR_POLICY_CONFIDENCE = 1, TR_POLICY_LINEAR = 2 };

typedef struct tr_ctx tr_ctx;

/* Model and capacity description. The decoder is the pre-norm GQA / RoPE (half-split pairing) / SwiGLU
 * stack of the model family named in Section 4.2. Supported shapes (anything else: tr_workspace_bytes
 * returns 0 and tr_create TR_ERR_SHAPE): head_dim 64 or 128; n_q_heads a multiple of n_kv_heads with at
 * most 8 query heads per kv head; d_model and d_ffn multiples of 8; router_hidden <= 1024 (and
 * d_model <= 4096 with a router). Every such shape runs on the streaming kernels; bf16 models whose
 * d_model and d_ffn are multiples of 16 (d_ffn of 32 when d_model > 896) and d_model <= 4096 additionally
 * run batches of 3 or more rows on the matrix cores. */
typedef struct tr_config {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_theta;
    int32_t dtype;         /* storage type of every weight tensor: TR_F32 or TR_BF16 */
    int32_t kv_dtype;      /* storage type of the key/value cache (values are rounded to nearest-even on write) */
    int32_t tie_lm_head;   /* 1: the LM head is the token embedding matrix */
    int32_t router_hidden; /* width of the router's hidden layer; 0 = no router (score = 1, flag = 0) */
    float threshold;       /* initial routing threshold */
    int32_t route_dir;     /* TR_ROUTE_IF_BELOW: flag = score < threshold (strict) */
    int32_t hidden_tap;    /* tensor returned as hidden state and fed to the router */
    int32_t max_batch;     /* number of sequence slots */
    int32_t max_seq;       /* cache capacity per slot, in tokens */
    int32_t route_policy;  /* TR_POLICY_*; router_hidden is ignored unless TR_POLICY_MLP */
    int32_t kv_page;       /* 0: every slot owns max_seq contiguous cache positions. > 0: paged cache (the cache management
                              for alternating prefill and decode stages that Section 3 of the paper asks for): positions
                              live in pages of kv_page tokens (a power of two >= 32; kv_dtype must be TR_BF16) taken from a
                              common pool as sequences grow and given back by tr_seq_truncate / tr_prefill; tr_seq_fork
                              shares pages and a shared page is copied only when one side is about to write into it */
    int32_t kv_pool_pages; /* pages in the pool; 0 = max_batch * ceil(max_seq / kv_page) (no call can run out). With a smaller
                              pool a call that needs more pages than are free returns TR_ERR_CAPACITY and changes nothing */
} tr_config;

/* DEVICE pointers, row-major [out][in], all in tr_config.dtype. BORROWED: they must stay valid and
 * unchanged for the life of the context; the library never writes them. The pointer arrays
 * themselves are HOST arrays of n_layers device pointers and are copied by tr_create.
 * bq/bk/bv (arrays or single entries) and r_b1/r_b2 may be NULL = no bias. */
typedef struct tr_weights {
    const void *tok_emb;    /* [vocab][d_model] */
    const void *lm_head;    /* [vocab][d_model]; NULL when tie_lm_head */
    const void *final_norm; /* [d_model] */
    const void *const *ln1, *const *wq, *const *wk, *const *wv, *const *bq, *const *bk, *const *bv;
    const void *const *wo, *const *ln2, *const *wg, *const *wu, *const *wd;
    const void *r_w1, *r_b1, *r_w2, *r_b2; /* router: [rh][d_model], [rh], [rh], [1]; TR_POLICY_LINEAR: r_w2 is [d_model] */
} tr_weights;

/* Caller-owned DEVICE output buffers; row i belongs to the i-th sequence of the call.
 * token/conf/score/flag are required; hidden and logits may be NULL. */
typedef struct tr_out {
    int32_t *token; /* greedy next token: lowest index attaining the maximum logit */
    float *conf;    /* its softmax probability (Figure 1: "low confidence") */
    float *score;   /* router output in (0,1) (Section 3.1) */
    int32_t *flag;  /* 1 = route this token to the large model */
    float *hidden;  /* [n][d_model] exposed last-layer hidden state (Section 3.3) */
    float *logits;  /* [n][vocab] full logits, for debugging and parity checks; costs a write of n*vocab*4 bytes */
} tr_out;

/* General: a context is not thread-safe (the caller serialises the calls on one context; different contexts are
 * independent). With a paged cache (kv_page > 0) tr_prefill, tr_decode_step, tr_extend and tr_seq_load_kv also return
 * TR_ERR_CAPACITY when the page pool cannot supply the pages the call needs; like every error, that leaves all state
 * (cache, page tables, lengths, counters) as it was. */

/* Bytes of device workspace tr_create needs for this configuration (cache, tables, scratch); 0 if the
 * configuration is invalid. */
size_t tr_workspace_bytes(const tr_config *cfg);

/* Build a context over a caller-provided device workspace (256-byte aligned, at least
 * tr_workspace_bytes(cfg) bytes, owned by the caller and dedicated to this context until tr_destroy).
 * Synchronous: uploads small tables and clears counters with blocking copies.
 * Errors: TR_ERR_INVALID_ARG (NULL/misaligned), TR_ERR_SHAPE (unsupported shape), TR_ERR_CAPACITY
 * (workspace too small), TR_ERR_HIP. */
int tr_create(const tr_config *cfg, const tr_weights *w, void *workspace, size_t workspace_bytes, tr_ctx **out);

/* Frees the host-side context only. The caller must have synchronised all streams it used. */
void tr_destroy(tr_ctx *ctx);

/* Prefill (the paper's TTFT phase, Section 4.1): run the prompts of n distinct slots through the model,
 * fill their caches from position 0, reset their counters, and return the outputs of each prompt's LAST
 * position (the prediction of the first generated token and its route flag).
 * slots [n], tokens_flat [offsets[n]], offsets [n+1] (offsets[0] = 0) are HOST arrays, read before return.
 * Errors: TR_ERR_INVALID_ARG (bad slot/duplicate/token out of range/empty prompt), TR_ERR_CAPACITY
 * (prompt longer than max_seq). */
int tr_prefill(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *tokens_flat,
               const int32_t *offsets, const tr_out *out);

/* One decode step for n distinct slots: in_tokens[i] is appended to slot slots[i] (the caller supplies it
 * every step, so a token generated by the large model can replace the small model's, Section 3.1), the
 * model attends over the slot's cache, and the routing tail produces the outputs. Lengths grow by one;
 * n_generated grows by one and n_routed by the flag.
 * slots and in_tokens are HOST arrays, read before return.
 * Errors: TR_ERR_STATE (slot never prefilled/loaded), TR_ERR_CAPACITY (slot full), TR_ERR_INVALID_ARG. */
int tr_decode_step(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *in_tokens,
                   const tr_out *out);

/* The same step with the input tokens in DEVICE memory (int32 [n]), e.g. the token field of the previous step's tr_out:
 * a caller that does not need the flags on the host every step (small_only mode, or between two routing decisions it
 * has already taken) can enqueue many steps without a device-to-host copy in between. The tokens cannot be checked on the
 * host: values outside [0, vocab) are clamped into that range by the kernel. slots is a HOST array as above. */
int tr_decode_step_dev(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *in_tokens_dev,
                       const tr_out *out);

/* Decode step of the sequences that DEVICE-side flags select: the alternation of the two models inside one request
 * (opening of Section 3, Figure 2; Section 3.1: a flagged token is produced by the large model) without a trip of the
 * flags to the host. The caller names n candidate slots (HOST array, distinct, at most 256); flags_dev and in_tokens_dev
 * are DEVICE int32 arrays [n], typically the flag output of the small model's step and the tokens the large model has to
 * ingest. The candidates whose flag is non-zero are taken in increasing index, at most n_max of them (3 <= n_max <=
 * max_batch): each takes one decode step exactly like tr_decode_step (input token appended at the slot's length,
 * counters updated). Everything is enqueued with launches sized for n_max rows; rows past the number taken are padding
 * that changes no state, and when no candidate is flagged the large kernels return at once.
 * Outputs: row r of out (n_max rows) belongs to the r-th taken candidate; padding rows report token -1, conf 0, score 0,
 * flag 0. active_dev (DEVICE int32 [2 + n_max], required): [0] = rows taken, [1] = candidates flagged (larger than [0]
 * when more than n_max were flagged: those were NOT stepped; call again), [2 + r] = candidate index of row r (-1 for
 * padding). next_tokens_dev (DEVICE int32 [n] or NULL): entry i receives the emitted token if candidate i was taken and
 * is left alone otherwise: pass the small model's next-input buffer and the large model's token replaces the small model's.
 * Sequence lengths: which slots grew is only known on the device. The library keeps a device-side length array and
 * brings the host's lengths up to date, by synchronising the stream of the last such call, inside the next call that
 * needs them (tr_seq_len, tr_prefill, tr_decode_step, tr_extend, ...); consecutive tr_decode_step_active calls need no
 * synchronisation. Until then a candidate slot is assumed to have grown in every call (capacity check).
 * Needs a bf16 model that runs on the matrix cores and a contiguous cache (TR_ERR_SHAPE otherwise). Errors:
 * TR_ERR_INVALID_ARG, TR_ERR_STATE (candidate never prefilled), TR_ERR_CAPACITY (a candidate may be full). */
int tr_decode_step_active(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *flags_dev,
                          const int32_t *in_tokens_dev, int32_t n_max, int32_t *active_dev, int32_t *next_tokens_dev,
                          const tr_out *out);

/* Catch-up ("extend") step: each listed slot ingests the T >= 1 tokens of its segment, which another model
 * produced (opening of Section 3 and Figure 2: several rounds of prefill and decode inside one request; the prototype of
 * Section 4.1 re-runs the whole prefix instead), at positions len .. len+T-1 over its existing cache, and
 * returns the outputs of the last of them: the same result as T decode steps of which only the last is
 * visible. The counters move as for one decode step. Segments are given like prompts: tokens_flat (HOST)
 * holds them back to back, offsets (HOST, n+1 entries, offsets[0] = 0) delimit them; row i of out belongs to
 * slots[i]. Errors (a slot without a cache, a segment that does not fit, an empty segment, a bad token) are
 * detected before anything is enqueued and leave all state unchanged (TR_ERR_HIP: see the general conventions). */
int tr_extend(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *tokens_flat,
              const int32_t *offsets, const tr_out *out);

/* The routing tail alone on n rows of residual stream x (DEVICE, fp32 [n][d_model]): final RMSNorm, LM
 * head, softmax confidence + argmax, router, flag, i.e. the "token routing selection module" of Section 3
 * (MLP classifier on the last-layer hidden state and threshold rule of Section 3.1, hidden state exposed as
 * in Section 3.3) applied to rows the caller supplies. Touches no sequence state and no counters.
 * n <= max_batch. */
int tr_tail(tr_ctx *ctx, void *hip_stream, int32_t n, const float *x, const tr_out *out);

/* tr_tail for callers that cannot allocate or hand over device memory for scratch at the time of the call (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same computation and arguments, but
 * every intermediate (normalised rows, per-slice softmax statistics, router partial sums and arrival counters) lives in
 * a fixed array inside the library's own device image, 3.1 MB per GPU, held until the process ends; the context's
 * workspace is not touched and nothing is allocated or freed, by the library or through any runtime call. Limits
 * (TR_ERR_CAPACITY beyond them): n <= 64 rows, d_model <= 4096, vocab <= 262144. It always runs the streaming
 * (vector-ALU) tail kernels on the borrowed weights, so for models whose tr_tail uses the matrix cores the outputs agree
 * with tr_tail's to the library's floating-point tolerance rather than bit for bit; otherwise they are identical.
 * All calls on one GPU share that GPU's array (whatever the context): calls that overlap in time on one GPU race;
 * the caller serialises them (one stream, or events). Enqueues on the stream and returns, like tr_tail. */
int tr_tail_noalloc(tr_ctx *ctx, void *hip_stream, int32_t n, const float *x, const tr_out *out);

/* Threshold slider and mode switch of Section 3.1; they apply to calls made afterwards. */
int tr_set_threshold(tr_ctx *ctx, float threshold);
int tr_set_mode(tr_ctx *ctx, int32_t mode);

/* Host-side sequence state (infrastructure; the paper's request only carries the position as "token_index",
 * Figure 5). tr_seq_len: number of cached tokens of a slot (0 for a slot never filled). tr_seq_truncate rolls a
 * slot back to its first new_len tokens, 0 <= new_len <= length (a paged cache gives the freed pages back):
 * the rollback a caller needs when a token is replaced after the fact; the cache management Section 3 asks for. */
int tr_seq_len(const tr_ctx *ctx, int32_t slot, int32_t *len);
int tr_seq_truncate(tr_ctx *ctx, int32_t slot, int32_t new_len);

/* Copy a slot's whole state (cache up to its length, length, counters) into another slot, after which the two
 * continue independently from the same prefix: a shared prompt, or a rollback point kept aside (the cache management
 * for alternating stages that Section 3 asks for). Contiguous cache: enqueues device-to-device copies of the slot's cache
 * on the stream. Paged cache: no data moves, the copy refers to the same pages (TR_ERR_CAPACITY cannot occur here; a later
 * write into a shared page takes one page from the pool for a private copy). */
int tr_seq_fork(tr_ctx *ctx, void *hip_stream, int32_t src_slot, int32_t dst_slot);

/* Overwrite a slot's cache with len tokens of given keys/values (DEVICE pointers in kv_dtype, layout
 * [layer][kv_head][len][head_dim], keys already rotated) and set its length; counters are cleared.
 * Infrastructure (no passage of the paper): imports a cache computed elsewhere, e.g. the synthetic
 * 2048-token contexts of the large-model workload. Errors: TR_ERR_CAPACITY (len outside [1, max_seq], or
 * the page pool cannot supply the pages). */
int tr_seq_load_kv(tr_ctx *ctx, void *hip_stream, int32_t slot, int32_t len, const void *k, const void *v);

/* Device address of the per-slot counters, int64 [max_batch][2] = {n_generated, n_routed}
 * (the routing history of Figure 5 as counts). They live in the workspace and are updated by the tail
 * kernel; read them with a device-to-host copy after synchronising. */
int tr_counters_ptr(const tr_ctx *ctx, const int64_t **dev_counters);

/* Kernel timing for benchmarks (infrastructure). The launches of a step belong to kernel families (TR_KERNEL_*);
 * while timing is enabled, ONE launch of the selected family per call (tr_decode_step, tr_tail, each pass of
 * tr_prefill / tr_extend) is bracketed by two HIP events on the launch stream, and a third event is recorded straight
 * after the second, so that the cost of an event pair with nothing in between is measured in the same place of the
 * same stream. A family with several launches per call (one per layer) is sampled in turn: call k brackets launch
 * k mod (launches per call), so the timed launch costs every call the same overhead whatever the family.
 * tr_profile_select chooses the family (default TR_KERNEL_LMHEAD) and clears the sums. tr_profile_read synchronises the
 * events and returns, summed over the bracketed launches since enabling, the bracketed duration (ms_total) and the
 * empty intervals (ms_empty_pairs), in milliseconds, and their number: (ms_total - ms_empty_pairs) / launches
 * estimates the duration of one launch of the family. */
enum { TR_KERNEL_SETUP = 0,      /* row set-up + embedding lookup */
       TR_KERNEL_PREP,           /* residual update + RMSNorm (+ pack) ahead of a matrix-core layer; final norm of the tail */
       TR_KERNEL_QKV,            /* q|k|v projection, rotary embedding, cache append */
       TR_KERNEL_ATTENTION,      /* attention over the cache (and its merge kernel where there is one) */
       TR_KERNEL_OPROJ,          /* attention output projection */
       TR_KERNEL_GATEUP,         /* gate/up projections + SwiGLU */
       TR_KERNEL_DOWN,           /* FFN output projection */
       TR_KERNEL_LMHEAD,         /* LM head with the running softmax statistics */
       TR_KERNEL_TAIL_MERGE,     /* merge of the slices, router, flag, counters */
       TR_KERNEL_QKV_ATTENTION,  /* 1-2 row steps: projection and attention in one launch */
       TR_KERNEL_FAMILIES };
int tr_profile_select(tr_ctx *ctx, int32_t family);
int tr_profile_enable(tr_ctx *ctx, int32_t on);
int tr_profile_read(tr_ctx *ctx, double *ms_total, double *ms_empty_pairs, int64_t *launches);

/* Benchmark infrastructure: enqueues `launches` launches, one after the other on the stream, of a kernel of
 * `workgroups` workgroups of 256 threads that does nothing but one 4-byte store per thread into buf (DEVICE,
 * workgroups * 256 int32). What such a chain costs per launch is the floor under any step built as a chain of
 * dependent kernels. */
int tr_profile_chain(void *hip_stream, int32_t *buf, int32_t workgroups, int32_t launches);

const char *tr_last_error(const tr_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif
