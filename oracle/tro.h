/*
 * tro — plain CPU oracle for the token-level routing decode path.
 *
 * TEST INFRASTRUCTURE ONLY. This is the slow, obviously-correct definition that the
 * GPU library is checked against; it shares no code with it. Nothing in the product
 * path may call it.
 *
 * What it computes (arxiv 2504.07878): the on-device small model's forward pass
 * (Section 3, "on-device small model inference module"; the model is the Qwen2.5
 * decoder family named in Section 4.2), with the last-layer hidden state exposed as an
 * extra output (Section 3.3, Figure 4), the MLP router scoring that hidden state and
 * the rule "route to the large model when the score falls below the threshold"
 * (Section 3.1), the joint / small_only modes (Section 3.1) and the per-request token
 * index and routing history (Figure 5) kept as integer counters.
 *
 * The paper prints no decoder equations; the decoder is the standard pre-norm
 * GQA / RoPE (half-split pairing) / SwiGLU stack of the model family it names.
 *
 * Precision: every tensor is fp32; every reduction (dot products, mean of squares,
 * softmax sums) is accumulated in double and rounded to fp32 once. bf16 weights are
 * widened exactly to fp32 before use.
 *
 * Parity status: all functions are pinned by tests (invariants, closed forms, brute
 * force, and a third-party implementation of the same decoder family) EXCEPT the
 * choice of ReLU as the router's hidden activation and of the post-final-norm tensor
 * as "last-layer hidden state" relative to the authors' trained router:
 * "parity unpinned" for those two readings (the trained router is not available).
 */
#ifndef TRO_H
#define TRO_H
#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { TRO_F32 = 0, TRO_BF16 = 1 };
enum { TRO_OK = 0, TRO_ERR_INVALID_ARG = -1, TRO_ERR_SHAPE = -2, TRO_ERR_CAPACITY = -3, TRO_ERR_STATE = -4 };
enum { TRO_JOINT = 0, TRO_SMALL_ONLY = 1 };
enum { TRO_ROUTE_IF_BELOW = 0, TRO_ROUTE_IF_ABOVE = 1 };
enum { TRO_POST_FINAL_NORM = 0, TRO_PRE_FINAL_NORM = 1 };
/* What the routing score is: the MLP router of Section 3.1 (default); the small model's own confidence, i.e. the
 * maximum softmax probability (the "low confidence" of Figure 1 taken literally; no router weights);
 * a single linear head with a sigmoid, the shape of a learned deferral probability compared with ">" (Section 2.2;
 * the head's weights are r_w2 [d] and r_b2). The rule (below / above the threshold) stays route_dir. */
enum { TRO_POLICY_MLP = 0, TRO_POLICY_CONFIDENCE = 1, TRO_POLICY_LINEAR = 2 };

typedef struct tro_config {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_theta;
    int32_t dtype;          /* storage type of every weight tensor: TRO_F32 or TRO_BF16 */
    int32_t kv_dtype;       /* TRO_F32: cached K/V kept as computed; TRO_BF16: each cached K/V value is rounded to the
                               nearest-even bf16 when it is produced (the cache format of a bf16 deployment) */
    int32_t tie_lm_head;    /* 1: LM head = token embedding */
    int32_t router_hidden;  /* 0: no router (large model); score = 1, flag = 0 */
    float threshold;
    int32_t route_dir;
    int32_t hidden_tap;
    int32_t max_batch, max_seq;
    int32_t route_policy;
} tro_config;

/* All pointers are HOST pointers, borrowed (must outlive the context), row-major [out][in]. */
typedef struct tro_weights {
    const void *tok_emb;    /* [vocab][d] */
    const void *lm_head;    /* [vocab][d] or NULL when tied */
    const void *final_norm; /* [d] */
    const void *const *ln1, *const *wq, *const *wk, *const *wv, *const *bq, *const *bk, *const *bv;
    const void *const *wo, *const *ln2, *const *wg, *const *wu, *const *wd; /* each [n_layers]; bq/bk/bv arrays or entries may be NULL */
    const void *r_w1, *r_b1, *r_w2, *r_b2; /* [rh][d], [rh], [rh], [1] */
} tro_weights;

/* Caller-owned host buffers, row i = i-th sequence of the call. hidden/logits may be NULL. */
typedef struct tro_out {
    int32_t *token;
    float *conf, *score;
    int32_t *flag;
    float *hidden; /* [n][d] */
    float *logits; /* [n][vocab] */
} tro_out;

typedef struct tro_ctx tro_ctx;

int tro_create(const tro_config *, const tro_weights *, tro_ctx **out);
void tro_destroy(tro_ctx *);
/* Brute-force forward over the whole prompt of each listed slot (no cache is read); fills the
 * slot's cache as a by-product, resets its counters, returns the last position's outputs. */
int tro_prefill(tro_ctx *, int32_t n, const int32_t *slots, const int32_t *tokens_flat, const int32_t *offsets, const tro_out *);
/* One token per listed slot, attending over the slot's cache. */
int tro_decode_step(tro_ctx *, int32_t n, const int32_t *slots, const int32_t *in_tokens, const tro_out *);
/* Catch-up ("extend") step: each listed slot ingests the T >= 1 tokens of its segment, which some other model produced
 * (opening of Section 3 and Figure 2: several rounds of prefill and decode inside one request; the prototype of Section 4.1 re-runs
 * the whole prefix instead), at positions len .. len+T-1 over its existing cache. By definition this is T cached
 * decode steps of which only the last one is visible: its outputs are returned and the counters move as for one
 * decode step. Segments are given like prompts (tokens_flat, offsets[n+1]). */
int tro_extend(tro_ctx *, int32_t n, const int32_t *slots, const int32_t *tokens_flat, const int32_t *offsets, const tro_out *);
int tro_set_threshold(tro_ctx *, float);
int tro_set_mode(tro_ctx *, int32_t);
int tro_seq_len(const tro_ctx *, int32_t slot, int32_t *len);
int tro_seq_truncate(tro_ctx *, int32_t slot, int32_t new_len);
/* Copy a slot's whole state (cache up to its length, length, counters) into another slot: both continue independently
 * from the same prefix (one way of sharing a prompt between requests, or of keeping a rollback point). */
int tro_seq_fork(tro_ctx *, int32_t src_slot, int32_t dst_slot);
/* counters[2] = {n_generated, n_routed} of a slot */
int tro_counters(const tro_ctx *, int32_t slot, int64_t *counters);
/* Overwrite a slot's cache with given K/V ([layer][kv_head][len][head_dim], fp32) and set its length. */
int tro_seq_load_kv(tro_ctx *, int32_t slot, int32_t len, const float *k, const float *v);
/* Read back one layer of a slot's cache ([kv_head][len][head_dim] each). */
int tro_seq_read_kv(const tro_ctx *, int32_t slot, int32_t layer, float *k, float *v);

/* Brute-force forward returning EVERY position (no cache read or written):
 * hidden_all [T][d] (the tapped tensor), logits_all [T][vocab] (may be NULL). */
int tro_forward_all(const tro_ctx *, int32_t T, const int32_t *tokens, float *hidden_all, float *logits_all);

/* ---- the pieces, exported so that each can be pinned on its own ---- */
void tro_rmsnorm(const float *x, const void *gain, int32_t dtype, int32_t d, float eps, float *out);
void tro_rope(float *u, int32_t head_dim, int32_t pos, float theta);
void tro_linear(const void *W, const void *bias, int32_t dtype, const float *in, int32_t N, int32_t K, float *out);
/* one query head against ctx cached positions; K,V rows are strided by kv_stride floats */
void tro_attend(const float *q, const float *K, const float *V, int32_t ctx, int32_t head_dim, int32_t kv_stride, float *out);
float tro_silu(float u);
void tro_softmax_stats(const float *z, int32_t V, int32_t *argmax, float *max_prob);
float tro_router_score(const float *u, const void *w1, const void *b1, const void *w2, const void *b2, int32_t dtype, int32_t d, int32_t rh);
/* sigmoid(w . u + b) */
float tro_linear_score(const float *u, const void *w, const void *b, int32_t dtype, int32_t d);
int32_t tro_route_flag(float score, float threshold, int32_t route_dir, int32_t mode);
float tro_bf16_to_f32(uint16_t);
float tro_round_to_bf16(float); /* nearest-even, result widened back to fp32 */

#ifdef __cplusplus
}
#endif
#endif
