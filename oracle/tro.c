/*
 * tro — plain CPU oracle (see tro.h). TEST INFRASTRUCTURE ONLY.
 *
 * Every function is the textbook definition written out: no blocking, no fusion, no
 * online softmax. fp32 tensors, double accumulators. OpenMP is used only across
 * independent output elements, so results do not depend on the thread count.
 */
#include "tro.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

struct tro_ctx {
    tro_config c;
    tro_weights w;
    /* copies of the per-layer pointer arrays (the caller's arrays need not outlive create) */
    const void **ln1, **wq, **wk, **wv, **bq, **bk, **bv, **wo, **ln2, **wg, **wu, **wd;
    float *kc, *vc;       /* [layer][slot][pos][n_kv_heads*head_dim] */
    int32_t *len;         /* [max_batch], -1 = never prefilled */
    int64_t *counters;    /* [max_batch][2] */
    float threshold;
    int32_t mode;
};

/* ---------------------------------------------------------------- element access */

float tro_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16; /* bf16 is the upper half of an IEEE fp32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* Round to the nearest bf16 (ties to even), returned as fp32. NaN stays NaN. */
float tro_round_to_bf16(float f)
{
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return f;
    uint32_t lower = u & 0xffffu, keep = u & 0xffff0000u;
    if (lower > 0x8000u || (lower == 0x8000u && (keep & 0x10000u))) keep += 0x10000u;
    memcpy(&f, &keep, sizeof f);
    return f;
}

static void kv_round(const tro_config *c, float *p, int32_t n)
{
    if (c->kv_dtype == TRO_BF16)
        for (int32_t i = 0; i < n; ++i) p[i] = tro_round_to_bf16(p[i]);
}

static inline float w_at(const void *W, int32_t dtype, size_t i)
{
    if (dtype == TRO_F32) return ((const float *)W)[i];
    return tro_bf16_to_f32(((const uint16_t *)W)[i]);
}

/* sum_k W[row][k] * x[k], accumulated in double */
static double dot_row(const void *W, int32_t dtype, size_t row, int32_t K, const float *x)
{
    double acc = 0.0;
    if (dtype == TRO_F32) {
        const float *w = (const float *)W + row * (size_t)K;
#pragma omp simd reduction(+ : acc)
        for (int32_t k = 0; k < K; ++k) acc += (double)w[k] * (double)x[k];
    } else {
        const uint16_t *w = (const uint16_t *)W + row * (size_t)K;
#pragma omp simd reduction(+ : acc)
        for (int32_t k = 0; k < K; ++k) {
            uint32_t u = (uint32_t)w[k] << 16;
            float f;
            memcpy(&f, &u, sizeof f);
            acc += (double)f * (double)x[k];
        }
    }
    return acc;
}

/* ---------------------------------------------------------------- the pieces */

/* RMSNorm: out_j = x_j * g_j / sqrt(mean_j(x_j^2) + eps) */
void tro_rmsnorm(const float *x, const void *gain, int32_t dtype, int32_t d, float eps, float *out)
{
    double ss = 0.0;
    for (int32_t j = 0; j < d; ++j) ss += (double)x[j] * (double)x[j];
    double r = 1.0 / sqrt(ss / (double)d + (double)eps);
    for (int32_t j = 0; j < d; ++j) out[j] = (float)((double)x[j] * r * (double)w_at(gain, dtype, (size_t)j));
}

/* Rotary embedding of one head at position pos, half-split pairing (j, j + dh/2):
 * angle_j = pos * theta^(-2j/dh). */
void tro_rope(float *u, int32_t head_dim, int32_t pos, float theta)
{
    int32_t half = head_dim / 2;
    for (int32_t j = 0; j < half; ++j) {
        double ang = (double)pos * pow((double)theta, -2.0 * (double)j / (double)head_dim);
        double c = cos(ang), s = sin(ang);
        double a = (double)u[j], b = (double)u[j + half];
        u[j] = (float)(a * c - b * s);
        u[j + half] = (float)(b * c + a * s);
    }
}

/* out[t][n] = sum_k W[n][k] in[t][k] + bias[n], for T input rows */
static void linear_rows(const void *W, const void *bias, int32_t dtype, const float *in, int32_t T, int32_t N, int32_t K,
                        float *out)
{
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n) {
        double b = bias ? (double)w_at(bias, dtype, (size_t)n) : 0.0;
        for (int32_t t = 0; t < T; ++t)
            out[(size_t)t * N + n] = (float)(dot_row(W, dtype, (size_t)n, K, in + (size_t)t * K) + b);
    }
}

void tro_linear(const void *W, const void *bias, int32_t dtype, const float *in, int32_t N, int32_t K, float *out)
{
    linear_rows(W, bias, dtype, in, 1, N, K, out);
}

/* softmax(q.K_j / sqrt(dh)) weighted sum of V_j over j = 0..ctx-1, one query head */
void tro_attend(const float *q, const float *K, const float *V, int32_t ctx, int32_t head_dim, int32_t kv_stride, float *out)
{
    double *s = (double *)malloc(sizeof(double) * (size_t)ctx);
    double scale = 1.0 / sqrt((double)head_dim);
    double m = -INFINITY;
    for (int32_t j = 0; j < ctx; ++j) {
        double acc = 0.0;
        const float *kj = K + (size_t)j * kv_stride;
        for (int32_t e = 0; e < head_dim; ++e) acc += (double)q[e] * (double)kj[e];
        s[j] = acc * scale;
        if (s[j] > m) m = s[j];
    }
    double denom = 0.0;
    for (int32_t j = 0; j < ctx; ++j) {
        s[j] = exp(s[j] - m);
        denom += s[j];
    }
    for (int32_t e = 0; e < head_dim; ++e) {
        double acc = 0.0;
        for (int32_t j = 0; j < ctx; ++j) acc += s[j] * (double)V[(size_t)j * kv_stride + e];
        out[e] = (float)(acc / denom);
    }
    free(s);
}

float tro_silu(float u)
{
    return (float)((double)u / (1.0 + exp(-(double)u)));
}

/* argmax = lowest index attaining the maximum; max_prob = 1 / sum_v exp(z_v - max) */
void tro_softmax_stats(const float *z, int32_t V, int32_t *argmax, float *max_prob)
{
    int32_t best = 0;
    for (int32_t v = 1; v < V; ++v)
        if (z[v] > z[best]) best = v;
    double sum = 0.0;
    for (int32_t v = 0; v < V; ++v) sum += exp((double)z[v] - (double)z[best]);
    *argmax = best;
    *max_prob = (float)(1.0 / sum);
}

/* score = sigmoid( w2 . relu(W1 u + b1) + b2 ) */
float tro_router_score(const float *u, const void *w1, const void *b1, const void *w2, const void *b2, int32_t dtype, int32_t d,
                       int32_t rh)
{
    double acc = b2 ? (double)w_at(b2, dtype, 0) : 0.0;
    for (int32_t j = 0; j < rh; ++j) {
        float h = (float)(dot_row(w1, dtype, (size_t)j, d, u) + (b1 ? (double)w_at(b1, dtype, (size_t)j) : 0.0));
        if (h < 0.0f) h = 0.0f;
        acc += (double)w_at(w2, dtype, (size_t)j) * (double)h;
    }
    return (float)(1.0 / (1.0 + exp(-acc)));
}

/* score = sigmoid( w . u + b ): a single linear head (Section 2.2's deferral probability has this shape) */
float tro_linear_score(const float *u, const void *w, const void *b, int32_t dtype, int32_t d)
{
    double acc = (b ? (double)w_at(b, dtype, 0) : 0.0) + dot_row(w, dtype, 0, d, u);
    return (float)(1.0 / (1.0 + exp(-acc)));
}

/* Section 3.1: route when the score falls below the threshold (strict); small_only disables routing.
 * TRO_ROUTE_IF_ABOVE is the opposite sense used by the deferral rule of Section 2.2. */
int32_t tro_route_flag(float score, float threshold, int32_t route_dir, int32_t mode)
{
    if (mode != TRO_JOINT) return 0;
    if (route_dir == TRO_ROUTE_IF_BELOW) return score < threshold ? 1 : 0;
    return score > threshold ? 1 : 0;
}

/* ---------------------------------------------------------------- context */

static int check_config(const tro_config *c)
{
    if (c->n_layers < 1 || c->d_model < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 2 || c->d_ffn < 1 ||
        c->vocab < 1 || c->max_batch < 1 || c->max_seq < 1)
        return TRO_ERR_SHAPE;
    if (c->head_dim % 2 || c->n_q_heads % c->n_kv_heads) return TRO_ERR_SHAPE;
    if (c->dtype != TRO_F32 && c->dtype != TRO_BF16) return TRO_ERR_INVALID_ARG;
    if (c->kv_dtype != TRO_F32 && c->kv_dtype != TRO_BF16) return TRO_ERR_INVALID_ARG;
    if (c->router_hidden < 0) return TRO_ERR_SHAPE;
    if (c->route_policy < TRO_POLICY_MLP || c->route_policy > TRO_POLICY_LINEAR) return TRO_ERR_INVALID_ARG;
    return TRO_OK;
}

static const void **copy_ptrs(const void *const *src, int32_t n)
{
    const void **dst = (const void **)calloc((size_t)n, sizeof(void *));
    if (src)
        for (int32_t i = 0; i < n; ++i) dst[i] = src[i];
    return dst;
}

int tro_create(const tro_config *c, const tro_weights *w, tro_ctx **out)
{
    if (!c || !w || !out) return TRO_ERR_INVALID_ARG;
    int rc = check_config(c);
    if (rc) return rc;
    if (!w->tok_emb || !w->final_norm || (!c->tie_lm_head && !w->lm_head)) return TRO_ERR_INVALID_ARG;
    if (!w->ln1 || !w->wq || !w->wk || !w->wv || !w->wo || !w->ln2 || !w->wg || !w->wu || !w->wd) return TRO_ERR_INVALID_ARG;
    if (c->route_policy == TRO_POLICY_MLP && c->router_hidden > 0 && (!w->r_w1 || !w->r_w2)) return TRO_ERR_INVALID_ARG;
    if (c->route_policy == TRO_POLICY_LINEAR && !w->r_w2) return TRO_ERR_INVALID_ARG;
    tro_ctx *x = (tro_ctx *)calloc(1, sizeof *x);
    x->c = *c;
    x->w = *w;
    int32_t L = c->n_layers;
    x->ln1 = copy_ptrs(w->ln1, L); x->wq = copy_ptrs(w->wq, L); x->wk = copy_ptrs(w->wk, L); x->wv = copy_ptrs(w->wv, L);
    x->bq = copy_ptrs(w->bq, L); x->bk = copy_ptrs(w->bk, L); x->bv = copy_ptrs(w->bv, L);
    x->wo = copy_ptrs(w->wo, L); x->ln2 = copy_ptrs(w->ln2, L); x->wg = copy_ptrs(w->wg, L); x->wu = copy_ptrs(w->wu, L);
    x->wd = copy_ptrs(w->wd, L);
    size_t kvw = (size_t)c->n_kv_heads * c->head_dim;
    size_t n = (size_t)L * c->max_batch * c->max_seq * kvw;
    x->kc = (float *)calloc(n, sizeof(float));
    x->vc = (float *)calloc(n, sizeof(float));
    x->len = (int32_t *)malloc(sizeof(int32_t) * (size_t)c->max_batch);
    for (int32_t i = 0; i < c->max_batch; ++i) x->len[i] = -1;
    x->counters = (int64_t *)calloc((size_t)c->max_batch * 2, sizeof(int64_t));
    x->threshold = c->threshold;
    x->mode = TRO_JOINT;
    if (!x->kc || !x->vc) { tro_destroy(x); return TRO_ERR_CAPACITY; }
    *out = x;
    return TRO_OK;
}

void tro_destroy(tro_ctx *x)
{
    if (!x) return;
    free(x->ln1); free(x->wq); free(x->wk); free(x->wv); free(x->bq); free(x->bk); free(x->bv);
    free(x->wo); free(x->ln2); free(x->wg); free(x->wu); free(x->wd);
    free(x->kc); free(x->vc); free(x->len); free(x->counters);
    free(x);
}

int tro_set_threshold(tro_ctx *x, float t) { if (!x) return TRO_ERR_INVALID_ARG; x->threshold = t; return TRO_OK; }
int tro_set_mode(tro_ctx *x, int32_t m)
{
    if (!x || (m != TRO_JOINT && m != TRO_SMALL_ONLY)) return TRO_ERR_INVALID_ARG;
    x->mode = m;
    return TRO_OK;
}
int tro_seq_len(const tro_ctx *x, int32_t slot, int32_t *len)
{
    if (!x || !len || slot < 0 || slot >= x->c.max_batch) return TRO_ERR_INVALID_ARG;
    *len = x->len[slot] < 0 ? 0 : x->len[slot];
    return TRO_OK;
}
int tro_seq_truncate(tro_ctx *x, int32_t slot, int32_t new_len)
{
    if (!x || slot < 0 || slot >= x->c.max_batch) return TRO_ERR_INVALID_ARG;
    if (x->len[slot] < 0) return TRO_ERR_STATE;
    if (new_len < 0 || new_len > x->len[slot]) return TRO_ERR_INVALID_ARG;
    x->len[slot] = new_len;
    return TRO_OK;
}
int tro_seq_fork(tro_ctx *x, int32_t src, int32_t dst)
{
    if (!x || src < 0 || src >= x->c.max_batch || dst < 0 || dst >= x->c.max_batch || src == dst) return TRO_ERR_INVALID_ARG;
    if (x->len[src] < 0) return TRO_ERR_STATE;
    const tro_config *c = &x->c;
    size_t kvw = (size_t)c->n_kv_heads * c->head_dim;
    for (int32_t l = 0; l < c->n_layers; ++l)
        for (int32_t p = 0; p < x->len[src]; ++p) {
            size_t so = (((size_t)l * c->max_batch + src) * c->max_seq + p) * kvw, d_ = (((size_t)l * c->max_batch + dst) * c->max_seq + p) * kvw;
            memcpy(x->kc + d_, x->kc + so, sizeof(float) * kvw);
            memcpy(x->vc + d_, x->vc + so, sizeof(float) * kvw);
        }
    x->len[dst] = x->len[src];
    x->counters[2 * dst] = x->counters[2 * src];
    x->counters[2 * dst + 1] = x->counters[2 * src + 1];
    return TRO_OK;
}

int tro_counters(const tro_ctx *x, int32_t slot, int64_t *counters)
{
    if (!x || !counters || slot < 0 || slot >= x->c.max_batch) return TRO_ERR_INVALID_ARG;
    counters[0] = x->counters[2 * slot];
    counters[1] = x->counters[2 * slot + 1];
    return TRO_OK;
}

static float *cache_at(float *base, const tro_config *c, int32_t layer, int32_t slot, int32_t pos)
{
    size_t kvw = (size_t)c->n_kv_heads * c->head_dim;
    return base + (((size_t)layer * c->max_batch + slot) * c->max_seq + pos) * kvw;
}

int tro_seq_load_kv(tro_ctx *x, int32_t slot, int32_t len, const float *k, const float *v)
{
    if (!x || !k || !v || slot < 0 || slot >= x->c.max_batch) return TRO_ERR_INVALID_ARG;
    if (len < 1 || len > x->c.max_seq) return TRO_ERR_CAPACITY;
    const tro_config *c = &x->c;
    int32_t dh = c->head_dim;
    for (int32_t l = 0; l < c->n_layers; ++l)
        for (int32_t g = 0; g < c->n_kv_heads; ++g)
            for (int32_t p = 0; p < len; ++p) {
                size_t src = (((size_t)l * c->n_kv_heads + g) * len + p) * dh;
                memcpy(cache_at(x->kc, c, l, slot, p) + g * dh, k + src, sizeof(float) * dh);
                memcpy(cache_at(x->vc, c, l, slot, p) + g * dh, v + src, sizeof(float) * dh);
                kv_round(c, cache_at(x->kc, c, l, slot, p) + g * dh, dh);
                kv_round(c, cache_at(x->vc, c, l, slot, p) + g * dh, dh);
            }
    x->len[slot] = len;
    x->counters[2 * slot] = 0;
    x->counters[2 * slot + 1] = 0;
    return TRO_OK;
}

int tro_seq_read_kv(const tro_ctx *x, int32_t slot, int32_t layer, float *k, float *v)
{
    if (!x || !k || !v || slot < 0 || slot >= x->c.max_batch || layer < 0 || layer >= x->c.n_layers) return TRO_ERR_INVALID_ARG;
    if (x->len[slot] < 0) return TRO_ERR_STATE;
    const tro_config *c = &x->c;
    int32_t dh = c->head_dim, len = x->len[slot];
    for (int32_t g = 0; g < c->n_kv_heads; ++g)
        for (int32_t p = 0; p < len; ++p) {
            memcpy(k + ((size_t)g * len + p) * dh, cache_at(x->kc, c, layer, slot, p) + g * dh, sizeof(float) * dh);
            memcpy(v + ((size_t)g * len + p) * dh, cache_at(x->vc, c, layer, slot, p) + g * dh, sizeof(float) * dh);
        }
    return TRO_OK;
}

/* ---------------------------------------------------------------- tail (one row) */

/* x: residual stream after the last layer. Writes the i-th row of out. */
static void tail_row(const tro_ctx *cx, const float *x, const tro_out *out, int32_t i, float *logits_tmp, int32_t *flag_out)
{
    const tro_config *c = &cx->c;
    int32_t d = c->d_model, V = c->vocab;
    float *hn = (float *)malloc(sizeof(float) * (size_t)d);
    tro_rmsnorm(x, cx->w.final_norm, c->dtype, d, c->rms_eps, hn);
    const void *head = c->tie_lm_head ? cx->w.tok_emb : cx->w.lm_head;
    float *z = (out && out->logits) ? out->logits + (size_t)i * V : logits_tmp;
    tro_linear(head, NULL, c->dtype, hn, V, d, z);
    int32_t tok;
    float conf;
    tro_softmax_stats(z, V, &tok, &conf);
    const float *tap = c->hidden_tap == TRO_POST_FINAL_NORM ? hn : x;
    float score = 1.0f;
    int32_t flag = 0;
    if (c->route_policy == TRO_POLICY_CONFIDENCE) {
        score = conf;
        flag = tro_route_flag(score, cx->threshold, c->route_dir, cx->mode);
    } else if (c->route_policy == TRO_POLICY_LINEAR) {
        score = tro_linear_score(tap, cx->w.r_w2, cx->w.r_b2, c->dtype, d);
        flag = tro_route_flag(score, cx->threshold, c->route_dir, cx->mode);
    } else if (c->router_hidden > 0) {
        score = tro_router_score(tap, cx->w.r_w1, cx->w.r_b1, cx->w.r_w2, cx->w.r_b2, c->dtype, d, c->router_hidden);
        flag = tro_route_flag(score, cx->threshold, c->route_dir, cx->mode);
    }
    if (out) {
        if (out->token) out->token[i] = tok;
        if (out->conf) out->conf[i] = conf;
        if (out->score) out->score[i] = score;
        if (out->flag) out->flag[i] = flag;
        if (out->hidden) memcpy(out->hidden + (size_t)i * d, tap, sizeof(float) * (size_t)d);
    }
    *flag_out = flag;
    free(hn);
}

/* ---------------------------------------------------------------- brute-force forward over a whole sequence */

/* Runs all layers over tokens[0..T). x_out [T][d] receives the residual stream after the last layer.
 * When kdst/vdst are given (a slot's cache base for layer 0 .. L-1 via cache_at), each layer's rotated K and V are stored. */
static void forward_sequence(const tro_ctx *cx, int32_t T, const int32_t *tokens, float *x, tro_ctx *store, int32_t store_slot)
{
    const tro_config *c = &cx->c;
    int32_t d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, dh = c->head_dim, F = c->d_ffn;
    int32_t qw = Hq * dh, kvw = Hkv * dh, group = Hq / Hkv;
    float *n = (float *)malloc(sizeof(float) * (size_t)T * d);
    float *q = (float *)malloc(sizeof(float) * (size_t)T * qw);
    float *k = (float *)malloc(sizeof(float) * (size_t)T * kvw);
    float *v = (float *)malloc(sizeof(float) * (size_t)T * kvw);
    float *a = (float *)malloc(sizeof(float) * (size_t)T * qw);
    float *o = (float *)malloc(sizeof(float) * (size_t)T * d);
    float *g = (float *)malloc(sizeof(float) * (size_t)T * F);
    float *u = (float *)malloc(sizeof(float) * (size_t)T * F);

    for (int32_t t = 0; t < T; ++t)
        for (int32_t j = 0; j < d; ++j) x[(size_t)t * d + j] = w_at(cx->w.tok_emb, c->dtype, (size_t)tokens[t] * d + j);

    for (int32_t l = 0; l < c->n_layers; ++l) {
        for (int32_t t = 0; t < T; ++t) tro_rmsnorm(x + (size_t)t * d, cx->ln1[l], c->dtype, d, c->rms_eps, n + (size_t)t * d);
        linear_rows(cx->wq[l], cx->bq[l], c->dtype, n, T, qw, d, q);
        linear_rows(cx->wk[l], cx->bk[l], c->dtype, n, T, kvw, d, k);
        linear_rows(cx->wv[l], cx->bv[l], c->dtype, n, T, kvw, d, v);
        for (int32_t t = 0; t < T; ++t) {
            for (int32_t h = 0; h < Hq; ++h) tro_rope(q + (size_t)t * qw + h * dh, dh, t, c->rope_theta);
            for (int32_t h = 0; h < Hkv; ++h) tro_rope(k + (size_t)t * kvw + h * dh, dh, t, c->rope_theta);
            kv_round(c, k + (size_t)t * kvw, kvw);
            kv_round(c, v + (size_t)t * kvw, kvw);
        }
        if (store)
            for (int32_t t = 0; t < T; ++t) {
                memcpy(cache_at(store->kc, c, l, store_slot, t), k + (size_t)t * kvw, sizeof(float) * kvw);
                memcpy(cache_at(store->vc, c, l, store_slot, t), v + (size_t)t * kvw, sizeof(float) * kvw);
            }
        /* causal: position t sees keys 0..t */
#pragma omp parallel for collapse(2) schedule(dynamic)
        for (int32_t t = 0; t < T; ++t)
            for (int32_t h = 0; h < Hq; ++h) {
                int32_t kvh = h / group;
                tro_attend(q + (size_t)t * qw + h * dh, k + kvh * dh, v + kvh * dh, t + 1, dh, kvw, a + (size_t)t * qw + h * dh);
            }
        linear_rows(cx->wo[l], NULL, c->dtype, a, T, d, qw, o);
        for (size_t i = 0; i < (size_t)T * d; ++i) x[i] += o[i];
        for (int32_t t = 0; t < T; ++t) tro_rmsnorm(x + (size_t)t * d, cx->ln2[l], c->dtype, d, c->rms_eps, n + (size_t)t * d);
        linear_rows(cx->wg[l], NULL, c->dtype, n, T, F, d, g);
        linear_rows(cx->wu[l], NULL, c->dtype, n, T, F, d, u);
        for (size_t i = 0; i < (size_t)T * F; ++i) g[i] = tro_silu(g[i]) * u[i];
        linear_rows(cx->wd[l], NULL, c->dtype, g, T, d, F, o);
        for (size_t i = 0; i < (size_t)T * d; ++i) x[i] += o[i];
    }
    free(n); free(q); free(k); free(v); free(a); free(o); free(g); free(u);
}

static int tokens_ok(const tro_config *c, const int32_t *tok, int32_t n)
{
    for (int32_t i = 0; i < n; ++i)
        if (tok[i] < 0 || tok[i] >= c->vocab) return 0;
    return 1;
}

int tro_forward_all(const tro_ctx *cx, int32_t T, const int32_t *tokens, float *hidden_all, float *logits_all)
{
    if (!cx || !tokens || T < 1) return TRO_ERR_INVALID_ARG;
    const tro_config *c = &cx->c;
    if (!tokens_ok(c, tokens, T)) return TRO_ERR_INVALID_ARG;
    int32_t d = c->d_model, V = c->vocab;
    float *x = (float *)malloc(sizeof(float) * (size_t)T * d);
    float *hn = (float *)malloc(sizeof(float) * (size_t)d);
    forward_sequence(cx, T, tokens, x, NULL, 0);
    const void *head = c->tie_lm_head ? cx->w.tok_emb : cx->w.lm_head;
    for (int32_t t = 0; t < T; ++t) {
        tro_rmsnorm(x + (size_t)t * d, cx->w.final_norm, c->dtype, d, c->rms_eps, hn);
        if (hidden_all)
            memcpy(hidden_all + (size_t)t * d, c->hidden_tap == TRO_POST_FINAL_NORM ? hn : x + (size_t)t * d, sizeof(float) * (size_t)d);
        if (logits_all) tro_linear(head, NULL, c->dtype, hn, V, d, logits_all + (size_t)t * V);
    }
    free(x); free(hn);
    return TRO_OK;
}

static int slots_ok(const tro_ctx *cx, int32_t n, const int32_t *slots)
{
    if (n < 1 || n > cx->c.max_batch) return 0;
    for (int32_t i = 0; i < n; ++i) {
        if (slots[i] < 0 || slots[i] >= cx->c.max_batch) return 0;
        for (int32_t j = 0; j < i; ++j)
            if (slots[j] == slots[i]) return 0;
    }
    return 1;
}

int tro_prefill(tro_ctx *cx, int32_t n, const int32_t *slots, const int32_t *tokens_flat, const int32_t *offsets, const tro_out *out)
{
    if (!cx || !slots || !tokens_flat || !offsets || !out) return TRO_ERR_INVALID_ARG;
    if (!slots_ok(cx, n, slots)) return TRO_ERR_INVALID_ARG;
    const tro_config *c = &cx->c;
    if (offsets[0] != 0) return TRO_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i) {
        int32_t T = offsets[i + 1] - offsets[i];
        if (T < 1) return TRO_ERR_INVALID_ARG;
        if (T > c->max_seq) return TRO_ERR_CAPACITY;
    }
    if (!tokens_ok(c, tokens_flat, offsets[n])) return TRO_ERR_INVALID_ARG;
    float *logits_tmp = (float *)malloc(sizeof(float) * (size_t)c->vocab);
    for (int32_t i = 0; i < n; ++i) {
        int32_t T = offsets[i + 1] - offsets[i], slot = slots[i], flag;
        float *x = (float *)malloc(sizeof(float) * (size_t)T * c->d_model);
        forward_sequence(cx, T, tokens_flat + offsets[i], x, cx, slot);
        tail_row(cx, x + (size_t)(T - 1) * c->d_model, out, i, logits_tmp, &flag);
        cx->len[slot] = T;
        cx->counters[2 * slot] = 1;
        cx->counters[2 * slot + 1] = flag;
        free(x);
    }
    free(logits_tmp);
    return TRO_OK;
}

/* ---------------------------------------------------------------- cached decode of one token per slot */

int tro_decode_step(tro_ctx *cx, int32_t n, const int32_t *slots, const int32_t *in_tokens, const tro_out *out)
{
    if (!cx || !slots || !in_tokens || !out) return TRO_ERR_INVALID_ARG;
    if (!slots_ok(cx, n, slots)) return TRO_ERR_INVALID_ARG;
    const tro_config *c = &cx->c;
    if (!tokens_ok(c, in_tokens, n)) return TRO_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i) {
        if (cx->len[slots[i]] < 0) return TRO_ERR_STATE;
        if (cx->len[slots[i]] >= c->max_seq) return TRO_ERR_CAPACITY;
    }
    int32_t d = c->d_model, Hq = c->n_q_heads, Hkv = c->n_kv_heads, dh = c->head_dim, F = c->d_ffn;
    int32_t qw = Hq * dh, kvw = Hkv * dh, group = Hq / Hkv;
    float *x = (float *)malloc(sizeof(float) * (size_t)d), *nrm = (float *)malloc(sizeof(float) * (size_t)d);
    float *q = (float *)malloc(sizeof(float) * (size_t)qw), *a = (float *)malloc(sizeof(float) * (size_t)qw);
    float *o = (float *)malloc(sizeof(float) * (size_t)d);
    float *g = (float *)malloc(sizeof(float) * (size_t)F), *u = (float *)malloc(sizeof(float) * (size_t)F);
    float *logits_tmp = (float *)malloc(sizeof(float) * (size_t)c->vocab);
    for (int32_t i = 0; i < n; ++i) {
        int32_t slot = slots[i], pos = cx->len[slot], flag;
        for (int32_t j = 0; j < d; ++j) x[j] = w_at(cx->w.tok_emb, c->dtype, (size_t)in_tokens[i] * d + j);
        for (int32_t l = 0; l < c->n_layers; ++l) {
            float *kn = cache_at(cx->kc, c, l, slot, pos), *vn = cache_at(cx->vc, c, l, slot, pos);
            tro_rmsnorm(x, cx->ln1[l], c->dtype, d, c->rms_eps, nrm);
            tro_linear(cx->wq[l], cx->bq[l], c->dtype, nrm, qw, d, q);
            tro_linear(cx->wk[l], cx->bk[l], c->dtype, nrm, kvw, d, kn);
            tro_linear(cx->wv[l], cx->bv[l], c->dtype, nrm, kvw, d, vn);
            for (int32_t h = 0; h < Hq; ++h) tro_rope(q + h * dh, dh, pos, c->rope_theta);
            for (int32_t h = 0; h < Hkv; ++h) tro_rope(kn + h * dh, dh, pos, c->rope_theta);
            kv_round(c, kn, kvw);
            kv_round(c, vn, kvw);
            const float *K0 = cache_at(cx->kc, c, l, slot, 0), *V0 = cache_at(cx->vc, c, l, slot, 0);
#pragma omp parallel for schedule(static)
            for (int32_t h = 0; h < Hq; ++h) {
                int32_t kvh = h / group;
                tro_attend(q + h * dh, K0 + kvh * dh, V0 + kvh * dh, pos + 1, dh, kvw, a + h * dh);
            }
            tro_linear(cx->wo[l], NULL, c->dtype, a, d, qw, o);
            for (int32_t j = 0; j < d; ++j) x[j] += o[j];
            tro_rmsnorm(x, cx->ln2[l], c->dtype, d, c->rms_eps, nrm);
            tro_linear(cx->wg[l], NULL, c->dtype, nrm, F, d, g);
            tro_linear(cx->wu[l], NULL, c->dtype, nrm, F, d, u);
            for (int32_t j = 0; j < F; ++j) g[j] = tro_silu(g[j]) * u[j];
            tro_linear(cx->wd[l], NULL, c->dtype, g, d, F, o);
            for (int32_t j = 0; j < d; ++j) x[j] += o[j];
        }
        tail_row(cx, x, out, i, logits_tmp, &flag);
        cx->len[slot] = pos + 1;
        cx->counters[2 * slot] += 1;
        cx->counters[2 * slot + 1] += flag;
    }
    free(x); free(nrm); free(q); free(a); free(o); free(g); free(u); free(logits_tmp);
    return TRO_OK;
}

/* ---------------------------------------------------------------- catch-up: T cached decode steps, the last one visible */

int tro_extend(tro_ctx *cx, int32_t n, const int32_t *slots, const int32_t *tokens_flat, const int32_t *offsets, const tro_out *out)
{
    if (!cx || !slots || !tokens_flat || !offsets || !out) return TRO_ERR_INVALID_ARG;
    if (!slots_ok(cx, n, slots)) return TRO_ERR_INVALID_ARG;
    const tro_config *c = &cx->c;
    if (offsets[0] != 0) return TRO_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i) {
        int32_t T = offsets[i + 1] - offsets[i];
        if (T < 1) return TRO_ERR_INVALID_ARG;
        if (cx->len[slots[i]] < 0) return TRO_ERR_STATE;
        if ((int64_t)cx->len[slots[i]] + T > c->max_seq) return TRO_ERR_CAPACITY;
    }
    if (!tokens_ok(c, tokens_flat, offsets[n])) return TRO_ERR_INVALID_ARG;
    /* outputs of the steps that stay invisible go here */
    int32_t tok_tmp, flag_tmp;
    float conf_tmp, score_tmp;
    tro_out hidden_steps = {&tok_tmp, &conf_tmp, &score_tmp, &flag_tmp, NULL, NULL};
    for (int32_t i = 0; i < n; ++i) {
        int32_t T = offsets[i + 1] - offsets[i], slot = slots[i];
        const int32_t *tok = tokens_flat + offsets[i];
        int64_t saved[2] = {cx->counters[2 * slot], cx->counters[2 * slot + 1]};
        for (int32_t t = 0; t + 1 < T; ++t) {
            int rc = tro_decode_step(cx, 1, &slot, tok + t, &hidden_steps);
            if (rc != TRO_OK) return rc;
        }
        cx->counters[2 * slot] = saved[0];
        cx->counters[2 * slot + 1] = saved[1];
        tro_out last = {out->token + i, out->conf + i, out->score + i, out->flag + i,
                        out->hidden ? out->hidden + (size_t)i * c->d_model : NULL, out->logits ? out->logits + (size_t)i * c->vocab : NULL};
        int rc = tro_decode_step(cx, 1, &slot, tok + T - 1, &last);
        if (rc != TRO_OK) return rc;
    }
    return TRO_OK;
}
