// Internal declarations shared by the host scheduler and the gfx950 kernels of libtokroute.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace tr {

typedef uint16_t bf16_t;  // bf16 bit pattern

enum { DT_F32 = 0, DT_BF16 = 1 };

struct Dims {
    int L, d, Hq, Hkv, dh, F, V, qw, kvw, G, rh, max_batch, max_seq;
    float eps;
};

// Weights of one decoder layer (device pointers in the model's storage type).
struct LayerW {
    const void *ln1, *wq, *wk, *wv, *bq, *bk, *bv, *wo, *ln2, *wg, *wu, *wd;
};

// Per-row metadata of the rows being processed (device arrays).
struct Rows {
    const int *slot, *pos, *tok;
    int n;
};

struct TailArgs {
    const void *head, *final_norm, *r_w1, *r_b1, *r_w2, *r_b2;
    const float *x;          // [n][d] residual stream (rows picked through gather when given)
    const int *gather;       // row of x for output i, or NULL = i
    const int *slot;         // slot of output i (for the counters), or NULL
    int n;
    float *hn;               // scratch [n][d]: normalised rows
    float *part;             // scratch [nslices][n][4]: slice max, argmax, sum-exp
    int nslices, slice_rows;
    int32_t *token; float *conf, *score; int32_t *flag; float *hidden, *logits;
    long long *counters;     // [max_batch][2] or NULL
    int counter_mode;        // 0 none, 1 add (decode), 2 set (prefill)
    float threshold; int route_dir, mode, hidden_tap;
};

// ---- launchers (enqueue only) ----
void launch_setup_rows(hipStream_t s, int n, const int *slots, const int *toks, const int *poss, int *d_slot, int *d_tok, int *d_pos);
void launch_iota_rows(hipStream_t s, int n, int slot, int *d_slot, int *d_pos);
void launch_embed(hipStream_t s, int wdt, const void *E, const int *tok, int R, int d, float *x);
void launch_qkv(hipStream_t s, int wdt, int kdt, const Dims &D, const LayerW &w, const float *x, Rows rows, const float2 *rope,
                float *q, void *kc, void *vc);
void launch_attention(hipStream_t s, int kdt, const Dims &D, const float *q, const void *kc, const void *vc, Rows rows, int max_ctx,
                      float *part, size_t part_floats, float *att);
void launch_oproj(hipStream_t s, int wdt, const Dims &D, const void *wo, const float *att, int R, float *x);
void launch_gateup(hipStream_t s, int wdt, const Dims &D, const LayerW &w, const float *x, int R, float *h);
void launch_down(hipStream_t s, int wdt, const Dims &D, const void *wd, const float *h, int R, float *x);
void launch_tail(hipStream_t s, int wdt, const Dims &D, const TailArgs &t, hipEvent_t ev0, hipEvent_t ev1);
void launch_load_kv(hipStream_t s, int kdt, const Dims &D, int slot, int len, const void *k, const void *v, void *kc, void *vc);
void launch_reset_counters(hipStream_t s, long long *counters, int slot);

int tail_slice_rows();

}  // namespace tr
