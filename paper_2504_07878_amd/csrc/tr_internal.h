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
    int vts;   // bf16 cache: V is stored transposed in blocks of 32 positions, [unit][kv head][position / 32][dim][position % 32]
               // (vts = positions per storage unit rounded up to 32), so that the V^T operand of one block of 32 keys is dh*64
               // consecutive bytes; 0: V is stored like K, [unit][kv head][position][dim] (fp32 cache)
    float eps;
    // Storage units of the cache. Contiguous cache (page = 0): one unit per slot, max_seq positions long. Paged cache:
    // a unit is a page of `page` positions (a power of two, multiple of 32) from a common pool of `units` pages; position
    // p of a slot lives in page ptab[slot * maxp + p / page] at position p % page.
    int page, maxp, units;
    const int *ptab;
};

__host__ __device__ inline int kv_unit_len(const Dims &D) { return D.page ? D.page : D.max_seq; }
__host__ __device__ inline int kv_unit_vts(const Dims &D) { return D.page ? D.page : D.vts; }

struct KvPlace { int unit, pos; };   // storage unit and position inside it
__device__ __forceinline__ KvPlace kv_place(const Dims &D, int slot, int pos)
{
    if (!D.page) return KvPlace{slot, pos};
    return KvPlace{D.ptab[(size_t)slot * D.maxp + pos / D.page], pos % D.page};
}

// element offsets of K[unit][head][pos][dim] and V[unit][head][pos][dim] inside one layer's cache (pos inside the unit)
__host__ __device__ inline size_t k_offset(const Dims &D, int unit, int head, int pos, int dim)
{
    return (((size_t)unit * D.Hkv + head) * kv_unit_len(D) + pos) * D.dh + dim;
}
__host__ __device__ inline size_t v_offset(const Dims &D, int unit, int head, int pos, int dim)
{
    const int vts = kv_unit_vts(D);
    return vts ? ((((size_t)unit * D.Hkv + head) * (vts >> 5) + (pos >> 5)) * D.dh + dim) * 32 + (pos & 31)
               : k_offset(D, unit, head, pos, dim);
}

// Weights of one decoder layer (device pointers in the model's storage type).
struct LayerW {
    const void *ln1, *wq, *wk, *wv, *bq, *bk, *bv, *wo, *ln2, *wg, *wu, *wd;
};

// Per-row metadata of the rows being processed (device arrays).
struct Rows {
    const int *slot, *pos, *tok;
    int n;
    // Device-side row count (NULL: all n rows are live). When given, only rows 0 .. *live - 1 belong to sequences: the rows
    // from *live on are padding of a launch whose size was fixed before the count was known. They are computed like any row
    // (on a valid slot at position 0) but must change no state, and with *live == 0 the large kernels return at once.
    const int *live;
};

// Attention partials that have not been merged yet: the consumer (the output projection of the GEMV path) merges them
// while it stages its activations, which saves a kernel when only a few rows are in flight.
struct AttnPending {
    const float *part;   // [row][head][nchunks][dh + 4]: unnormalised weighted V sums, then running max and sum of exponentials
    const int *pos;
    int nchunks, chunk;  // nchunks == 0: nothing pending, the merged rows are in the fp32 buffer
    // Set by the fused q|k|v + attention kernel: its partials cover the keys cached BEFORE the step only, and the row's own
    // new key and value join in the merge. qn: rotated queries [row][q width]; kvn: the new key and value as the cache holds
    // them (rounded to its type), [row][2][kv width]. NULL: the partials already cover the new key.
    const float *qn, *kvn;
    int G, kvw;
};

constexpr int MAX_SPLITS = 32;   // most split-K partial buffers a linear layer may produce

// residual update + RMSNorm + pack (see mfma_kernels.hip)
struct PrepArgs {
    float *x;                // residual stream, row of output m is gather[m], or row0 + m without a gather list
    int row0;
    const int *gather;
    const float *part;       // [nsplit][part_M][d] split-K partials to add first (rows indexed like x)
    int nsplit, part_M;
    int M, d;
    float eps;
    const bf16_t *gain;
    uint4 *pack;             // packed hi/lo activations out, or NULL: only the residual update is wanted
    int ncb;
    float *hn;               // optional fp32 copy of the normalised rows [M][d]
    float *hidden;           // optional exposed hidden state [M][d]
    int hidden_tap;
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
    int policy;              // TR_POLICY_*
    float *rpart;            // [n][TAIL_ROUTER_PARTS]: partial pre-activations of the router's output unit, one per workgroup of a row
    int *rcnt;               // [n]: arrival counters of those workgroups, zero before and after every launch (NULL: one workgroup per row)
    const float *r1;         // [n][r1_stride]: sums W1 . hidden of the router's first layer, computed by the LM-head launch (NULL: computed here)
    int r1_stride;
    const int *live;         // device-side row count (see Rows::live); rows from *live on report token -1, score 0, flag 0 and count nothing
    const int *cand;         // with scatter: index of output i in the caller's candidate list
    int32_t *scatter;        // scatter[cand[i]] = token of live row i (the other model's next-input buffer), or NULL
};
constexpr int TAIL_ROUTER_PARTS = 4;

// ---- launchers (enqueue only) ----
// rows 0..n-1 of one slot at positions base..base+n-1
void launch_iota_rows(hipStream_t s, int n, int slot, int base, int *d_slot, int *d_pos);
void launch_embed(hipStream_t s, int wdt, const void *E, const int *tok, int R, int d, float *x);
// row metadata from host arrays (passed in the kernel arguments, 256 rows per launch) and the embedding lookup of those rows
void launch_setup_rows_embed(hipStream_t s, int n, const int *slots, const int *toks, const int *poss, int *d_slot, int *d_tok, int *d_pos, int wdt,
                             const void *E, int d, float *x, const int *dev_toks, int vocab);   // dev_toks: device tokens [n] instead of toks (then NULL)
void launch_qkv(hipStream_t s, int wdt, int kdt, const Dims &D, const LayerW &w, const float *x, Rows rows, const float2 *rope,
                float *q, void *kc, void *vc);
// One or two decode rows of DIFFERENT slots, bf16 weights and cache, 64-wide heads, d <= 1024: the q|k|v projection and the attention
// over the cached keys in one launch (see qkv_attn_kernel). Returns false, having done nothing, when the case is not covered.
// kvn: scratch [rows][2][kv width] floats. The partials are left for the output projection to merge (pend).
bool launch_qkv_attention(hipStream_t s, int wdt, int kdt, const Dims &D, const LayerW &w, const float *x, Rows rows, int max_ctx,
                          const float2 *rope, float *q, void *kc, void *vc, float *part, size_t part_floats, float *kvn, AttnPending *pend);
// cnt: one zero-initialised int per (row, kv head), left at zero again by every launch (arrival counters of the
// workgroups that share a row when its context is split)
void launch_attention(hipStream_t s, int kdt, const Dims &D, const float *q, const void *kc, const void *vc, Rows rows, int max_ctx,
                      float *part, size_t part_floats, int *cnt, float *att, void *pack, int ncb, AttnPending *defer);
// bf16 cache, many rows of few sequences (prompts, catch-up segments): blocks of up to attention_block_rows() consecutive query
// rows of one slot share the keys and values they read. qblock[b] = first row * 8 + rows in block b (device array).
int attention_block_rows(const Dims &D);
void launch_attention_blocks(hipStream_t s, const Dims &D, const float *q, const void *kc, const void *vt, Rows rows, const int *qblock, int nblocks,
                             float *att, void *pack, int ncb);
void launch_attention_mfma(hipStream_t s, const Dims &D, const float *q, const void *kc, const void *vt, Rows rows, int max_ctx, float *part,
                           size_t part_floats, int *cnt, float *att, void *pack, int ncb, AttnPending *defer);
void launch_attn_merge(hipStream_t s, const Dims &D, const float *part, int nchunks, Rows rows, int chunk, float *att, void *pack, int ncb);
void launch_oproj(hipStream_t s, int wdt, const Dims &D, const void *wo, const float *att, const AttnPending &pend, int R, float *x);
// bf16 models wider than 1024 columns, up to 4 rows: launch_gateup / launch_down run kernels that keep the activations in registers
// (one workgroup per compute unit walks the output features) instead of staging them in LDS per group of features
bool ffn_rows_supported(int wdt, const Dims &D, int R);
void launch_gateup(hipStream_t s, int wdt, const Dims &D, const LayerW &w, const float *x, int R, float *h);
void launch_down(hipStream_t s, int wdt, const Dims &D, const void *wd, const float *h, int R, float *x);
void launch_tail(hipStream_t s, int wdt, const Dims &D, const TailArgs &t);
void launch_load_kv(hipStream_t s, int kdt, const Dims &D, int slot, int len, const void *k, const void *v, void *kc, void *vc);
void launch_reset_counters(hipStream_t s, long long *counters, int slot);
void launch_fill_int(hipStream_t s, int *p, int n, int value);   // p[0..n) = value
// Device-side selection of the rows of a decode step. Candidates i = 0..n-1 (slot cand_slot[i], input token tokens_dev[i]) whose
// flags_dev[i] is non-zero are taken in increasing i, at most n_max of them: row r gets the r-th of them, at the position the
// device-side length array holds for its slot, and that length grows by one. host_len[i] >= 0 first sets the slot's device-side
// length (the host knew it); -1 keeps the device's value. Rows past the count are padding: slot cand_slot[0], position 0, token 0.
// active[0] = rows taken, active[1] = candidates flagged, active[2 + r] = candidate of row r (-1 for padding). n <= 256.
void launch_active_setup(hipStream_t s, int n, const int *cand_slot, const int *host_len, const int *flags_dev, const int *tokens_dev, int n_max,
                         int vocab, int *dev_len, int *d_slot, int *d_tok, int *d_pos, int *active);

int tail_slice_rows();
void launch_tail_norm(hipStream_t s, int wdt, const Dims &D, const TailArgs &t);   // final RMSNorm of the streaming tail: t.x -> t.hn (and t.hidden)
void launch_tail_final(hipStream_t s, int wdt, const Dims &D, const TailArgs &t);
void launch_lmhead_gemv(hipStream_t s, int wdt, const Dims &D, const TailArgs &t);

// matrix-core path (bf16 weights, more than a few rows)
// pair_dh > 0: rows of each head reordered so that rotary partners are adjacent (q, k, v matrices), see repack_kernel
void launch_repack(hipStream_t s, const void *W, int N, int K, void *Wt, int dst_tile0, int dst_tile_stride, int pair_dh);
void launch_widen_bias(hipStream_t s, const void *b, int n, float *out);
void launch_prep(hipStream_t s, const PrepArgs &p);
void launch_pack(hipStream_t s, const float *in, int M, int K, void *pack, int ncb);
int mfma_ncb(int M);
// live (also below): device-side row count or NULL; the kernel returns at once when it is zero
void launch_gemm_partial(hipStream_t s, const void *Wt, const void *pack, int K, int N, int M, float *part, int *nsplit_out, const int *live = nullptr);
void launch_gemm_qkv(hipStream_t s, int kdt, const Dims &D, const void *Wt, const void *pack, const float *bias, Rows rows, const float2 *rope,
                     float *q, void *kc, void *vc);
// sumsq != NULL: the packed activations lack the 1/rms factor; it is applied to the sums from the rows' sums of squares sumsq[row * ss_stride + i], i < n_ss <= 32 <= ss_stride (a multiple of 4: every thread reads 8 consecutive floats of its row's first 32)
void launch_gemm_swiglu(hipStream_t s, const Dims &D, const void *Wt, const void *pack, int M, void *hpack, const int *live = nullptr,
                        const float *sumsq = nullptr, int n_ss = 0, int ss_stride = 0);
// Output projection without split-K whose epilogue updates the residual stream x and writes the next linear layer's packed input as
// x * gain (no 1/rms) together with the rows' sums of squares per tile range (returns how many tile ranges: the consumer's n_ss).
// Needs the whole reduction dimension inside one workgroup: gemm_oproj_residual_supported().
bool gemm_oproj_residual_supported(const Dims &D);
int launch_gemm_oproj_residual(hipStream_t s, const Dims &D, const void *Wt, const void *pack_a, int M, float *x, const void *gain, void *pack_out,
                               float *sumsq, int ss_stride, const int *live = nullptr);
// Wide models (K beyond what one workgroup keeps resident): every linear layer goes through split-K partials, and the
// layers with a non-linear epilogue are finished by a small kernel of their own.
// number of partial buffers launch_gemm_partial will produce for a K x N layer
int gemm_partial_splits(int K, int N);
// floats of partial sums such a layer may produce for any number of rows up to max_rows
size_t gemm_partial_floats(int K, int N, int max_rows);
// [q|k|v] = sum of partials + bias, rotary embedding, q out, cache append
void launch_qkv_finish(hipStream_t s, int kdt, const Dims &D, const float *part, int nsplit, const float *bias, Rows rows, const float2 *rope, float *q,
                       void *kc, void *vc);
// h = silu(gate) * up from the partials of the interleaved gate/up tiles, written as packed activations
void launch_swiglu_finish(hipStream_t s, const Dims &D, const float *part, int nsplit, int M, void *hpack);
// Softmax statistics of vocabulary slices of LMHEAD_FINISH_COLS columns from split-K partial logits [nsplit][M][V]:
// writes slice_part[slice][m] = {max, lowest argmax, sum-exp} (what the tail's final kernel merges) and, when asked, the logits.
constexpr int LMHEAD_FINISH_COLS = 2048;
void launch_lmhead_finish(hipStream_t s, const float *part, int nsplit, int M, int V, float *slice_part, float *logits);
int lmhead_mfma_wgs(int V, int router_tiles, int M);   // workgroups per 64-row group that own tiles, for M rows (most at M <= 64)
// router_tiles > 0: the matrix holds that many extra tiles after the vocabulary (the router's first layer); their raw sums go to r1[row][router_tiles * 32]
void launch_gemm_lmhead(hipStream_t s, const Dims &D, const void *Wt, const void *pack, int M, float *part, float *logits, float *r1, int router_tiles,
                        const int *live = nullptr);

}  // namespace tr
