// Host side of libtokroute: the C ABI declared in include/tokroute.h. Validates arguments, keeps the per-slot
// bookkeeping (sequence lengths on the host; n_generated / n_routed counters on the device, next to the
// flags that feed them) and enqueues the fixed kernel sequence of a step on the caller's stream.
#include "../../include/tokroute.h"
#include "tr_internal.h"
#include "kv_pages.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace tr;

// ---- scratch of the entry point that allocates nothing (tr_tail_noalloc): one fixed array per GPU, held until the
// process ends. In host code the array's NAME is only a handle for the runtime: the device address is looked up once per
// device with hipGetSymbolAddress and only that address is ever handed to kernels.
constexpr int NOALLOC_MAX_ROWS = 64, NOALLOC_MAX_D = 4096, NOALLOC_MAX_SLICES = 2048;
constexpr size_t NOALLOC_HN = 0;                                                              // [rows][d] normalised rows
constexpr size_t NOALLOC_PART = NOALLOC_HN + (size_t)NOALLOC_MAX_ROWS * NOALLOC_MAX_D;        // [slices][rows] x 4 floats
constexpr size_t NOALLOC_RPART = NOALLOC_PART + (size_t)NOALLOC_MAX_SLICES * NOALLOC_MAX_ROWS * 4;   // [rows][TAIL_ROUTER_PARTS]
constexpr size_t NOALLOC_RCNT = NOALLOC_RPART + (size_t)NOALLOC_MAX_ROWS * TAIL_ROUTER_PARTS; // [rows] ints
constexpr size_t NOALLOC_FLOATS = NOALLOC_RCNT + NOALLOC_MAX_ROWS;
static __device__ __align__(256) float scratch[NOALLOC_FLOATS];


namespace {

constexpr size_t ALIGN = 256;
size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct Layout {
    size_t k_layer_bytes, v_layer_bytes;
    size_t kc, vc, rope, counters, slot, tok, pos, gather, out_slot, x, q, att, h, hn, attn_part, tail_part, total;
    size_t attn_part_floats;
    size_t attn_cnt;
    size_t tail_rpart, tail_rcnt;
    size_t ptab;       // paged cache: device page table [max_batch][maxp]
    size_t r1;         // sums of the router's first layer, [max_batch][router_tiles * 32], written by the LM-head launch
    int router_tiles;  // tiles of router weight rows appended to the repacked head matrix (0: the merge kernel computes the router itself)
    size_t qblock;     // query-row blocks of a pass (prompts, catch-up segments): first row * 8 + rows
    size_t kvn;        // new keys and values of up to two decode rows, [row][2][kv width] floats (fused q|k|v + attention kernel)
    size_t dev_len;    // device-side sequence lengths [max_batch], used by the steps whose rows are selected on the device
    size_t sumsq;      // rows' sums of squares per tile range of the output projection, [max_rows][ss_stride] floats (deferred RMSNorm)
    int ss_stride;     // floats per row: 32, the most tile ranges the fused output projection has (one cache line per row)
    int maxp, pool;    // pages per slot (table row length) and pages in the pool; 0 for the contiguous cache
    int max_rows, nslices;
    // matrix-core paths: repacked weights, packed activations, split-K partials.
    // mfma: K of the layers with a non-linear epilogue fits one workgroup (d <= 896), those layers are fused GEMMs and the
    // LM head runs on the matrix cores too. split: wider models, every layer through split-K partials plus finishing kernels.
    bool mfma, split;
    bool split_head;   // wide model whose LM head runs through split-K partial logits (vocabulary a multiple of 8)
    size_t wt_layers, wt_layer_stride, wt_qkv, wt_o, wt_gu, wt_d, wt_head, bias, bias_stride;
    size_t pack_d, pack_a, pack_h, part;
};

// Up to this many rows the streaming GEMV kernels are used where the matrix-core path exists. Measured decode step of the
// 0.5B-class model (context 256): 0.63 ms at 1 row and 0.83 at 2 on the streaming kernels, which then climb to 1.15 (3 rows),
// 1.26 (4) and 1.40 (8), while the matrix-core path takes 1.05 ms from 3 to 16 rows.
constexpr int GEMV_MAX_ROWS = 2;

// The matrix-core kernels keep 896 columns of K per workgroup resident, and the layers with a non-linear
// epilogue (rotary, SwiGLU, softmax statistics) cannot split K across workgroups.
bool mfma_supported(const tr_config *c)
{
    return c->dtype == TR_BF16 && c->d_model % 16 == 0 && c->d_model <= 896 && c->d_ffn % 16 == 0 && c->head_dim % 32 == 0 &&
           (c->max_batch > GEMV_MAX_ROWS || c->max_seq > GEMV_MAX_ROWS);
}

bool split_supported(const tr_config *c)
{
    return c->dtype == TR_BF16 && c->d_model % 16 == 0 && c->d_model > 896 && c->d_model <= 4096 && c->d_ffn % 32 == 0 &&
           c->head_dim % 32 == 0 && (c->max_batch > 4 || c->max_seq > 4);
}

size_t elem_size(int dt) { return dt == TR_F32 ? 4 : 2; }

int check_config(const tr_config *c)
{
    if (!c) return TR_ERR_INVALID_ARG;
    if (c->n_layers < 1 || c->d_model < 8 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 8 || c->vocab < 1 || c->max_batch < 1 ||
        c->max_seq < 1)
        return TR_ERR_SHAPE;
    if (c->head_dim != 64 && c->head_dim != 128) return TR_ERR_SHAPE;           // attention kernels are built for these
    if (c->n_q_heads % c->n_kv_heads || c->n_q_heads / c->n_kv_heads > 8) return TR_ERR_SHAPE;
    if (c->d_model % 8 || c->d_ffn % 8) return TR_ERR_SHAPE;                    // 16-byte loads along the reduction dimension
    if (c->router_hidden < 0 || c->router_hidden > 1024 || (c->router_hidden > 0 && c->d_model > 4096)) return TR_ERR_SHAPE;
    if ((c->dtype != TR_F32 && c->dtype != TR_BF16) || (c->kv_dtype != TR_F32 && c->kv_dtype != TR_BF16)) return TR_ERR_INVALID_ARG;
    if (c->route_dir != TR_ROUTE_IF_BELOW && c->route_dir != TR_ROUTE_IF_ABOVE) return TR_ERR_INVALID_ARG;
    if (c->route_policy < TR_POLICY_MLP || c->route_policy > TR_POLICY_LINEAR) return TR_ERR_INVALID_ARG;
    if (c->hidden_tap != TR_POST_FINAL_NORM && c->hidden_tap != TR_PRE_FINAL_NORM) return TR_ERR_INVALID_ARG;
    if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f)) return TR_ERR_INVALID_ARG;
    if ((long long)c->max_batch * c->max_seq >= (1ll << 31)) return TR_ERR_CAPACITY;   // row and position indices are ints
    if (c->kv_page < 0 || c->kv_pool_pages < 0 || (c->kv_page == 0 && c->kv_pool_pages != 0)) return TR_ERR_INVALID_ARG;
    if (c->kv_page) {   // pages: a power of two of at least 32 positions; the matrix-core attention kernels (bf16 cache) walk them
        if (c->kv_page < 32 || (c->kv_page & (c->kv_page - 1)) || c->kv_dtype != TR_BF16) return TR_ERR_SHAPE;
        const long long per_slot = (c->max_seq + (long long)c->kv_page - 1) / c->kv_page;
        const long long pool = c->kv_pool_pages ? c->kv_pool_pages : c->max_batch * per_slot;
        if (pool * c->kv_page >= (1ll << 31)) return TR_ERR_CAPACITY;
    }
    return TR_OK;
}

Layout make_layout(const tr_config *c)
{
    Layout L{};
    const size_t kvw = (size_t)c->n_kv_heads * c->head_dim, qw = (size_t)c->n_q_heads * c->head_dim;
    const int vts = c->kv_dtype == TR_BF16 ? (c->max_seq + 31) / 32 * 32 : 0;   // bf16 cache: V transposed, rows padded to 32 positions
    L.maxp = c->kv_page ? (c->max_seq + c->kv_page - 1) / c->kv_page : 0;
    L.pool = c->kv_page ? (c->kv_pool_pages ? c->kv_pool_pages : c->max_batch * L.maxp) : 0;
    if (c->kv_page) {   // a pool of pages instead of one block per slot
        L.k_layer_bytes = L.v_layer_bytes = (size_t)L.pool * c->kv_page * kvw * elem_size(c->kv_dtype);
    } else {
        L.k_layer_bytes = (size_t)c->max_batch * c->max_seq * kvw * elem_size(c->kv_dtype);
        L.v_layer_bytes = (size_t)c->max_batch * (vts ? vts : c->max_seq) * kvw * elem_size(c->kv_dtype);
    }
    // rows of one pass over the weights: a decode batch, one whole prompt, and room to pack several prompts or catch-up
    // segments into a pass (more 64-row groups per launch: the activations a workgroup keeps are reused for more tiles)
    L.max_rows = std::max({c->max_batch, c->max_seq, std::min(8192, c->max_batch * c->max_seq)});
    L.nslices = (c->vocab + tail_slice_rows() - 1) / tail_slice_rows();
    const size_t R = (size_t)L.max_rows;
    // room for up to 32 context splits of a full decode batch
    L.attn_part_floats = (size_t)c->max_batch * c->n_q_heads * 32 * (c->head_dim + 4);
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.kc = take(L.k_layer_bytes * c->n_layers); L.vc = take(L.v_layer_bytes * c->n_layers);
    L.rope = take((size_t)c->max_seq * (c->head_dim / 2) * sizeof(float2));
    L.counters = take((size_t)c->max_batch * 2 * sizeof(long long));
    L.slot = take(R * 4); L.tok = take(R * 4); L.pos = take(R * 4); L.gather = take((size_t)c->max_batch * 4); L.out_slot = take((size_t)c->max_batch * 4);
    L.x = take(R * c->d_model * 4); L.q = take(R * qw * 4); L.att = take(R * qw * 4); L.h = take(R * c->d_ffn * 4);
    L.hn = take((size_t)c->max_batch * c->d_model * 4);
    L.attn_part = take(L.attn_part_floats * 4);
    L.attn_cnt = take(R * c->n_kv_heads * 4);
    L.tail_rpart = take((size_t)c->max_batch * TAIL_ROUTER_PARTS * 4); L.tail_rcnt = take((size_t)c->max_batch * 4);
    L.ptab = take((size_t)c->max_batch * (L.maxp ? L.maxp : 1) * 4);
    L.mfma = mfma_supported(c);
    L.split = split_supported(c);
    // fused matrix-core tail with the MLP router on the normalised hidden state: the router's first layer rides along in the LM-head launch
    L.router_tiles = (L.mfma && c->route_policy == TR_POLICY_MLP && c->router_hidden > 0 && c->hidden_tap == TR_POST_FINAL_NORM) ? (c->router_hidden + 31) / 32 : 0;
    L.r1 = take((size_t)c->max_batch * (L.router_tiles ? L.router_tiles : 1) * 32 * 4);
    const int head_wgs = L.mfma ? lmhead_mfma_wgs(c->vocab, L.router_tiles, 1) : 0;
    L.tail_part = take((size_t)(L.nslices > head_wgs ? L.nslices : head_wgs) * c->max_batch * sizeof(float4));
    if (L.mfma || L.split) {
        const size_t d = (size_t)c->d_model, F = (size_t)c->d_ffn;
        auto tiles = [](size_t n) { return (n + 31) / 32; };
        const size_t tile_d = d / 16 * 1024, tile_q = qw / 16 * 1024, tile_f = F / 16 * 1024;   // bytes of one 32-row tile over K
        size_t o2 = 0;
        L.wt_qkv = o2; o2 += tiles(qw + 2 * kvw) * tile_d;
        L.wt_o = o2;   o2 += tiles(d) * tile_q;
        L.wt_gu = o2;  o2 += 2 * tiles(F) * tile_d;
        L.wt_d = o2;   o2 += tiles(d) * tile_f;
        L.wt_layer_stride = align_up(o2);
        L.wt_layers = take(L.wt_layer_stride * c->n_layers);
        L.wt_head = (L.mfma || (L.split && c->vocab % 8 == 0)) ? take((tiles((size_t)c->vocab) + L.router_tiles) * tile_d) : 0;
        L.split_head = L.split && c->vocab % 8 == 0;
        L.bias_stride = align_up((qw + 2 * kvw) * 4);
        L.bias = take(L.bias_stride * c->n_layers);
        const size_t groups = (R + 63) / 64;
        L.pack_d = take(groups * (d / 16) * 4 * 1024);
        L.pack_a = take(groups * (qw / 16) * 4 * 1024);
        L.pack_h = take(groups * (F / 16) * 4 * 1024);
        // largest set of split-K partials any layer leaves, over all row counts of a pass
        const int Ri = (int)R;
        size_t part_floats = std::max(gemm_partial_floats((int)qw, (int)d, Ri), gemm_partial_floats((int)F, (int)d, Ri));
        if (L.split) {
            const size_t n_qkv = qw + 2 * kvw, n_gu = 2 * tiles(F) * 32;
            part_floats = std::max({part_floats, gemm_partial_floats((int)d, (int)n_qkv, Ri), gemm_partial_floats((int)d, (int)n_gu, Ri)});
        }
        if (L.split_head)   // partial logits of a tail call: up to max_batch rows
            part_floats = std::max(part_floats, gemm_partial_floats((int)d, c->vocab, c->max_batch));
        const size_t part_bytes = part_floats * 4;
        L.part = take(part_bytes);
    }
    L.qblock = take(R * 4);
    L.kvn = take(2 * 2 * kvw * 4);
    L.dev_len = take((size_t)c->max_batch * 4);
    L.ss_stride = 32;
    L.sumsq = take((size_t)L.ss_stride * R * 4);
    L.total = off;
    return L;
}

constexpr int MAX_DEVICES = 64;
float *g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each GPU, looked up on first use

// Device address of the static scratch array on the current device (looked up once per device), or an error.
hipError_t scratch_address(float **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        float *p = nullptr;
        e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct tr_ctx {
    tr_config c;
    Dims D;
    Layout lay;
    char *ws;
    std::vector<LayerW> layers;
    const void *tok_emb, *head, *final_norm, *r_w1, *r_b1, *r_w2, *r_b2;
    std::vector<int> len;   // -1 = never prefilled
    KvPages pages;          // paged cache only (c.kv_page > 0)
    int qblocks = 0;        // > 0: the rows of the current pass are grouped into this many query-row blocks (see ingest)
    // Steps whose rows are selected on the device (tr_decode_step_active) advance the lengths of the selected slots in a device
    // array; the host does not know which slots those were. Until the next call that needs lengths, len[] of a candidate slot
    // is what the host last knew, ahead[] counts the steps it may have taken since, and the device array is the truth.
    std::vector<int> ahead;
    bool unsynced = false;
    hipStream_t active_stream = nullptr;
    const int *live = nullptr;       // device-side row count of the pass being enqueued (NULL: every row is live)
    const int *cand = nullptr;       // ... and the candidate index of each of its rows, for the token scatter
    int32_t *scatter = nullptr;
    float threshold;
    int mode;
    std::string err;
    // kernel timing: while enabled, ONE launch of the selected kernel family per call is bracketed by events (the launches of
    // the family take turns from call to call, so that every layer is sampled)
    bool profile = false;
    std::vector<hipEvent_t> ev;   // triples: before the kernel, after it, and once more straight away
    size_t ev_used = 0;
    double prof_ms = 0.0, prof_gap_ms = 0.0;
    long long prof_launches = 0;
    int prof_family = TR_KERNEL_LMHEAD;
    int prof_seen = 0, prof_pick = 0;   // launches of the family seen in this call; the one to bracket

    template <typename T> T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }
    void *kc_layer(int l) const { return ws + lay.kc + (size_t)l * lay.k_layer_bytes; }
    void *vc_layer(int l) const { return ws + lay.vc + (size_t)l * lay.v_layer_bytes; }
    char *wt(int l, size_t which) const { return ws + lay.wt_layers + (size_t)l * lay.wt_layer_stride + which; }
    float *bias(int l) const { return reinterpret_cast<float *>(ws + lay.bias + (size_t)l * lay.bias_stride); }
    bool use_mfma(int rows) const { return lay.mfma && rows > GEMV_MAX_ROWS; }
    // wide models: the streaming kernels that stage the rows in LDS slow down with the rows (7B-class gate/up: 46 us at 1 row, 52 at 2,
    // 69 at 4) while the matrix-core path is nearly flat in them: it takes over from 3 rows on, except where run_layers finds the
    // register-resident streaming kernels usable (2 to 4 rows)
    bool use_split(int rows) const { return lay.split && rows > 2; }
};

namespace {

int fail(tr_ctx *ctx, int code, const char *msg)
{
    if (ctx) ctx->err = msg;
    return code;
}

int fail_hip(tr_ctx *ctx, hipError_t e, const char *what)
{
    if (ctx) ctx->err = std::string(what) + ": " + hipGetErrorString(e);
    return TR_ERR_HIP;
}

bool check_out(const tr_out *o) { return o && o->token && o->conf && o->score && o->flag; }

bool slots_ok(const tr_ctx *ctx, int n, const int32_t *slots)
{
    if (n < 1 || n > ctx->c.max_batch) return false;
    std::vector<char> seen((size_t)ctx->c.max_batch, 0);
    for (int i = 0; i < n; ++i) {
        if (slots[i] < 0 || slots[i] >= ctx->c.max_batch || seen[(size_t)slots[i]]) return false;
        seen[(size_t)slots[i]] = 1;
    }
    return true;
}

void drain_profile(tr_ctx *ctx)
{
    for (size_t i = 0; i + 2 < ctx->ev_used; i += 3) {
        float ms = 0.f, gap = 0.f;
        if (hipEventSynchronize(ctx->ev[i + 2]) == hipSuccess && hipEventElapsedTime(&ms, ctx->ev[i], ctx->ev[i + 1]) == hipSuccess &&
            hipEventElapsedTime(&gap, ctx->ev[i + 1], ctx->ev[i + 2]) == hipSuccess) {
            ctx->prof_ms += ms;
            ctx->prof_gap_ms += gap;
            ctx->prof_launches += 1;
        }
    }
    ctx->ev_used = 0;
}

void next_events(tr_ctx *ctx, hipEvent_t *e0, hipEvent_t *e1, hipEvent_t *e2)
{
    *e0 = *e1 = *e2 = nullptr;
    if (!ctx->profile) return;
    if (ctx->ev_used + 3 > ctx->ev.size()) drain_profile(ctx);
    *e0 = ctx->ev[ctx->ev_used];
    *e1 = ctx->ev[ctx->ev_used + 1];
    *e2 = ctx->ev[ctx->ev_used + 2];
    ctx->ev_used += 3;
}

// Brackets the launches made during its lifetime with events when they belong to the selected family and it is this
// launch's turn (see tr_ctx::prof_pick).
struct Bracket {
    hipStream_t s;
    hipEvent_t e1 = nullptr, e2 = nullptr;
    Bracket(tr_ctx *ctx, hipStream_t stream, int family) : s(stream)
    {
        if (!ctx->profile || family != ctx->prof_family) return;
        if (ctx->prof_seen++ != ctx->prof_pick) return;
        hipEvent_t e0;
        next_events(ctx, &e0, &e1, &e2);
        if (e0) (void)hipEventRecord(e0, s);
    }
    ~Bracket()
    {
        if (e1) (void)hipEventRecord(e1, s);
        if (e2) (void)hipEventRecord(e2, s);
    }
    Bracket(const Bracket &) = delete;
    Bracket &operator=(const Bracket &) = delete;
};

// End of a call's launches: the next call brackets the family's next launch.
void profile_next_turn(tr_ctx *ctx)
{
    if (ctx->profile) ctx->prof_pick = ctx->prof_seen > 0 ? (ctx->prof_pick + 1) % ctx->prof_seen : 0;
    ctx->prof_seen = 0;
}

// All layers over the rows currently described by the device row arrays. Returns the number of split-K partial
// buffers of the last down projection that still have to be added to the residual stream (matrix-core path).
// distinct_slots: every row belongs to a different slot (a decode step), so no row reads a key another row appends.
int run_layers(tr_ctx *ctx, hipStream_t s, int R, int max_ctx, bool embed = true, bool distinct_slots = false)
{
    const Dims &D = ctx->D;
    const Layout &L = ctx->lay;
    Rows rows{ctx->at<int>(L.slot), ctx->at<int>(L.pos), ctx->at<int>(L.tok), R, ctx->live};
    const int *live = ctx->live;
    float *x = ctx->at<float>(L.x), *q = ctx->at<float>(L.q), *att = ctx->at<float>(L.att), *h = ctx->at<float>(L.h);
    const size_t attn_part_floats = R <= ctx->c.max_batch ? L.attn_part_floats : 0;
    if (embed) { Bracket br(ctx, s, TR_KERNEL_SETUP); launch_embed(s, ctx->c.dtype, ctx->tok_emb, rows.tok, R, D.d, x); }
    // attention of one layer: blocks of query rows that share their keys when the pass was grouped that way, rows one by one otherwise
    auto attend = [&](int l, const float *q_, Rows rows_, int max_ctx_, float *part_, size_t part_floats_, int *cnt_, float *att_, void *pack_, int ncb_,
                      AttnPending *defer_) {
        Bracket br(ctx, s, TR_KERNEL_ATTENTION);
        if (ctx->qblocks > 0) {
            if (defer_) defer_->nchunks = 0;
            launch_attention_blocks(s, D, q_, ctx->kc_layer(l), ctx->vc_layer(l), rows_, ctx->at<int>(L.qblock), ctx->qblocks, att_, pack_, ncb_);
        } else {
            launch_attention(s, ctx->c.kv_dtype, D, q_, ctx->kc_layer(l), ctx->vc_layer(l), rows_, max_ctx_, part_, part_floats_, cnt_, att_, pack_, ncb_, defer_);
        }
    };
    // Wide model, 3 and 4 rows whose count the host knows: the streaming kernels that keep the rows in registers (the last branch below)
    // take fewer launches than the matrix-core path with its partials and finishing kernels (7B-class step at 3 rows: 3.9 -> 3.5 ms).
    const bool rows_kernels = !live && ffn_rows_supported(ctx->c.dtype, D, R);
    if (ctx->use_split(R) && !rows_kernels) {
        // wide model: every linear layer leaves split-K partials; rotary/cache append and SwiGLU are finished by kernels of their own
        const int ncb = mfma_ncb(R);
        float *part = ctx->at<float>(L.part);
        int pending = 0, ns = 0;
        for (int l = 0; l < D.L; ++l) {
            const LayerW &w = ctx->layers[(size_t)l];
            PrepArgs p{};
            p.x = x; p.row0 = 0; p.part = part; p.nsplit = pending; p.part_M = R; p.M = R; p.d = D.d; p.eps = D.eps;
            p.gain = (const bf16_t *)w.ln1; p.pack = ctx->at<uint4>(L.pack_d); p.ncb = ncb;
            { Bracket br(ctx, s, TR_KERNEL_PREP); launch_prep(s, p); }
            {
                Bracket br(ctx, s, TR_KERNEL_QKV);
                launch_gemm_partial(s, ctx->wt(l, L.wt_qkv), ctx->at<uint4>(L.pack_d), D.d, D.qw + 2 * D.kvw, R, part, &ns, live);
                launch_qkv_finish(s, ctx->c.kv_dtype, D, part, ns, ctx->bias(l), rows, ctx->at<float2>(L.rope), q, ctx->kc_layer(l), ctx->vc_layer(l));
            }
            attend(l, q, rows, max_ctx, ctx->at<float>(L.attn_part),
                             attn_part_floats, ctx->at<int>(L.attn_cnt), att, ctx->at<uint4>(L.pack_a), ncb, nullptr);
            { Bracket br(ctx, s, TR_KERNEL_OPROJ); launch_gemm_partial(s, ctx->wt(l, L.wt_o), ctx->at<uint4>(L.pack_a), D.qw, D.d, R, part, &pending, live); }
            p.nsplit = pending; p.gain = (const bf16_t *)w.ln2;
            { Bracket br(ctx, s, TR_KERNEL_PREP); launch_prep(s, p); }
            {
                Bracket br(ctx, s, TR_KERNEL_GATEUP);
                launch_gemm_partial(s, ctx->wt(l, L.wt_gu), ctx->at<uint4>(L.pack_d), D.d, 2 * ((D.F + 31) / 32) * 32, R, part, &ns, live);
                launch_swiglu_finish(s, D, part, ns, R, ctx->at<uint4>(L.pack_h));
            }
            { Bracket br(ctx, s, TR_KERNEL_DOWN); launch_gemm_partial(s, ctx->wt(l, L.wt_d), ctx->at<uint4>(L.pack_h), D.F, D.d, R, part, &pending, live); }
        }
        return pending;
    }
    if (!ctx->use_mfma(R) || rows_kernels) {
        AttnPending pend{};
        for (int l = 0; l < D.L; ++l) {
            const LayerW &w = ctx->layers[(size_t)l];
            // one or two rows of a decode step: projection and attention over the cached keys in one launch, merged by the output projection
            bool fused = false;
            if (distinct_slots) {
                Bracket br(ctx, s, TR_KERNEL_QKV_ATTENTION);
                fused = launch_qkv_attention(s, ctx->c.dtype, ctx->c.kv_dtype, D, w, x, rows, max_ctx, ctx->at<float2>(L.rope), q, ctx->kc_layer(l),
                                             ctx->vc_layer(l), ctx->at<float>(L.attn_part), attn_part_floats, ctx->at<float>(L.kvn), &pend);
            }
            if (!fused) {
                { Bracket br(ctx, s, TR_KERNEL_QKV); launch_qkv(s, ctx->c.dtype, ctx->c.kv_dtype, D, w, x, rows, ctx->at<float2>(L.rope), q, ctx->kc_layer(l), ctx->vc_layer(l)); }
                attend(l, q, rows, max_ctx, ctx->at<float>(L.attn_part),
                                 attn_part_floats, ctx->at<int>(L.attn_cnt), att, nullptr, 0, &pend);
            }
            { Bracket br(ctx, s, TR_KERNEL_OPROJ); launch_oproj(s, ctx->c.dtype, D, w.wo, att, pend, R, x); }
            { Bracket br(ctx, s, TR_KERNEL_GATEUP); launch_gateup(s, ctx->c.dtype, D, w, x, R, h); }
            { Bracket br(ctx, s, TR_KERNEL_DOWN); launch_down(s, ctx->c.dtype, D, w.wd, h, R, x); }
        }
        return 0;
    }
    const int ncb = mfma_ncb(R);
    float *part = ctx->at<float>(L.part);
    int pending = 0;
    const bool fuse_oproj = gemm_oproj_residual_supported(D);
    for (int l = 0; l < D.L; ++l) {
        const LayerW &w = ctx->layers[(size_t)l];
        PrepArgs p{};
        p.x = x; p.row0 = 0; p.part = part; p.nsplit = pending; p.part_M = R; p.M = R; p.d = D.d; p.eps = D.eps;
        p.gain = (const bf16_t *)w.ln1; p.pack = ctx->at<uint4>(L.pack_d); p.ncb = ncb;
        { Bracket br(ctx, s, TR_KERNEL_PREP); launch_prep(s, p); }
        {
            Bracket br(ctx, s, TR_KERNEL_QKV);
            launch_gemm_qkv(s, ctx->c.kv_dtype, D, ctx->wt(l, L.wt_qkv), ctx->at<uint4>(L.pack_d), ctx->bias(l), rows, ctx->at<float2>(L.rope), q,
                            ctx->kc_layer(l), ctx->vc_layer(l));
        }
        attend(l, q, rows, max_ctx, ctx->at<float>(L.attn_part),
                         attn_part_floats, ctx->at<int>(L.attn_cnt), att, ctx->at<uint4>(L.pack_a), ncb, nullptr);
        if (fuse_oproj) {
            // the output projection updates the residual stream and packs the FFN input itself; the 1/rms factor follows in the gate/up epilogue
            int n_ss;
            { Bracket br(ctx, s, TR_KERNEL_OPROJ);
              n_ss = launch_gemm_oproj_residual(s, D, ctx->wt(l, L.wt_o), ctx->at<uint4>(L.pack_a), R, x, w.ln2, ctx->at<uint4>(L.pack_d), ctx->at<float>(L.sumsq), L.ss_stride, live); }
            { Bracket br(ctx, s, TR_KERNEL_GATEUP);
              launch_gemm_swiglu(s, D, ctx->wt(l, L.wt_gu), ctx->at<uint4>(L.pack_d), R, ctx->at<uint4>(L.pack_h), live, ctx->at<float>(L.sumsq), n_ss, L.ss_stride); }
        } else {
            { Bracket br(ctx, s, TR_KERNEL_OPROJ); launch_gemm_partial(s, ctx->wt(l, L.wt_o), ctx->at<uint4>(L.pack_a), D.qw, D.d, R, part, &pending, live); }
            p.nsplit = pending; p.gain = (const bf16_t *)w.ln2;
            { Bracket br(ctx, s, TR_KERNEL_PREP); launch_prep(s, p); }
            { Bracket br(ctx, s, TR_KERNEL_GATEUP); launch_gemm_swiglu(s, D, ctx->wt(l, L.wt_gu), ctx->at<uint4>(L.pack_d), R, ctx->at<uint4>(L.pack_h), live); }
        }
        { Bracket br(ctx, s, TR_KERNEL_DOWN); launch_gemm_partial(s, ctx->wt(l, L.wt_d), ctx->at<uint4>(L.pack_h), D.F, D.d, R, part, &pending, live); }
    }
    return pending;
}

// The routing tail on n rows of the residual stream x starting at row0. `pending` split-K partials (rows indexed
// like x, part_M rows per split) are added first.
void run_tail(tr_ctx *ctx, hipStream_t s, TailArgs t, float *x, int row0, int pending, int part_M)
{
    const Dims &D = ctx->D;
    const Layout &L = ctx->lay;
    if (ctx->lay.split_head && t.n > 2) {
        // wide model, more rows than one pass of the streaming head takes: final norm + pack, the head as split-K partial
        // logits on the matrix cores, softmax statistics per vocabulary slice from the partials
        PrepArgs p{};
        p.x = x; p.row0 = row0; p.gather = t.gather; p.part = ctx->at<float>(L.part); p.nsplit = pending; p.part_M = part_M; p.M = t.n; p.d = D.d;
        p.eps = D.eps;
        p.gain = (const bf16_t *)ctx->final_norm; p.pack = ctx->at<uint4>(L.pack_d); p.ncb = mfma_ncb(t.n);
        p.hn = t.hn; p.hidden = t.hidden; p.hidden_tap = t.hidden_tap;
        { Bracket br(ctx, s, TR_KERNEL_PREP); launch_prep(s, p); }
        t.x = x + (size_t)row0 * D.d;
        int ns = 0;
        { Bracket br(ctx, s, TR_KERNEL_LMHEAD); launch_gemm_partial(s, ctx->ws + L.wt_head, ctx->at<uint4>(L.pack_d), D.d, D.V, t.n, ctx->at<float>(L.part), &ns, ctx->live); }
        Bracket br(ctx, s, TR_KERNEL_TAIL_MERGE);
        launch_lmhead_finish(s, ctx->at<float>(L.part), ns, t.n, D.V, t.part, t.logits);
        t.nslices = (D.V + LMHEAD_FINISH_COLS - 1) / LMHEAD_FINISH_COLS;
        launch_tail_final(s, ctx->c.dtype, D, t);
        return;
    }
    if (!ctx->lay.mfma) {
        if (pending > 0) {   // wide model: add the last down projection's partials to the rows the tail reads
            PrepArgs p{};
            p.x = x; p.row0 = row0; p.gather = t.gather; p.part = ctx->at<float>(L.part); p.nsplit = pending; p.part_M = part_M; p.M = t.n; p.d = D.d;
            p.eps = D.eps;
            Bracket br(ctx, s, TR_KERNEL_PREP);
            launch_prep(s, p);
        }
        t.x = x + (size_t)row0 * D.d;
        { Bracket br(ctx, s, TR_KERNEL_PREP); launch_tail_norm(s, ctx->c.dtype, D, t); }
        { Bracket br(ctx, s, TR_KERNEL_LMHEAD); launch_lmhead_gemv(s, ctx->c.dtype, D, t); }
        Bracket br(ctx, s, TR_KERNEL_TAIL_MERGE);
        launch_tail_final(s, ctx->c.dtype, D, t);
        return;
    }
    PrepArgs p{};
    p.x = x; p.row0 = row0; p.gather = t.gather; p.part = ctx->at<float>(L.part); p.nsplit = pending; p.part_M = part_M; p.M = t.n; p.d = D.d;
    p.eps = D.eps;
    p.gain = (const bf16_t *)ctx->final_norm; p.pack = ctx->at<uint4>(L.pack_d); p.ncb = mfma_ncb(t.n);
    p.hn = t.hn; p.hidden = t.hidden; p.hidden_tap = t.hidden_tap;
    { Bracket br(ctx, s, TR_KERNEL_PREP); launch_prep(s, p); }
    t.x = x + (size_t)row0 * D.d;
    // the head is streamed by the matrix-core kernel for any row count: one row costs the same bytes as 32
    t.nslices = lmhead_mfma_wgs(D.V, L.router_tiles, t.n);
    {
        Bracket br(ctx, s, TR_KERNEL_LMHEAD);
        launch_gemm_lmhead(s, D, ctx->ws + L.wt_head, ctx->at<uint4>(L.pack_d), t.n, t.part, t.logits, ctx->at<float>(L.r1), L.router_tiles, ctx->live);
    }
    if (L.router_tiles) { t.r1 = ctx->at<float>(L.r1); t.r1_stride = L.router_tiles * 32; }
    Bracket br(ctx, s, TR_KERNEL_TAIL_MERGE);
    launch_tail_final(s, ctx->c.dtype, D, t);
}

TailArgs tail_args(tr_ctx *ctx, const tr_out *out, int out_offset, int n)
{
    const Layout &L = ctx->lay;
    TailArgs t{};
    t.head = ctx->head; t.final_norm = ctx->final_norm;
    t.r_w1 = ctx->r_w1; t.r_b1 = ctx->r_b1; t.r_w2 = ctx->r_w2; t.r_b2 = ctx->r_b2;
    t.n = n;
    t.hn = ctx->at<float>(L.hn);
    t.part = ctx->at<float>(L.tail_part);
    t.nslices = L.nslices; t.slice_rows = tail_slice_rows();
    t.token = out->token + out_offset; t.conf = out->conf + out_offset; t.score = out->score + out_offset; t.flag = out->flag + out_offset;
    t.hidden = out->hidden ? out->hidden + (size_t)out_offset * ctx->D.d : nullptr;
    t.logits = out->logits ? out->logits + (size_t)out_offset * ctx->D.V : nullptr;
    t.counters = ctx->at<long long>(L.counters);
    t.threshold = ctx->threshold; t.route_dir = ctx->c.route_dir; t.mode = ctx->mode; t.hidden_tap = ctx->c.hidden_tap;
    t.policy = ctx->c.route_policy;
    t.rpart = ctx->at<float>(L.tail_rpart); t.rcnt = ctx->at<int>(L.tail_rcnt);
    t.live = ctx->live; t.cand = ctx->cand; t.scatter = ctx->scatter;
    return t;
}

}  // namespace

// Brings the host's sequence lengths up to date after steps whose rows were selected on the device: waits for the stream those
// steps were enqueued on and reads the device-side lengths of the slots that were candidates. TR_OK or TR_ERR_HIP.
static int sync_lengths(tr_ctx *ctx)
{
    if (!ctx->unsynced) return TR_OK;
    std::vector<int> dev((size_t)ctx->c.max_batch);
    hipError_t e = hipMemcpyAsync(dev.data(), ctx->ws + ctx->lay.dev_len, dev.size() * 4, hipMemcpyDeviceToHost, ctx->active_stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->active_stream);
    if (e != hipSuccess) return fail_hip(ctx, e, "reading back the device-side sequence lengths");
    for (size_t b = 0; b < dev.size(); ++b)
        if (ctx->ahead[b] > 0) { ctx->len[b] = dev[b]; ctx->ahead[b] = 0; }
    ctx->unsynced = false;
    return TR_OK;
}

// Segments of several slots through all layers in as few passes as the row buffers allow (whole segments per pass):
// segment i is tokens_flat[offsets[i] .. offsets[i+1]) at positions base_i .. base_i+T_i-1, base_i = the slot's length
// (from_len) or 0. Keys and values of all rows are appended before any row attends, each row over positions 0..its own;
// the tail runs on the last row of every segment. counter_mode: 1 add, 2 set. Returns TR_OK or an error code.
static int ingest(tr_ctx *ctx, hipStream_t s, int n, const int32_t *slots, const int32_t *tokens_flat, const int32_t *offsets, bool from_len,
                  const tr_out *out, int counter_mode, const char *who)
{
    const Layout &L = ctx->lay;
    struct Pass { std::vector<int> slot, pos, gather, out_slot, qblock; };
    const int block_rows = attention_block_rows(ctx->D);
    std::vector<Pass> passes;   // kept until the end: the uploads below read them
    passes.reserve((size_t)n);
    int i = 0;
    while (i < n) {
        passes.emplace_back();
        Pass &ps = passes.back();
        int rows = 0, max_ctx = 0, j = i;
        bool one_token_each = true;   // every segment of the pass is a single token: its rows belong to different slots, like a decode step's
        for (; j < n; ++j) {
            const int T = offsets[j + 1] - offsets[j], base = from_len ? ctx->len[(size_t)slots[j]] : 0;
            if (j > i && rows + T > L.max_rows) break;
            if (T != 1) one_token_each = false;
            for (int t = 0; t < T; ++t) { ps.slot.push_back(slots[j]); ps.pos.push_back(base + t); }
            for (int t = 0; t < T; t += block_rows) ps.qblock.push_back((rows + t) * 8 + std::min(block_rows, T - t));
            rows += T;
            ps.gather.push_back(rows - 1);
            ps.out_slot.push_back(slots[j]);
            if (base + T > max_ctx) max_ctx = base + T;
        }
        // pageable sources: each copy has left the host array when the call returns
        hipError_t e = hipMemcpyAsync(ctx->at<int>(L.tok), tokens_flat + offsets[i], (size_t)rows * 4, hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(ctx->at<int>(L.slot), ps.slot.data(), (size_t)rows * 4, hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(ctx->at<int>(L.pos), ps.pos.data(), (size_t)rows * 4, hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(ctx->at<int>(L.gather), ps.gather.data(), (size_t)(j - i) * 4, hipMemcpyHostToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(ctx->at<int>(L.out_slot), ps.out_slot.data(), (size_t)(j - i) * 4, hipMemcpyHostToDevice, s);
        // bf16 cache and enough blocks of query rows to fill the chip: the rows of a block share the keys and values they read
        const bool blocks = ctx->c.kv_dtype == TR_BF16 && ps.qblock.size() * (size_t)ctx->D.Hkv >= 256 && ps.qblock.size() < (size_t)rows;
        if (blocks && e == hipSuccess) e = hipMemcpyAsync(ctx->at<int>(L.qblock), ps.qblock.data(), ps.qblock.size() * 4, hipMemcpyHostToDevice, s);
        if (e != hipSuccess) return fail_hip(ctx, e, who);
        ctx->qblocks = blocks ? (int)ps.qblock.size() : 0;
        const int pending = run_layers(ctx, s, rows, max_ctx, true, one_token_each);
        ctx->qblocks = 0;
        TailArgs t = tail_args(ctx, out, i, j - i);
        t.gather = ctx->at<int>(L.gather);
        t.slot = ctx->at<int>(L.out_slot);
        t.counter_mode = counter_mode;
        run_tail(ctx, s, t, ctx->at<float>(L.x), 0, pending, rows);
        profile_next_turn(ctx);
        i = j;
    }
    return TR_OK;
}

// Paged cache: room for the writes [old_len[i], new_len[i]) of the listed slots. All or nothing: when the pool cannot
// supply the pages, nothing has changed and TR_ERR_CAPACITY is returned. Otherwise the copies of shared pages that are about
// to be written and the changed rows of the page table are enqueued on the stream, ahead of the kernels of the call.
static int reserve_pages(tr_ctx *ctx, hipStream_t s, int n, const int *slots, const int *old_len, const int *new_len, const char *who)
{
    if (!ctx->c.kv_page) return TR_OK;
    KvPages &P = ctx->pages;
    if (P.demand(n, slots, old_len, new_len) > P.free_count()) return fail(ctx, TR_ERR_CAPACITY, "the page pool of the cache is exhausted");
    std::vector<KvPages::Copy> copies;
    const Layout &L = ctx->lay;
    for (int i = 0; i < n; ++i) {
        if (!P.grow(slots[i], old_len[i], new_len[i], copies)) continue;
        // pageable source: the copy has left the host array when the call returns
        const hipError_t e = hipMemcpyAsync(ctx->ws + L.ptab + (size_t)slots[i] * L.maxp * 4, P.row(slots[i]), (size_t)P.npages[(size_t)slots[i]] * 4,
                                            hipMemcpyHostToDevice, s);
        if (e != hipSuccess) return fail_hip(ctx, e, who);
    }
    const size_t page_bytes = L.k_layer_bytes / (size_t)L.pool;   // one page of one layer, K or V
    for (const KvPages::Copy &c : copies)
        for (int l = 0; l < ctx->D.L; ++l) {
            char *k = static_cast<char *>(ctx->kc_layer(l)), *v = static_cast<char *>(ctx->vc_layer(l));
            hipError_t e = hipMemcpyAsync(k + (size_t)c.to * page_bytes, k + (size_t)c.from * page_bytes, page_bytes, hipMemcpyDeviceToDevice, s);
            if (e == hipSuccess) e = hipMemcpyAsync(v + (size_t)c.to * page_bytes, v + (size_t)c.from * page_bytes, page_bytes, hipMemcpyDeviceToDevice, s);
            if (e != hipSuccess) return fail_hip(ctx, e, who);
        }
    return TR_OK;
}

extern "C" {

size_t tr_workspace_bytes(const tr_config *cfg)
{
    if (check_config(cfg) != TR_OK) return 0;
    return make_layout(cfg).total;
}

int tr_create(const tr_config *cfg, const tr_weights *w, void *workspace, size_t workspace_bytes, tr_ctx **out)
{
    if (!cfg || !w || !workspace || !out) return TR_ERR_INVALID_ARG;
    int rc = check_config(cfg);
    if (rc) return rc;
    if ((uintptr_t)workspace % ALIGN) return TR_ERR_INVALID_ARG;
    if (!w->tok_emb || !w->final_norm || (!cfg->tie_lm_head && !w->lm_head)) return TR_ERR_INVALID_ARG;
    if (!w->ln1 || !w->wq || !w->wk || !w->wv || !w->wo || !w->ln2 || !w->wg || !w->wu || !w->wd) return TR_ERR_INVALID_ARG;
    if (cfg->route_policy == TR_POLICY_MLP && cfg->router_hidden > 0 && (!w->r_w1 || !w->r_w2)) return TR_ERR_INVALID_ARG;
    if (cfg->route_policy == TR_POLICY_LINEAR && !w->r_w2) return TR_ERR_INVALID_ARG;
    Layout lay = make_layout(cfg);
    if (workspace_bytes < lay.total) return TR_ERR_CAPACITY;

    tr_ctx *ctx = new tr_ctx();
    ctx->c = *cfg;
    ctx->lay = lay;
    ctx->ws = static_cast<char *>(workspace);
    Dims &D = ctx->D;
    D.L = cfg->n_layers; D.d = cfg->d_model; D.Hq = cfg->n_q_heads; D.Hkv = cfg->n_kv_heads; D.dh = cfg->head_dim; D.F = cfg->d_ffn;
    D.V = cfg->vocab; D.qw = D.Hq * D.dh; D.kvw = D.Hkv * D.dh; D.G = D.Hq / D.Hkv; D.rh = cfg->router_hidden;
    D.max_batch = cfg->max_batch; D.max_seq = cfg->max_seq; D.eps = cfg->rms_eps;
    D.vts = cfg->kv_dtype == TR_BF16 ? (cfg->max_seq + 31) / 32 * 32 : 0;
    D.page = cfg->kv_page; D.maxp = lay.maxp; D.units = cfg->kv_page ? lay.pool : cfg->max_batch;
    D.ptab = reinterpret_cast<const int *>(ctx->ws + lay.ptab);
    if (cfg->kv_page) ctx->pages.init(cfg->max_batch, cfg->kv_page, lay.maxp, lay.pool);
    bool aligned = true;
    auto chk = [&](const void *p) { if (p && (uintptr_t)p % 16) aligned = false; return p; };
    ctx->layers.resize((size_t)D.L);
    for (int l = 0; l < D.L; ++l) {
        LayerW &lw = ctx->layers[(size_t)l];
        lw.ln1 = chk(w->ln1[l]); lw.wq = chk(w->wq[l]); lw.wk = chk(w->wk[l]); lw.wv = chk(w->wv[l]);
        lw.bq = w->bq ? w->bq[l] : nullptr; lw.bk = w->bk ? w->bk[l] : nullptr; lw.bv = w->bv ? w->bv[l] : nullptr;
        lw.wo = chk(w->wo[l]); lw.ln2 = chk(w->ln2[l]); lw.wg = chk(w->wg[l]); lw.wu = chk(w->wu[l]); lw.wd = chk(w->wd[l]);
        if (!lw.ln1 || !lw.wq || !lw.wk || !lw.wv || !lw.wo || !lw.ln2 || !lw.wg || !lw.wu || !lw.wd) { delete ctx; return TR_ERR_INVALID_ARG; }
    }
    ctx->tok_emb = chk(w->tok_emb);
    ctx->head = chk(cfg->tie_lm_head ? w->tok_emb : w->lm_head);
    ctx->final_norm = chk(w->final_norm);
    ctx->r_w1 = chk(w->r_w1); ctx->r_b1 = w->r_b1; ctx->r_w2 = w->r_w2; ctx->r_b2 = w->r_b2;
    if (!aligned) { delete ctx; return TR_ERR_INVALID_ARG; }
    ctx->len.assign((size_t)cfg->max_batch, -1);
    ctx->ahead.assign((size_t)cfg->max_batch, 0);
    ctx->threshold = cfg->threshold;
    ctx->mode = TR_JOINT;

    // rotary table: cos/sin of pos * theta^(-2j/dh), computed in double
    const int half = D.dh / 2;
    std::vector<float2> rope((size_t)cfg->max_seq * half);
    for (int j = 0; j < half; ++j) {
        const double inv = std::pow((double)cfg->rope_theta, -2.0 * j / (double)D.dh);
        for (int p = 0; p < cfg->max_seq; ++p) {
            const double a = (double)p * inv;
            rope[(size_t)p * half + j] = make_float2((float)std::cos(a), (float)std::sin(a));
        }
    }
    hipError_t e = hipMemcpy(ctx->ws + lay.rope, rope.data(), rope.size() * sizeof(float2), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemset(ctx->ws + lay.counters, 0, (size_t)cfg->max_batch * 2 * sizeof(long long));
    // the attention kernels read whole 32-key blocks and mask afterwards: cache positions never written must hold finite values
    if (e == hipSuccess) e = hipMemset(ctx->ws + lay.kc, 0, lay.rope - lay.kc);
    if (e == hipSuccess) e = hipMemset(ctx->ws + lay.attn_cnt, 0, (size_t)lay.max_rows * cfg->n_kv_heads * 4);
    if (e == hipSuccess) e = hipMemset(ctx->ws + lay.tail_rcnt, 0, (size_t)cfg->max_batch * 4);
    if (e == hipSuccess) e = hipMemset(ctx->ws + lay.ptab, 0, (size_t)cfg->max_batch * (lay.maxp ? lay.maxp : 1) * 4);   // page 0: a valid page
    if (e == hipSuccess && (lay.mfma || lay.split)) {
        // one-time repack of the bf16 matrices into matrix-core tiles; q|k|v are concatenated, gate/up interleaved
        for (int l = 0; l < D.L; ++l) {
            const LayerW &lw = ctx->layers[(size_t)l];
            launch_repack(nullptr, lw.wq, D.qw, D.d, ctx->wt(l, lay.wt_qkv), 0, 1, D.dh);
            launch_repack(nullptr, lw.wk, D.kvw, D.d, ctx->wt(l, lay.wt_qkv), D.qw / 32, 1, D.dh);
            launch_repack(nullptr, lw.wv, D.kvw, D.d, ctx->wt(l, lay.wt_qkv), (D.qw + D.kvw) / 32, 1, D.dh);
            launch_repack(nullptr, lw.wo, D.d, D.qw, ctx->wt(l, lay.wt_o), 0, 1, 0);
            launch_repack(nullptr, lw.wg, D.F, D.d, ctx->wt(l, lay.wt_gu), 0, 2, 0);
            launch_repack(nullptr, lw.wu, D.F, D.d, ctx->wt(l, lay.wt_gu), 1, 2, 0);
            launch_repack(nullptr, lw.wd, D.d, D.F, ctx->wt(l, lay.wt_d), 0, 1, 0);
            launch_widen_bias(nullptr, lw.bq, D.qw, ctx->bias(l));
            launch_widen_bias(nullptr, lw.bk, D.kvw, ctx->bias(l) + D.qw);
            launch_widen_bias(nullptr, lw.bv, D.kvw, ctx->bias(l) + D.qw + D.kvw);
        }
        if (lay.mfma || lay.split_head) launch_repack(nullptr, ctx->head, D.V, D.d, ctx->ws + lay.wt_head, 0, 1, 0);
        if (lay.router_tiles) launch_repack(nullptr, ctx->r_w1, D.rh, D.d, ctx->ws + lay.wt_head, (D.V + 31) / 32, 1, 0);
        e = hipMemset(ctx->ws + lay.pack_d, 0, lay.part - lay.pack_d);   // padding rows of the packed activations stay zero
    }
    if (e == hipSuccess) { float *sc = nullptr; e = scratch_address(&sc); }   // static scratch of tr_tail_noalloc: address on this device
    // everything above ran on the null stream; the caller's streams need not be ordered after it, so finish it here
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e == hipSuccess) e = hipGetLastError();
    if (e != hipSuccess) { delete ctx; return TR_ERR_HIP; }
    *out = ctx;
    return TR_OK;
}

void tr_destroy(tr_ctx *ctx)
{
    if (!ctx) return;
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    delete ctx;
}

const char *tr_last_error(const tr_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int tr_profile_chain(void *hip_stream, int32_t *buf, int32_t workgroups, int32_t launches)
{
    if (!buf || workgroups < 1 || workgroups > 65536 || launches < 1) return TR_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    for (int i = 0; i < launches; ++i) launch_fill_int(s, buf, workgroups * 256, i);   // each launch overwrites what the one before wrote
    return hipGetLastError() == hipSuccess ? TR_OK : TR_ERR_HIP;
}

int tr_set_threshold(tr_ctx *ctx, float t)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    ctx->threshold = t;
    return TR_OK;
}

int tr_set_mode(tr_ctx *ctx, int32_t mode)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (mode != TR_JOINT && mode != TR_SMALL_ONLY) return fail(ctx, TR_ERR_INVALID_ARG, "tr_set_mode: unknown mode");
    ctx->mode = mode;
    return TR_OK;
}

int tr_seq_len(const tr_ctx *ctx, int32_t slot, int32_t *len)
{
    if (!ctx || !len || slot < 0 || slot >= ctx->c.max_batch) return TR_ERR_INVALID_ARG;
    { const int src = sync_lengths(const_cast<tr_ctx *>(ctx)); if (src != TR_OK) return src; }
    *len = ctx->len[(size_t)slot] < 0 ? 0 : ctx->len[(size_t)slot];
    return TR_OK;
}

int tr_seq_truncate(tr_ctx *ctx, int32_t slot, int32_t new_len)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (slot < 0 || slot >= ctx->c.max_batch) return fail(ctx, TR_ERR_INVALID_ARG, "tr_seq_truncate: slot out of range");
    { const int src = sync_lengths(ctx); if (src != TR_OK) return src; }
    if (ctx->len[(size_t)slot] < 0) return fail(ctx, TR_ERR_STATE, "tr_seq_truncate: slot was never filled");
    if (new_len < 0 || new_len > ctx->len[(size_t)slot]) return fail(ctx, TR_ERR_INVALID_ARG, "tr_seq_truncate: new_len outside [0, len]");
    ctx->len[(size_t)slot] = new_len;
    if (ctx->c.kv_page) ctx->pages.shrink(slot, new_len);   // pages past the new length go back to the pool
    return TR_OK;
}

int tr_counters_ptr(const tr_ctx *ctx, const int64_t **dev_counters)
{
    if (!ctx || !dev_counters) return TR_ERR_INVALID_ARG;
    *dev_counters = reinterpret_cast<const int64_t *>(ctx->ws + ctx->lay.counters);
    return TR_OK;
}

int tr_prefill(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *tokens_flat, const int32_t *offsets,
               const tr_out *out)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (!slots || !tokens_flat || !offsets || !check_out(out)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_prefill: null argument");
    { const int src = sync_lengths(ctx); if (src != TR_OK) return src; }
    if (!slots_ok(ctx, n, slots)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_prefill: bad slot list");
    if (offsets[0] != 0) return fail(ctx, TR_ERR_INVALID_ARG, "tr_prefill: offsets[0] must be 0");
    for (int i = 0; i < n; ++i) {
        const long long T = (long long)offsets[i + 1] - offsets[i];
        if (T < 1) return fail(ctx, TR_ERR_INVALID_ARG, "tr_prefill: empty prompt");
        if (T > ctx->c.max_seq) return fail(ctx, TR_ERR_CAPACITY, "tr_prefill: prompt longer than max_seq");
    }
    for (int i = 0; i < offsets[n]; ++i)
        if (tokens_flat[i] < 0 || tokens_flat[i] >= ctx->c.vocab) return fail(ctx, TR_ERR_INVALID_ARG, "tr_prefill: token out of range");

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (ctx->c.kv_page) {   // the slots start over: their pages go back to the pool, then the prompts take what they need
        const KvPages before = ctx->pages;
        std::vector<int> zero((size_t)n, 0), want((size_t)n);
        for (int i = 0; i < n; ++i) { ctx->pages.shrink(slots[i], 0); want[(size_t)i] = offsets[i + 1] - offsets[i]; }
        const int prc = reserve_pages(ctx, s, n, slots, zero.data(), want.data(), "tr_prefill: page table");
        if (prc != TR_OK) { ctx->pages = before; return prc; }
    }
    const int rc = ingest(ctx, s, n, slots, tokens_flat, offsets, false, out, 2, "tr_prefill");
    if (rc != TR_OK) return rc;
    for (int i = 0; i < n; ++i) ctx->len[(size_t)slots[i]] = offsets[i + 1] - offsets[i];
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(ctx, e, "tr_prefill: launch");
    return TR_OK;
}

int tr_extend(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *tokens_flat, const int32_t *offsets,
              const tr_out *out)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (!slots || !tokens_flat || !offsets || !check_out(out)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_extend: null argument");
    { const int src = sync_lengths(ctx); if (src != TR_OK) return src; }
    if (!slots_ok(ctx, n, slots)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_extend: bad slot list");
    if (offsets[0] != 0) return fail(ctx, TR_ERR_INVALID_ARG, "tr_extend: offsets[0] must be 0");
    for (int i = 0; i < n; ++i) {
        const long long T = (long long)offsets[i + 1] - offsets[i];
        const int len = ctx->len[(size_t)slots[i]];
        if (T < 1) return fail(ctx, TR_ERR_INVALID_ARG, "tr_extend: empty segment");
        if (len < 0) return fail(ctx, TR_ERR_STATE, "tr_extend: slot was never prefilled");
        if (len + T > ctx->c.max_seq) return fail(ctx, TR_ERR_CAPACITY, "tr_extend: segment does not fit the cache");
    }
    for (int i = 0; i < offsets[n]; ++i)
        if (tokens_flat[i] < 0 || tokens_flat[i] >= ctx->c.vocab) return fail(ctx, TR_ERR_INVALID_ARG, "tr_extend: token out of range");

    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (ctx->c.kv_page) {
        std::vector<int> from((size_t)n), to((size_t)n);
        for (int i = 0; i < n; ++i) { from[(size_t)i] = ctx->len[(size_t)slots[i]]; to[(size_t)i] = from[(size_t)i] + offsets[i + 1] - offsets[i]; }
        const int prc = reserve_pages(ctx, s, n, slots, from.data(), to.data(), "tr_extend: page table");
        if (prc != TR_OK) return prc;
    }
    const int rc = ingest(ctx, s, n, slots, tokens_flat, offsets, true, out, 1, "tr_extend");
    if (rc != TR_OK) return rc;
    for (int i = 0; i < n; ++i) ctx->len[(size_t)slots[i]] += offsets[i + 1] - offsets[i];
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(ctx, e, "tr_extend: launch");
    return TR_OK;
}

// one decode step; the input tokens are either a host array (checked here) or a device array (clamped by the kernel)
static int decode_step_impl(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *in_tokens, const int32_t *dev_tokens,
                            const tr_out *out)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (!slots || (!in_tokens && !dev_tokens) || !check_out(out)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_decode_step: null argument");
    { const int src = sync_lengths(ctx); if (src != TR_OK) return src; }
    if (!slots_ok(ctx, n, slots)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_decode_step: bad slot list");
    int max_ctx = 0;
    std::vector<int> pos((size_t)n);
    for (int i = 0; i < n; ++i) {
        if (in_tokens && (in_tokens[i] < 0 || in_tokens[i] >= ctx->c.vocab)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_decode_step: token out of range");
        const int len = ctx->len[(size_t)slots[i]];
        if (len < 0) return fail(ctx, TR_ERR_STATE, "tr_decode_step: slot was never prefilled");
        if (len >= ctx->c.max_seq) return fail(ctx, TR_ERR_CAPACITY, "tr_decode_step: slot is full");
        pos[(size_t)i] = len;
        if (len + 1 > max_ctx) max_ctx = len + 1;
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const Layout &L = ctx->lay;
    if (ctx->c.kv_page) {
        std::vector<int> to((size_t)n);
        for (int i = 0; i < n; ++i) to[(size_t)i] = pos[(size_t)i] + 1;
        const int prc = reserve_pages(ctx, s, n, slots, pos.data(), to.data(), "tr_decode_step: page table");
        if (prc != TR_OK) return prc;
    }
    {
        Bracket br(ctx, s, TR_KERNEL_SETUP);
        launch_setup_rows_embed(s, n, slots, in_tokens, pos.data(), ctx->at<int>(L.slot), ctx->at<int>(L.tok), ctx->at<int>(L.pos), ctx->c.dtype,
                                ctx->tok_emb, ctx->D.d, ctx->at<float>(L.x), dev_tokens, ctx->c.vocab);
    }
    const int pending = run_layers(ctx, s, n, max_ctx, false, true);
    TailArgs t = tail_args(ctx, out, 0, n);
    t.gather = nullptr;
    t.slot = ctx->at<int>(L.slot);
    t.counter_mode = 1;
    run_tail(ctx, s, t, ctx->at<float>(L.x), 0, pending, n);
    profile_next_turn(ctx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(ctx, e, "tr_decode_step: launch");
    for (int i = 0; i < n; ++i) ctx->len[(size_t)slots[i]] += 1;
    return TR_OK;
}

int tr_decode_step(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *in_tokens, const tr_out *out)
{
    if (!in_tokens) return ctx ? fail(ctx, TR_ERR_INVALID_ARG, "tr_decode_step: null argument") : TR_ERR_INVALID_ARG;
    return decode_step_impl(ctx, hip_stream, n, slots, in_tokens, nullptr, out);
}

int tr_decode_step_dev(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *in_tokens_dev, const tr_out *out)
{
    if (!in_tokens_dev) return ctx ? fail(ctx, TR_ERR_INVALID_ARG, "tr_decode_step_dev: null argument") : TR_ERR_INVALID_ARG;
    return decode_step_impl(ctx, hip_stream, n, slots, nullptr, in_tokens_dev, out);
}

int tr_decode_step_active(tr_ctx *ctx, void *hip_stream, int32_t n, const int32_t *slots, const int32_t *flags_dev, const int32_t *in_tokens_dev,
                          int32_t n_max, int32_t *active_dev, int32_t *next_tokens_dev, const tr_out *out)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (!slots || !flags_dev || !in_tokens_dev || !active_dev || !check_out(out)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_decode_step_active: null argument");
    if (!slots_ok(ctx, n, slots) || n > 256) return fail(ctx, TR_ERR_INVALID_ARG, "tr_decode_step_active: bad candidate list (distinct slots, at most 256)");
    if (n_max < 3 || n_max > ctx->c.max_batch) return fail(ctx, TR_ERR_INVALID_ARG, "tr_decode_step_active: n_max outside [3, max_batch]");
    if (!(ctx->use_mfma(n_max) || ctx->use_split(n_max)) || ctx->c.kv_page)
        return fail(ctx, TR_ERR_SHAPE, "tr_decode_step_active: needs a bf16 model on the matrix-core path and a contiguous cache");
    int max_ctx = 0;
    std::vector<int> host_len((size_t)n);
    for (int i = 0; i < n; ++i) {
        const size_t b = (size_t)slots[i];
        if (ctx->len[b] < 0) return fail(ctx, TR_ERR_STATE, "tr_decode_step_active: slot was never prefilled");
        const int most = ctx->len[b] + ctx->ahead[b];   // the slot's length is at most this
        if (most >= ctx->c.max_seq) return fail(ctx, TR_ERR_CAPACITY, "tr_decode_step_active: a candidate slot may be full");
        host_len[(size_t)i] = ctx->ahead[b] ? -1 : ctx->len[b];
        if (most + 1 > max_ctx) max_ctx = most + 1;
    }
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const Layout &L = ctx->lay;
    launch_active_setup(s, n, slots, host_len.data(), flags_dev, in_tokens_dev, n_max, ctx->c.vocab, ctx->at<int>(L.dev_len), ctx->at<int>(L.slot),
                        ctx->at<int>(L.tok), ctx->at<int>(L.pos), active_dev);
    ctx->live = active_dev; ctx->cand = active_dev + 2; ctx->scatter = next_tokens_dev;
    const int pending = run_layers(ctx, s, n_max, max_ctx, true, false);
    TailArgs t = tail_args(ctx, out, 0, n_max);
    t.gather = nullptr;
    t.slot = ctx->at<int>(L.slot);
    t.counter_mode = 1;
    run_tail(ctx, s, t, ctx->at<float>(L.x), 0, pending, n_max);
    profile_next_turn(ctx);
    ctx->live = ctx->cand = nullptr; ctx->scatter = nullptr;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(ctx, e, "tr_decode_step_active: launch");
    for (int i = 0; i < n; ++i) ctx->ahead[(size_t)slots[i]] += 1;
    ctx->unsynced = true;
    ctx->active_stream = s;
    return TR_OK;
}

int tr_tail(tr_ctx *ctx, void *hip_stream, int32_t n, const float *x, const tr_out *out)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (!x || !check_out(out)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_tail: null argument");
    if (n < 1 || n > ctx->c.max_batch) return fail(ctx, TR_ERR_INVALID_ARG, "tr_tail: n outside [1, max_batch]");
    if ((uintptr_t)x % 16) return fail(ctx, TR_ERR_INVALID_ARG, "tr_tail: x must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    TailArgs t = tail_args(ctx, out, 0, n);
    t.gather = nullptr;
    t.slot = nullptr;
    t.counters = nullptr;
    t.counter_mode = 0;
    run_tail(ctx, s, t, const_cast<float *>(x), 0, 0, n);   // no partials pending: x is only read
    profile_next_turn(ctx);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(ctx, e, "tr_tail: launch");
    return TR_OK;
}

int tr_tail_noalloc(tr_ctx *ctx, void *hip_stream, int32_t n, const float *x, const tr_out *out)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (!x || !check_out(out)) return fail(ctx, TR_ERR_INVALID_ARG, "tr_tail_noalloc: null argument");
    if ((uintptr_t)x % 16) return fail(ctx, TR_ERR_INVALID_ARG, "tr_tail_noalloc: x must be 16-byte aligned");
    const int nslices = (ctx->c.vocab + tail_slice_rows() - 1) / tail_slice_rows();
    if (n < 1 || n > NOALLOC_MAX_ROWS) return fail(ctx, TR_ERR_CAPACITY, "tr_tail_noalloc: n outside [1, 64]");
    if (ctx->c.d_model > NOALLOC_MAX_D || nslices > NOALLOC_MAX_SLICES)
        return fail(ctx, TR_ERR_CAPACITY, "tr_tail_noalloc: d_model above 4096 or vocabulary above 262144");
    float *sc = nullptr;
    const hipError_t ea = scratch_address(&sc);
    if (ea != hipSuccess) return fail_hip(ctx, ea, "tr_tail_noalloc: hipGetSymbolAddress");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    TailArgs t = tail_args(ctx, out, 0, n);
    t.gather = nullptr;
    t.slot = nullptr;
    t.counters = nullptr;
    t.counter_mode = 0;
    t.x = x;
    t.hn = sc + NOALLOC_HN;
    t.part = sc + NOALLOC_PART;
    t.nslices = nslices;
    t.rpart = sc + NOALLOC_RPART;
    t.rcnt = reinterpret_cast<int *>(sc + NOALLOC_RCNT);
    // the array keeps what the last call left: the arrival counters must start at zero (a fill kernel, not a memset node,
    // so that the call can be captured into a graph)
    launch_fill_int(s, t.rcnt, n, 0);
    launch_tail(s, ctx->c.dtype, ctx->D, t);   // the streaming kernels, on the borrowed weights
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(ctx, e, "tr_tail_noalloc: launch");
    return TR_OK;
}

int tr_seq_fork(tr_ctx *ctx, void *hip_stream, int32_t src, int32_t dst)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (src < 0 || src >= ctx->c.max_batch || dst < 0 || dst >= ctx->c.max_batch || src == dst)
        return fail(ctx, TR_ERR_INVALID_ARG, "tr_seq_fork: bad slot pair");
    { const int src = sync_lengths(ctx); if (src != TR_OK) return src; }
    if (ctx->len[(size_t)src] < 0) return fail(ctx, TR_ERR_STATE, "tr_seq_fork: source slot was never filled");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const Layout &L = ctx->lay;
    if (ctx->c.kv_page) {
        // paged cache: the copy refers to the same pages; a page is copied only when one of the two is about to write into it
        KvPages &P = ctx->pages;
        P.shrink(dst, 0);
        P.share(src, dst);
        if (P.npages[(size_t)dst] > 0) {
            const hipError_t e = hipMemcpyAsync(ctx->ws + L.ptab + (size_t)dst * L.maxp * 4, P.row(dst), (size_t)P.npages[(size_t)dst] * 4, hipMemcpyHostToDevice, s);
            if (e != hipSuccess) return fail_hip(ctx, e, "tr_seq_fork: page table");
        }
    }
    // contiguous cache: a slot's keys (and values) of one layer are one block; whole blocks are copied, whatever the length
    const size_t kb = L.k_layer_bytes / (size_t)ctx->c.max_batch, vb = L.v_layer_bytes / (size_t)ctx->c.max_batch;
    for (int l = 0; l < (ctx->c.kv_page ? 0 : ctx->D.L); ++l) {
        char *k = static_cast<char *>(ctx->kc_layer(l)), *v = static_cast<char *>(ctx->vc_layer(l));
        hipError_t e = hipMemcpyAsync(k + (size_t)dst * kb, k + (size_t)src * kb, kb, hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(v + (size_t)dst * vb, v + (size_t)src * vb, vb, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail_hip(ctx, e, "tr_seq_fork: copy");
    }
    long long *cnt = ctx->at<long long>(L.counters);
    hipError_t e = hipMemcpyAsync(cnt + 2 * (size_t)dst, cnt + 2 * (size_t)src, 2 * sizeof(long long), hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return fail_hip(ctx, e, "tr_seq_fork: copy");
    ctx->len[(size_t)dst] = ctx->len[(size_t)src];
    return TR_OK;
}

int tr_seq_load_kv(tr_ctx *ctx, void *hip_stream, int32_t slot, int32_t len, const void *k, const void *v)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (!k || !v) return fail(ctx, TR_ERR_INVALID_ARG, "tr_seq_load_kv: null argument");
    if (slot < 0 || slot >= ctx->c.max_batch) return fail(ctx, TR_ERR_INVALID_ARG, "tr_seq_load_kv: slot out of range");
    { const int src = sync_lengths(ctx); if (src != TR_OK) return src; }
    if (len < 1 || len > ctx->c.max_seq) return fail(ctx, TR_ERR_CAPACITY, "tr_seq_load_kv: len outside [1, max_seq]");
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (ctx->c.kv_page) {
        const KvPages before = ctx->pages;
        const int zero = 0, sl = slot, want = len;
        ctx->pages.shrink(slot, 0);
        const int prc = reserve_pages(ctx, s, 1, &sl, &zero, &want, "tr_seq_load_kv: page table");
        if (prc != TR_OK) { ctx->pages = before; return prc; }
    }
    launch_load_kv(s, ctx->c.kv_dtype, ctx->D, slot, len, k, v, ctx->ws + ctx->lay.kc, ctx->ws + ctx->lay.vc);
    launch_reset_counters(s, ctx->at<long long>(ctx->lay.counters), slot);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(ctx, e, "tr_seq_load_kv: launch");
    ctx->len[(size_t)slot] = len;
    return TR_OK;
}

int tr_profile_enable(tr_ctx *ctx, int32_t on)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (on && ctx->ev.empty()) {
        ctx->ev.resize(3 * 256);
        for (auto &e : ctx->ev) {
            hipError_t rc = hipEventCreate(&e);
            if (rc != hipSuccess) {
                for (hipEvent_t *made = ctx->ev.data(); made != &e; ++made) (void)hipEventDestroy(*made);
                ctx->ev.clear();
                return fail_hip(ctx, rc, "tr_profile_enable: hipEventCreate");
            }
        }
    }
    if (on && !ctx->profile) { ctx->prof_ms = ctx->prof_gap_ms = 0.0; ctx->prof_launches = 0; ctx->ev_used = 0; ctx->prof_seen = ctx->prof_pick = 0; }
    if (!on && ctx->profile) drain_profile(ctx);
    ctx->profile = on != 0;
    return TR_OK;
}

int tr_profile_select(tr_ctx *ctx, int32_t family)
{
    if (!ctx) return TR_ERR_INVALID_ARG;
    if (family < 0 || family >= TR_KERNEL_FAMILIES) return fail(ctx, TR_ERR_INVALID_ARG, "tr_profile_select: unknown kernel family");
    if (ctx->profile) drain_profile(ctx);
    ctx->prof_family = family;
    ctx->prof_ms = ctx->prof_gap_ms = 0.0; ctx->prof_launches = 0; ctx->ev_used = 0; ctx->prof_seen = ctx->prof_pick = 0;
    return TR_OK;
}

int tr_profile_read(tr_ctx *ctx, double *ms_total, double *ms_empty_pairs, int64_t *launches)
{
    if (!ctx || !ms_total || !ms_empty_pairs || !launches) return TR_ERR_INVALID_ARG;
    drain_profile(ctx);
    *ms_total = ctx->prof_ms;
    *ms_empty_pairs = ctx->prof_gap_ms;
    *launches = ctx->prof_launches;
    return TR_OK;
}

}  // extern "C"
