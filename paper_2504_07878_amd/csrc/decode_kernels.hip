// Streaming (GEMV-class) kernels of the decode step for gfx950: fp32 activations, fp32 or bf16 weights,
// fp32 accumulation. One 64-lane wavefront owns a few output rows and strides over the reduction
// dimension with 16-byte loads; reductions are wavefront shuffles in a fixed order, so results are
// bit-identical from run to run.
//
// The step follows the decoder of the model family named in Section 4.2 of arxiv 2504.07878
// (pre-norm, grouped-query attention, rotary embedding with half-split pairing, SwiGLU FFN);
// the tail (final norm, LM head, confidence, router, flag) is in tail_kernels.hip.
#include "tr_internal.h"

namespace tr {

// ------------------------------------------------------------------ small device helpers

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }

// nearest-even rounding of fp32 to bf16 (NaN kept quiet)
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

__device__ __forceinline__ void load8(const float *p, float (&w)[8])
{
    float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
}

__device__ __forceinline__ void load8(const bf16_t *p, float (&w)[8])
{
    uint4 v = *reinterpret_cast<const uint4 *>(p);
    w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xffff0000u);
    w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xffff0000u);
    w[4] = __uint_as_float(v.z << 16); w[5] = __uint_as_float(v.z & 0xffff0000u);
    w[6] = __uint_as_float(v.w << 16); w[7] = __uint_as_float(v.w & 0xffff0000u);
}

__device__ __forceinline__ float widen(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float widen(const bf16_t *p, size_t i) { return bf16_to_f32(p[i]); }

__device__ __forceinline__ void store_kv(float *p, float v) { *p = v; }
__device__ __forceinline__ void store_kv(bf16_t *p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

template <typename KT> struct Raw8;
template <> struct Raw8<bf16_t> {
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void get(float (&w)[8]) const
    {
        w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xffff0000u);
        w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xffff0000u);
        w[4] = __uint_as_float(v.z << 16); w[5] = __uint_as_float(v.z & 0xffff0000u);
        w[6] = __uint_as_float(v.w << 16); w[7] = __uint_as_float(v.w & 0xffff0000u);
    }
};
template <> struct Raw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float *p) { a = *reinterpret_cast<const float4 *>(p); b = *reinterpret_cast<const float4 *>(p + 4); }
    __device__ __forceinline__ void get(float (&w)[8]) const { w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w; }
};

// One 512-column step of the dot products of NR weight rows with MB activation rows (staged in LDS).
template <typename WT, int NR, int MB>
__device__ __forceinline__ void dots_step(const Raw8<WT> (&rw)[NR], const float *const (&xrow)[MB], int k, float (&acc)[NR][MB])
{
    float w[NR][8];
#pragma unroll
    for (int r = 0; r < NR; ++r) rw[r].get(w[r]);
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        float xv[8];
        load8(xrow[m] + k, xv);
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int r = 0; r < NR; ++r) acc[r][m] = fmaf(w[r][i], xv[i], acc[r][m]);
    }
}

// Activation columns staged in LDS at a time: two weight batches of U 512-column steps (U = 4 up to two activation rows,
// U = 2 at four), so that the buffer is 16 KiB for one row and 32 KiB otherwise.
template <int MB> struct DotsCfg {
    static constexpr int U = MB > 2 ? 2 : 4;
    static constexpr int BATCH = U * 512;
    static constexpr int KC = 2 * BATCH;
    static constexpr int LDS_FLOATS = MB * KC + 4 * MB;   // the staged chunk, then one sum of squares per wavefront and row
};

// Where the staged activations come from: plain fp32 rows ...
struct StageRows {
    static constexpr bool direct = true;    // plain rows in memory: lanes may fetch their own columns
    const float *x;
    size_t stride;
    __device__ __forceinline__ float4 load(int m, int k) const { return *reinterpret_cast<const float4 *>(x + (size_t)m * stride + k); }
    __device__ __forceinline__ void advance(int rows) { x += (size_t)rows * stride; }
};
// ... or attention partials merged on the fly (fixed order over the chunks)
struct StageAttn {
    static constexpr bool direct = false;   // a staged value costs a merge over the chunks: stage once per workgroup
    AttnPending a;
    int Hq, dh, r0;
    // up to 16 chunks (the launcher defers the merge only then); all requests of a phase are issued together, with
    // indices clamped to the live chunks and weight 0 past them
    __device__ __forceinline__ float4 load(int m, int k) const
    {
        const int r = r0 + m, head = k / dh, d0 = k % dh, ps = dh + 4;
        // chunks that hold keys: positions 0..pos, or 0..pos-1 when the new key joins here (chunk 0 is always written then)
        const int live = a.qn ? max(1, min(a.nchunks, (a.pos[r] + a.chunk - 1) / a.chunk)) : min(a.nchunks, (a.pos[r] + a.chunk) / a.chunk);
        const float *pp = a.part + ((size_t)r * Hq + head) * a.nchunks * ps;
        // the row's own key: its score is taken here, from the rotated query and the key as the cache holds it. The 16 lanes
        // that stage one 64-wide head (consecutive lanes, 4 dims each) share the dot product.
        float snew = -INFINITY;
        float4 vnew = make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.qn) {
            const float *kp = a.kvn + (size_t)r * 2 * a.kvw + (size_t)(head / a.G) * dh;
            const float4 qv = *reinterpret_cast<const float4 *>(a.qn + (size_t)r * Hq * dh + k), kv = *reinterpret_cast<const float4 *>(kp + d0);
            vnew = *reinterpret_cast<const float4 *>(kp + a.kvw + d0);
            float dot = fmaf(qv.x, kv.x, fmaf(qv.y, kv.y, fmaf(qv.z, kv.z, qv.w * kv.w)));
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) dot += __shfl_xor(dot, o, 64);
            snew = dot * 0.125f;   // 1 / sqrt(64)
        }
        float mc[16], lc[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const float *pc = pp + min(c, live - 1) * ps + dh;
            mc[c] = pc[0]; lc[c] = pc[1];
        }
        float M = snew;
#pragma unroll
        for (int c = 0; c < 16; ++c) M = fmaxf(M, mc[c]);   // clamped entries repeat a live chunk
        const float wnew = __expf(snew - M);                 // 0 when no new key joins
        float L = wnew;
        float4 o = make_float4(vnew.x * wnew, vnew.y * wnew, vnew.z * wnew, vnew.w * wnew);
#pragma unroll
        for (int c0 = 0; c0 < 16; c0 += 8) {
            if (c0 >= live) break;
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const float4 *>(pp + min(c0 + u, live - 1) * ps + d0);
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float w = c0 + u < live ? __expf(mc[c0 + u] - M) : 0.f;
                L = fmaf(lc[c0 + u], w, L);
                o.x = fmaf(v[u].x, w, o.x); o.y = fmaf(v[u].y, w, o.y); o.z = fmaf(v[u].z, w, o.z); o.w = fmaf(v[u].w, w, o.w);
            }
        }
        const float inv = 1.0f / L;
        return make_float4(o.x * inv, o.y * inv, o.z * inv, o.w * inv);
    }
    __device__ __forceinline__ void advance(int rows) { r0 += rows; }
};

// Workgroup-wide GEMV step: the 4 wavefronts of a workgroup each own NR weight rows; the MB activation
// rows are staged through LDS in chunks of KC columns (read once from memory per workgroup, then broadcast from LDS,
// which keeps the vector-memory pipe free for the weight stream). With NORM the staged values are x*gain and the rows'
// sums of squares are accumulated while staging, so that W.(g*x/rms) = W.(g*x) / rms needs no normalisation pass and
// no per-weight work. The weight stream does not depend on the staging, so it runs one batch ahead of the arithmetic
// in two register sets: the first batch is requested before the activations are staged, and each later batch while
// the previous one is consumed, across chunk boundaries. Requests past the end of a row are
// redirected to its last 16 bytes (one cache line for the whole wavefront) and their result is unused, which keeps
// every request unconditional and the number in flight known at compile time.
// Every wavefront of the workgroup must call this (barriers inside). xs: LDS buffer of DotsCfg<MB>::LDS_FLOATS floats.
// Rows m >= mvalid are read as zeros. K % 8 == 0. Results are valid in every lane.
// (Several row groups per wavefront, which would amortise the staging, were measured 5 % to 17 % slower on the
// 7B-class FFN: too few wavefronts are left to fill the chip evenly.)
template <typename WT, int NR, int MB, bool NORM, class Stage>
__device__ __forceinline__ void wg_dots(const WT *const (&wrow)[NR], const WT *gain, const Stage &src, int mvalid, int K, float *xs,
                                        float (&acc)[NR][MB], float (&ss)[MB])
{
    constexpr int U = DotsCfg<MB>::U, BATCH = DotsCfg<MB>::BATCH, KC = DotsCfg<MB>::KC;
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        ss[m] = 0.f;
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[r][m] = 0.f;
    }
    Raw8<WT> rw[2][U][NR];
    const float *xr[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) xr[m] = xs + m * KC;

#define TR_ISSUE(SET, K0)                                                                     \
    _Pragma("unroll") for (int u = 0; u < U; ++u) {                                           \
        const int kk = min((K0) + u * 512 + lane * 8, K - 8);                                 \
        _Pragma("unroll") for (int r = 0; r < NR; ++r) rw[SET][u][r].load(wrow[r] + kk);      \
    }
#define TR_CONSUME(SET, K0, KC0)                                                              \
    if ((K0) + BATCH <= K) {                                                                  \
        _Pragma("unroll") for (int u = 0; u < U; ++u)                                         \
            dots_step<WT, NR, MB>(rw[SET][u], xr, (K0) - (KC0) + u * 512 + lane * 8, acc);    \
    } else {                                                                                  \
        _Pragma("unroll") for (int u = 0; u < U; ++u)                                         \
            if ((K0) + u * 512 + lane * 8 < K)                                                \
                dots_step<WT, NR, MB>(rw[SET][u], xr, (K0) - (KC0) + u * 512 + lane * 8, acc);    \
    }

    // stages columns kc0 .. kc0+kc-1 of the MB rows (gain applied, sums of squares taken); barriers on both sides
    auto stage = [&](int kc0, int kc) {
        __syncthreads();
        for (int c = threadIdx.x * 4; c < kc; c += 1024) {
            float4 g = make_float4(1.f, 1.f, 1.f, 1.f);
            if (NORM) g = make_float4(widen(gain, kc0 + c), widen(gain, kc0 + c + 1), widen(gain, kc0 + c + 2), widen(gain, kc0 + c + 3));
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (m < mvalid) v = src.load(m, kc0 + c);
                if (NORM) {
                    ss[m] = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, fmaf(v.w, v.w, ss[m]))));
                    v = make_float4(v.x * g.x, v.y * g.y, v.z * g.z, v.w * g.w);
                }
                *reinterpret_cast<float4 *>(xs + m * KC + c) = v;
            }
        }
        __syncthreads();
    };
    if (K <= 1024) {
        // short rows (the 0.5B-class model's d = 896): two steps cover a row, so there is nothing to run ahead of and
        // no request is made that is not used
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int kk = min(u * 512 + lane * 8, K - 8);
#pragma unroll
            for (int r = 0; r < NR; ++r) rw[0][u][r].load(wrow[r] + kk);
        }
        if constexpr (MB <= 2 && Stage::direct) {
            // one or two plain activation rows: every lane fetches the 16 columns it multiplies (and their gains) together
            // with the weights, each wavefront sees the whole rows, so nothing goes through LDS and no barrier is needed
            float4 xa[MB][2][2];
            Raw8<WT> gr[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int kk = min(u * 512 + lane * 8, K - 8);
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    const int mm = m < mvalid ? m : 0;   // a missing second row repeats the first; its results are dropped by the caller
                    xa[m][u][0] = src.load(mm, kk); xa[m][u][1] = src.load(mm, kk + 4);
                }
                if (NORM) gr[u].load(gain + kk);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u)
                if (u * 512 + lane * 8 < K) {
                    float g[8];
                    if (NORM) gr[u].get(g);
                    float w[NR][8];
#pragma unroll
                    for (int r = 0; r < NR; ++r) rw[0][u][r].get(w[r]);
#pragma unroll
                    for (int m = 0; m < MB; ++m) {
                        float xe[8] = {xa[m][u][0].x, xa[m][u][0].y, xa[m][u][0].z, xa[m][u][0].w, xa[m][u][1].x, xa[m][u][1].y, xa[m][u][1].z, xa[m][u][1].w};
                        if (NORM) {
#pragma unroll
                            for (int e = 0; e < 8; ++e) { ss[m] = fmaf(xe[e], xe[e], ss[m]); xe[e] *= g[e]; }
                        }
#pragma unroll
                        for (int r = 0; r < NR; ++r)
#pragma unroll
                            for (int e = 0; e < 8; ++e) acc[r][m] = fmaf(w[r][e], xe[e], acc[r][m]);
                    }
                }
#pragma unroll
            for (int m = 0; m < MB; ++m) {
#pragma unroll
                for (int r = 0; r < NR; ++r) acc[r][m] = wave_sum(acc[r][m]);
                if (NORM) ss[m] = wave_sum(ss[m]);
            }
            return;
        }
        stage(0, K);
#pragma unroll
        for (int u = 0; u < 2; ++u)
            if (u * 512 + lane * 8 < K) dots_step<WT, NR, MB>(rw[0][u], xr, u * 512 + lane * 8, acc);
    } else {
        TR_ISSUE(0, 0)
        int kc0 = 0;
        for (; kc0 + KC < K; kc0 += KC) {   // chunks with a successor: every request of the steady state is unconditional
            stage(kc0, KC);
            TR_ISSUE(1, kc0 + BATCH)
            TR_CONSUME(0, kc0, kc0)
            TR_ISSUE(0, kc0 + KC)
            TR_CONSUME(1, kc0 + BATCH, kc0)
        }
        stage(kc0, K - kc0);                // last chunk: nothing is requested beyond the row
        if (kc0 + BATCH < K) {
            TR_ISSUE(1, kc0 + BATCH)
            TR_CONSUME(0, kc0, kc0)
            TR_CONSUME(1, kc0 + BATCH, kc0)
        } else {
            TR_CONSUME(0, kc0, kc0)
        }
    }
#undef TR_ISSUE
#undef TR_CONSUME
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int r = 0; r < NR; ++r) acc[r][m] = wave_sum(acc[r][m]);
    if (NORM) {
        float *red = xs + MB * KC;
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            const float t = wave_sum(ss[m]);
            if (lane == 0) red[(threadIdx.x >> 6) * MB + m] = t;
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < MB; ++m) ss[m] = (red[m] + red[MB + m]) + (red[2 * MB + m] + red[3 * MB + m]);
    }
}

// ------------------------------------------------------------------ row metadata

struct SetupArgs {
    int n;
    int slot[256], tok[256], pos[256];
};

__global__ void iota_rows_kernel(int n, int slot, int base, int *d_slot, int *d_pos)
{
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        d_slot[i] = slot;
        d_pos[i] = base + i;
    }
}

void launch_iota_rows(hipStream_t s, int n, int slot, int base, int *d_slot, int *d_pos)
{
    hipLaunchKernelGGL(iota_rows_kernel, dim3((n + 255) / 256), dim3(256), 0, s, n, slot, base, d_slot, d_pos);
}

__global__ void reset_counters_kernel(long long *counters, int slot)
{
    counters[2 * slot + threadIdx.x] = 0;
}

void launch_reset_counters(hipStream_t s, long long *counters, int slot)
{
    hipLaunchKernelGGL(reset_counters_kernel, dim3(1), dim3(2), 0, s, counters, slot);
}

__global__ void fill_int_kernel(int *p, int n, int value)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

void launch_fill_int(hipStream_t s, int *p, int n, int value)
{
    hipLaunchKernelGGL(fill_int_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n, value);
}

// ------------------------------------------------------------------ device-side selection of a step's rows
// (the flags a router left in device memory pick the sequences the other model steps; the host never sees them)

struct ActiveArgs {
    int n;
    int slot[256], len[256];   // candidates: slot, and its length where the host knows it (-1: the device-side array is ahead of the host)
};

__global__ __launch_bounds__(256) void active_setup_kernel(ActiveArgs a, const int *flags, const int *tokens, int n_max, int vocab, int *dev_len,
                                                           int *d_slot, int *d_tok, int *d_pos, int *active)
{
    __shared__ int s_scan[256];
    const int i = threadIdx.x;
    const bool cand = i < a.n;
    const int f = cand && flags[i] != 0 ? 1 : 0;
    if (cand && a.len[i] >= 0) dev_len[a.slot[i]] = a.len[i];   // slots are distinct: one writer per entry
    s_scan[i] = f;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {   // inclusive scan in a fixed order
        const int v = i >= o ? s_scan[i - o] : 0;
        __syncthreads();
        s_scan[i] += v;
        __syncthreads();
    }
    const int total = s_scan[255], count = min(total, n_max), rank = s_scan[i] - f;
    if (f && rank < n_max) {
        const int slot = a.slot[i], len = dev_len[slot];   // this thread's own write above, or the value an earlier step left
        d_slot[rank] = slot;
        d_pos[rank] = len;
        d_tok[rank] = min(max(tokens[i], 0), vocab - 1);
        dev_len[slot] = len + 1;
        active[2 + rank] = i;
    }
    for (int r = count + i; r < n_max; r += 256) {   // padding rows: a valid slot at position 0, no state changes
        d_slot[r] = a.slot[0]; d_pos[r] = 0; d_tok[r] = 0;
        active[2 + r] = -1;
    }
    if (i == 0) { active[0] = count; active[1] = total; }
}

void launch_active_setup(hipStream_t s, int n, const int *cand_slot, const int *host_len, const int *flags_dev, const int *tokens_dev, int n_max,
                         int vocab, int *dev_len, int *d_slot, int *d_tok, int *d_pos, int *active)
{
    ActiveArgs a;
    a.n = n;
    for (int i = 0; i < 256; ++i) { a.slot[i] = i < n ? cand_slot[i] : 0; a.len[i] = i < n ? host_len[i] : -1; }
    hipLaunchKernelGGL(active_setup_kernel, dim3(1), dim3(256), 0, s, a, flags_dev, tokens_dev, n_max, vocab, dev_len, d_slot, d_tok, d_pos, active);
}

// ------------------------------------------------------------------ embedding lookup: x[r] = E[tok[r]]

template <typename WT>
__global__ void embed_kernel(const WT *E, const int *tok, int d, float *x)
{
    const int r = blockIdx.x;
    const WT *e = E + (size_t)tok[r] * d;
    for (int j = threadIdx.x; j < d; j += blockDim.x) x[(size_t)r * d + j] = widen(e, j);
}

// Row metadata from the kernel arguments and the embedding lookup of the same rows in one launch (a decode step's first kernel)
// dev_tok != NULL: the tokens come from device memory (e.g. the previous step's output) instead of the arguments; they cannot
// be checked on the host, so values outside the vocabulary are clamped into it.
template <typename WT>
__global__ void setup_embed_kernel(SetupArgs a, int *d_slot, int *d_tok, int *d_pos, int base, const WT *E, int d, float *x, const int *dev_tok, int vocab)
{
    const int i = blockIdx.x, r = base + i;
    const int tok = dev_tok ? min(max(dev_tok[r], 0), vocab - 1) : a.tok[i];
    if (threadIdx.x == 0) {
        d_slot[r] = a.slot[i];
        d_tok[r] = tok;
        d_pos[r] = a.pos[i];
    }
    const WT *e = E + (size_t)tok * d;
    for (int j = threadIdx.x; j < d; j += blockDim.x) x[(size_t)r * d + j] = widen(e, j);
}

void launch_setup_rows_embed(hipStream_t s, int n, const int *slots, const int *toks, const int *poss, int *d_slot, int *d_tok, int *d_pos, int wdt,
                             const void *E, int d, float *x, const int *dev_toks, int vocab)
{
    for (int base = 0; base < n; base += 256) {
        SetupArgs a;
        a.n = n - base < 256 ? n - base : 256;
        for (int i = 0; i < a.n; ++i) {
            a.slot[i] = slots[base + i];
            a.tok[i] = toks ? toks[base + i] : 0;
            a.pos[i] = poss[base + i];
        }
        if (wdt == DT_F32)
            hipLaunchKernelGGL(setup_embed_kernel<float>, dim3(a.n), dim3(256), 0, s, a, d_slot, d_tok, d_pos, base, (const float *)E, d, x, dev_toks, vocab);
        else
            hipLaunchKernelGGL(setup_embed_kernel<bf16_t>, dim3(a.n), dim3(256), 0, s, a, d_slot, d_tok, d_pos, base, (const bf16_t *)E, d, x, dev_toks, vocab);
    }
}

void launch_embed(hipStream_t s, int wdt, const void *E, const int *tok, int R, int d, float *x)
{
    if (wdt == DT_F32) hipLaunchKernelGGL(embed_kernel<float>, dim3(R), dim3(256), 0, s, (const float *)E, tok, d, x);
    else hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3(R), dim3(256), 0, s, (const bf16_t *)E, tok, d, x);
}

// ------------------------------------------------------------------ attention input:
// n = RMSNorm(x; ln1); [q|k|v] = W n + b; rotate q and k at the row's position; append k, v to the cache.
// One wavefront computes the two output rows (j, j + dh/2) of one head that the rotation pairs up.

template <typename WT, typename KT, int MB>
__global__ __launch_bounds__(256) void qkv_kernel(Dims D, LayerW w, const float *x, Rows rows, const float2 *rope, float *q, KT *kc,
                                                  KT *vc)
{
    __shared__ __attribute__((aligned(16))) float xs[DotsCfg<MB>::LDS_FLOATS];
    const int half = D.dh / 2;
    const int npairs = (D.Hq + 2 * D.Hkv) * half;
    const int pair_raw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int pair = pair_raw < npairs ? pair_raw : npairs - 1;   // surplus wavefronts redo the last pair and drop it
    const int hh = pair / half, j = pair % half;
    const WT *W, *bias;
    int head;  // head index inside its own matrix
    if (hh < D.Hq) { W = (const WT *)w.wq; bias = (const WT *)w.bq; head = hh; }
    else if (hh < D.Hq + D.Hkv) { W = (const WT *)w.wk; bias = (const WT *)w.bk; head = hh - D.Hq; }
    else { W = (const WT *)w.wv; bias = (const WT *)w.bv; head = hh - D.Hq - D.Hkv; }
    const int n1 = head * D.dh + j, n2 = n1 + half;
    const WT *const wrow[2] = {W + (size_t)n1 * D.d, W + (size_t)n2 * D.d};
    const int r0 = blockIdx.y * MB;
    // what the epilogue needs from memory is requested now (position -> rotary pair is a chain of two dependent loads)
    // and arrives while the weights stream
    KvPlace place[MB];   // where the row's new key and value go
    float2 cs[MB];
    float b1 = 0.f, b2 = 0.f;
    if (bias) { b1 = widen(bias, n1); b2 = widen(bias, n2); }
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const int r = min(r0 + m, rows.n - 1);
        const int pos = rows.pos[r];
        place[m] = kv_place(D, rows.slot[r], pos);
        cs[m] = rope[(size_t)pos * half + j];
    }
    float acc[2][MB], ss[MB];
    wg_dots<WT, 2, MB, true>(wrow, (const WT *)w.ln1, StageRows{x + (size_t)r0 * D.d, (size_t)D.d}, rows.n - r0, D.d, xs, acc, ss);
    if ((threadIdx.x & 63) != 0 || pair_raw >= npairs) return;
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const int r = r0 + m;
        if (r >= rows.n) break;
        const float rstd = 1.0f / sqrtf(ss[m] / (float)D.d + D.eps);
        float y1 = acc[0][m] * rstd + b1, y2 = acc[1][m] * rstd + b2;
        if (hh < D.Hq + D.Hkv) {
            const float o1 = y1 * cs[m].x - y2 * cs[m].y, o2 = y2 * cs[m].x + y1 * cs[m].y;
            y1 = o1; y2 = o2;
        }
        if (hh < D.Hq) {
            q[(size_t)r * D.qw + n1] = y1;
            q[(size_t)r * D.qw + n2] = y2;
        } else if (hh < D.Hq + D.Hkv) {
            KT *dst = kc + k_offset(D, place[m].unit, head, place[m].pos, 0);
            store_kv(dst + j, y1);
            store_kv(dst + j + half, y2);
        } else {
            store_kv(vc + v_offset(D, place[m].unit, head, place[m].pos, j), y1);
            store_kv(vc + v_offset(D, place[m].unit, head, place[m].pos, j + half), y2);
        }
    }
}

template <typename WT, typename KT>
static void launch_qkv_t(hipStream_t s, const Dims &D, const LayerW &w, const float *x, Rows rows, const float2 *rope, float *q, void *kc,
                         void *vc)
{
    const int pairs = (D.Hq + 2 * D.Hkv) * (D.dh / 2), gx = (pairs + 3) / 4;
    if (rows.n == 1)
        hipLaunchKernelGGL((qkv_kernel<WT, KT, 1>), dim3(gx, 1), dim3(256), 0, s, D, w, x, rows, rope, q, (KT *)kc, (KT *)vc);
    else if (rows.n == 2)
        hipLaunchKernelGGL((qkv_kernel<WT, KT, 2>), dim3(gx, 1), dim3(256), 0, s, D, w, x, rows, rope, q, (KT *)kc, (KT *)vc);
    else
        hipLaunchKernelGGL((qkv_kernel<WT, KT, 4>), dim3(gx, (rows.n + 3) / 4), dim3(256), 0, s, D, w, x, rows, rope, q, (KT *)kc, (KT *)vc);
}

// 2 to 4 rows of a wide bf16 model, rows kept in registers (qkv_rows_kernel below); false: not served
static bool launch_qkv_rows(hipStream_t s, int wdt, int kdt, const Dims &D, const LayerW &w, const float *x, Rows rows, const float2 *rope, float *q,
                            void *kc, void *vc);

void launch_qkv(hipStream_t s, int wdt, int kdt, const Dims &D, const LayerW &w, const float *x, Rows rows, const float2 *rope, float *q,
                void *kc, void *vc)
{
    if (launch_qkv_rows(s, wdt, kdt, D, w, x, rows, rope, q, kc, vc)) return;
    if (wdt == DT_F32 && kdt == DT_F32) launch_qkv_t<float, float>(s, D, w, x, rows, rope, q, kc, vc);
    else if (wdt == DT_F32) launch_qkv_t<float, bf16_t>(s, D, w, x, rows, rope, q, kc, vc);
    else if (kdt == DT_F32) launch_qkv_t<bf16_t, float>(s, D, w, x, rows, rope, q, kc, vc);
    else launch_qkv_t<bf16_t, bf16_t>(s, D, w, x, rows, rope, q, kc, vc);
}

// ------------------------------------------------------------------ q|k|v projection and attention in one launch
// (one or two decode rows, bf16 weights and cache, 64-wide heads, d <= 1024).
// A decode step of one sequence is a chain of small dependent kernels, each costing several microseconds whatever it
// does; this kernel removes one link per layer. Two kinds of workgroups (8 wavefronts):
//  * (query head h, chunk c of the keys cached BEFORE this step): computes q_h = rotate(W_q[h] n + b) itself -- 64 weight
//    rows of d columns, re-read from L2 by the other chunks of the head -- while its keys and values are already on
//    their way, then scores its chunk (one key per 4 lanes), and leaves (weighted V sum, max, sum of exponentials) as a
//    partial. Chunk 0 also stores q_h.
//  * k/v workgroups: the new key (rotated) and value of the row, appended to the cache and also left, as the cache holds
//    them, in kvn.
// No workgroup has both q_h and the new key, so the new key's score and its share of the softmax are taken by the
// consumer of the partials (StageAttn) in the output projection.
// Rows must belong to different slots: a row's keys are read while other rows' keys are being appended.

// dot products of NR weight rows with one activation row of K <= 1024 columns (gain applied, sum of squares taken):
// each lane fetches the 16 columns it multiplies; results in every lane
template <int NR>
struct RowDots {
    Raw8<bf16_t> rw[2][NR], gr[2];
    float4 xa[2][2];
    __device__ __forceinline__ void request(const bf16_t *const (&wrow)[NR], const bf16_t *gain, const float *xrow, int K)
    {
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int kk = min(u * 512 + lane * 8, K - 8);
#pragma unroll
            for (int r = 0; r < NR; ++r) rw[u][r].load(wrow[r] + kk);
            xa[u][0] = *reinterpret_cast<const float4 *>(xrow + kk); xa[u][1] = *reinterpret_cast<const float4 *>(xrow + kk + 4);
            gr[u].load(gain + kk);
        }
    }
    __device__ __forceinline__ void finish(int K, float (&acc)[NR], float &ss)
    {
    const int lane = threadIdx.x & 63;
    ss = 0.f;
#pragma unroll
    for (int r = 0; r < NR; ++r) acc[r] = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
        if (u * 512 + lane * 8 < K) {
            float xe[8] = {xa[u][0].x, xa[u][0].y, xa[u][0].z, xa[u][0].w, xa[u][1].x, xa[u][1].y, xa[u][1].z, xa[u][1].w};
            float g[8];
            gr[u].get(g);
#pragma unroll
            for (int e = 0; e < 8; ++e) { ss = fmaf(xe[e], xe[e], ss); xe[e] *= g[e]; }
#pragma unroll
            for (int r = 0; r < NR; ++r) {
                float wv[8];
                rw[u][r].get(wv);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[r] = fmaf(wv[e], xe[e], acc[r]);
            }
        }
    ss = wave_sum(ss);
    }
};

// Sums each of NR (a power of two <= 16) per-lane values over the wavefront with NR - 1 + log2(64 / NR) exchanges instead of
// 6 NR: every step halves the number of values a lane carries. Afterwards lane L holds the total of value L / (64 / NR).
template <int N, int O>   // one halving step: N values remain afterwards, exchanged with the lane O away
__device__ __forceinline__ void wave_sum_step(float *v)
{
    const bool up = threadIdx.x & O;
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const float keep = up ? v[i + N] : v[i], send = up ? v[i] : v[i + N];
        v[i] = keep + __shfl_xor(send, O, 64);
    }
}
template <int NR>
__device__ __forceinline__ float wave_sum_n(float (&v)[NR])
{
    static_assert(NR == 4 || NR == 8 || NR == 16, "4, 8 or 16 values");
    // every array index below is a compile-time constant: the values stay in registers
    if constexpr (NR == 16) { wave_sum_step<8, 32>(v); wave_sum_step<4, 16>(v); wave_sum_step<2, 8>(v); wave_sum_step<1, 4>(v); }
    if constexpr (NR == 8) { wave_sum_step<4, 32>(v); wave_sum_step<2, 16>(v); wave_sum_step<1, 8>(v); }
    if constexpr (NR == 4) { wave_sum_step<2, 32>(v); wave_sum_step<1, 16>(v); }
    float t = v[0];
#pragma unroll
    for (int o = 64 / NR / 2; o >= 1; o >>= 1) t += __shfl_xor(t, o, 64);
    return t;
}

constexpr int QA_WAVES = 8;                  // wavefronts per workgroup (measured at a context of 384: 8.3 us per launch; 16 wavefronts 8.6 us; 4 spill registers)
constexpr int QA_PAIRS = 32 / QA_WAVES;       // rotary pairs (two weight rows each) per wavefront
constexpr int QA_NR = 2 * QA_PAIRS;
constexpr int QA_LG = 64 / QA_NR;             // lanes that end up with the same sum
constexpr int QA_KEYS = 128 / QA_WAVES;       // keys a wavefront scores at a time
constexpr int QA_LPK = 64 / QA_KEYS;          // lanes per key
constexpr int QA_DPL = 64 / QA_LPK;           // dims of a key per lane
constexpr int QA_STRIDE = QA_WAVES * QA_KEYS; // 128 keys per trip of a workgroup

__global__ __launch_bounds__(64 * QA_WAVES) void qkv_attn_kernel(Dims D, LayerW w, const float *x, Rows rows, const float2 *rope, float *q, bf16_t *kc,
                                                                 bf16_t *vc, int chunk, int nchunks, float *part, float *kvn)
{
    constexpr int DH = 64, HALF = 32, PS = DH + 4;
    __shared__ __attribute__((aligned(16))) float q_s[DH];
    __shared__ float wp[QA_WAVES][DH + 2];
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6), lane = threadIdx.x & 63;
    const int r = blockIdx.y, pos = rows.pos[r], slot = rows.slot[r];
    const float *xrow = x + (size_t)r * D.d;
    const int n_att = D.Hq * nchunks;
    const int grp = lane / QA_LG;                            // which of the wavefront's sums this lane ends up with
    const bool second = grp >= QA_PAIRS;                     // ... the second row of its rotary pair
    const int jpair = wave * QA_PAIRS + (grp % QA_PAIRS);    // rotary pair (jpair, jpair + 32) of the head
    const int dim_own = jpair + (second ? HALF : 0);

    if ((int)blockIdx.x >= n_att) {
        // ---- new key and value of the row: workgroup i takes kv "head" i (keys of head i, then values of head i - Hkv)
        const int hk = blockIdx.x - n_att;
        const bool is_k = hk < D.Hkv;
        const int head = is_k ? hk : hk - D.Hkv;
        const bf16_t *W = (const bf16_t *)(is_k ? w.wk : w.wv), *bias = (const bf16_t *)(is_k ? w.bk : w.bv);
        const bf16_t *wrow[QA_NR];
#pragma unroll
        for (int i = 0; i < QA_PAIRS; ++i) {
            wrow[i] = W + (size_t)(head * DH + wave * QA_PAIRS + i) * D.d;
            wrow[i + QA_PAIRS] = wrow[i] + (size_t)HALF * D.d;
        }
        RowDots<QA_NR> rd;
        rd.request(wrow, (const bf16_t *)w.ln1, xrow, D.d);
        const float b_own = bias ? widen(bias, head * DH + dim_own) : 0.f;
        const float2 cs = rope[(size_t)pos * HALF + jpair];
        const KvPlace place = kv_place(D, slot, pos);
        float acc[QA_NR], ss;
        rd.finish(D.d, acc, ss);
        const float rstd = 1.0f / sqrtf(ss / (float)D.d + D.eps);
        const float y_own = wave_sum_n<QA_NR>(acc) * rstd + b_own;
        const float y_other = __shfl_xor(y_own, 32, 64);
        float y = y_own;
        if (is_k) y = second ? y_own * cs.x + y_other * cs.y : y_own * cs.x - y_other * cs.y;
        if (lane % QA_LG == 0) {
            const bf16_t yb = f32_to_bf16(y);
            if (is_k) kc[k_offset(D, place.unit, head, place.pos, dim_own)] = yb;
            else vc[v_offset(D, place.unit, head, place.pos, dim_own)] = yb;
            kvn[((size_t)r * 2 + (is_k ? 0 : 1)) * D.kvw + head * DH + dim_own] = bf16_to_f32(yb);
        }
        return;
    }

    // ---- query head h over chunk c of the cached keys
    const int h = blockIdx.x / nchunks, c = blockIdx.x % nchunks, g = h / D.G;
    const int j0 = c * chunk, j1 = min(pos, j0 + chunk);       // keys j0 .. j1-1, all cached before this step
    if (c > 0 && j0 >= pos) return;                            // nothing here; the merge does not read this partial
    const int kk = lane / QA_LPK, qd = lane % QA_LPK;          // scores: key of the group and part of its dims
    const int last = max(j1 - 1, 0);                           // requests past the chunk are redirected to its last key and unused
    uint4 kraw[QA_DPL / 8], vraw[QA_KEYS / 8];
    auto request = [&](int t) {
        const KvPlace pk = kv_place(D, slot, min(t + kk, last));
        const bf16_t *kp = kc + k_offset(D, pk.unit, g, pk.pos, qd * QA_DPL);
#pragma unroll
        for (int i = 0; i < QA_DPL / 8; ++i) kraw[i] = *reinterpret_cast<const uint4 *>(kp + 8 * i);
        const KvPlace pv = kv_place(D, slot, min(t, last & ~(QA_KEYS - 1)));
        const bf16_t *vp = vc + v_offset(D, pv.unit, g, pv.pos, lane);     // QA_KEYS consecutive positions of dim `lane`
#pragma unroll
        for (int i = 0; i < QA_KEYS / 8; ++i) vraw[i] = *reinterpret_cast<const uint4 *>(vp + 8 * i);
    };
    const bf16_t *wrow[QA_NR];
#pragma unroll
    for (int i = 0; i < QA_PAIRS; ++i) {
        wrow[i] = (const bf16_t *)w.wq + (size_t)(h * DH + wave * QA_PAIRS + i) * D.d;
        wrow[i + QA_PAIRS] = wrow[i] + (size_t)HALF * D.d;
    }
    // the weights are requested first (their addresses need nothing from memory), then the keys and values, whose
    // addresses wait for the row's slot and position
    RowDots<QA_NR> rd;
    rd.request(wrow, (const bf16_t *)w.ln1, xrow, D.d);
    int t = j0 + wave * QA_KEYS;
    request(t);
    const float b_own = w.bq ? widen((const bf16_t *)w.bq, h * DH + dim_own) : 0.f;
    const float2 cs = rope[(size_t)pos * HALF + jpair];
    float acc[QA_NR], ss;
    rd.finish(D.d, acc, ss);
    const float rstd = 1.0f / sqrtf(ss / (float)D.d + D.eps);
    const float y_own = wave_sum_n<QA_NR>(acc) * rstd + b_own;
    const float y_other = __shfl_xor(y_own, 32, 64);
    const float yq = second ? y_own * cs.x + y_other * cs.y : y_own * cs.x - y_other * cs.y;
    if (lane % QA_LG == 0) {
        q_s[dim_own] = yq * (1.0f / sqrtf((float)DH));
        if (c == 0) q[(size_t)r * D.qw + h * DH + dim_own] = yq;
    }
    __syncthreads();

    float qv[QA_DPL];
#pragma unroll
    for (int e = 0; e < QA_DPL; e += 4) {
        const float4 a = *reinterpret_cast<const float4 *>(q_s + qd * QA_DPL + e);
        qv[e] = a.x; qv[e + 1] = a.y; qv[e + 2] = a.z; qv[e + 3] = a.w;
    }
    float m_run = -INFINITY, l_run = 0.f, o_run = 0.f;         // o_run: dim `lane` of the weighted V sum
    for (; t < j1; t += QA_STRIDE) {
        float kf[QA_DPL], vf[QA_KEYS];
#pragma unroll
        for (int i = 0; i < QA_DPL / 8; ++i) {
            float a[8];
            Raw8<bf16_t> ra{kraw[i]};
            ra.get(a);
#pragma unroll
            for (int e = 0; e < 8; ++e) kf[8 * i + e] = a[e];
        }
#pragma unroll
        for (int i = 0; i < QA_KEYS / 8; ++i) {
            float a[8];
            Raw8<bf16_t> ra{vraw[i]};
            ra.get(a);
#pragma unroll
            for (int e = 0; e < 8; ++e) vf[8 * i + e] = a[e];
        }
        if (t + QA_STRIDE < j1) request(t + QA_STRIDE);        // the next group, while this one is consumed
        float sc = 0.f;
#pragma unroll
        for (int e = 0; e < QA_DPL; ++e) sc = fmaf(qv[e], kf[e], sc);
#pragma unroll
        for (int o = 1; o < QA_LPK; o <<= 1) sc += __shfl_xor(sc, o, 64);
        if (t + kk >= j1) sc = -INFINITY;
        float bm = sc;                                         // the lanes of a key agree already
#pragma unroll
        for (int o = 32; o >= QA_LPK; o >>= 1) bm = fmaxf(bm, __shfl_xor(bm, o, 64));
        const float m_new = fmaxf(m_run, bm);                  // finite: key t is valid
        const float corr = __expf(m_run - m_new);              // 0 the first time
        const float p = __expf(sc - m_new);
        float psum = p;
#pragma unroll
        for (int o = 32; o >= QA_LPK; o >>= 1) psum += __shfl_xor(psum, o, 64);
        l_run = l_run * corr + psum;
        o_run *= corr;
#pragma unroll
        for (int e = 0; e < QA_KEYS; ++e) o_run = fmaf(__shfl(p, QA_LPK * e, 64), vf[e], o_run);
        m_run = m_new;
    }
    wp[wave][lane] = o_run;
    if (lane == 0) { wp[wave][DH] = m_run; wp[wave][DH + 1] = l_run; }
    __syncthreads();
    if (wave != 0) return;
    float M = -INFINITY;
#pragma unroll
    for (int i = 0; i < QA_WAVES; ++i) M = fmaxf(M, wp[i][DH]);
    float L = 0.f, O = 0.f;
    if (M > -INFINITY) {
#pragma unroll
        for (int i = 0; i < QA_WAVES; ++i) {
            const float wgt = __expf(wp[i][DH] - M);            // 0 for a wavefront that saw no key
            L = fmaf(wp[i][DH + 1], wgt, L);
            O = fmaf(wp[i][lane], wgt, O);
        }
    }
    float *dst = part + (((size_t)r * D.Hq + h) * nchunks + c) * PS;
    dst[lane] = O;
    if (lane == 0) { dst[DH] = M; dst[DH + 1] = L; }
}

bool launch_qkv_attention(hipStream_t s, int wdt, int kdt, const Dims &D, const LayerW &w, const float *x, Rows rows, int max_ctx,
                          const float2 *rope, float *q, void *kc, void *vc, float *part, size_t part_floats, float *kvn, AttnPending *pend)
{
    if (wdt != DT_BF16 || kdt != DT_BF16 || D.dh != 64 || D.d > 1024 || D.d % 8 || rows.n < 1 || rows.n > 2 || !pend) return false;
    // chunks of 128 cached keys (16 per wavefront), longer ones when the consumer's limit of 16 chunks asks for it
    const int cached = max_ctx > 1 ? max_ctx - 1 : 0;
    int chunk = QA_STRIDE, nchunks = (cached + chunk - 1) / chunk;
    if (nchunks > 16) {
        chunk = QA_STRIDE * ((cached + QA_STRIDE * 16 - 1) / (QA_STRIDE * 16));
        nchunks = (cached + chunk - 1) / chunk;
    }
    if (nchunks < 1) nchunks = 1;
    if ((size_t)rows.n * D.Hq * nchunks * (D.dh + 4) > part_floats) return false;
    const dim3 grid(D.Hq * nchunks + 2 * D.Hkv, rows.n);
    hipLaunchKernelGGL(qkv_attn_kernel, grid, dim3(64 * QA_WAVES), 0, s, D, w, x, rows, rope, q, (bf16_t *)kc, (bf16_t *)vc, chunk, nchunks, part, kvn);
    pend->part = part; pend->pos = rows.pos; pend->nchunks = nchunks; pend->chunk = chunk;
    pend->qn = q; pend->kvn = kvn; pend->G = D.G; pend->kvw = D.kvw;
    return true;
}

// ------------------------------------------------------------------ grouped-query attention over the cache.
// One workgroup (4 wavefronts) serves one query row, one kv head (all G query heads of its group share the
// K/V loads) and one contiguous chunk of the context ("split"); partial (max, sum, weighted V) triples of
// the splits are merged afterwards. Scores: one key per lane. Weighted sum of V: 8 dims per lane, 16-byte loads.

constexpr int MAXG = 8;

template <typename KT, int DH>
__global__ __launch_bounds__(256) void attn_kernel(Dims D, const float *q, const KT *kc, const KT *vc, Rows rows, int chunk, int nsplit,
                                                   float *part, float *att)
{
    constexpr int DG = DH / 8;    // lanes that cover one V row
    constexpr int KG = 64 / DG;   // V rows covered by one wavefront load
    __shared__ float q_s[MAXG][DH];
    __shared__ float p_s[4][MAXG][64];
    __shared__ float red_o[4][MAXG][DH];
    __shared__ float red_m[4][MAXG], red_l[4][MAXG];

    const int r = blockIdx.x, g = blockIdx.y, sp = blockIdx.z;
    const int G = D.G, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int ctx = rows.pos[r] + 1;
    const int j0 = sp * chunk, j1 = min(ctx, j0 + chunk);
    const float scale = 1.0f / sqrtf((float)DH);
    for (int i = threadIdx.x; i < G * DH; i += 256) q_s[i / DH][i % DH] = q[(size_t)r * D.qw + (size_t)g * G * DH + i] * scale;
    __syncthreads();

    const KT *Kb = kc + ((size_t)rows.slot[r] * D.Hkv + g) * (size_t)D.max_seq * DH;
    const KT *Vb = vc + ((size_t)rows.slot[r] * D.Hkv + g) * (size_t)D.max_seq * DH;
    const int dgrp = lane % DG, kgrp = lane / DG;

    float m[MAXG], l[MAXG], o[MAXG][8];
#pragma unroll
    for (int h = 0; h < MAXG; ++h) {
        m[h] = -INFINITY; l[h] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[h][i] = 0.f;
    }

    for (int t0 = j0; t0 < j1; t0 += 256) {
        const int t = t0 + wave * 64;          // first key of this wavefront's tile
        const bool tile_live = t < j1;         // wavefront-uniform
        if (tile_live) {
            const int j = t + lane;
            const bool valid = j < j1;
            float sc[MAXG];
#pragma unroll
            for (int h = 0; h < MAXG; ++h) sc[h] = 0.f;
            if (valid) {
                const KT *kr = Kb + (size_t)j * DH;
#pragma unroll 2
                for (int e = 0; e < DH; e += 8) {
                    float kv[8];
                    load8(kr + e, kv);
#pragma unroll
                    for (int h = 0; h < MAXG; ++h)
                        if (h < G) {
#pragma unroll
                            for (int i = 0; i < 8; ++i) sc[h] = fmaf(q_s[h][e + i], kv[i], sc[h]);
                        }
                }
            }
#pragma unroll
            for (int h = 0; h < MAXG; ++h)
                if (h < G) {
                    const float s = valid ? sc[h] : -INFINITY;
                    const float mn = fmaxf(m[h], wave_max(s));     // finite: lane 0 of a live tile is valid
                    const float p = valid ? expf(s - mn) : 0.f;
                    const float corr = expf(m[h] - mn);            // exp(-inf) = 0 on the first tile
                    l[h] = l[h] * corr + wave_sum(p);
#pragma unroll
                    for (int i = 0; i < 8; ++i) o[h][i] *= corr;
                    m[h] = mn;
                    p_s[wave][h][lane] = p;
                }
        }
        __syncthreads();
        if (tile_live) {
#pragma unroll 2
            for (int i = 0; i < 64 / KG; ++i) {
                const int jj = i * KG + kgrp, j = t + jj;
                if (j < j1) {
                    float vv[8];
                    load8(Vb + (size_t)j * DH + dgrp * 8, vv);
#pragma unroll
                    for (int h = 0; h < MAXG; ++h)
                        if (h < G) {
                            const float p = p_s[wave][h][jj];
#pragma unroll
                            for (int e = 0; e < 8; ++e) o[h][e] = fmaf(p, vv[e], o[h][e]);
                        }
                }
            }
        }
        __syncthreads();
    }

    // sum the per-key-group partial outputs inside the wavefront, then merge the 4 wavefronts
#pragma unroll
    for (int h = 0; h < MAXG; ++h)
        if (h < G) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float v = o[h][e];
#pragma unroll
                for (int off = DG; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
                o[h][e] = v;
            }
            if (kgrp == 0) {
#pragma unroll
                for (int e = 0; e < 8; ++e) red_o[wave][h][dgrp * 8 + e] = o[h][e];
            }
            if (lane == 0) { red_m[wave][h] = m[h]; red_l[wave][h] = l[h]; }
        }
    __syncthreads();
    for (int i = threadIdx.x; i < G * DH; i += 256) {
        const int h = i / DH, e = i % DH;
        float M = -INFINITY;
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) M = fmaxf(M, red_m[w2][h]);
        float Lsum = 0.f, O = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w2 = 0; w2 < 4; ++w2) {
                const float c = expf(red_m[w2][h] - M);
                Lsum += red_l[w2][h] * c;
                O += red_o[w2][h][e] * c;
            }
        }
        const int head = g * G + h;
        if (nsplit == 1) {
            att[(size_t)r * D.qw + head * DH + e] = O / Lsum;
        } else {
            float *pp = part + (((size_t)r * D.Hq + head) * nsplit + sp) * (DH + 2);
            pp[e] = O;
            if (e == 0) { pp[DH] = M; pp[DH + 1] = Lsum; }
        }
    }
}

template <int DH>
__global__ void attn_merge_kernel(Dims D, const float *part, int nsplit, float *att)
{
    const int r = blockIdx.x, head = blockIdx.y, e = threadIdx.x;
    const float *pp = part + ((size_t)r * D.Hq + head) * nsplit * (DH + 2);
    float M = -INFINITY;
    for (int s = 0; s < nsplit; ++s) M = fmaxf(M, pp[s * (DH + 2) + DH]);
    float Lsum = 0.f, O = 0.f;
    for (int s = 0; s < nsplit; ++s) {
        const float ms = pp[s * (DH + 2) + DH];
        if (ms > -INFINITY) {
            const float c = expf(ms - M);
            Lsum += pp[s * (DH + 2) + DH + 1] * c;
            O += pp[s * (DH + 2) + e] * c;
        }
    }
    att[(size_t)r * D.qw + head * DH + e] = O / Lsum;
}

// ---- decode variant: one wavefront per (query row, kv head, chunk of the context), no workgroup barrier in the
// loop. Every chunk writes an unnormalised partial (weighted V sum, running max, sum of exponentials); the merge
// kernel combines them in a fixed order. K and V of a tile are requested together, so a tile costs one memory
// round trip; with one tile per wavefront the whole context of a batch is in flight at once.

template <typename KT, int DH>
__global__ __launch_bounds__(256) void attn_wave_kernel(Dims D, const float *q, const KT *kc, const KT *vc, Rows rows, int chunk, int nchunks,
                                                        float *part)
{
    constexpr int DG = DH / 8, KG = 64 / DG, PS = DH + 4;   // PS: floats per partial (16-byte aligned rows)
    __shared__ float q_s[MAXG][DH];
    __shared__ float p_s[4][MAXG][64];
    const int r = blockIdx.x, g = blockIdx.y;
    const int G = D.G, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float scale = 1.0f / sqrtf((float)DH);
    for (int i = threadIdx.x; i < G * DH; i += 256) q_s[i / DH][i % DH] = q[(size_t)r * D.qw + (size_t)g * G * DH + i] * scale;
    __syncthreads();   // the only workgroup barrier
    const int c = blockIdx.z * 4 + wave;
    if (c >= nchunks) return;
    const int ctx = rows.pos[r] + 1;
    const int j0 = c * chunk, j1 = min(ctx, j0 + chunk);
    const KT *Kb = kc + ((size_t)rows.slot[r] * D.Hkv + g) * (size_t)D.max_seq * DH;
    const KT *Vb = vc + ((size_t)rows.slot[r] * D.Hkv + g) * (size_t)D.max_seq * DH;
    const int dgrp = lane % DG, kgrp = lane / DG;

    float m[MAXG], l[MAXG], o[MAXG][8];
#pragma unroll
    for (int h = 0; h < MAXG; ++h) {
        m[h] = -INFINITY; l[h] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) o[h][i] = 0.f;
    }
    for (int t = j0; t < j1; t += 64) {
        // request K (one key per lane) and V (8 dims per lane, KG keys per load) of this tile together
        const int jk = min(t + lane, j1 - 1);
        Raw8<KT> kraw[DH / 8], vraw[64 / KG];
#pragma unroll
        for (int e = 0; e < DH / 8; ++e) kraw[e].load(Kb + (size_t)jk * DH + e * 8);
#pragma unroll
        for (int i = 0; i < 64 / KG; ++i) vraw[i].load(Vb + (size_t)min(t + i * KG + kgrp, j1 - 1) * DH + dgrp * 8);
        const bool valid = t + lane < j1;
        float sc[MAXG];
#pragma unroll
        for (int h = 0; h < MAXG; ++h) sc[h] = 0.f;
#pragma unroll
        for (int e = 0; e < DH / 8; ++e) {
            float kv[8];
            kraw[e].get(kv);
#pragma unroll
            for (int h = 0; h < MAXG; ++h)
                if (h < G) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) sc[h] = fmaf(q_s[h][e * 8 + i], kv[i], sc[h]);
                }
        }
        // tile maximum and sum of exponentials per head; the G butterflies are interleaved so that their
        // cross-lane exchanges overlap
        float tm[MAXG], ts[MAXG], pv[MAXG];
#pragma unroll
        for (int h = 0; h < MAXG; ++h) tm[h] = (valid && h < G) ? sc[h] : -INFINITY;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            float other[MAXG];
#pragma unroll
            for (int h = 0; h < MAXG; ++h) if (h < G) other[h] = __shfl_xor(tm[h], off, 64);
#pragma unroll
            for (int h = 0; h < MAXG; ++h) if (h < G) tm[h] = fmaxf(tm[h], other[h]);
        }
#pragma unroll
        for (int h = 0; h < MAXG; ++h) {
            pv[h] = 0.f; ts[h] = 0.f;
            if (h < G) {
                tm[h] = fmaxf(m[h], tm[h]);                          // finite: lane 0 of a tile is always valid
                pv[h] = valid ? __expf(sc[h] - tm[h]) : 0.f;
                ts[h] = pv[h];
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            float other[MAXG];
#pragma unroll
            for (int h = 0; h < MAXG; ++h) if (h < G) other[h] = __shfl_xor(ts[h], off, 64);
#pragma unroll
            for (int h = 0; h < MAXG; ++h) if (h < G) ts[h] += other[h];
        }
#pragma unroll
        for (int h = 0; h < MAXG; ++h)
            if (h < G) {
                const float corr = __expf(m[h] - tm[h]);             // 0 on the first tile
                l[h] = l[h] * corr + ts[h];
#pragma unroll
                for (int i = 0; i < 8; ++i) o[h][i] *= corr;
                m[h] = tm[h];
                p_s[wave][h][lane] = pv[h];                          // read back by other lanes of this wavefront only
            }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < 64 / KG; ++i) {
            const int jj = i * KG + kgrp;
            if (t + jj < j1) {
                float vv[8];
                vraw[i].get(vv);
#pragma unroll
                for (int h = 0; h < MAXG; ++h)
                    if (h < G) {
                        const float p = p_s[wave][h][jj];
#pragma unroll
                        for (int e = 0; e < 8; ++e) o[h][e] = fmaf(p, vv[e], o[h][e]);
                    }
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
#pragma unroll
    for (int h = 0; h < MAXG; ++h)
        if (h < G) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float v = o[h][e];
#pragma unroll
                for (int off = DG; off < 64; off <<= 1) v += __shfl_xor(v, off, 64);
                o[h][e] = v;
            }
            float *pp = part + (((size_t)r * D.Hq + g * G + h) * nchunks + c) * PS;
            if (kgrp == 0) {
                *reinterpret_cast<float4 *>(pp + dgrp * 8) = make_float4(o[h][0], o[h][1], o[h][2], o[h][3]);
                *reinterpret_cast<float4 *>(pp + dgrp * 8 + 4) = make_float4(o[h][4], o[h][5], o[h][6], o[h][7]);
            }
            if (lane == 0) { pp[DH] = m[h]; pp[DH + 1] = l[h]; }
        }
}

template <typename KT, int DH>
static void launch_attention_t(hipStream_t s, const Dims &D, const float *q, const void *kc, const void *vc, Rows rows, int max_ctx,
                               float *part, size_t part_floats, float *att)
{
    // enough splits to give the chip ~1024 workgroups, at least 256 keys each, bounded by the partials buffer
    int nsplit = (1024 + rows.n * D.Hkv - 1) / (rows.n * D.Hkv);
    const int by_ctx = (max_ctx + 255) / 256;
    if (nsplit > by_ctx) nsplit = by_ctx;
    const size_t per_split = (size_t)rows.n * D.Hq * (DH + 2);
    if ((size_t)nsplit * per_split > part_floats) nsplit = (int)(part_floats / per_split);
    if (nsplit < 1) nsplit = 1;
    int chunk = (max_ctx + nsplit - 1) / nsplit;
    chunk = (chunk + 255) / 256 * 256;
    nsplit = (max_ctx + chunk - 1) / chunk;
    hipLaunchKernelGGL((attn_kernel<KT, DH>), dim3(rows.n, D.Hkv, nsplit), dim3(256), 0, s, D, q, (const KT *)kc, (const KT *)vc, rows, chunk,
                       nsplit, part, att);
    if (nsplit > 1) hipLaunchKernelGGL((attn_merge_kernel<DH>), dim3(rows.n, D.Hq), dim3(DH), 0, s, D, part, nsplit, att);
}

template <typename KT, int DH>
static bool launch_attention_wave(hipStream_t s, const Dims &D, const float *q, const void *kc, const void *vc, Rows rows, int max_ctx,
                                  float *part, size_t part_floats, float *att, void *pack, int ncb)
{
    int chunk = 64 * ((max_ctx + 64 * 32 - 1) / (64 * 32));   // at most 32 chunks per row
    const int nchunks = (max_ctx + chunk - 1) / chunk;
    if ((size_t)rows.n * D.Hq * nchunks * (DH + 4) > part_floats) return false;
    hipLaunchKernelGGL((attn_wave_kernel<KT, DH>), dim3(rows.n, D.Hkv, (nchunks + 3) / 4), dim3(256), 0, s, D, q, (const KT *)kc, (const KT *)vc,
                       rows, chunk, nchunks, part);
    launch_attn_merge(s, D, part, nchunks, rows, chunk, pack ? nullptr : att, pack, ncb);
    return true;
}

// att (fp32 [R][qw]) and/or pack (packed hi/lo activations of the output projection) receive the result.
void launch_attention(hipStream_t s, int kdt, const Dims &D, const float *q, const void *kc, const void *vc, Rows rows, int max_ctx,
                      float *part, size_t part_floats, int *cnt, float *att, void *pack, int ncb, AttnPending *defer)
{
    if (defer) { defer->nchunks = 0; defer->qn = defer->kvn = nullptr; }
    if (kdt == DT_BF16) {   // bf16 cache: V is stored transposed and attention runs on the matrix cores
        launch_attention_mfma(s, D, q, kc, vc, rows, max_ctx, part, part_floats, cnt, att, pack, ncb, defer);
        return;
    }
    bool done = false;
    if (D.dh == 64) done = kdt == DT_F32 ? launch_attention_wave<float, 64>(s, D, q, kc, vc, rows, max_ctx, part, part_floats, att, pack, ncb)
                                         : launch_attention_wave<bf16_t, 64>(s, D, q, kc, vc, rows, max_ctx, part, part_floats, att, pack, ncb);
    else done = kdt == DT_F32 ? launch_attention_wave<float, 128>(s, D, q, kc, vc, rows, max_ctx, part, part_floats, att, pack, ncb)
                              : launch_attention_wave<bf16_t, 128>(s, D, q, kc, vc, rows, max_ctx, part, part_floats, att, pack, ncb);
    if (done) return;
    // many rows (a prompt): one workgroup per row and kv head over the whole context
    if (D.dh == 64) {
        if (kdt == DT_F32) launch_attention_t<float, 64>(s, D, q, kc, vc, rows, max_ctx, part, 0, att);
        else launch_attention_t<bf16_t, 64>(s, D, q, kc, vc, rows, max_ctx, part, 0, att);
    } else {
        if (kdt == DT_F32) launch_attention_t<float, 128>(s, D, q, kc, vc, rows, max_ctx, part, 0, att);
        else launch_attention_t<bf16_t, 128>(s, D, q, kc, vc, rows, max_ctx, part, 0, att);
    }
    if (pack) launch_pack(s, att, rows.n, D.qw, pack, ncb);
}

// ------------------------------------------------------------------ attention output: x += Wo a

template <typename WT, int MB, class Stage>
__global__ __launch_bounds__(256) void residual_gemv_kernel(const WT *W, Stage in, int R, int N, int K, float *x)
{
    __shared__ __attribute__((aligned(16))) float xs[DotsCfg<MB>::LDS_FLOATS];
    const int n_raw = (blockIdx.x * 4 + (threadIdx.x >> 6)) * 2;     // two consecutive output rows per wavefront
    const int n = n_raw < N ? n_raw : 0, n2 = n_raw + 1 < N ? n_raw + 1 : n;
    const WT *const wrow[2] = {W + (size_t)n * K, W + (size_t)n2 * K};
    const int r0 = blockIdx.y * MB;
    // the old residual values are requested before the weights stream (each is owned by exactly one wavefront)
    float xa[MB], xb[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const size_t row = (size_t)min(r0 + m, R - 1) * N;
        xa[m] = x[row + n]; xb[m] = x[row + n2];
    }
    float acc[2][MB], ss[MB];
    Stage src = in;
    src.advance(r0);
    wg_dots<WT, 2, MB, false>(wrow, nullptr, src, R - r0, K, xs, acc, ss);
    if ((threadIdx.x & 63) != 0 || n_raw >= N) return;
#pragma unroll
    for (int m = 0; m < MB; ++m)
        if (r0 + m < R) {
            x[(size_t)(r0 + m) * N + n_raw] = xa[m] + acc[0][m];
            if (n_raw + 1 < N) x[(size_t)(r0 + m) * N + n_raw + 1] = xb[m] + acc[1][m];
        }
}

// One or two activation rows and weight rows of 1025 to 8192 columns (the 0.5B-class FFN output: 896 rows of 4864): the four
// wavefronts of a workgroup share two output rows and split their columns (wavefront w takes the 512-column steps
// w, w + 4, ...), so that a row is ONE round of requests instead of several dependent ones and four times as many
// wavefronts stream. Each wavefront reads the activations of its own columns straight from memory, together with the
// weights. The partial sums meet in LDS and are added in wavefront order. SPW: steps per wavefront.
// MB: activation rows (1 or 2; row m of `in` has K columns, row m of x has N).
template <typename WT, int SPW, int MB>
__global__ __launch_bounds__(256) void residual_splitk_kernel(const WT *W, const float *in, int N, int K, float *x)
{
    __shared__ float s_p[4][2][MB];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x * 2, n2 = min(n + 1, N - 1);
    const WT *const wrow[2] = {W + (size_t)n * K, W + (size_t)n2 * K};
    float xold = 0.f;   // thread t < 2 * MB owns output t % 2 of row t / 2
    if (threadIdx.x < 2 * MB) xold = x[(size_t)(threadIdx.x >> 1) * N + min(n + (int)(threadIdx.x & 1), N - 1)];
    Raw8<WT> rw[SPW][2];
    float4 xv[SPW][MB][2];
#pragma unroll
    for (int i = 0; i < SPW; ++i) {
        const int k = min((wave + 4 * i) * 512 + lane * 8, K - 8);   // requests past the end of the row are redirected and unused
        rw[i][0].load(wrow[0] + k); rw[i][1].load(wrow[1] + k);
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            xv[i][m][0] = *reinterpret_cast<const float4 *>(in + (size_t)m * K + k);
            xv[i][m][1] = *reinterpret_cast<const float4 *>(in + (size_t)m * K + k + 4);
        }
    }
    float acc[2][MB];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int m = 0; m < MB; ++m) acc[r][m] = 0.f;
#pragma unroll
    for (int i = 0; i < SPW; ++i)
        if ((wave + 4 * i) * 512 + lane * 8 < K) {
            float w[2][8];
            rw[i][0].get(w[0]); rw[i][1].get(w[1]);
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                const float xe[8] = {xv[i][m][0].x, xv[i][m][0].y, xv[i][m][0].z, xv[i][m][0].w, xv[i][m][1].x, xv[i][m][1].y, xv[i][m][1].z, xv[i][m][1].w};
#pragma unroll
                for (int r = 0; r < 2; ++r)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[r][m] = fmaf(w[r][e], xe[e], acc[r][m]);
            }
        }
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            const float t = wave_sum(acc[r][m]);
            if (lane == 0) s_p[wave][r][m] = t;
        }
    __syncthreads();
    const int t = threadIdx.x, r = t & 1, m = t >> 1;
    if (t < 2 * MB && n + r < N) x[(size_t)m * N + n + r] = xold + ((s_p[0][r][m] + s_p[1][r][m]) + (s_p[2][r][m] + s_p[3][r][m]));
}

template <typename WT, int MB>
static void launch_residual_splitk_mb(hipStream_t s, const WT *w, const float *in, int N, int K, float *x)
{
    const int spw = ((K + 511) / 512 + 3) / 4;
    const dim3 grid((N + 1) / 2), block(256);
    if (spw == 1) hipLaunchKernelGGL((residual_splitk_kernel<WT, 1, MB>), grid, block, 0, s, w, in, N, K, x);
    else if (spw == 2) hipLaunchKernelGGL((residual_splitk_kernel<WT, 2, MB>), grid, block, 0, s, w, in, N, K, x);
    else if (spw == 3) hipLaunchKernelGGL((residual_splitk_kernel<WT, 3, MB>), grid, block, 0, s, w, in, N, K, x);
    else hipLaunchKernelGGL((residual_splitk_kernel<WT, 4, MB>), grid, block, 0, s, w, in, N, K, x);
}

template <typename WT>
static bool launch_residual_splitk(hipStream_t s, const void *W, const float *in, int R, int N, int K, float *x)
{
    if (R < 1 || R > 2 || K <= 1024 || K > 8192) return false;
    if (R == 1) launch_residual_splitk_mb<WT, 1>(s, (const WT *)W, in, N, K, x);
    else launch_residual_splitk_mb<WT, 2>(s, (const WT *)W, in, N, K, x);
    return true;
}

template <typename WT, class Stage>
static void launch_residual_gemv(hipStream_t s, const void *W, const Stage &in, int R, int N, int K, float *x)
{
    const int gx = (N + 7) / 8;
    // merging attention partials while staging is a chain of dependent loads per row: two rows go to two workgroups (the
    // weights are re-read from L2) rather than one after the other in the same one (0.5B-class output projection: 6.4 -> 5.1 us per launch)
    if (R == 1 || (R == 2 && !Stage::direct))
        hipLaunchKernelGGL((residual_gemv_kernel<WT, 1, Stage>), dim3(gx, R), dim3(256), 0, s, (const WT *)W, in, R, N, K, x);
    else if (R == 2) hipLaunchKernelGGL((residual_gemv_kernel<WT, 2, Stage>), dim3(gx, 1), dim3(256), 0, s, (const WT *)W, in, R, N, K, x);
    else hipLaunchKernelGGL((residual_gemv_kernel<WT, 4, Stage>), dim3(gx, (R + 3) / 4), dim3(256), 0, s, (const WT *)W, in, R, N, K, x);
}

// x += W in for 2 to 4 plain rows of a wide bf16 matrix, with the rows kept in registers (down_rows_kernel below); false: not served
static bool launch_residual_rows(hipStream_t s, int wdt, const void *W, const float *in, int R, int N, int K, float *x);

void launch_oproj(hipStream_t s, int wdt, const Dims &D, const void *wo, const float *att, const AttnPending &pend, int R, float *x)
{
    if (pend.nchunks == 0 && launch_residual_rows(s, wdt, wo, att, R, D.d, D.qw, x)) return;
    if (pend.nchunks > 0) {
        const StageAttn st{pend, D.Hq, D.dh, 0};
        if (wdt == DT_F32) launch_residual_gemv<float>(s, wo, st, R, D.d, D.qw, x);
        else launch_residual_gemv<bf16_t>(s, wo, st, R, D.d, D.qw, x);
        return;
    }
    const StageRows st{att, (size_t)D.qw};
    if (wdt == DT_F32) { if (!launch_residual_splitk<float>(s, wo, att, R, D.d, D.qw, x)) launch_residual_gemv<float>(s, wo, st, R, D.d, D.qw, x); }
    else if (!launch_residual_splitk<bf16_t>(s, wo, att, R, D.d, D.qw, x)) launch_residual_gemv<bf16_t>(s, wo, st, R, D.d, D.qw, x);
}

// ------------------------------------------------------------------ FFN input: h = silu(Wg n) * (Wu n), n = RMSNorm(x; ln2)

template <typename WT, int MB>
__global__ __launch_bounds__(256) void gateup_kernel(Dims D, const WT *wg, const WT *wu, const WT *gain, const float *x, int R, float *h)
{
    __shared__ __attribute__((aligned(16))) float xs[DotsCfg<MB>::LDS_FLOATS];
    const int f_raw = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int f = f_raw < D.F ? f_raw : D.F - 1;
    const WT *const wrow[2] = {wg + (size_t)f * D.d, wu + (size_t)f * D.d};
    const int r0 = blockIdx.y * MB;
    float acc[2][MB], ss[MB];
    wg_dots<WT, 2, MB, true>(wrow, gain, StageRows{x + (size_t)r0 * D.d, (size_t)D.d}, R - r0, D.d, xs, acc, ss);
    if ((threadIdx.x & 63) != 0 || f_raw >= D.F) return;
#pragma unroll
    for (int m = 0; m < MB; ++m)
        if (r0 + m < R) {
            const float rstd = 1.0f / sqrtf(ss[m] / (float)D.d + D.eps);
            const float gt = acc[0][m] * rstd, up = acc[1][m] * rstd;
            h[(size_t)(r0 + m) * D.F + f] = gt / (1.0f + expf(-gt)) * up;
        }
}

// ------------------------------------------------------------------ wide models, up to 4 rows: FFN with the activations in registers
// The kernels above stage the activation rows in LDS once per workgroup of 4 output features; with thousands of such
// workgroups and rows of 3584 to 18944 columns the staging traffic and the LDS reads per weight (32 bytes per row and
// 16-byte weight load) cost as much as the weight stream itself from two rows on. Here a launch has ONE workgroup per compute
// unit, whose wavefronts keep their share of the activation columns in registers for the whole launch and walk the output
// features; per feature a wavefront only streams its share of the weight row (several features in flight) and adds across its
// lanes. Reductions have a fixed shape (lanes: a fixed tree; wavefronts: in index order), so results are the same from run to run.

// Sums each of v[0..NV) over the 64 lanes. Halving steps first (lanes whose bit `mask` is set keep the upper half of the values
// and hand the lower half to their partner), so NV values cost NV - 1 + log2(64 / NV) exchanges instead of 6 NV. Returns the
// total of value `idx`, which differs by lane: idx = the top log2(NV) bits of the lane index.
template <int N, int NV>
__device__ __forceinline__ void lanes_halve(float (&v)[NV], int lane, int mask, int &idx)
{
    const bool up = (lane & mask) != 0;
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
        const float keep = up ? v[N / 2 + i] : v[i], send = up ? v[i] : v[N / 2 + i];
        v[i] = keep + __shfl_xor(send, mask, 64);
    }
    idx = 2 * idx + (up ? 1 : 0);
}

template <int NV>
__device__ __forceinline__ float lanes_sum_scatter(float (&v)[NV], int lane, int &idx)
{
    static_assert(NV == 1 || NV == 2 || NV == 4 || NV == 8, "power of two");
    int mask = 32;
    idx = 0;
    if constexpr (NV == 8) { lanes_halve<8>(v, lane, 32, idx); lanes_halve<4>(v, lane, 16, idx); lanes_halve<2>(v, lane, 8, idx); mask = 4; }
    else if constexpr (NV == 4) { lanes_halve<4>(v, lane, 32, idx); lanes_halve<2>(v, lane, 16, idx); mask = 8; }
    else if constexpr (NV == 2) { lanes_halve<2>(v, lane, 32, idx); mask = 16; }
    float r = v[0];
    for (; mask > 0; mask >>= 1) r += __shfl_xor(r, mask, 64);
    return r;
}

constexpr int ROWS_WAVES = 8;        // wavefronts per workgroup
constexpr int GU_MAX_FEATURES = 64;  // output features a pair of wavefronts may own (LDS for their partial sums)

// h = silu(Wg n) * (Wu n), n = RMSNorm(x; gain), for R <= MB rows. The 8 wavefronts form 4 pairs; the two wavefronts of a pair
// split the columns (512-column chunks: the first NCH to one, the rest to the other) and pair p of workgroup b owns the
// features 4 b + p, + 4 gridDim.x, ... . K <= 2 * NCH * 512, K % 8 == 0.
template <int MB, int NCH>
__global__ __launch_bounds__(64 * ROWS_WAVES) void gateup_rows_kernel(Dims D, const bf16_t *wg, const bf16_t *wu, const bf16_t *gain, const float *x, int R,
                                                                        float *h)
{
    constexpr int NV = 2 * MB;
    __shared__ float s_ss[ROWS_WAVES][MB];
    __shared__ float s_part[ROWS_WAVES][GU_MAX_FEATURES][NV];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, pair = wave >> 1, half = wave & 1;
    const int K = D.d, F = D.F;
    // this wavefront's columns: chunk c covers 512 c + 8 lane .. + 7
    int kcol[NCH];
    bool klive[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int k = (half * NCH + c) * 512 + lane * 8;
        klive[c] = k < K;
        kcol[c] = klive[c] ? k : K - 8;   // a column group past the row: its activations are zero, its weight requests repeat the row's last 16 bytes
    }
    const int stride = gridDim.x * 4, f0 = blockIdx.x * 4 + pair;
    const int nf = f0 < F ? (F - f0 + stride - 1) / stride : 0;   // features of this pair (<= GU_MAX_FEATURES: the launcher sees to it)
    uint4 w[3][2][NCH];
    auto request = [&](int i, uint4 (&ws)[2][NCH]) {   // unconditional: past the last feature the last one is requested again
        const size_t f = (size_t)(f0 + min(i, nf - 1) * stride);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            ws[0][c] = *reinterpret_cast<const uint4 *>(wg + f * K + kcol[c]);
            ws[1][c] = *reinterpret_cast<const uint4 *>(wu + f * K + kcol[c]);
        }
    };
    // the first weight rows are requested before the activations: their addresses do not depend on them
    if (nf > 0) {
        request(0, w[0]);
        request(1, w[1]);
    }
    float xa[NCH][8][MB];
    float ss[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) ss[m] = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        float g[8];
        load8(gain + kcol[c], g);
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = 0.f;
            if (klive[c] && m < R) load8(x + (size_t)m * K + kcol[c], v);
#pragma unroll
            for (int e = 0; e < 8; ++e) { ss[m] = fmaf(v[e], v[e], ss[m]); xa[c][e][m] = v[e] * g[e]; }
        }
    }
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const float t = wave_sum(ss[m]);
        if (lane == 0) s_ss[wave][m] = t;
    }
    auto consume = [&](int i, const uint4 (&ws)[2][NCH]) {
        float acc[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) acc[j] = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const uint32_t u[4] = {ws[r][c].x, ws[r][c].y, ws[r][c].z, ws[r][c].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float wv = __uint_as_float((e & 1) ? (u[e >> 1] & 0xffff0000u) : (u[e >> 1] << 16));
#pragma unroll
                    for (int m = 0; m < MB; ++m) acc[r * MB + m] = fmaf(wv, xa[c][e][m], acc[r * MB + m]);
                }
            }
        int idx;
        const float t = lanes_sum_scatter<NV>(acc, lane, idx);
        if ((lane & (64 / NV - 1)) == 0) s_part[wave][i][idx] = t;
    };
    if (nf > 0) {
        for (int i = 0; i < nf; i += 3) {   // two features are in flight while one is multiplied
            request(i + 2, w[2]);
            consume(i, w[0]);
            if (i + 1 >= nf) break;
            request(i + 3, w[0]);
            consume(i + 1, w[1]);
            if (i + 2 >= nf) break;
            request(i + 4, w[1]);
            consume(i + 2, w[2]);
        }
    }
    __syncthreads();
    // (pair, feature, row): the halves are added in index order, then 1/rms, SiLU and the product
    for (int t = threadIdx.x; t < 4 * GU_MAX_FEATURES * MB; t += blockDim.x) {
        const int m = t % MB, i = (t / MB) % GU_MAX_FEATURES, p = t / (MB * GU_MAX_FEATURES);
        const int f = blockIdx.x * 4 + p + i * stride;
        if (m >= R || f >= F) continue;
        const float tot = s_ss[0][m] + s_ss[1][m];   // every pair saw the whole row: the two halves of pair 0
        const float rstd = 1.0f / sqrtf(tot / (float)K + D.eps);
        const float gt = (s_part[2 * p][i][m] + s_part[2 * p + 1][i][m]) * rstd, up = (s_part[2 * p][i][MB + m] + s_part[2 * p + 1][i][MB + m]) * rstd;
        h[(size_t)m * F + f] = gt / (1.0f + expf(-gt)) * up;
    }
}

constexpr int QKV_MAX_PAIRS = 16;   // rotary pairs a group of four wavefronts may own

// [q|k|v] = W n + b, n = RMSNorm(x; gain), rotation of q and k at the row's position, k and v appended to the cache, for R <= MB
// rows. As in the kernel above, with the two output rows (j, j + dh/2) of a head that the rotation pairs up in place of (gate, up),
// and four wavefronts per pair of rows (two groups per workgroup; wavefront g of a group owns the 512-column chunks g NCH .. g NCH + NCH - 1):
// there are fewer output rows here, and a finer share per wavefront spreads them more evenly. K <= 4 * NCH * 512, K % 8 == 0.
template <typename KT, int MB, int NCH>
__global__ __launch_bounds__(64 * ROWS_WAVES) void qkv_rows_kernel(Dims D, LayerW lw, const float *x, Rows rows, const float2 *rope, float *q, KT *kc, KT *vc)
{
    constexpr int NV = 2 * MB;
    __shared__ float s_ss[ROWS_WAVES][MB];
    __shared__ float s_part[ROWS_WAVES][QKV_MAX_PAIRS][NV];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, group = wave >> 2, part = wave & 3;
    const int K = D.d, R = rows.n, half = D.dh / 2, npairs = (D.Hq + 2 * D.Hkv) * half;
    int kcol[NCH];
    bool klive[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int k = (part * NCH + c) * 512 + lane * 8;
        klive[c] = k < K;
        kcol[c] = klive[c] ? k : K - 8;
    }
    const int stride = gridDim.x * 2, p0 = blockIdx.x * 2 + group;
    const int nf = p0 < npairs ? (npairs - p0 + stride - 1) / stride : 0;   // <= QKV_MAX_PAIRS: the launcher sees to it
    // the two weight rows of pair index pi
    auto pair_rows = [&](int pi, const bf16_t *&r1, const bf16_t *&r2) {
        const int hh = pi / half, j = pi % half;
        const bf16_t *W = hh < D.Hq ? (const bf16_t *)lw.wq : hh < D.Hq + D.Hkv ? (const bf16_t *)lw.wk : (const bf16_t *)lw.wv;
        const int head = hh < D.Hq ? hh : hh < D.Hq + D.Hkv ? hh - D.Hq : hh - D.Hq - D.Hkv;
        r1 = W + (size_t)(head * D.dh + j) * K;
        r2 = r1 + (size_t)half * K;
    };
    uint4 w[3][2][NCH];
    auto request = [&](int i, uint4 (&ws)[2][NCH]) {   // unconditional: past the last pair the last one is requested again
        const bf16_t *r1, *r2;
        pair_rows(p0 + min(i, nf - 1) * stride, r1, r2);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            ws[0][c] = *reinterpret_cast<const uint4 *>(r1 + kcol[c]);
            ws[1][c] = *reinterpret_cast<const uint4 *>(r2 + kcol[c]);
        }
    };
    if (nf > 0) {   // before the activations: the addresses do not depend on them
        request(0, w[0]);
        request(1, w[1]);
    }
    float xa[NCH][8][MB];
    float ss[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) ss[m] = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        float g[8];
        load8((const bf16_t *)lw.ln1 + kcol[c], g);
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = 0.f;
            if (klive[c] && m < R) load8(x + (size_t)m * K + kcol[c], v);
#pragma unroll
            for (int e = 0; e < 8; ++e) { ss[m] = fmaf(v[e], v[e], ss[m]); xa[c][e][m] = v[e] * g[e]; }
        }
    }
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const float t = wave_sum(ss[m]);
        if (lane == 0) s_ss[wave][m] = t;
    }
    auto consume = [&](int i, const uint4 (&ws)[2][NCH]) {
        float acc[NV];
#pragma unroll
        for (int j = 0; j < NV; ++j) acc[j] = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const uint32_t u[4] = {ws[r][c].x, ws[r][c].y, ws[r][c].z, ws[r][c].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float wv = __uint_as_float((e & 1) ? (u[e >> 1] & 0xffff0000u) : (u[e >> 1] << 16));
#pragma unroll
                    for (int m = 0; m < MB; ++m) acc[r * MB + m] = fmaf(wv, xa[c][e][m], acc[r * MB + m]);
                }
            }
        int idx;
        const float t = lanes_sum_scatter<NV>(acc, lane, idx);
        if ((lane & (64 / NV - 1)) == 0) s_part[wave][i][idx] = t;
    };
    for (int i = 0; i < nf; i += 3) {   // two pairs are in flight while one is multiplied
        request(i + 2, w[2]);
        consume(i, w[0]);
        if (i + 1 >= nf) break;
        request(i + 3, w[0]);
        consume(i + 1, w[1]);
        if (i + 2 >= nf) break;
        request(i + 4, w[1]);
        consume(i + 2, w[2]);
    }
    __syncthreads();
    // (group, pair, row): the four column shares are added in index order, then 1/rms, bias, rotation, and the stores
    for (int t = threadIdx.x; t < 2 * QKV_MAX_PAIRS * MB; t += blockDim.x) {
        const int m = t % MB, i = (t / MB) % QKV_MAX_PAIRS, g = t / (MB * QKV_MAX_PAIRS);
        const int pi = blockIdx.x * 2 + g + i * stride;
        if (m >= R || pi >= npairs) continue;
        const int hh = pi / half, j = pi % half;
        const float tot = (s_ss[0][m] + s_ss[1][m]) + (s_ss[2][m] + s_ss[3][m]);   // the four shares of group 0: the whole row
        const float rstd = 1.0f / sqrtf(tot / (float)K + D.eps);
        const float a1 = (s_part[4 * g][i][m] + s_part[4 * g + 1][i][m]) + (s_part[4 * g + 2][i][m] + s_part[4 * g + 3][i][m]);
        const float a2 = (s_part[4 * g][i][MB + m] + s_part[4 * g + 1][i][MB + m]) + (s_part[4 * g + 2][i][MB + m] + s_part[4 * g + 3][i][MB + m]);
        const bf16_t *bias = hh < D.Hq ? (const bf16_t *)lw.bq : hh < D.Hq + D.Hkv ? (const bf16_t *)lw.bk : (const bf16_t *)lw.bv;
        const int head = hh < D.Hq ? hh : hh < D.Hq + D.Hkv ? hh - D.Hq : hh - D.Hq - D.Hkv;
        const int n1 = head * D.dh + j, n2 = n1 + half;
        float y1 = a1 * rstd + (bias ? widen(bias, n1) : 0.f), y2 = a2 * rstd + (bias ? widen(bias, n2) : 0.f);
        const int pos = rows.pos[m];
        if (hh < D.Hq + D.Hkv) {
            const float2 cs = rope[(size_t)pos * half + j];
            const float o1 = y1 * cs.x - y2 * cs.y, o2 = y2 * cs.x + y1 * cs.y;
            y1 = o1; y2 = o2;
        }
        if (hh < D.Hq) {
            q[(size_t)m * D.qw + n1] = y1;
            q[(size_t)m * D.qw + n2] = y2;
        } else {
            const KvPlace place = kv_place(D, rows.slot[m], pos);
            if (hh < D.Hq + D.Hkv) {
                KT *dst = kc + k_offset(D, place.unit, head, place.pos, 0);
                store_kv(dst + j, y1);
                store_kv(dst + j + half, y2);
            } else {
                store_kv(vc + v_offset(D, place.unit, head, place.pos, j), y1);
                store_kv(vc + v_offset(D, place.unit, head, place.pos, j + half), y2);
            }
        }
    }
}

template <typename KT, int MB>
static void launch_qkv_rows_mb(hipStream_t s, const Dims &D, const LayerW &w, const float *x, Rows rows, const float2 *rope, float *q, void *kc, void *vc)
{
    const int npairs = (D.Hq + 2 * D.Hkv) * (D.dh / 2), grid = std::min(256, (npairs + 1) / 2);
    const int chunks = (D.d + 511) / 512;
    if (chunks <= 4) hipLaunchKernelGGL((qkv_rows_kernel<KT, MB, 1>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, D, w, x, rows, rope, q, (KT *)kc, (KT *)vc);
    else hipLaunchKernelGGL((qkv_rows_kernel<KT, MB, 2>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, D, w, x, rows, rope, q, (KT *)kc, (KT *)vc);
}

static bool launch_qkv_rows(hipStream_t s, int wdt, int kdt, const Dims &D, const LayerW &w, const float *x, Rows rows, const float2 *rope, float *q,
                            void *kc, void *vc)
{
    const int npairs = (D.Hq + 2 * D.Hkv) * (D.dh / 2);
    if (wdt != DT_BF16 || rows.n < 1 || rows.n > 4 || rows.live || D.d <= 1024 || D.d > 4096 || D.d % 8 || npairs > QKV_MAX_PAIRS * 512) return false;
    auto go = [&](auto kt) {
        using KT = decltype(kt);
        if (rows.n == 1) launch_qkv_rows_mb<KT, 1>(s, D, w, x, rows, rope, q, kc, vc);
        else if (rows.n == 2) launch_qkv_rows_mb<KT, 2>(s, D, w, x, rows, rope, q, kc, vc);
        else launch_qkv_rows_mb<KT, 4>(s, D, w, x, rows, rope, q, kc, vc);
    };
    if (kdt == DT_F32) go(float{}); else go(bf16_t{});
    return true;
}

constexpr int DOWN_MAX_FEATURES = 32;   // output features a workgroup may own

// x[m] += Wd h[m] for R <= MB rows. The 8 wavefronts split the columns (512-column chunk c goes to wavefront c % 8, NCH chunks
// each at most) and the workgroup owns the features blockIdx.x, + gridDim.x, ... . K <= 8 * NCH * 512, K % 8 == 0.
template <int MB, int NCH>
__global__ __launch_bounds__(64 * ROWS_WAVES) void down_rows_kernel(const bf16_t *wd, const float *hin, int R, int N, int K, float *x)
{
    constexpr int DEPTH = 3;   // two features in flight while one is multiplied (twelve, for wavefronts that own one chunk, measured slower)
    __shared__ float s_part[ROWS_WAVES][DOWN_MAX_FEATURES][MB];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    int kcol[NCH];
    bool klive[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
        const int k = (c * ROWS_WAVES + wave) * 512 + lane * 8;
        klive[c] = k < K;
        kcol[c] = klive[c] ? k : K - 8;
    }
    const int stride = gridDim.x, f0 = blockIdx.x;
    const int nf = f0 < N ? (N - f0 + stride - 1) / stride : 0;   // <= DOWN_MAX_FEATURES: the launcher sees to it
    uint4 w[DEPTH][NCH];
    // unconditional, so that the number of requests in flight is known at compile time and a feature can be waited for alone (requests
    // under a condition measured 6.1-7.1 -> 7.5 us on the 7B-class output projection); past the last feature the last one is requested again
    auto request = [&](int i, uint4 (&ws)[NCH]) {
        const size_t f = (size_t)(f0 + min(i, nf - 1) * stride);
#pragma unroll
        for (int c = 0; c < NCH; ++c) ws[c] = *reinterpret_cast<const uint4 *>(wd + f * K + kcol[c]);
    };
    if (nf > 0) {   // before the activations: the addresses do not depend on them
#pragma unroll
        for (int d = 0; d < DEPTH - 1; ++d) request(d, w[d]);
    }
    float xa[NCH][8][MB];
#pragma unroll
    for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int m = 0; m < MB; ++m) {
            float v[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = 0.f;
            if (klive[c] && m < R) load8(hin + (size_t)m * K + kcol[c], v);
#pragma unroll
            for (int e = 0; e < 8; ++e) xa[c][e][m] = v[e];
        }
    auto consume = [&](int i, const uint4 (&ws)[NCH]) {
        float acc[MB];
#pragma unroll
        for (int m = 0; m < MB; ++m) acc[m] = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const uint32_t u[4] = {ws[c].x, ws[c].y, ws[c].z, ws[c].w};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float wv = __uint_as_float((e & 1) ? (u[e >> 1] & 0xffff0000u) : (u[e >> 1] << 16));
#pragma unroll
                for (int m = 0; m < MB; ++m) acc[m] = fmaf(wv, xa[c][e][m], acc[m]);
            }
        }
        int idx;
        const float t = lanes_sum_scatter<MB>(acc, lane, idx);
        if ((lane & (64 / MB - 1)) == 0) s_part[wave][i][idx] = t;
    };
    for (int i = 0; i < nf; i += DEPTH) {   // DEPTH - 1 features are in flight while one is multiplied
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (i + d >= nf) break;
            request(i + d + DEPTH - 1, w[(d + DEPTH - 1) % DEPTH]);
            consume(i + d, w[d]);
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < DOWN_MAX_FEATURES * MB; t += blockDim.x) {
        const int m = t % MB, i = t / MB, f = f0 + i * stride;
        if (m >= R || i >= nf) continue;
        float tot = 0.f;
#pragma unroll
        for (int wv = 0; wv < ROWS_WAVES; ++wv) tot += s_part[wv][i][m];   // wavefronts in index order
        x[(size_t)m * N + f] += tot;
    }
}

// The two kernels above serve bf16 models wider than 1024 columns at 2 to 4 rows, within the column counts their register
// arrays are built for (7B-class FFN, kernel time at 1 / 2 / 4 rows: gate/up 44.0 / 44.8 / 50.3 us against 43.4 / 48.4 / 69 us for the
// kernel that stages the rows in LDS, down 22.9 / 23.6 / 26.9 against 23.3 / 28.3 / 41 us: one row stays where it was).
bool ffn_rows_supported(int wdt, const Dims &D, int R)
{
    return wdt == DT_BF16 && R >= 2 && R <= 4 && D.d > 1024 && D.d <= 4096 && D.d % 8 == 0 && D.F % 8 == 0 && D.F <= 5 * ROWS_WAVES * 512 &&
           D.F <= GU_MAX_FEATURES * 1024 && D.d <= DOWN_MAX_FEATURES * 256 && D.qw > 1024 && D.qw % 8 == 0 && D.qw <= 5 * ROWS_WAVES * 512;   // (the output projection too)
}

template <int MB>
static void launch_gateup_rows(hipStream_t s, const Dims &D, const LayerW &w, const float *x, int R, float *h)
{
    const int grid = std::min(256, (D.F + 3) / 4);   // one workgroup per compute unit; every pair then owns at most F / 1024 features (rounded up)
    const bf16_t *wg = (const bf16_t *)w.wg, *wu = (const bf16_t *)w.wu, *ln = (const bf16_t *)w.ln2;
    const int chunks = (D.d + 511) / 512;
    if (chunks <= 4) hipLaunchKernelGGL((gateup_rows_kernel<MB, 2>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, D, wg, wu, ln, x, R, h);
    else if (chunks <= 6) hipLaunchKernelGGL((gateup_rows_kernel<MB, 3>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, D, wg, wu, ln, x, R, h);
    else hipLaunchKernelGGL((gateup_rows_kernel<MB, 4>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, D, wg, wu, ln, x, R, h);
}

template <int MB>
static void launch_residual_rows_mb(hipStream_t s, const void *W, const float *in, int R, int N, int K, float *x)
{
    const int grid = std::min(256, N);
    const int per = ((K + 511) / 512 + ROWS_WAVES - 1) / ROWS_WAVES;   // chunks per wavefront
    const bf16_t *w = (const bf16_t *)W;
    if (per <= 1) hipLaunchKernelGGL((down_rows_kernel<MB, 1>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, w, in, R, N, K, x);
    else if (per <= 2) hipLaunchKernelGGL((down_rows_kernel<MB, 2>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, w, in, R, N, K, x);
    else if (per <= 3) hipLaunchKernelGGL((down_rows_kernel<MB, 3>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, w, in, R, N, K, x);
    else if (per <= 4) hipLaunchKernelGGL((down_rows_kernel<MB, 4>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, w, in, R, N, K, x);
    else hipLaunchKernelGGL((down_rows_kernel<MB, 5>), dim3(grid), dim3(64 * ROWS_WAVES), 0, s, w, in, R, N, K, x);
}

static bool launch_residual_rows(hipStream_t s, int wdt, const void *W, const float *in, int R, int N, int K, float *x)
{
    if (wdt != DT_BF16 || R < 2 || R > 4 || K <= 1024 || K % 8 || K > 5 * ROWS_WAVES * 512 || N > DOWN_MAX_FEATURES * 256) return false;
    if (R == 2) launch_residual_rows_mb<2>(s, W, in, R, N, K, x);
    else launch_residual_rows_mb<4>(s, W, in, R, N, K, x);
    return true;
}

void launch_down(hipStream_t s, int wdt, const Dims &D, const void *wd, const float *h, int R, float *x)
{
    if (ffn_rows_supported(wdt, D, R) && launch_residual_rows(s, wdt, wd, h, R, D.d, D.F, x)) return;
    const StageRows st{h, (size_t)D.F};
    if (wdt == DT_F32) { if (!launch_residual_splitk<float>(s, wd, h, R, D.d, D.F, x)) launch_residual_gemv<float>(s, wd, st, R, D.d, D.F, x); }
    else if (!launch_residual_splitk<bf16_t>(s, wd, h, R, D.d, D.F, x)) launch_residual_gemv<bf16_t>(s, wd, st, R, D.d, D.F, x);
}

template <typename WT>
static void launch_gateup_t(hipStream_t s, const Dims &D, const LayerW &w, const float *x, int R, float *h)
{
    const int gx = (D.F + 3) / 4;
    const WT *wg = (const WT *)w.wg, *wu = (const WT *)w.wu, *ln = (const WT *)w.ln2;
    if (R == 1) hipLaunchKernelGGL((gateup_kernel<WT, 1>), dim3(gx, 1), dim3(256), 0, s, D, wg, wu, ln, x, R, h);
    else if (R == 2) hipLaunchKernelGGL((gateup_kernel<WT, 2>), dim3(gx, 1), dim3(256), 0, s, D, wg, wu, ln, x, R, h);
    else hipLaunchKernelGGL((gateup_kernel<WT, 4>), dim3(gx, (R + 3) / 4), dim3(256), 0, s, D, wg, wu, ln, x, R, h);
}

void launch_gateup(hipStream_t s, int wdt, const Dims &D, const LayerW &w, const float *x, int R, float *h)
{
    if (ffn_rows_supported(wdt, D, R)) {
        if (R == 1) launch_gateup_rows<1>(s, D, w, x, R, h);
        else if (R == 2) launch_gateup_rows<2>(s, D, w, x, R, h);
        else launch_gateup_rows<4>(s, D, w, x, R, h);
        return;
    }
    if (wdt == DT_F32) launch_gateup_t<float>(s, D, w, x, R, h);
    else launch_gateup_t<bf16_t>(s, D, w, x, R, h);
}

// ------------------------------------------------------------------ cache import: [layer][kv_head][len][dh] -> the slot's cache

template <typename KT>
__global__ void load_kv_kernel(Dims D, int slot, int len, const KT *k, const KT *v, KT *kc, KT *vc)
{
    const size_t per_layer_src = (size_t)D.Hkv * len * D.dh;
    const size_t total = (size_t)D.L * per_layer_src;
    const size_t layer_stride = (size_t)D.units * D.Hkv * kv_unit_len(D) * D.dh;
    const size_t v_layer_stride = (size_t)D.units * D.Hkv * D.dh * (kv_unit_vts(D) ? kv_unit_vts(D) : kv_unit_len(D));
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const size_t l = i / per_layer_src, rem = i % per_layer_src;
        const size_t g = rem / ((size_t)len * D.dh), pe = rem % ((size_t)len * D.dh);
        const KvPlace at = kv_place(D, slot, (int)(pe / D.dh));
        kc[l * layer_stride + k_offset(D, at.unit, (int)g, at.pos, (int)(pe % D.dh))] = k[i];
        vc[l * v_layer_stride + v_offset(D, at.unit, (int)g, at.pos, (int)(pe % D.dh))] = v[i];
    }
}

void launch_load_kv(hipStream_t s, int kdt, const Dims &D, int slot, int len, const void *k, const void *v, void *kc, void *vc)
{
    const size_t total = (size_t)D.L * D.Hkv * len * D.dh;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (kdt == DT_F32) hipLaunchKernelGGL(load_kv_kernel<float>, dim3(blocks), dim3(256), 0, s, D, slot, len, (const float *)k, (const float *)v, (float *)kc, (float *)vc);
    else hipLaunchKernelGGL(load_kv_kernel<bf16_t>, dim3(blocks), dim3(256), 0, s, D, slot, len, (const bf16_t *)k, (const bf16_t *)v, (bf16_t *)kc, (bf16_t *)vc);
}

}  // namespace tr
