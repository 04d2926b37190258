// Routing tail for gfx950: final RMSNorm -> LM head over the whole vocabulary -> softmax confidence and greedy
// argmax -> MLP router on the exposed last-layer hidden state -> route flag -> per-slot counters.
//
// The rule (arxiv 2504.07878, Section 3.1): a token is routed to the large model when the router's score,
// computed by an MLP classifier on the last-layer hidden state of the small model, falls below the threshold;
// the small_only mode disables routing. The hidden state is an output of the model (Section 3.3, Figure 4).
//
// The logits are never written to memory unless a debug buffer is given: every workgroup streams one slice
// of the head matrix, keeps a running (max, lowest argmax, sum of exponentials) per row, and the slices'
// triples are merged in a fixed order, so results are bit-identical from run to run.
#include "tr_internal.h"
#include <algorithm>

namespace tr {

__device__ __forceinline__ float t_bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ float t_widen(const float *p, size_t i) { return p[i]; }
__device__ __forceinline__ float t_widen(const bf16_t *p, size_t i) { return t_bf16_to_f32(p[i]); }

__device__ __forceinline__ void t_load8(const float *p, float (&w)[8])
{
    float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w;
}

__device__ __forceinline__ void t_load8(const bf16_t *p, float (&w)[8])
{
    uint4 v = *reinterpret_cast<const uint4 *>(p);
    w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xffff0000u);
    w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xffff0000u);
    w[4] = __uint_as_float(v.z << 16); w[5] = __uint_as_float(v.z & 0xffff0000u);
    w[6] = __uint_as_float(v.w << 16); w[7] = __uint_as_float(v.w & 0xffff0000u);
}

__device__ __forceinline__ float t_wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

constexpr int SLICE_ROWS = 128;  // vocabulary rows per workgroup (32 per wavefront)
int tail_slice_rows() { return SLICE_ROWS; }

// ------------------------------------------------------------------ final RMSNorm; exposes the hidden state

template <typename WT>
__global__ __launch_bounds__(256) void tail_norm_kernel(int d, float eps, const WT *gain, const float *x, const int *gather, float *hn,
                                                        float *hidden, int hidden_tap)
{
    __shared__ float red[4];
    const int i = blockIdx.x;
    const float *xr = x + (size_t)(gather ? gather[i] : i) * d;
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) ss = fmaf(xr[j], xr[j], ss);
    ss = t_wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float rstd = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
    for (int j = threadIdx.x; j < d; j += 256) {
        const float v = xr[j] * rstd * t_widen(gain, j);
        hn[(size_t)i * d + j] = v;
        if (hidden) hidden[(size_t)i * d + j] = hidden_tap == 0 ? v : xr[j];
    }
}

// ------------------------------------------------------------------ LM head slice: running softmax statistics

// part[slice][row] = {max, argmax (as int bits), sum exp(z - max), unused}
template <typename WT, int MB>
__global__ __launch_bounds__(256) void lmhead_kernel(const WT *head, int V, int d, const float *hn, int n, float4 *part, float *logits)
{
    __shared__ float4 wpart[4][MB];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int r0 = blockIdx.y * MB;
    const float *xrow[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) xrow[m] = hn + (size_t)(r0 + m < n ? r0 + m : r0) * d;
    float mx[MB], sum[MB];
    int idx[MB];
#pragma unroll
    for (int m = 0; m < MB; ++m) { mx[m] = -INFINITY; sum[m] = 0.f; idx[m] = 0x7fffffff; }

    const int v_begin = blockIdx.x * SLICE_ROWS + wave * (SLICE_ROWS / 4);
    for (int v0 = v_begin; v0 < v_begin + SLICE_ROWS / 4 && v0 < V; v0 += 4) {
        float acc[4][MB];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int m = 0; m < MB; ++m) acc[r][m] = 0.f;
        for (int k = lane * 8; k < d; k += 512) {
            float w[4][8];
#pragma unroll
            for (int r = 0; r < 4; ++r) t_load8(head + (size_t)(v0 + r < V ? v0 + r : v0) * d + k, w[r]);
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                float xv[8];
                t_load8(xrow[m] + k, xv);
#pragma unroll
                for (int i = 0; i < 8; ++i)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[r][m] = fmaf(w[r][i], xv[i], acc[r][m]);
            }
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int v = v0 + r;
            if (v < V) {
#pragma unroll
                for (int m = 0; m < MB; ++m) {
                    const float z = t_wave_sum(acc[r][m]);
                    if (logits && lane == 0 && r0 + m < n) logits[(size_t)(r0 + m) * V + v] = z;
                    if (z > mx[m]) {   // strict: the lowest index wins ties
                        sum[m] = sum[m] * expf(mx[m] - z) + 1.0f;
                        mx[m] = z; idx[m] = v;
                    } else {
                        sum[m] += expf(z - mx[m]);
                    }
                }
            }
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int m = 0; m < MB; ++m) wpart[wave][m] = make_float4(mx[m], __int_as_float(idx[m]), sum[m], 0.f);
    }
    __syncthreads();
    if (threadIdx.x < MB && r0 + threadIdx.x < n) {
        const int m = threadIdx.x;
        float M = -INFINITY; int I = 0x7fffffff;
        for (int w = 0; w < 4; ++w) {      // wavefronts hold increasing vocabulary ranges
            const float4 p = wpart[w][m];
            if (p.x > M) { M = p.x; I = __float_as_int(p.y); }
        }
        float S = 0.f;
        for (int w = 0; w < 4; ++w) {
            const float4 p = wpart[w][m];
            if (p.x > -INFINITY) S += p.z * expf(p.x - M);
        }
        part[(size_t)blockIdx.x * n + r0 + m] = make_float4(M, __int_as_float(I), S, 0.f);
    }
}

// ------------------------------------------------------------------ merge the slices, run the router, set the flag

// 16 wavefronts per workgroup; gridDim.y workgroups per batch row. Reductions are wavefront shuffles plus one
// fixed-order pass over the 16 wavefront results, so the outcome does not depend on timing. The kernel is a chain of
// dependent steps on few compute units, so its time is memory round trips plus the issue time of the router's
// first layer (rh x d multiply-adds and as many widenings on ONE compute unit take ~10 us at 256 x 896). Hence: the
// slice triples are read once and kept in registers for both merge passes; the router's hidden units are split over
// the row's workgroups (part 0 also merges the slices), whose partial pre-activations meet in memory: each part
// leaves its sum with a device-coherent store and counts in, and the last one to arrive adds them in part order
// (bit-identical whoever is last), applies the sigmoid and the threshold, and leaves the counter at zero.
constexpr int TF_WAVES = 16;
constexpr int TF_THREADS = 64 * TF_WAVES;
constexpr int RQ = 4;   // hidden units of the router per wavefront and batch of requests (8 requests in flight per lane)

template <typename WT> struct TRaw8;
template <> struct TRaw8<float> {
    float4 a, b;
    __device__ __forceinline__ void load(const float *p) { a = *reinterpret_cast<const float4 *>(p); b = *reinterpret_cast<const float4 *>(p + 4); }
    __device__ __forceinline__ void widen(float (&w)[8]) const { w[0] = a.x; w[1] = a.y; w[2] = a.z; w[3] = a.w; w[4] = b.x; w[5] = b.y; w[6] = b.z; w[7] = b.w; }
};
template <> struct TRaw8<bf16_t> {
    uint4 v;
    __device__ __forceinline__ void load(const bf16_t *p) { v = *reinterpret_cast<const uint4 *>(p); }
    __device__ __forceinline__ void widen(float (&w)[8]) const
    {
        w[0] = __uint_as_float(v.x << 16); w[1] = __uint_as_float(v.x & 0xffff0000u);
        w[2] = __uint_as_float(v.y << 16); w[3] = __uint_as_float(v.y & 0xffff0000u);
        w[4] = __uint_as_float(v.z << 16); w[5] = __uint_as_float(v.z & 0xffff0000u);
        w[6] = __uint_as_float(v.w << 16); w[7] = __uint_as_float(v.w & 0xffff0000u);
    }
};

template <typename WT>
__global__ __launch_bounds__(TF_THREADS) void tail_final_kernel(int d, int rh, TailArgs t)
{
    __shared__ float s_wm[TF_WAVES];
    __shared__ int s_wi[TF_WAVES];
    __shared__ float s_ws[2][TF_WAVES];
    __shared__ float s_h[1024];
    __shared__ __attribute__((aligned(16))) float s_u[4096];
    const int i = blockIdx.x, part_id = blockIdx.y, nparts = gridDim.y, tid = threadIdx.x, lane = tid & 63, n = t.n;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const float4 *part = reinterpret_cast<const float4 *>(t.part);
    const bool mlp = t.policy == 0 && rh > 0, linear = t.policy == 2;   // several parts only with the MLP
    const WT *w1 = (const WT *)t.r_w1;
    const int per = (rh + nparts - 1) / nparts, j_lo = part_id * per, j_hi = min(rh, j_lo + per);   // this part's hidden units

    // requests first: this thread's slice triple, the router's input row, the first batch of router weights
    const bool has = part_id == 0 && tid < t.nslices;
    const float4 p0 = part[(size_t)min(tid, t.nslices - 1) * n + i];
    const float *u = t.hidden_tap == 0 ? t.hn + (size_t)i * d : t.x + (size_t)(t.gather ? t.gather[i] : i) * d;
    TRaw8<WT> rw[RQ][2];
    // weight rows j0 + q*TF_WAVES (clamped to the last row), columns k0 + h*512 + lane*8 (clamped to the last 8)
    auto issue = [&](int j0, int k0) {
#pragma unroll
        for (int q = 0; q < RQ; ++q)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                rw[q][h].load(w1 + (size_t)min(j0 + q * TF_WAVES, rh - 1) * d + min(k0 + h * 512 + lane * 8, d - 8));
    };
    const bool given = mlp && t.r1 != nullptr;   // the first layer's sums were computed by the LM-head launch
    if (mlp && !given) {
        for (int k = tid; k < d; k += TF_THREADS) s_u[k] = u[k];
        issue(j_lo + wave, 0);
    }

    float M = -INFINITY, S = 0.f; int I = 0x7fffffff;
    if (part_id == 0) {
        // 1. global maximum and the lowest index that attains it
        if (has) { M = p0.x; I = __float_as_int(p0.y); }
        for (int s = tid + TF_THREADS; s < t.nslices; s += TF_THREADS) {
            const float4 p = part[(size_t)s * n + i];
            const int pi = __float_as_int(p.y);
            if (p.x > M || (p.x == M && pi < I)) { M = p.x; I = pi; }
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const float m2 = __shfl_xor(M, o, 64); const int i2 = __shfl_xor(I, o, 64);
            if (m2 > M || (m2 == M && i2 < I)) { M = m2; I = i2; }
        }
        if (lane == 0) { s_wm[wave] = M; s_wi[wave] = I; }
        __syncthreads();
        M = -INFINITY; I = 0x7fffffff;
        for (int w = 0; w < TF_WAVES; ++w) {
            const float m2 = s_wm[w]; const int i2 = s_wi[w];
            if (m2 > M || (m2 == M && i2 < I)) { M = m2; I = i2; }
        }
        // 2. sum of exponentials relative to the global maximum
        if (has && p0.x > -INFINITY) S = p0.z * expf(p0.x - M);
        for (int s = tid + TF_THREADS; s < t.nslices; s += TF_THREADS) {
            const float4 p = part[(size_t)s * n + i];
            if (p.x > -INFINITY) S += p.z * expf(p.x - M);
        }
        S = t_wave_sum(S);
        if (lane == 0) s_ws[0][wave] = S;
    }

    // 3. router: score = sigmoid(w2 . relu(W1 u + b1) + b2) on the tapped hidden state. A wavefront takes RQ hidden
    //    units at a time; its lanes split the columns, so every weight row is read as consecutive 16-byte pieces.
    if (linear) {   // one linear head: the block's threads split the columns
        const WT *w = (const WT *)t.r_w2;
        float a = 0.f;
        for (int k = tid; k < d; k += TF_THREADS) a = fmaf(t_widen(w, k), u[k], a);
        a = t_wave_sum(a);
        if (lane == 0) s_ws[1][wave] = a;
    }
    if (given) {
        const WT *b1 = (const WT *)t.r_b1, *w2 = (const WT *)t.r_w2;
        float a = 0.f;
        for (int j = tid; j < rh; j += TF_THREADS) {
            const float hb = t.r1[(size_t)i * t.r1_stride + j] + (b1 ? t_widen(b1, j) : 0.f);
            a = fmaf(t_widen(w2, j), hb > 0.f ? hb : 0.f, a);
        }
        a = t_wave_sum(a);
        if (lane == 0) s_ws[1][wave] = a;
    } else if (mlp) {
        const WT *b1 = (const WT *)t.r_b1, *w2 = (const WT *)t.r_w2;
        __syncthreads();   // s_u is complete
        for (int j0 = j_lo + wave; j0 < j_hi; j0 += RQ * TF_WAVES) {
            float acc[RQ];
#pragma unroll
            for (int q = 0; q < RQ; ++q) acc[q] = 0.f;
            for (int k0 = 0; k0 < d; k0 += 1024) {
                if (j0 != j_lo + wave || k0 != 0) issue(j0, k0);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int k = k0 + h * 512 + lane * 8;
                    const float4 x0 = *reinterpret_cast<const float4 *>(s_u + min(k, d - 8)), x1 = *reinterpret_cast<const float4 *>(s_u + min(k, d - 8) + 4);
                    const float keep = k < d ? 1.f : 0.f;   // clamped requests contribute nothing
                    const float xv[8] = {x0.x * keep, x0.y * keep, x0.z * keep, x0.w * keep, x1.x * keep, x1.y * keep, x1.z * keep, x1.w * keep};
#pragma unroll
                    for (int q = 0; q < RQ; ++q) {
                        float w[8];
                        rw[q][h].widen(w);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[q] = fmaf(w[e], xv[e], acc[q]);
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < RQ; ++q) {
                const float h = t_wave_sum(acc[q]);
                const int j = j0 + q * TF_WAVES;
                if (lane == 0 && j < j_hi) {
                    const float hb = h + (b1 ? t_widen(b1, j) : 0.f);
                    s_h[j - j_lo] = hb > 0.f ? hb : 0.f;
                }
            }
        }
        __syncthreads();
        float a = 0.f;
        for (int j = j_lo + tid; j < j_hi; j += TF_THREADS) a = fmaf(t_widen(w2, j), s_h[j - j_lo], a);
        a = t_wave_sum(a);
        if (lane == 0) s_ws[1][wave] = a;
    }
    __syncthreads();
    if (tid != 0) return;
    // padding row of a launch sized before the row count was known: fixed outputs, nothing counted or scattered
    const bool dead = t.live && i >= *t.live;
    float conf = 0.f;
    if (part_id == 0) {
        float Ssum = 0.f;
        for (int w = 0; w < TF_WAVES; ++w) Ssum += s_ws[0][w];
        conf = 1.0f / Ssum;
        t.token[i] = dead ? -1 : I; t.conf[i] = dead ? 0.f : conf;
        if (t.scatter && !dead) t.scatter[t.cand[i]] = I;
    }
    float score = 1.0f;
    int flag = 0;
    if (mlp || linear) {
        float pre = 0.f;
        for (int w = 0; w < TF_WAVES; ++w) pre += s_ws[1][w];
        if (nparts > 1) {
            __hip_atomic_store(t.rpart + (size_t)i * nparts + part_id, pre, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the device-coherent store has been acknowledged (vmcnt counts stores on this architecture)
            const int old = __hip_atomic_fetch_add(t.rcnt + i, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old != nparts - 1) return;
            __hip_atomic_store(t.rcnt + i, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // every part has counted: ready for the next launch
            pre = 0.f;
            for (int q = 0; q < nparts; ++q) pre += __hip_atomic_load(t.rpart + (size_t)i * nparts + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        pre += t.r_b2 ? t_widen((const WT *)t.r_b2, 0) : 0.f;
        score = 1.0f / (1.0f + expf(-pre));
    } else if (t.policy == 1) {
        score = conf;
    }
    if ((mlp || linear || t.policy == 1) && t.mode == 0) flag = t.route_dir == 0 ? (score < t.threshold) : (score > t.threshold);
    if (dead) { t.score[i] = 0.f; t.flag[i] = 0; return; }
    t.score[i] = score; t.flag[i] = flag;
    if (t.counters && t.counter_mode) {
        long long *c = t.counters + 2 * (size_t)t.slot[i];
        if (t.counter_mode == 1) { c[0] += 1; c[1] += flag; }
        else { c[0] = 1; c[1] = flag; }
    }
}

template <typename WT>
static void launch_lmhead_gemv_t(hipStream_t s, const Dims &D, const TailArgs &t)
{
    if (t.n == 1)
        hipLaunchKernelGGL((lmhead_kernel<WT, 1>), dim3(t.nslices, 1), dim3(256), 0, s, (const WT *)t.head, D.V, D.d, t.hn, t.n,
                           (float4 *)t.part, t.logits);
    else if (t.n == 2)
        hipLaunchKernelGGL((lmhead_kernel<WT, 2>), dim3(t.nslices, 1), dim3(256), 0, s, (const WT *)t.head, D.V, D.d, t.hn, t.n,
                           (float4 *)t.part, t.logits);
    else
        hipLaunchKernelGGL((lmhead_kernel<WT, 4>), dim3(t.nslices, (t.n + 3) / 4), dim3(256), 0, s, (const WT *)t.head, D.V, D.d, t.hn, t.n,
                           (float4 *)t.part, t.logits);
}

void launch_lmhead_gemv(hipStream_t s, int wdt, const Dims &D, const TailArgs &t)
{
    if (wdt == DT_F32) launch_lmhead_gemv_t<float>(s, D, t);
    else launch_lmhead_gemv_t<bf16_t>(s, D, t);
}

void launch_tail_final(hipStream_t s, int wdt, const Dims &D, const TailArgs &t)
{
    // the MLP router's hidden units go to up to TAIL_ROUTER_PARTS workgroups per row, at least 64 units each, as long
    // as all workgroups of the launch fit the chip at once (beyond that the split only adds the exchange)
    int parts = 1;
    if (t.policy == 0 && D.rh > 0 && t.rpart && t.rcnt && !t.r1) parts = std::max(1, std::min({TAIL_ROUTER_PARTS, (D.rh + 63) / 64, 256 / t.n}));
    if (wdt == DT_F32) hipLaunchKernelGGL(tail_final_kernel<float>, dim3(t.n, parts), dim3(TF_THREADS), 0, s, D.d, D.rh, t);
    else hipLaunchKernelGGL(tail_final_kernel<bf16_t>, dim3(t.n, parts), dim3(TF_THREADS), 0, s, D.d, D.rh, t);
}

void launch_tail_norm(hipStream_t s, int wdt, const Dims &D, const TailArgs &t)
{
    if (wdt == DT_F32)
        hipLaunchKernelGGL(tail_norm_kernel<float>, dim3(t.n), dim3(256), 0, s, D.d, D.eps, (const float *)t.final_norm, t.x, t.gather, t.hn,
                           t.hidden, t.hidden_tap);
    else
        hipLaunchKernelGGL(tail_norm_kernel<bf16_t>, dim3(t.n), dim3(256), 0, s, D.d, D.eps, (const bf16_t *)t.final_norm, t.x, t.gather, t.hn,
                           t.hidden, t.hidden_tap);
}

// the all-streaming tail: norm, LM head slices, merge + router
void launch_tail(hipStream_t s, int wdt, const Dims &D, const TailArgs &t)
{
    launch_tail_norm(s, wdt, D, t);
    launch_lmhead_gemv(s, wdt, D, t);
    launch_tail_final(s, wdt, D, t);
}

}  // namespace tr
