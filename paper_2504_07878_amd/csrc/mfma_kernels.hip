// Batched (more than a few rows) linear layers of the decode step on the gfx950 matrix cores.
//
// Shape of the problem: Y[M][N] = A[M][K] . W[N][K]^T with M = rows of the batch (tens), N and K in the
// hundreds to hundred-thousands, W in bf16. The work is bound by streaming W from HBM once, so the kernel is
// built around that stream:
//   * W is repacked once, when the context is created, into 32-row x 16-column tiles stored in the exact
//     register layout of the v_mfma_f32_32x32x16_bf16 "A" operand: one wavefront load of a tile is 1 KiB of
//     consecutive bytes.
//   * The activations are the stationary operand. Every wavefront keeps the "B" operands of its share of K
//     (at most 14 k-steps of 16) resident in registers for the whole kernel, so the inner loop is one
//     coalesced 16-byte load per lane per MFMA group and no LDS traffic.
//   * fp32 activations are carried as two bf16 terms (value = hi + lo), both multiplied against the same W
//     registers, which keeps about 16 mantissa bits; W itself is exact.
//   * The four wavefronts of a workgroup split K; their partial tiles are added through LDS in a fixed order,
//     then an epilogue functor consumes the 32x64 tile (rotary + cache append, SwiGLU, split-K partials, or the
//     running softmax statistics of the LM head). Everything is deterministic.
#include "tr_internal.h"

namespace tr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int MAXKW = 14;  // k-steps a wavefront keeps resident (4 wavefronts x 14 x 16 = 896 columns of K per workgroup)

__device__ __forceinline__ bf16_t m_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float m_bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }

// value = hi + lo with hi = bf16(value), lo = bf16(value - hi)
__device__ __forceinline__ void split_hi_lo(const float (&v)[8], uint4 &hi, uint4 &lo)
{
    uint32_t h[8], l[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const bf16_t hb = m_f32_to_bf16(v[e]);
        h[e] = hb;
        l[e] = m_f32_to_bf16(v[e] - m_bf16_to_f32(hb));
    }
    hi = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    lo = make_uint4(l[0] | (l[1] << 16), l[2] | (l[3] << 16), l[4] | (l[5] << 16), l[6] | (l[7] << 16));
}

// Packed activations of one group of up to 64 rows: [k-step][column block][lane] of 16 bytes, column blocks =
// {hi rows 0-31, (hi rows 32-63), lo rows 0-31, (lo rows 32-63)}; lane = row%32 + 32*(k%16 / 8).
__device__ __forceinline__ void store_packed(uint4 *pack, int ncb, int row_in_group, int k8 /* index of the 8-column chunk */,
                                             const float (&v)[8])
{
    uint4 hi, lo;
    split_hi_lo(v, hi, lo);
    const int ks = k8 >> 1, lane = (row_in_group & 31) + 32 * (k8 & 1), cb = row_in_group >> 5;
    pack[((size_t)ks * ncb + cb) * 64 + lane] = hi;
    pack[((size_t)ks * ncb + (ncb >> 1) + cb) * 64 + lane] = lo;
}

// ------------------------------------------------------------------ one-time weight repack

__global__ void repack_kernel(const bf16_t *W, int N, int K, uint4 *Wt, int KS, int dst_tile0, int dst_tile_stride, int n_tiles)
{
    const size_t total = (size_t)n_tiles * KS * 64;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(i & 63);
        const size_t rest = i >> 6;
        const int ks = (int)(rest % KS), t = (int)(rest / KS);
        const int row = t * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8;
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = (row < N && k + e < K) ? W[(size_t)row * K + k + e] : 0;
        Wt[((size_t)(dst_tile0 + t * dst_tile_stride) * KS + ks) * 64 + lane] =
            make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
}

void launch_repack(hipStream_t s, const void *W, int N, int K, void *Wt, int dst_tile0, int dst_tile_stride)
{
    const int KS = (K + 15) / 16, n_tiles = (N + 31) / 32;
    const size_t total = (size_t)n_tiles * KS * 64;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(repack_kernel, dim3(blocks), dim3(256), 0, s, (const bf16_t *)W, N, K, (uint4 *)Wt, KS, dst_tile0, dst_tile_stride, n_tiles);
}

__global__ void widen_bias_kernel(const bf16_t *b, int n, float *out)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = b ? m_bf16_to_f32(b[i]) : 0.f;
}

void launch_widen_bias(hipStream_t s, const void *b, int n, float *out)
{
    hipLaunchKernelGGL(widen_bias_kernel, dim3((n + 255) / 256), dim3(256), 0, s, (const bf16_t *)b, n, out);
}

// ------------------------------------------------------------------ residual update + RMSNorm + pack
// x[m] += sum of the split-K partials of the previous linear layer (fixed order), then
// n = x * g / rms(x) is written as packed hi/lo activations. One workgroup per row.

__global__ __launch_bounds__(128) void prep_kernel(PrepArgs p)
{
    __shared__ float red[2];
    const int m = blockIdx.x, tid = threadIdx.x;
    const int d = p.d, k0 = tid * 8;
    const bool live = k0 < d;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.f;
    float *xr = p.x + (size_t)(p.row0 + m) * d;
    if (live) {
        const float4 a = *reinterpret_cast<const float4 *>(xr + k0), b = *reinterpret_cast<const float4 *>(xr + k0 + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        for (int s = 0; s < p.nsplit; ++s) {
            const float *pr = p.part + ((size_t)s * p.part_M + p.row0 + m) * d + k0;
            const float4 c = *reinterpret_cast<const float4 *>(pr), e2 = *reinterpret_cast<const float4 *>(pr + 4);
            v[0] += c.x; v[1] += c.y; v[2] += c.z; v[3] += c.w; v[4] += e2.x; v[5] += e2.y; v[6] += e2.z; v[7] += e2.w;
        }
        if (p.nsplit > 0) {
            *reinterpret_cast<float4 *>(xr + k0) = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float4 *>(xr + k0 + 4) = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
    float ss = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) ss = fmaf(v[e], v[e], ss);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float rstd = 1.0f / sqrtf((red[0] + red[1]) / (float)d + p.eps);
    if (!live) return;
    const uint4 gbits = *reinterpret_cast<const uint4 *>(p.gain + k0);
    const uint32_t gw[4] = {gbits.x, gbits.y, gbits.z, gbits.w};
    float n[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float g = __uint_as_float((e & 1) ? (gw[e >> 1] & 0xffff0000u) : (gw[e >> 1] << 16));
        n[e] = v[e] * rstd * g;
    }
    if (p.hn) {
        *reinterpret_cast<float4 *>(p.hn + (size_t)m * d + k0) = make_float4(n[0], n[1], n[2], n[3]);
        *reinterpret_cast<float4 *>(p.hn + (size_t)m * d + k0 + 4) = make_float4(n[4], n[5], n[6], n[7]);
    }
    if (p.hidden) {
        const float *src = p.hidden_tap == 0 ? n : v;
        *reinterpret_cast<float4 *>(p.hidden + (size_t)m * d + k0) = make_float4(src[0], src[1], src[2], src[3]);
        *reinterpret_cast<float4 *>(p.hidden + (size_t)m * d + k0 + 4) = make_float4(src[4], src[5], src[6], src[7]);
    }
    const int KS = d / 16;
    uint4 *pack = p.pack + (size_t)(m >> 6) * KS * p.ncb * 64;
    store_packed(pack, p.ncb, m & 63, tid, n);
}

void launch_prep(hipStream_t s, const PrepArgs &p)
{
    hipLaunchKernelGGL(prep_kernel, dim3(p.M), dim3(128), 0, s, p);
}

// fp32 rows -> packed hi/lo activations (attention output ahead of the output projection)
__global__ void pack_kernel(const float *in, int M, int K, uint4 *pack, int ncb)
{
    const int m = blockIdx.x;
    const int KS = K / 16;
    uint4 *dst = pack + (size_t)(m >> 6) * KS * ncb * 64;
    for (int k8 = threadIdx.x; k8 < K / 8; k8 += blockDim.x) {
        const float *src = in + (size_t)m * K + k8 * 8;
        const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
        const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        store_packed(dst, ncb, m & 63, k8, v);
    }
}

void launch_pack(hipStream_t s, const float *in, int M, int K, void *pack, int ncb)
{
    hipLaunchKernelGGL(pack_kernel, dim3(M), dim3(128), 0, s, in, M, K, (uint4 *)pack, ncb);
}

// ------------------------------------------------------------------ the GEMM

struct GemmArgs {
    const uint4 *Wt;    // tiled weights [tile][KS][64]
    const uint4 *pack;  // packed activations [group][KS][NCB][64]
    int KS;             // K / 16
    int ksw;            // k-steps per workgroup (<= 56)
    int n_tiles;
    int tiles_per_wg;
    int M;              // rows in total (groups of 64 along gridDim.z)
};

// Epilogues receive, per thread, 8 consecutive output features (rows i0..i0+7 of tile t) of one batch row.

struct EpiPartial {   // split-K partial sums: part[split][m][n]
    float *part;
    int N, M;
    __device__ void begin() {}
    __device__ void tile(int t, int m, int i0, const float (&v)[8])
    {
        const int n = t * 32 + i0;
        if (m < M && n < N) {
            float *dst = part + ((size_t)blockIdx.y * M + m) * N + n;
            *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
    __device__ void end(float *) {}
};

template <typename KT>
struct EpiQkv {       // bias, rotary embedding, q out, cache append
    const float *bias;        // concatenated [qw + 2 kvw]
    const float2 *rope;
    const int *slot, *pos;
    float *q;
    KT *kc, *vc;
    int M, Hq, Hkv, dh, max_seq, qw;
    float hold[2][8];
    __device__ void begin() {}
    __device__ void tile(int t, int m, int i0, const float (&v)[8])
    {
        const int tph = dh >> 5, halfp = tph >> 1;          // tiles per head, tiles per rotary half
        const int hh = t / tph, sub = t % tph;
        float y[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] = v[e] + bias[t * 32 + i0 + e];
        if (sub < halfp) {
#pragma unroll
            for (int e = 0; e < 8; ++e) hold[sub & 1][e] = y[e];
            return;
        }
        if (m >= M) return;
        const int e0 = (sub - halfp) * 32 + i0;              // index inside the first half of the head
        const int half = dh >> 1, p = pos[m];
        float lo[8], hi[8];
        if (hh < Hq + Hkv) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float2 cs = rope[(size_t)p * half + e0 + e];
                const float a = hold[(sub - halfp) & 1][e], b = y[e];
                lo[e] = a * cs.x - b * cs.y;
                hi[e] = b * cs.x + a * cs.y;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) { lo[e] = hold[(sub - halfp) & 1][e]; hi[e] = y[e]; }
        }
        if (hh < Hq) {
            float *dst = q + (size_t)m * qw + hh * dh + e0;
            *reinterpret_cast<float4 *>(dst) = make_float4(lo[0], lo[1], lo[2], lo[3]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(lo[4], lo[5], lo[6], lo[7]);
            *reinterpret_cast<float4 *>(dst + half) = make_float4(hi[0], hi[1], hi[2], hi[3]);
            *reinterpret_cast<float4 *>(dst + half + 4) = make_float4(hi[4], hi[5], hi[6], hi[7]);
        } else {
            const int head = hh < Hq + Hkv ? hh - Hq : hh - Hq - Hkv;
            KT *dst = (hh < Hq + Hkv ? kc : vc) + (((size_t)slot[m] * Hkv + head) * max_seq + p) * dh + e0;
            store8(dst, lo);
            store8(dst + half, hi);
        }
    }
    __device__ static void store8(float *dst, const float (&v)[8])
    {
        *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4 *>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
    __device__ static void store8(bf16_t *dst, const float (&v)[8])
    {
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = m_f32_to_bf16(v[e]);
        *reinterpret_cast<uint4 *>(dst) = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
    __device__ void end(float *) {}
};

struct EpiSwiglu {    // tiles alternate gate, up; h = silu(gate) * up, written as packed activations of the down projection
    uint4 *hpack;     // [group][F/16][NCB][64]
    int M, F, ncb;
    float hold[8];
    __device__ void begin() {}
    __device__ void tile(int t, int m, int i0, const float (&v)[8])
    {
        if ((t & 1) == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) hold[e] = v[e];
            return;
        }
        if (m >= M) return;
        float h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = hold[e] / (1.0f + expf(-hold[e])) * v[e];
        const int f0 = (t >> 1) * 32 + i0;
        if (f0 < F) store_packed(hpack + (size_t)(m >> 6) * (F / 16) * ncb * 64, ncb, m & 63, f0 >> 3, h);
    }
    __device__ void end(float *) {}
};

struct EpiLmHead {    // running softmax statistics per batch row; logits optionally dumped
    float4 *part;     // [gridDim.x][M]
    float *logits;
    int M, V;
    float mx, sum;
    int idx;
    __device__ void begin() { mx = -INFINITY; sum = 0.f; idx = 0x7fffffff; }
    __device__ void tile(int t, int m, int i0, const float (&v)[8])
    {
        if (m >= M) return;
        const int n0 = t * 32 + i0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int n = n0 + e;
            if (n < V) {
                const float z = v[e];
                if (logits) logits[(size_t)m * V + n] = z;
                if (z > mx) { sum = sum * expf(mx - z) + 1.0f; mx = z; idx = n; }
                else sum += expf(z - mx);
            }
        }
    }
    // the four threads that share a batch row (one per 8-row band) merge through LDS
    __device__ void end(float *lds)
    {
        float4 *s = reinterpret_cast<float4 *>(lds);
        __syncthreads();
        s[threadIdx.x] = make_float4(mx, __int_as_float(idx), sum, 0.f);
        __syncthreads();
        const int j = threadIdx.x;
        const int m = blockIdx.z * 64 + j;
        if (j < 64 && m < M) {
            float Mx = -INFINITY; int I = 0x7fffffff;
            for (int b = 0; b < 4; ++b) {
                const float4 p = s[b * 64 + j];
                const int pi = __float_as_int(p.y);
                if (p.x > Mx || (p.x == Mx && pi < I)) { Mx = p.x; I = pi; }
            }
            float S = 0.f;
            for (int b = 0; b < 4; ++b) {
                const float4 p = s[b * 64 + j];
                if (p.x > -INFINITY) S += p.z * expf(p.x - Mx);
            }
            part[(size_t)blockIdx.x * M + m] = make_float4(Mx, __int_as_float(I), S, 0.f);
        }
    }
};

template <int NCB, class Epi>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_kernel(GemmArgs a, Epi epi_in)
{
    Epi epi = epi_in;   // per-thread epilogue state lives in registers
    constexpr int NCO = NCB / 2;
    __shared__ float red[4][32][65];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int ks0 = blockIdx.y * a.ksw, ks1 = min(a.KS, ks0 + a.ksw);
    const int per = (ks1 - ks0 + 3) >> 2;
    const int wk0 = ks0 + wave * per;
    const int nk = max(0, min(ks1, wk0 + per) - wk0);
    const int group = blockIdx.z;

    // resident activations of this wavefront's k-steps
    bf16x8 b[MAXKW][NCB];
    {
        const uint4 *pk = a.pack + ((size_t)group * a.KS + wk0) * NCB * 64 + lane;
#pragma unroll
        for (int kk = 0; kk < MAXKW; ++kk)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb) {
                uint4 u = make_uint4(0, 0, 0, 0);
                if (kk < nk) u = pk[((size_t)kk * NCB + cb) * 64];
                b[kk][cb] = __builtin_bit_cast(bf16x8, u);
            }
    }

    const int t0 = blockIdx.x * a.tiles_per_wg, t1 = min(a.n_tiles, t0 + a.tiles_per_wg);
    uint4 wc[MAXKW], wn[MAXKW];
#pragma unroll
    for (int kk = 0; kk < MAXKW; ++kk) { wc[kk] = make_uint4(0, 0, 0, 0); wn[kk] = make_uint4(0, 0, 0, 0); }
    if (t0 < t1) {
        const uint4 *wp = a.Wt + ((size_t)t0 * a.KS + wk0) * 64 + lane;
#pragma unroll
        for (int kk = 0; kk < MAXKW; ++kk)
            if (kk < nk) wc[kk] = wp[(size_t)kk * 64];
    }
    epi.begin();
    const int j = threadIdx.x & 63, i0 = (threadIdx.x >> 6) * 8;
    for (int t = t0; t < t1; ++t) {
        if (t + 1 < t1) {
            const uint4 *wp = a.Wt + ((size_t)(t + 1) * a.KS + wk0) * 64 + lane;
#pragma unroll
            for (int kk = 0; kk < MAXKW; ++kk)
                if (kk < nk) wn[kk] = wp[(size_t)kk * 64];
        }
        f32x16 acc[NCO];
#pragma unroll
        for (int co = 0; co < NCO; ++co)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[co][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < MAXKW; ++kk)
            if (kk < nk) {
                const bf16x8 w = __builtin_bit_cast(bf16x8, wc[kk]);
#pragma unroll
                for (int co = 0; co < NCO; ++co) {
                    acc[co] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, b[kk][co], acc[co], 0, 0, 0);
                    acc[co] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w, b[kk][NCO + co], acc[co], 0, 0, 0);
                }
            }
        __syncthreads();   // the previous tile has been read
#pragma unroll
        for (int co = 0; co < NCO; ++co)
#pragma unroll
            for (int r = 0; r < 16; ++r) red[wave][(r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)][co * 32 + (lane & 31)] = acc[co][r];
        __syncthreads();
        float v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = 0.f;
        if (j < 32 * NCO) {
#pragma unroll
            for (int r = 0; r < 8; ++r) v[r] = (red[0][i0 + r][j] + red[1][i0 + r][j]) + (red[2][i0 + r][j] + red[3][i0 + r][j]);
        }
        epi.tile(t, group * 64 + j, i0, v);
#pragma unroll
        for (int kk = 0; kk < MAXKW; ++kk) wc[kk] = wn[kk];
    }
    epi.end(&red[0][0][0]);
}

template <class Epi>
static void launch_gemm(hipStream_t s, const GemmArgs &a, int nsplit, const Epi &epi)
{
    const int groups = (a.M + 63) / 64;
    const dim3 grid((a.n_tiles + a.tiles_per_wg - 1) / a.tiles_per_wg, nsplit, groups);
    if (a.M <= 32) hipLaunchKernelGGL((gemm_kernel<2, Epi>), grid, dim3(256), 0, s, a, epi);
    else hipLaunchKernelGGL((gemm_kernel<4, Epi>), grid, dim3(256), 0, s, a, epi);
}

int mfma_ncb(int M) { return M <= 32 ? 2 : 4; }

// split-K plan for the linear layers whose epilogue is a plain sum
void plan_partial(int KS, int n_tiles, int *nsplit, int *ksw, int *tiles_per_wg)
{
    int S = (KS + 4 * MAXKW - 1) / (4 * MAXKW);
    const int want = 256 / (n_tiles > 0 ? n_tiles : 1);
    if (want > S) S = want;
    if (S > MAX_SPLITS) S = MAX_SPLITS;
    if (S > KS) S = KS;
    int w = (KS + S - 1) / S;
    S = (KS + w - 1) / w;
    *nsplit = S;
    *ksw = w;
    int tpw = (n_tiles * S + 255) / 256;
    *tiles_per_wg = tpw < 1 ? 1 : tpw;
}

void launch_gemm_partial(hipStream_t s, const void *Wt, const void *pack, int K, int N, int M, float *part, int *nsplit_out)
{
    GemmArgs a{};
    a.Wt = (const uint4 *)Wt; a.pack = (const uint4 *)pack; a.KS = K / 16; a.n_tiles = (N + 31) / 32; a.M = M;
    int S, ksw, tpw;
    plan_partial(a.KS, a.n_tiles, &S, &ksw, &tpw);
    a.ksw = ksw; a.tiles_per_wg = tpw;
    EpiPartial e{part, N, M};
    launch_gemm(s, a, S, e);
    *nsplit_out = S;
}

void launch_gemm_qkv(hipStream_t s, int kdt, const Dims &D, const void *Wt, const void *pack, const float *bias, Rows rows, const float2 *rope,
                     float *q, void *kc, void *vc)
{
    GemmArgs a{};
    a.Wt = (const uint4 *)Wt; a.pack = (const uint4 *)pack; a.KS = D.d / 16; a.ksw = a.KS; a.n_tiles = (D.qw + 2 * D.kvw) / 32; a.M = rows.n;
    a.tiles_per_wg = D.dh / 32;   // one head per workgroup
    if (kdt == DT_F32) {
        EpiQkv<float> e{bias, rope, rows.slot, rows.pos, q, (float *)kc, (float *)vc, rows.n, D.Hq, D.Hkv, D.dh, D.max_seq, D.qw, {}};
        launch_gemm(s, a, 1, e);
    } else {
        EpiQkv<bf16_t> e{bias, rope, rows.slot, rows.pos, q, (bf16_t *)kc, (bf16_t *)vc, rows.n, D.Hq, D.Hkv, D.dh, D.max_seq, D.qw, {}};
        launch_gemm(s, a, 1, e);
    }
}

void launch_gemm_swiglu(hipStream_t s, const Dims &D, const void *Wt, const void *pack, int M, void *hpack)
{
    GemmArgs a{};
    a.Wt = (const uint4 *)Wt; a.pack = (const uint4 *)pack; a.KS = D.d / 16; a.ksw = a.KS; a.n_tiles = 2 * ((D.F + 31) / 32); a.M = M;
    a.tiles_per_wg = 2 * ((a.n_tiles / 2 + 255) / 256);
    EpiSwiglu e{(uint4 *)hpack, M, D.F, mfma_ncb(M), {}};
    launch_gemm(s, a, 1, e);
}

int lmhead_mfma_wgs(int V)
{
    const int n_tiles = (V + 31) / 32;
    const int tpw = (n_tiles + 255) / 256;
    return (n_tiles + tpw - 1) / tpw;
}

void launch_gemm_lmhead(hipStream_t s, const Dims &D, const void *Wt, const void *pack, int M, float *part, float *logits)
{
    GemmArgs a{};
    a.Wt = (const uint4 *)Wt; a.pack = (const uint4 *)pack; a.KS = D.d / 16; a.ksw = a.KS; a.n_tiles = (D.V + 31) / 32; a.M = M;
    a.tiles_per_wg = (a.n_tiles + 255) / 256;
    EpiLmHead e{(float4 *)part, logits, M, D.V, 0.f, 0.f, 0};
    launch_gemm(s, a, 1, e);
}

}  // namespace tr
