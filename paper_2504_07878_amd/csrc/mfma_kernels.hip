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
#include <algorithm>
#include <type_traits>

namespace tr {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;

constexpr int NWAVES = 4;  // wavefronts per workgroup (one per SIMD, 512 registers each); they split K
constexpr int MAXKW = 14;  // k-steps a wavefront keeps resident (4 wavefronts x 14 x 16 = 896 columns of K per workgroup)

// Waits until every vector-memory operation this wavefront has issued (loads AND stores: gfx9-family parts count both in
// vmcnt) has completed. After device-coherent (write-through) stores this is the point from which another workgroup's
// device-coherent load returns the stored values.
__device__ __forceinline__ void wait_vector_memory() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ bf16_t m_f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float m_bf16_to_f32(bf16_t h) { return __uint_as_float((uint32_t)h << 16); }

// value = hi + lo with hi = bf16(value), lo = bf16(value - hi), both rounded to nearest even by the hardware's packed
// conversion (two values per instruction)
__device__ __forceinline__ void split_hi_lo(const float (&v)[8], uint4 &hi, uint4 &lo)
{
    uint32_t h[4], l[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const f32x2 x = {v[2 * p], v[2 * p + 1]};
        h[p] = __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
        const f32x2 rest = {v[2 * p] - __uint_as_float(h[p] << 16), v[2 * p + 1] - __uint_as_float(h[p] & 0xffff0000u)};
        l[p] = __builtin_bit_cast(uint32_t, __builtin_convertvector(rest, bf16x2));
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]);
    lo = make_uint4(l[0], l[1], l[2], l[3]);
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

// pair_dh > 0 (q, k, v matrices, pair_dh = head dim): the rows of a head are reordered so that tile row 2p holds dim
// 16*sub + p and tile row 2p + 1 its rotary partner dim 16*sub + p + pair_dh/2 (sub = tile index inside the head): the
// two features a rotation pairs up then sit next to each other in one thread of the GEMM epilogue.
__device__ __forceinline__ int paired_row(int t, int i, int pair_dh)
{
    const int tph = pair_dh >> 5, head = t / tph, sub = t % tph;
    return head * pair_dh + sub * 16 + (i >> 1) + (i & 1) * (pair_dh >> 1);
}

// MFMA row rho of a tile (the accumulator holds rows 8*qd + 4*hf + e in register 4*qd + e of the lanes with lane/32 = hf)
// carries the tile's feature tile_feature(rho): features are placed so that the accumulator registers {8a .. 8a+7} of
// one lane, a = 0 or 1, are 8 CONSECUTIVE features 16a + 8hf .. + 7. A wavefront can then hand half of its accumulator
// to another wavefront and keep, per lane, whole runs of 8 features.
__host__ __device__ __forceinline__ int tile_feature(int rho)
{
    const int qd = rho >> 3, hf = (rho >> 2) & 1, e = rho & 3;
    return 16 * (qd >> 1) + 8 * hf + 4 * (qd & 1) + e;
}

__global__ void repack_kernel(const bf16_t *W, int N, int K, uint4 *Wt, int KS, int dst_tile0, int dst_tile_stride, int n_tiles, int pair_dh)
{
    const size_t total = (size_t)n_tiles * KS * 64;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(i & 63);
        const size_t rest = i >> 6;
        const int ks = (int)(rest % KS), t = (int)(rest / KS);
        const int feat = tile_feature(lane & 31);
        const int row = pair_dh ? paired_row(t, feat, pair_dh) : t * 32 + feat, k = ks * 16 + (lane >> 5) * 8;
        uint32_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = (row < N && k + e < K) ? W[(size_t)row * K + k + e] : 0;
        Wt[((size_t)(dst_tile0 + t * dst_tile_stride) * KS + ks) * 64 + lane] =
            make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    }
}

void launch_repack(hipStream_t s, const void *W, int N, int K, void *Wt, int dst_tile0, int dst_tile_stride, int pair_dh)
{
    const int KS = (K + 15) / 16, n_tiles = (N + 31) / 32;
    const size_t total = (size_t)n_tiles * KS * 64;
    int blocks = (int)((total + 255) / 256);
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(repack_kernel, dim3(blocks), dim3(256), 0, s, (const bf16_t *)W, N, K, (uint4 *)Wt, KS, dst_tile0, dst_tile_stride, n_tiles, pair_dh);
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

__global__ __launch_bounds__(512) void prep_kernel(PrepArgs p)   // d / 8 threads rounded up to whole wavefronts, d <= 4096
{
    __shared__ float red[8];
    const int m = blockIdx.x, tid = threadIdx.x;
    const int d = p.d, k0 = tid * 8;
    const bool live = k0 < d;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = 0.f;
    const int row = p.gather ? p.gather[m] : p.row0 + m;
    float *xr = p.x + (size_t)row * d;
    if (live) {
        const float4 a = *reinterpret_cast<const float4 *>(xr + k0), b = *reinterpret_cast<const float4 *>(xr + k0 + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        // the partials are requested eight at a time (indices clamped) and added in their fixed order
        for (int s0 = 0; s0 < p.nsplit; s0 += 8) {
            float4 c[8], e2[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const float *pr = p.part + ((size_t)min(s0 + u, p.nsplit - 1) * p.part_M + row) * d + k0;
                c[u] = *reinterpret_cast<const float4 *>(pr); e2[u] = *reinterpret_cast<const float4 *>(pr + 4);
            }
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (s0 + u < p.nsplit) {
                    v[0] += c[u].x; v[1] += c[u].y; v[2] += c[u].z; v[3] += c[u].w;
                    v[4] += e2[u].x; v[5] += e2[u].y; v[6] += e2[u].z; v[7] += e2[u].w;
                }
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
    if (!live || !p.pack) return;
    float tot = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) tot += red[w];
    const float rstd = 1.0f / sqrtf(tot / (float)d + p.eps);
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
    const int threads = p.d / 8 <= 128 ? 128 : (p.d / 8 + 63) / 64 * 64;
    hipLaunchKernelGGL(prep_kernel, dim3(p.M), dim3(threads), 0, s, p);
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

// Merge of the per-chunk attention partials of one row (fixed order over chunks), written as fp32 rows and/or as
// packed hi/lo activations for the output projection. One thread per 8 consecutive dims of a head.
__global__ void attn_merge_kernel2(int Hq, int dh, int qw, const float *part, int nchunks, const int *pos, int chunk, float *att, uint4 *pack, int ncb)
{
    const int r = blockIdx.x, ps = dh + 4;
    const int p = pos[r];
    const int live = min(nchunks, (p + chunk) / chunk);   // chunks that hold at least one key of this row
    for (int k8 = threadIdx.x; k8 < qw / 8; k8 += blockDim.x) {
        const int head = (k8 * 8) / dh, d0 = (k8 * 8) % dh;
        const float *pp = part + ((size_t)r * Hq + head) * nchunks * ps;
        // chunks are taken four at a time with their loads issued together (indices clamped, weight 0 past the end)
        float M = -INFINITY;
        for (int c0 = 0; c0 < live; c0 += 4) {
            float mc[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) mc[u] = pp[min(c0 + u, live - 1) * ps + dh];
#pragma unroll
            for (int u = 0; u < 4; ++u) M = fmaxf(M, mc[u]);
        }
        float L = 0.f, o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.f;
        for (int c0 = 0; c0 < live; c0 += 4) {
            float mc[4], lc[4];
            float4 a[4], b[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float *pc = pp + min(c0 + u, live - 1) * ps;
                mc[u] = pc[dh]; lc[u] = pc[dh + 1];
                a[u] = *reinterpret_cast<const float4 *>(pc + d0); b[u] = *reinterpret_cast<const float4 *>(pc + d0 + 4);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float w = c0 + u < live ? __expf(mc[u] - M) : 0.f;
                L = fmaf(lc[u], w, L);
                o[0] = fmaf(a[u].x, w, o[0]); o[1] = fmaf(a[u].y, w, o[1]); o[2] = fmaf(a[u].z, w, o[2]); o[3] = fmaf(a[u].w, w, o[3]);
                o[4] = fmaf(b[u].x, w, o[4]); o[5] = fmaf(b[u].y, w, o[5]); o[6] = fmaf(b[u].z, w, o[6]); o[7] = fmaf(b[u].w, w, o[7]);
            }
        }
        const float inv = 1.0f / L;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= inv;
        if (att) {
            *reinterpret_cast<float4 *>(att + (size_t)r * qw + k8 * 8) = make_float4(o[0], o[1], o[2], o[3]);
            *reinterpret_cast<float4 *>(att + (size_t)r * qw + k8 * 8 + 4) = make_float4(o[4], o[5], o[6], o[7]);
        }
        if (pack) store_packed(pack + (size_t)(r >> 6) * (qw / 16) * ncb * 64, ncb, r & 63, k8, o);
    }
}

// The same merge for a few rows with many chunks: one workgroup per (row, head), the chunks spread over 16 thread
// groups whose results are combined through LDS in a fixed order, so that no thread walks more than
// ceil(nchunks / 16) chunks one after the other. Up to 64 chunks, dh <= 128.
__global__ __launch_bounds__(256) void attn_merge_wide_kernel(int Hq, int dh, int qw, const float *part, int nchunks, const int *pos,
                                                              int chunk, float *att, uint4 *pack, int ncb)
{
    __shared__ float s_m[64];
    __shared__ float s_l[16];
    __shared__ __attribute__((aligned(16))) float s_o[16][128];
    const int r = blockIdx.x, head = blockIdx.y, ps = dh + 4, tid = threadIdx.x;
    const int p = pos[r];
    const int live = min(nchunks, (p + chunk) / chunk);
    const float *pp = part + ((size_t)r * Hq + head) * nchunks * ps;
    if (tid < 64) s_m[tid] = tid < live ? pp[tid * ps + dh] : -INFINITY;
    __syncthreads();
    float M = -INFINITY;
    for (int c = 0; c < live; ++c) M = fmaxf(M, s_m[c]);
    const int d8 = dh / 8, cl = tid / d8, k8 = tid % d8;      // 16 chunk lanes x dh/8 thread columns (cl < 16 when tid < 2*dh)
    if (cl < 16) {
        float L = 0.f, o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int c = cl + 16 * u;
            const float *pc = pp + min(c, live - 1) * ps;
            const float w = c < live ? __expf(s_m[min(c, 63)] - M) : 0.f;
            const float lc = pc[dh + 1];
            const float4 a = *reinterpret_cast<const float4 *>(pc + k8 * 8), b = *reinterpret_cast<const float4 *>(pc + k8 * 8 + 4);
            L = fmaf(lc, w, L);
            o[0] = fmaf(a.x, w, o[0]); o[1] = fmaf(a.y, w, o[1]); o[2] = fmaf(a.z, w, o[2]); o[3] = fmaf(a.w, w, o[3]);
            o[4] = fmaf(b.x, w, o[4]); o[5] = fmaf(b.y, w, o[5]); o[6] = fmaf(b.z, w, o[6]); o[7] = fmaf(b.w, w, o[7]);
        }
        *reinterpret_cast<float4 *>(&s_o[cl][k8 * 8]) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4 *>(&s_o[cl][k8 * 8 + 4]) = make_float4(o[4], o[5], o[6], o[7]);
        if (k8 == 0) s_l[cl] = L;
    }
    __syncthreads();
    if (tid < d8) {
        float L = 0.f, o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.f;
        for (int g = 0; g < 16; ++g) {
            L += s_l[g];
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] += s_o[g][tid * 8 + e];
        }
        const float inv = 1.0f / L;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] *= inv;
        const int col8 = (head * dh) / 8 + tid;
        if (att) {
            *reinterpret_cast<float4 *>(att + (size_t)r * qw + col8 * 8) = make_float4(o[0], o[1], o[2], o[3]);
            *reinterpret_cast<float4 *>(att + (size_t)r * qw + col8 * 8 + 4) = make_float4(o[4], o[5], o[6], o[7]);
        }
        if (pack) store_packed(pack + (size_t)(r >> 6) * (qw / 16) * ncb * 64, ncb, r & 63, col8, o);
    }
}

void launch_attn_merge(hipStream_t s, const Dims &D, const float *part, int nchunks, Rows rows, int chunk, float *att, void *pack, int ncb)
{
    if (rows.n <= 8 && nchunks > 8 && nchunks <= 64 && D.dh <= 128) {
        hipLaunchKernelGGL(attn_merge_wide_kernel, dim3(rows.n, D.Hq), dim3(256), 0, s, D.Hq, D.dh, D.qw, part, nchunks, rows.pos, chunk, att,
                           (uint4 *)pack, ncb);
        return;
    }
    const int threads = D.qw / 8 >= 512 ? 512 : (D.qw / 8 + 63) / 64 * 64;
    hipLaunchKernelGGL(attn_merge_kernel2, dim3(rows.n), dim3(threads), 0, s, D.Hq, D.dh, D.qw, part, nchunks, rows.pos, chunk, att, (uint4 *)pack, ncb);
}

// ------------------------------------------------------------------ grouped-query attention on the matrix cores
// (bf16 cache, V stored transposed). One wavefront owns one (query row, kv head, chunk of the context) and walks its
// chunk in blocks of 32 keys:
//   S[key][head]  = K[key][:] . q[head][:]   v_mfma 32x32x16, A = K rows straight from the cache, B = q as hi+lo bf16
//   O[dim][head] += V^T[dim][key] . P[head][key]          A = V^T rows straight from the cache, B = P as hi+lo bf16
// The 32 accumulator columns are the query heads of the group (7 of 32 used). In the accumulator layout a lane holds
// one head column, so the softmax of a block is in-register arithmetic plus one exchange between lanes l and l^32,
// and the probabilities already sit where the second product wants its B operand: K rows are fetched in the order
// "bits 2 and 3 of the row index swapped", which makes the 8 accumulator registers of one k-step hold 8 consecutive keys.

__device__ __forceinline__ void to_hi_lo(const float (&v)[8], bf16x8 &hi, bf16x8 &lo)
{
    uint4 h, l;
    split_hi_lo(v, h, l);
    hi = __builtin_bit_cast(bf16x8, h);
    lo = __builtin_bit_cast(bf16x8, l);
}

// The walk of one wavefront over the blocks of 32 keys t_begin, t_begin + t_step, ... < j1 of one (row, kv head):
// running maximum m and sum l of its head column (both lanes of a head agree on m; l is per lane) and the
// unnormalised output o, accumulator register rr of block db = dim db*32 + 8*(rr/4) + 4*hf + rr%4 of head j.
// kc, vt: one layer's K cache and transposed V cache; PAGED: the row's keys live in pages looked up per block of 32 keys.
// MULTI: the 32 accumulator columns hold the heads of nq <= 32/G consecutive query rows of one sequence (column c = row c/G,
// head c%G) instead of one row's heads in the first G columns: the keys and values of the context are fetched once for all of
// them (the rows of a prompt). qrow is then the first of these rows, j1 the context of the LAST one; row i sees j1 - (nq-1) + i keys.
template <int DH, bool PAGED, bool MULTI = false, int NBLK = (DH == 64 ? 2 : 1)>
struct AttnWave {
    static constexpr int KSQ = DH / 16, DB = DH / 32;
    float m, l;
    f32x16 o[DB];

    __device__ __forceinline__ void run(const Dims &D, const float *qrow /* q of this row */, const bf16_t *kc, const bf16_t *vt, int slot, int g,
                                        int t_begin, int t_step, int j1, int nq = 1)
    {
        const int ulen = PAGED ? D.page : D.max_seq, uvts = PAGED ? D.page : D.vts;   // positions per storage unit
        const bf16_t *Kb = kc + ((size_t)slot * D.Hkv + g) * (size_t)ulen * DH, *Vb = vt + ((size_t)slot * D.Hkv + g) * (size_t)DH * uvts;   // contiguous cache
        [[maybe_unused]] const int t_last = (j1 - 1) & ~31;   // last block of 32 keys that holds a key of this row
        const int lane = threadIdx.x & 63, j = lane & 31, hf = lane >> 5, G = D.G;
        const int rq = MULTI ? j / G : 0, hq = MULTI ? j % G : j;          // query row and head of this lane's column
        const bool used = MULTI ? rq < nq : j < G;
        const int j1c = MULTI ? j1 - (nq - 1) + rq : j1;                    // keys this column sees
        const int j1min = MULTI ? j1 - (nq - 1) : j1;
        bf16x8 qh[KSQ], ql[KSQ];
        {
            const float scale = 1.0f / sqrtf((float)DH);
            const float *qp = qrow + (size_t)(used ? rq : 0) * D.qw + (size_t)(g * G + (used ? hq : 0)) * DH + hf * 8;
#pragma unroll
            for (int ks = 0; ks < KSQ; ++ks) {
                float v[8];
                const float4 a = *reinterpret_cast<const float4 *>(qp + ks * 16), b = *reinterpret_cast<const float4 *>(qp + ks * 16 + 4);
                v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = used ? v[e] * scale : 0.f;
                to_hi_lo(v, qh[ks], ql[ks]);
            }
        }
        const int krow = (j & 0x13) | ((j & 4) << 1) | ((j & 8) >> 1);   // row j of the A operand holds key krow (bits 2,3 swapped)
        m = -INFINITY; l = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int rr = 0; rr < 16; ++rr) o[db][rr] = 0.f;

        // NB blocks of 32 keys are requested together (64-wide heads: 64 keys in flight at once; three or four at once measured no faster:
        // a compute unit's requests in flight are limited well below what one wavefront can ask for)
        constexpr int NB = NBLK;
        for (int t0 = t_begin; t0 < j1; t0 += NB * t_step) {
            uint4 ka[NB][KSQ], va[NB][2][DB];
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                int t = t0 + nb * t_step;   // may start past j1 in the last trip
                const bf16_t *kp;
                int tv;                     // start of the block of V^T rows inside its storage unit
                if constexpr (PAGED) {
                    t = min(t, t_last);     // such a block's requests are redirected to the row's last block and unused
                    const int unit = D.ptab[(size_t)slot * D.maxp + t / D.page];
                    Kb = kc + ((size_t)unit * D.Hkv + g) * (size_t)ulen * DH;
                    Vb = vt + ((size_t)unit * D.Hkv + g) * (size_t)DH * uvts;
                    tv = t % D.page;
                    kp = Kb + (size_t)(tv + min(krow, j1 - 1 - t)) * DH + hf * 8;
                } else {                    // rows are clamped, V^T rows are padded to 32
                    t = min(t, t_last);     // a block past the context: its requests repeat the row's last block and are not used
                    kp = Kb + (size_t)min(t + krow, j1 - 1) * DH + hf * 8;
                    tv = min(t, D.vts - 32);
                }
#pragma unroll
                for (int ks = 0; ks < KSQ; ++ks) ka[nb][ks] = *reinterpret_cast<const uint4 *>(kp + ks * 16);
#pragma unroll
                for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                    for (int db = 0; db < DB; ++db)
                        va[nb][kk][db] = *reinterpret_cast<const uint4 *>(Vb + ((size_t)(tv >> 5) * DH + db * 32 + j) * 32 + 16 * kk + 8 * hf);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int t = t0 + nb * t_step;
                if (t >= j1) break;   // uniform over the wavefront
                f32x16 sacc;
#pragma unroll
                for (int rr = 0; rr < 16; ++rr) sacc[rr] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KSQ; ++ks) {
                    const bf16x8 kv = __builtin_bit_cast(bf16x8, ka[nb][ks]);
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv, qh[ks], sacc, 0, 0, 0);
                    sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kv, ql[ks], sacc, 0, 0, 0);
                }
                // register rr of this lane is key t + 16*(rr/8) + 8*hf + rr%8 of head j
                if (t + 32 > j1min) {   // the last block of a row's context may be ragged
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr)
                        if (t + 16 * (rr >> 3) + 8 * hf + (rr & 7) >= j1c) sacc[rr] = -INFINITY;
                }
                float bm = -INFINITY;
#pragma unroll
                for (int rr = 0; rr < 16; ++rr) bm = fmaxf(bm, sacc[rr]);
                bm = fmaxf(bm, __shfl_xor(bm, 32, 64));      // one row: key t is valid, so the pair maximum is finite
                const float mraw = fmaxf(m, bm);
                // a column whose row ends before this block and that has seen nothing yet keeps m = -inf; its exponentials take 0 as reference and vanish
                const float mn = (MULTI && mraw == -INFINITY) ? 0.f : mraw;
                const float corr = __expf(m - mn);           // 0 on the first block
                float p[16], ps = 0.f;
#pragma unroll
                for (int rr = 0; rr < 16; ++rr) { p[rr] = __expf(sacc[rr] - mn); ps += p[rr]; }
                l = l * corr + ps;
                m = mraw;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int rr = 0; rr < 16; ++rr) o[db][rr] *= corr;
#pragma unroll
                for (int kk = 0; kk < 2; ++kk) {
                    const float pk[8] = {p[8 * kk], p[8 * kk + 1], p[8 * kk + 2], p[8 * kk + 3], p[8 * kk + 4], p[8 * kk + 5], p[8 * kk + 6], p[8 * kk + 7]};
                    bf16x8 ph, pl;
                    to_hi_lo(pk, ph, pl);
#pragma unroll
                    for (int db = 0; db < DB; ++db) {
                        const bf16x8 vv = __builtin_bit_cast(bf16x8, va[nb][kk][db]);
                        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv, ph, o[db], 0, 0, 0);
                        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vv, pl, o[db], 0, 0, 0);
                    }
                }
            }
        }
    }
};

// One wavefront per (query row, chunk of the context), kv head along gridDim.y: partials for the merge, or the final
// rows when there is a single chunk.
template <int DH, bool PAGED>
__global__ __launch_bounds__(256) void attn_mfma_kernel(Dims D, const float *q, const bf16_t *kc, const bf16_t *vt, Rows rows, int chunk,
                                                        int nchunks, float *part, float *att)
{
    constexpr int DB = DH / 32, PS = DH + 4;
    const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (item >= rows.n * nchunks) return;
    if (rows.live && *rows.live == 0) return;   // uniform over the launch
    const int r = __builtin_amdgcn_readfirstlane(item / nchunks), c = item % nchunks, g = blockIdx.y;   // one row per wavefront
    const int lane = threadIdx.x & 63, j = lane & 31, hf = lane >> 5, G = D.G;
    const int ctx = rows.pos[r] + 1;
    const int j0 = c * chunk, j1 = min(ctx, j0 + chunk);
    const int slot = rows.slot[r];
    if (j0 >= ctx) return;   // no key of this row in the chunk: the merge never reads its partial

    AttnWave<DH, PAGED> w;
    w.run(D, q + (size_t)r * D.qw, kc, vt, slot, g, j0, 32, j1);
    const float lt = w.l + __shfl_xor(w.l, 32, 64);      // both lanes of a head used the same running maximum
    if (j >= G) return;
    const int head = g * G + j;
    if (nchunks == 1) {
        const float inv = 1.0f / lt;
        float *dst = att + (size_t)r * D.qw + (size_t)head * DH;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                *reinterpret_cast<float4 *>(dst + db * 32 + qd * 8 + hf * 4) =
                    make_float4(w.o[db][4 * qd] * inv, w.o[db][4 * qd + 1] * inv, w.o[db][4 * qd + 2] * inv, w.o[db][4 * qd + 3] * inv);
    } else {
        float *pp = part + (((size_t)r * D.Hq + head) * nchunks + c) * PS;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)
                *reinterpret_cast<float4 *>(pp + db * 32 + qd * 8 + hf * 4) = make_float4(w.o[db][4 * qd], w.o[db][4 * qd + 1], w.o[db][4 * qd + 2], w.o[db][4 * qd + 3]);
        if (hf == 0) { pp[DH] = w.m; pp[DH + 1] = lt; }
    }
}

// One workgroup of 8 wavefronts per (query row, kv head, part of the context). A row is split into as few parts as
// `span` (the longest part allowed, a multiple of 256 keys) permits, of equal length so that they finish together;
// wavefront w walks the key blocks w, w + 8, ... of its part and the eight results are combined through LDS in a
// fixed order. A row whose context fits one part is finished there. Otherwise every part leaves its (max, sum,
// output) in `part` and counts itself in on cnt[row][kv head]; the workgroup that arrives last combines the parts in
// their fixed order (whoever arrives last, the arithmetic is the same) and puts the counter back to zero. Nobody
// waits for anybody. Output: fp32 rows and/or packed hi/lo activations. For batches with enough (row, kv head)
// pairs to fill the chip this replaces the chunked kernel plus the separate merge.
constexpr int ATT_ROW_WAVES = 8;

template <int DH, bool PAGED>
__global__ __launch_bounds__(64 * ATT_ROW_WAVES) void attn_rows_kernel(Dims D, const float *q, const bf16_t *kc, const bf16_t *vt, Rows rows,
                                                                      int span, float *part, int *cnt, float *att, uint4 *pack, int ncb)
{
    constexpr int DB = DH / 32, NW = ATT_ROW_WAVES, GMAX = 8, PS = DH + 4;
    __shared__ float s_m[NW][GMAX], s_l[NW][GMAX];
    __shared__ __attribute__((aligned(16))) float s_o[NW][GMAX][DH];
    __shared__ int s_last;
    const int r = blockIdx.x, g = blockIdx.y, pt = blockIdx.z, P = gridDim.z, wv = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63, j = lane & 31, hf = lane >> 5, G = D.G;
    if (rows.live && *rows.live == 0) return;   // uniform over the launch, before any barrier
    const int ctx = rows.pos[r] + 1;
    const int slot = rows.slot[r];
    const int parts = (ctx + span - 1) / span;        // parts this row is split into: as few as the longest part allows ...
    if (pt >= parts) return;                          // (uniform over the workgroup, before any barrier)
    const int len = 256 * ((ctx + 256 * parts - 1) / (256 * parts));   // ... and of equal length, so that they finish together
    const int j0 = pt * len, j1 = min(ctx, j0 + len);

    if (j0 + wv * 32 < j1) {
        AttnWave<DH, PAGED> w;
        w.run(D, q + (size_t)r * D.qw, kc, vt, slot, g, j0 + wv * 32, NW * 32, j1);
        const float lt = w.l + __shfl_xor(w.l, 32, 64);
        if (j < G) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)
                    *reinterpret_cast<float4 *>(&s_o[wv][j][db * 32 + qd * 8 + hf * 4]) =
                        make_float4(w.o[db][4 * qd], w.o[db][4 * qd + 1], w.o[db][4 * qd + 2], w.o[db][4 * qd + 3]);
            if (hf == 0) { s_m[wv][j] = w.m; s_l[wv][j] = lt; }
        }
    }
    __syncthreads();
    const int live = min(NW, (j1 - j0 + 31) / 32);   // wavefronts that had keys
    const int task = threadIdx.x;                    // (head of the group, 8 dims)
    const bool worker = task < G * (DH / 8);
    const int h = task / (DH / 8), d0 = (task % (DH / 8)) * 8;
    float M = -INFINITY, L = 0.f, o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
    if (worker) {
        for (int w2 = 0; w2 < live; ++w2) M = fmaxf(M, s_m[w2][h]);
        for (int w2 = 0; w2 < live; ++w2) {
            const float c = __expf(s_m[w2][h] - M);
            L = fmaf(s_l[w2][h], c, L);
            const float4 a = *reinterpret_cast<const float4 *>(&s_o[w2][h][d0]), b = *reinterpret_cast<const float4 *>(&s_o[w2][h][d0 + 4]);
            o[0] = fmaf(a.x, c, o[0]); o[1] = fmaf(a.y, c, o[1]); o[2] = fmaf(a.z, c, o[2]); o[3] = fmaf(a.w, c, o[3]);
            o[4] = fmaf(b.x, c, o[4]); o[5] = fmaf(b.y, c, o[5]); o[6] = fmaf(b.z, c, o[6]); o[7] = fmaf(b.w, c, o[7]);
        }
    }
    if (parts > 1) {
        // leave this part's result, count in, and go on only as the last arrival of the row
        // The exchange goes through device-coherent accesses only (write-through stores, loads that bypass the
        // non-coherent cache levels): each is visible device-wide once it has completed. The ordering is made explicit:
        // every storing wavefront waits until its outstanding vector-memory operations have been acknowledged (on this
        // architecture the vector-memory counter covers stores) BEFORE the barrier that precedes the counter update, so
        // the counter can only reach `parts` after every part's data has landed; the last arriver issues its loads only
        // after its own read-modify-write has returned. No cache is flushed or invalidated as a whole (a device-scope
        // release fence writes back the entire L2 of the XCD, far more than this exchange is worth).
        if (worker) {
            float *pp = part + (((size_t)r * D.Hq + g * G + h) * P + pt) * PS;
#pragma unroll
            for (int e = 0; e < 8; ++e) __hip_atomic_store(pp + d0 + e, o[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (d0 == 0) {
                __hip_atomic_store(pp + DH, M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(pp + DH + 1, L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
        wait_vector_memory();   // this wavefront's device-coherent stores have been acknowledged
        __syncthreads();
        if (threadIdx.x == 0) {
            int *c = cnt + (size_t)r * D.Hkv + g;
            const int old = __hip_atomic_fetch_add(c, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = old == parts - 1;
            if (old == parts - 1) __hip_atomic_store(c, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // every part has counted: ready for the next launch
        }
        __syncthreads();
        if (!s_last) return;
        if (worker) {
            // four parts at a time, all their loads in flight together (indices clamped to the parts that exist, weight 0 past them)
            const float *pp = part + ((size_t)r * D.Hq + g * G + h) * P * PS;
            M = -INFINITY; L = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = 0.f;
            for (int c0 = 0; c0 < parts; c0 += 4) {
                float mc[4], lc[4], v[4][8];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float *pc = pp + min(c0 + u, parts - 1) * PS;
                    mc[u] = __hip_atomic_load(pc + DH, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    lc[u] = __hip_atomic_load(pc + DH + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[u][e] = __hip_atomic_load(pc + d0 + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                float Mn = M;
#pragma unroll
                for (int u = 0; u < 4; ++u) Mn = fmaxf(Mn, mc[u]);      // clamped entries repeat an existing part
                const float corr = __expf(M - Mn);                      // 0 in the first round
                L *= corr;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] *= corr;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float wgt = c0 + u < parts ? __expf(mc[u] - Mn) : 0.f;
                    L = fmaf(lc[u], wgt, L);
#pragma unroll
                    for (int e = 0; e < 8; ++e) o[e] = fmaf(v[u][e], wgt, o[e]);
                }
                M = Mn;
            }
        }
    }
    if (!worker) return;
    const float inv = 1.0f / L;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] *= inv;
    const int col = (g * G + h) * DH + d0;
    if (att) {
        *reinterpret_cast<float4 *>(att + (size_t)r * D.qw + col) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4 *>(att + (size_t)r * D.qw + col + 4) = make_float4(o[4], o[5], o[6], o[7]);
    }
    if (pack) store_packed(pack + (size_t)(r >> 6) * (D.qw / 16) * ncb * 64, ncb, r & 63, col >> 3, o);
}

// Prompts and catch-up segments: one workgroup of 8 wavefronts per (block of up to 32/G consecutive query rows of one
// sequence, kv head). The rows share every key and value they read (a wavefront's 32 accumulator columns hold the heads of
// all the rows, see AttnWave MULTI), so a prompt's cache is walked once per block of rows instead of once per row.
// Wavefront w walks the key blocks w, w + 8, ... of the whole context; the eight results are combined through LDS in a fixed
// order. qblock[b] = first row * 8 + number of rows of block b (consecutive positions of one slot).
template <int DH, bool PAGED>
__global__ __launch_bounds__(64 * ATT_ROW_WAVES) void attn_block_kernel(Dims D, const float *q, const bf16_t *kc, const bf16_t *vt, Rows rows,
                                                                       const int *qblock, float *att, uint4 *pack, int ncb)
{
    constexpr int DB = DH / 32, NW = ATT_ROW_WAVES;
    __shared__ float s_m[NW][32], s_l[NW][32];
    __shared__ __attribute__((aligned(16))) float s_o[NW][32][DH];
    const int code = qblock[blockIdx.x], r0 = code >> 3, nq = code & 7, g = blockIdx.y, wv = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63, j = lane & 31, hf = lane >> 5, G = D.G;
    const int j1 = rows.pos[r0] + nq;   // context of the block's last row
    const int slot = rows.slot[r0];
    if (wv * 32 < j1) {
        AttnWave<DH, PAGED, true> w;
        w.run(D, q + (size_t)r0 * D.qw, kc, vt, slot, g, wv * 32, NW * 32, j1, nq);
        const float lt = w.l + __shfl_xor(w.l, 32, 64);
        if (j < nq * G) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int qd = 0; qd < 4; ++qd)
                    *reinterpret_cast<float4 *>(&s_o[wv][j][db * 32 + qd * 8 + hf * 4]) =
                        make_float4(w.o[db][4 * qd], w.o[db][4 * qd + 1], w.o[db][4 * qd + 2], w.o[db][4 * qd + 3]);
            if (hf == 0) { s_m[wv][j] = w.m; s_l[wv][j] = lt; }
        }
    }
    __syncthreads();
    const int live = min(NW, (j1 + 31) / 32);        // wavefronts that had keys
    const int task = threadIdx.x;                    // (column = row and head, 8 dims)
    if (task >= nq * G * (DH / 8)) return;
    const int c = task / (DH / 8), d0 = (task % (DH / 8)) * 8, r = r0 + c / G, h = c % G;
    float M = -INFINITY, L = 0.f, o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.f;
    for (int w2 = 0; w2 < live; ++w2) M = fmaxf(M, s_m[w2][c]);     // finite: key 0 is seen by every row
    for (int w2 = 0; w2 < live; ++w2) {
        const float f = __expf(s_m[w2][c] - M);                     // 0 for a wavefront whose keys all lie past this row
        L = fmaf(s_l[w2][c], f, L);
        const float4 a = *reinterpret_cast<const float4 *>(&s_o[w2][c][d0]), b = *reinterpret_cast<const float4 *>(&s_o[w2][c][d0 + 4]);
        o[0] = fmaf(a.x, f, o[0]); o[1] = fmaf(a.y, f, o[1]); o[2] = fmaf(a.z, f, o[2]); o[3] = fmaf(a.w, f, o[3]);
        o[4] = fmaf(b.x, f, o[4]); o[5] = fmaf(b.y, f, o[5]); o[6] = fmaf(b.z, f, o[6]); o[7] = fmaf(b.w, f, o[7]);
    }
    const float inv = 1.0f / L;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] *= inv;
    const int col = (g * G + h) * DH + d0;
    if (att) {
        *reinterpret_cast<float4 *>(att + (size_t)r * D.qw + col) = make_float4(o[0], o[1], o[2], o[3]);
        *reinterpret_cast<float4 *>(att + (size_t)r * D.qw + col + 4) = make_float4(o[4], o[5], o[6], o[7]);
    }
    if (pack) store_packed(pack + (size_t)(r >> 6) * (D.qw / 16) * ncb * 64, ncb, r & 63, col >> 3, o);
}

int attention_block_rows(const Dims &D) { return std::min(4, 32 / D.G); }

void launch_attention_blocks(hipStream_t s, const Dims &D, const float *q, const void *kc, const void *vt, Rows rows, const int *qblock, int nblocks,
                             float *att, void *pack, int ncb)
{
    const dim3 grid(nblocks, D.Hkv);
    auto go = [&](auto kern) {
        hipLaunchKernelGGL(kern, grid, dim3(64 * ATT_ROW_WAVES), 0, s, D, q, (const bf16_t *)kc, (const bf16_t *)vt, rows, qblock, pack ? nullptr : att,
                           (uint4 *)pack, ncb);
    };
    if (D.dh == 64) { if (D.page) go(attn_block_kernel<64, true>); else go(attn_block_kernel<64, false>); }
    else { if (D.page) go(attn_block_kernel<128, true>); else go(attn_block_kernel<128, false>); }
}

void launch_attention_mfma(hipStream_t s, const Dims &D, const float *q, const void *kc, const void *vt, Rows rows, int max_ctx, float *part,
                           size_t part_floats, int *cnt, float *att, void *pack, int ncb, AttnPending *defer)
{
    if (defer) defer->nchunks = 0;
    // Few rows whose partials the consumer can merge while it stages them (the output projection of the GEMV path) keep the
    // chunked kernel below; everything else takes one workgroup per (row, kv head, part of the context), whose last arriver
    // merges the parts: no merge kernel.
    const bool consumer_merges = defer && !pack && rows.n <= 4 && max_ctx <= 16 * 64;
    // (128-wide heads with few rows stay on the chunked kernel too: the 7B-class routed-subset step measured 3.25 ms with it and
    // the merge kernel, 3.31 ms with parts of 256 keys here)
    const bool many = rows.n * D.Hkv >= 64;
    if (D.G <= 8 && (many || (!consumer_merges && D.dh == 64))) {
        // enough (row, kv head) pairs to fill the chip with one workgroup each: parts of 768 keys (three key blocks per
        // wavefront; measured best among 256..1024 on the ragged 64-sequence workload); fewer pairs: parts of 512 keys, so
        // that more compute units take part (0.5B-class step at 4 / 16 / 28 rows and contexts of ~1350: 1.031 / 1.049 / 1.063 ms;
        // with 256 keys 1.025 / 1.046 / 1.172, with 768 keys 1.072 / 1.085 / 1.095). Longer parts when the partials buffer
        // or the limit of 16 parts asks for it.
        size_t room = part_floats / ((size_t)rows.n * D.Hq * (D.dh + 4));
        if (room > 16) room = 16;
        if (room < 1) room = 1;
        int span = 768;
        if (many) {   // longer parts rather than a second round of workgroups (64 rows at contexts of ~1900: 1.390 -> 1.303 ms/step)
            const int max_parts = std::max(1, 256 / (rows.n * D.Hkv));
            span = std::max(768, 256 * ((max_ctx + 256 * max_parts - 1) / (256 * max_parts)));
        }
        if (!many) {   // parts of 512 keys, longer ones when the launch would otherwise exceed one round of 256 workgroups
            const int max_parts = std::max(1, 256 / (rows.n * D.Hkv));
            span = std::max(512, 256 * ((max_ctx + 256 * max_parts - 1) / (256 * max_parts)));
        }
        if ((size_t)(max_ctx + span - 1) / span > room) span = 256 * (int)((max_ctx + 256 * room - 1) / (256 * room));
        const int P = (max_ctx + span - 1) / span;
        const dim3 grid(rows.n, D.Hkv, P);
        auto go = [&](auto kern) {
            hipLaunchKernelGGL(kern, grid, dim3(64 * ATT_ROW_WAVES), 0, s, D, q, (const bf16_t *)kc, (const bf16_t *)vt, rows, span, part, cnt,
                               pack ? nullptr : att, (uint4 *)pack, ncb);
        };
        if (D.dh == 64) { if (D.page) go(attn_rows_kernel<64, true>); else go(attn_rows_kernel<64, false>); }
        else { if (D.page) go(attn_rows_kernel<128, true>); else go(attn_rows_kernel<128, false>); }
        return;
    }
    // decode: up to 32 chunks of the context per row, merged afterwards; prompts: one wavefront walks the whole context of a row
    size_t room = part_floats / ((size_t)rows.n * D.Hq * (D.dh + 4));   // chunks per row that fit the partials buffer
    if (room > 64) room = 64;
    int chunk = (max_ctx + 63) / 64 * 64, nchunks = 1;
    if (room >= 2) {
        chunk = 64 * (int)((max_ctx + 64 * room - 1) / (64 * room));
        nchunks = (max_ctx + chunk - 1) / chunk;
    }
    const dim3 grid((rows.n * nchunks + 3) / 4, D.Hkv);
    float *direct = nchunks == 1 ? att : nullptr;
    auto go = [&](auto kern) { hipLaunchKernelGGL(kern, grid, dim3(256), 0, s, D, q, (const bf16_t *)kc, (const bf16_t *)vt, rows, chunk, nchunks, part, direct); };
    if (D.dh == 64) { if (D.page) go(attn_mfma_kernel<64, true>); else go(attn_mfma_kernel<64, false>); }
    else { if (D.page) go(attn_mfma_kernel<128, true>); else go(attn_mfma_kernel<128, false>); }
    if (nchunks > 1 && defer && !pack && rows.n <= 4 && nchunks <= 16) {   // the consumer merges
        defer->part = part; defer->pos = rows.pos; defer->nchunks = nchunks; defer->chunk = chunk;
        return;
    }
    if (nchunks > 1) launch_attn_merge(s, D, part, nchunks, rows, chunk, pack ? nullptr : att, pack, ncb);
    else if (pack) launch_pack(s, att, rows.n, D.qw, pack, ncb);
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
    int half;           // 1: every 64-row group is served by two workgroups of 32 rows each (more workgroups for short tile ranges)
    int remap_groups;   // > 0: 1-D grid; the row groups of one tile range are placed on the same XCD, next to each other in time
    const int *live;    // device-side row count or NULL: with zero live rows the whole launch returns at once
};

// Epilogues receive, per thread, 8 consecutive output features (rows i0..i0+7 of tile t) of one batch row. PAR is the
// parity of the tile's index inside its workgroup's range, known at compile time. An epilogue does its arithmetic
// unconditionally and keeps conditions to its stores at the very end: the arithmetic then shares a basic block with the
// MFMAs of the next tile, which the matrix pipe executes while the vector ALUs do the epilogue.

struct EpiPartial {   // split-K partial sums: part[split][m][n]
    static constexpr bool half_only = false;
    float *part;
    int N, M;
    __device__ void block(int, int) {}
    __device__ void begin() {}
    __device__ void row(int, int) {}
    __device__ void row_ready(float *, int, int) {}
    template <int PAR> __device__ void tile(int t, int m, int i0, const float (&v)[8])
    {
        const int n = t * 32 + i0;
        if (m < M && n < N) {
            float *dst = part + ((size_t)blockIdx.y * M + m) * N + n;
            *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
        }
    }
    __device__ void end(float *, int, int) {}
};

template <typename KT>
struct EpiQkv {       // bias, rotary embedding, q out, cache append; tiles hold rotary pairs next to each other (see repack_kernel)
    static constexpr bool half_only = true;   // launched with GemmArgs::half = 1: 32-row workgroups only
    const float *bias;        // concatenated [qw + 2 kvw], natural feature order
    const float2 *rope;
    const int *slot, *pos;
    float *q;
    KT *kc, *vc;
    int M, Hq, Hkv, dh, max_seq, qw, vts;   // max_seq, vts: positions per storage unit of the cache (a slot or a page)
    const int *ptab;          // paged cache: page table [slot][maxp] and page length; page = 0: the unit is the slot
    int page, maxp;
    int rpos, runit, rupos;   // position of this thread's batch row (for the rotation) and where its key and value go:
                              // storage unit and position inside it, fetched ahead of the weight stream
    const int *live;          // device-side row count or NULL: rows from *live on are padding and store nothing
    __device__ void block(int, int) {}
    __device__ void begin() {}
    __device__ void row(int m, int)
    {
        rpos = pos[min(m, M - 1)]; runit = slot[min(m, M - 1)]; rupos = rpos;
        if (page) { runit = ptab[(size_t)runit * maxp + rpos / page]; rupos = rpos % page; }
        if (live) M = min(M, *live);
    }
    __device__ void row_ready(float *, int, int) {}
    // v: tile rows i0..i0+7 = the pairs (j, j + dh/2), j = 16*sub + i0/2 .. +3, as (first, partner) x 4
    template <int PAR> __device__ void tile(int t, int m, int i0, const float (&v)[8])
    {
        if (m >= M) return;
        const int tph = dh >> 5, half = dh >> 1, hh = t / tph, j0 = (t % tph) * 16 + (i0 >> 1), p = rpos;
        const float4 ba = *reinterpret_cast<const float4 *>(bias + hh * dh + j0), bb = *reinterpret_cast<const float4 *>(bias + hh * dh + half + j0);
        const float a[4] = {v[0] + ba.x, v[2] + ba.y, v[4] + ba.z, v[6] + ba.w}, b[4] = {v[1] + bb.x, v[3] + bb.y, v[5] + bb.z, v[7] + bb.w};
        float lo[4], hi[4];
        if (hh < Hq + Hkv) {
            const float4 *rp = reinterpret_cast<const float4 *>(rope + (size_t)p * half + j0);   // 4 (cos, sin) pairs, 32 bytes, aligned
            const float4 c0 = rp[0], c1 = rp[1];
            const float cx[4] = {c0.x, c0.z, c1.x, c1.z}, sy[4] = {c0.y, c0.w, c1.y, c1.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                lo[e] = a[e] * cx[e] - b[e] * sy[e];
                hi[e] = b[e] * cx[e] + a[e] * sy[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) { lo[e] = a[e]; hi[e] = b[e]; }
        }
        if (hh < Hq) {
            float *dst = q + (size_t)m * qw + hh * dh + j0;
            *reinterpret_cast<float4 *>(dst) = make_float4(lo[0], lo[1], lo[2], lo[3]);
            *reinterpret_cast<float4 *>(dst + half) = make_float4(hi[0], hi[1], hi[2], hi[3]);
        } else {
            const int head = hh < Hq + Hkv ? hh - Hq : hh - Hq - Hkv;
            if (hh < Hq + Hkv || vts == 0) {
                KT *dst = (hh < Hq + Hkv ? kc : vc) + (((size_t)runit * Hkv + head) * max_seq + rupos) * dh + j0;
                store4(dst, lo);
                store4(dst + half, hi);
            } else {   // block-transposed V: one position of 8 dim rows
                KT *dst = vc + ((((size_t)runit * Hkv + head) * (vts >> 5) + (rupos >> 5)) * dh + j0) * 32 + (rupos & 31);
#pragma unroll
                for (int e = 0; e < 4; ++e) { store1(dst + e * 32, lo[e]); store1(dst + (half + e) * 32, hi[e]); }
            }
        }
    }
    __device__ static void store4(float *dst, const float (&v)[4]) { *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]); }
    __device__ static void store4(bf16_t *dst, const float (&v)[4])
    {
        const f32x2 x0 = {v[0], v[1]}, x1 = {v[2], v[3]};
        *reinterpret_cast<uint2 *>(dst) = make_uint2(__builtin_bit_cast(uint32_t, __builtin_convertvector(x0, bf16x2)),
                                                     __builtin_bit_cast(uint32_t, __builtin_convertvector(x1, bf16x2)));
    }
    __device__ static void store1(float *dst, float v) { *dst = v; }
    __device__ static void store1(bf16_t *dst, float v)
    {
        const f32x2 x = {v, 0.f};
        *dst = (bf16_t)__builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));
    }
    __device__ void end(float *, int, int) {}
};

// RAGGED: F is not a multiple of 32, the last tile pair is partly empty.
// DEFER: deferred RMSNorm. The packed activations are x * gain WITHOUT the 1/rms factor (they were written by the epilogue of the
// output projection, which only knows its own 32 features of a row); W.(g*x/rms) = W.(g*x) / rms, so the factor is applied to the
// sums here. sumsq[m * ss_stride + i], i < n_ss <= 32: the row's sum of squares over the features of tile range i (ss_stride >= 32, a
// multiple of 4). The four threads that finish a row (one per band of 8 features) each fetch a quarter of the row's values and add
// them through LDS in band order: 8 registers per thread while the resident activations are being requested, not 32.
template <bool RAGGED, bool DEFER>
struct EpiSwiglu {    // tiles alternate gate, up; h = silu(gate) * up, written as packed activations of the down projection
    static constexpr bool half_only = false;
    uint4 *hpack;     // [group][F/16][NCB][64]
    int M, F, ncb;
    float hold[8];
    const float *sumsq;
    int n_ss, ss_stride;
    float eps, inv_d;
    float rstd;
    float4 raw[2];
    __device__ void block(int, int) {}
    __device__ void begin() {}
    // requests only: the values are used in row_ready(), after the kernel has requested its activations, so that nothing waits here
    __device__ void row(int m, int band)
    {
        if (DEFER) {
            const float4 *sp = reinterpret_cast<const float4 *>(sumsq + (size_t)min(m, M - 1) * ss_stride) + 2 * band;
            raw[0] = sp[0]; raw[1] = sp[1];
        }
    }
    // lds: 256 floats that nothing else uses before the workgroup's next barrier; every thread of the workgroup calls this
    __device__ void row_ready(float *lds, int row_local, int band)
    {
        if (DEFER) {
            const int i = 8 * band;   // entries past n_ss are not the row's
            float p = i < n_ss ? raw[0].x : 0.f;
            p += i + 1 < n_ss ? raw[0].y : 0.f; p += i + 2 < n_ss ? raw[0].z : 0.f; p += i + 3 < n_ss ? raw[0].w : 0.f;
            p += i + 4 < n_ss ? raw[1].x : 0.f; p += i + 5 < n_ss ? raw[1].y : 0.f; p += i + 6 < n_ss ? raw[1].z : 0.f; p += i + 7 < n_ss ? raw[1].w : 0.f;
            lds[band * 64 + row_local] = p;
            __syncthreads();
            const float tot = (lds[row_local] + lds[64 + row_local]) + (lds[128 + row_local] + lds[192 + row_local]);
            rstd = 1.0f / sqrtf(tot * inv_d + eps);
        }
    }
    // a workgroup's tile range starts at a gate tile (even index), so PAR = 0 is a gate tile, PAR = 1 its up tile
    template <int PAR> __device__ void tile(int t, int m, int i0, const float (&v)[8])
    {
        if (PAR == 0) {
#pragma unroll
            for (int e = 0; e < 8; ++e) hold[e] = DEFER ? v[e] * rstd : v[e];
            return;
        }
        float h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = hold[e] * __frcp_rn(1.0f + __expf(-hold[e])) * (DEFER ? v[e] * rstd : v[e]);   // hardware exp2 and reciprocal (1 ulp each)
        const int f0 = (t >> 1) * 32 + i0;
        // rows past M are written too: they lie inside the padded 64-row group and are never read back as valid rows
        if (!RAGGED || f0 < F) store_packed(hpack + (size_t)(m >> 6) * (F / 16) * ncb * 64, ncb, m & 63, f0 >> 3, h);
    }
    __device__ void end(float *, int, int) {}
};

// Output projection with the residual update and the next layer input's packing in its epilogue (no split-K, no separate
// residual + norm launch): x += tile; the packed activations of the FFN input are written as x * gain, hi/lo split, and the
// 1/rms factor is left to the consumer (EpiSwiglu::sumsq), for which every workgroup leaves its rows' sums of squares over its own
// tile range: sumsq[row][tile range]. The four threads that hold one row (one per band of 8 features) add their sums through LDS in
// band order, and a workgroup's tiles are taken in index order, so the value is the same from run to run.
struct EpiResidualNorm {
    static constexpr bool half_only = true;   // 32-row workgroups (GemmArgs::half = 1)
    float *x;              // residual stream [M][d], updated in place
    const bf16_t *gain;    // gain of the norm that follows
    uint4 *pack;           // packed activations of the next linear layer, [group][d/16][ncb][64]
    float *sumsq;          // [row][ss_stride], entry = index of the workgroup's tile range
    int M, d, ncb, ss_stride;
    int bx, m;
    float ss;
    __device__ void block(int b, int) { bx = b; }
    __device__ void begin() { ss = 0.f; }
    __device__ void row(int r, int) { m = r; }
    __device__ void row_ready(float *, int, int) {}
    template <int PAR> __device__ void tile(int t, int mm, int i0, const float (&v)[8])
    {
        const int n0 = t * 32 + i0;
        if (mm >= M || n0 >= d) return;   // d is a multiple of 8: a band is whole or absent
        float *xr = x + (size_t)mm * d + n0;
        const float4 a = *reinterpret_cast<const float4 *>(xr), b = *reinterpret_cast<const float4 *>(xr + 4);
        const uint4 gbits = *reinterpret_cast<const uint4 *>(gain + n0);
        const float xn[8] = {a.x + v[0], a.y + v[1], a.z + v[2], a.w + v[3], b.x + v[4], b.y + v[5], b.z + v[6], b.w + v[7]};
        *reinterpret_cast<float4 *>(xr) = make_float4(xn[0], xn[1], xn[2], xn[3]);
        *reinterpret_cast<float4 *>(xr + 4) = make_float4(xn[4], xn[5], xn[6], xn[7]);
        const uint32_t gw[4] = {gbits.x, gbits.y, gbits.z, gbits.w};
        float gx[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            ss = fmaf(xn[e], xn[e], ss);
            gx[e] = xn[e] * __uint_as_float((e & 1) ? (gw[e >> 1] & 0xffff0000u) : (gw[e >> 1] << 16));
        }
        store_packed(pack + (size_t)(mm >> 6) * (d / 16) * ncb * 64, ncb, mm & 63, n0 >> 3, gx);
    }
    __device__ void end(float *lds, int row_local, int band)
    {
        __syncthreads();
        lds[band * 64 + row_local] = ss;
        __syncthreads();
        if (band == 0 && row_local < 32 && m < M)
            sumsq[(size_t)m * ss_stride + bx] = (lds[row_local] + lds[64 + row_local]) + (lds[128 + row_local] + lds[192 + row_local]);
    }
};

// DUMP = false keeps every vector-memory store out of the tile loop, so that the wait counters of the weight stream stay exact.
// RAGGED: the vocabulary is not a multiple of 32.
template <bool DUMP, bool RAGGED>
struct EpiLmHead {    // running softmax statistics per batch row; logits optionally dumped
    static constexpr bool half_only = false;
    float4 *part;     // [gridDim.x][M]
    float *logits;
    int M, V;
    float mx, sum;
    int idx, bx, grp, nwg;   // nwg: workgroups that own tiles (the grid may be padded)
    // The tiles from index vt on are not vocabulary rows but the hidden units of the router's first layer (its weight
    // rows are appended to the head matrix: same activations, so the product comes for free inside this launch): their
    // raw sums go to r1[row][unit] and are kept out of the softmax statistics. vt = INT_MAX: no such tiles.
    float *r1;
    int vt, r1_stride;
    __device__ void block(int b, int g) { bx = b; grp = g; }
    __device__ void begin() { mx = -INFINITY; sum = 0.f; idx = 0x7fffffff; }
    __device__ void row(int, int) {}
    __device__ void row_ready(float *, int, int) {}
    // Branch-free: rows past M have all-zero activations, so their statistics are finite and simply never written.
    template <int PAR> __device__ void tile(int t, int m, int i0, const float (&vin)[8])
    {
        const int n0 = t * 32 + i0;
        if (DUMP) {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (m < M && n0 + e < V) logits[(size_t)m * V + n0 + e] = vin[e];
        }
        const bool router_tile = t >= vt;   // uniform over the workgroup
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = ((!RAGGED || n0 + e < V) && !router_tile) ? vin[e] : -INFINITY;   // a vocabulary tile holds at least one real row
        float lm = v[7];
        int li = 7;
#pragma unroll
        for (int e = 6; e >= 0; --e)
            if (v[e] >= lm) { lm = v[e]; li = e; }                  // descending scan: the lowest index wins ties
        const float nm = fmaxf(mx, lm);
        const float ref = nm == -INFINITY ? 0.f : nm;               // nothing but router tiles so far: every exponential below is 0
        idx = lm > mx ? n0 + li : idx;                              // strict: earlier tiles win ties
        float add = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) add += __expf(v[e] - ref);      // exp(-inf) = 0 for the rows past the vocabulary
        sum = fmaf(sum, __expf(mx - ref), add);                     // mx = -inf before the first tile: factor 0 on a zero sum
        mx = nm;
        if (router_tile && m < M) {
            float *dst = r1 + (size_t)m * r1_stride + (t - vt) * 32 + i0;
            *reinterpret_cast<float4 *>(dst) = make_float4(vin[0], vin[1], vin[2], vin[3]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(vin[4], vin[5], vin[6], vin[7]);
        }
    }
    // the four threads that share a batch row (one per band of 8 features) merge through LDS; row_local: the thread's
    // batch row inside its 64-row group, band: which 8 features of every tile it held
    __device__ void end(float *lds, int row_local, int band)
    {
        float4 *s = reinterpret_cast<float4 *>(lds);
        __syncthreads();
        s[band * 64 + row_local] = make_float4(mx, __int_as_float(idx), sum, 0.f);
        __syncthreads();
        const int j = threadIdx.x;
        const int m = grp * 64 + j;
        if (j < 64 && m < M && bx < nwg) {
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
            part[(size_t)bx * M + m] = make_float4(Mx, __int_as_float(I), S, 0.f);
        }
    }
};

// 256 threads = 4 wavefronts, each owning KW consecutive k-steps (compile time, so that every load of the steady
// state is unconditional and the hardware wait counters can be exact). The weight tiles of a wavefront alternate
// between two register sets; a set is refilled (tile t + 2) right after the MFMAs that read it have been issued.
// (Two dependent MFMAs on one accumulator run at half rate; the hi and lo products of the two column blocks are
// interleaved so that consecutive MFMAs never share an accumulator.)
constexpr int RED_FLOATS = NWAVES * 64 * 36;   // [wavefront][batch column][feature row padded to 36]

template <int NCB, int KW, class Epi>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm_kernel(GemmArgs a, Epi epi_in)
{
    constexpr int NCO = NCB / 2;
    __shared__ __attribute__((aligned(16))) float red[2 * RED_FLOATS];
    if (a.live && *a.live == 0) return;   // uniform over the launch
    Epi epi = epi_in;   // per-thread epilogue state lives in registers
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int ks0 = blockIdx.y * a.ksw, ks1 = min(a.KS, ks0 + a.ksw);
    const int per = (ks1 - ks0 + NWAVES - 1) / NWAVES;   // <= KW
    const int wk0 = ks0 + wave * per;
    const int nk = max(0, min(ks1, wk0 + per) - wk0);
    int bx = blockIdx.x, group = blockIdx.z;
    if (a.remap_groups > 0) {   // workgroups are dealt to the 8 XCDs round-robin: keep the groups of a tile range on one XCD
        const int xcd = bx & 7, slot = bx >> 3;
        group = slot % a.remap_groups;
        bx = (slot / a.remap_groups) * 8 + xcd;
    }
    epi.block(bx, group);
    // half mode: the packed activations hold 4 column blocks per 64-row group; this workgroup takes {h, 2 + h}
    const int pgroup = a.half ? group >> 1 : group, hsel = a.half ? group & 1 : 0, pncb = a.half ? 4 : NCB;
    const int row0 = pgroup * 64 + hsel * 32;
    // what the epilogue needs per batch row is requested first: it is then the oldest request in flight and can be waited for
    // without waiting for anything younger
    epi.row(row0 + (threadIdx.x & 63), threadIdx.x >> 6);

    // resident activations of this wavefront's k-steps (zero beyond its share, so the extra products vanish)
    bf16x8 b[KW][NCB];
    int koff[KW];   // k-step of each resident slot, clamped into the matrix
#pragma unroll
    for (int kk = 0; kk < KW; ++kk) {
        koff[kk] = min(wk0 + kk, a.KS - 1);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
            uint4 u = make_uint4(0, 0, 0, 0);
            if (kk < nk) u = a.pack[(((size_t)pgroup * a.KS + wk0 + kk) * pncb + (a.half ? cb * 2 + hsel : cb)) * 64 + lane];
            b[kk][cb] = __builtin_bit_cast(bf16x8, u);
        }
    }

    const int t0 = min(bx * a.tiles_per_wg, a.n_tiles), t1 = min(a.n_tiles, t0 + a.tiles_per_wg);
    const size_t tile_stride = (size_t)a.KS * 64;
    uint4 w[2][KW];
    f32x16 acc[NCO];
    const int j = threadIdx.x & 63, i0 = (threadIdx.x >> 6) * 8, rho0 = (i0 >> 4) * 16 + ((i0 >> 3) & 1) * 4;

    auto load_tile = [&](int t, uint4 (&ws)[KW]) {   // unconditional: t must be a valid tile
        const uint4 *wp = a.Wt + (size_t)t * tile_stride + lane;
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) ws[kk] = wp[(size_t)koff[kk] * 64];
    };
    auto mfma_step = [&](const uint4 &wk, int kk) {
        const bf16x8 wv = __builtin_bit_cast(bf16x8, wk);
#pragma unroll
        for (int hl = 0; hl < 2; ++hl)
#pragma unroll
            for (int co = 0; co < NCO; ++co) acc[co] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, b[kk][hl * NCO + co], acc[co], 0, 0, 0);
    };
    // The cross-wavefront sum of a tile goes through one of two LDS buffers, so a tile costs ONE barrier, and the sum and
    // epilogue of tile t sit in the same straight-line stretch as the MFMAs of tile t + 1 (independent work that can
    // fill the matrix pipe's shadow): put(t) | barrier | MFMAs(t + 1), refill, get(t), epilogue(t) | put(t + 1) | ...
    // A buffer is rewritten two barriers after it was read, and every wavefront reads before it reaches the next barrier.
    auto put = [&](float *rb) {
#pragma unroll
        for (int co = 0; co < NCO; ++co)
#pragma unroll
            for (int qd = 0; qd < 4; ++qd)   // registers 4qd..4qd+3 are the 4 consecutive MFMA rows 8qd + 4(lane/32) .. of one batch column
                *reinterpret_cast<float4 *>(&rb[(wave * 64 + co * 32 + (lane & 31)) * 36 + qd * 8 + (lane >> 5) * 4]) =
                    make_float4(acc[co][4 * qd], acc[co][4 * qd + 1], acc[co][4 * qd + 2], acc[co][4 * qd + 3]);
    };
    auto finish = [&](auto par, int t, const float *rb) {
        float v[8];
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = 0.f;
        if (j < 32 * NCO) {   // lanes past the column blocks of this workgroup hold nothing
#pragma unroll
            for (int ww = 0; ww < NWAVES; ++ww) {
                // features i0..i0+3 and i0+4..i0+7 sit in MFMA rows rho0.. and rho0+8.. (see tile_feature)
                const float4 lo4 = *reinterpret_cast<const float4 *>(&rb[(ww * 64 + j) * 36 + rho0]);
                const float4 hi4 = *reinterpret_cast<const float4 *>(&rb[(ww * 64 + j) * 36 + rho0 + 8]);
                v[0] += lo4.x; v[1] += lo4.y; v[2] += lo4.z; v[3] += lo4.w;
                v[4] += hi4.x; v[5] += hi4.y; v[6] += hi4.z; v[7] += hi4.w;
            }
            epi.template tile<decltype(par)::value>(t, row0 + j, i0, v);
        }
    };
    using Par0 = std::integral_constant<int, 0>;
    using Par1 = std::integral_constant<int, 1>;
    auto mfma_tile = [&](const uint4 (&ws)[KW]) {
#pragma unroll
        for (int co = 0; co < NCO; ++co)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[co][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < KW; ++kk) mfma_step(ws[kk], kk);
    };
    float *const red0 = red, *const red1 = red + RED_FLOATS;
    epi.begin();
    int t = t0;
    if (t0 < t1) {
        load_tile(t0, w[0]);
        if (t0 + 1 < t1) load_tile(t0 + 1, w[1]);
        // per-row inputs: they were requested before everything else, and nothing younger is waited for here.
        // The second LDS buffer is first written after the tile loop's first barrier.
        epi.row_ready(red1, threadIdx.x & 63, threadIdx.x >> 6);
        mfma_tile(w[0]);
        if (t0 + 2 < t1) load_tile(t0 + 2, w[0]);
        // from here on: acc = sums of tile t, w[1] = tile t + 1, w[0] = tile t + 2 (where they exist).
        // Long tile ranges: nothing conditional inside, so the compiler can wait for exactly the registers it needs
        // and leave the younger loads in flight.
        for (; t + 4 < t1; t += 2) {
            put(red0);
            __syncthreads();
            mfma_tile(w[1]);
            load_tile(t + 3, w[1]);
            finish(Par0{}, t, red0);
            put(red1);
            __syncthreads();
            mfma_tile(w[0]);
            load_tile(t + 4, w[0]);
            finish(Par1{}, t + 1, red1);
        }
        // up to four tiles are left
        auto tail_step = [&](auto ic) {
            constexpr int i = decltype(ic)::value;
            if (t + i < t1) {
                put(i & 1 ? red1 : red0);
                __syncthreads();
                if (t + i + 1 < t1) {
                    mfma_tile(w[(i + 1) & 1]);
                    if (t + i + 3 < t1) load_tile(t + i + 3, w[(i + 1) & 1]);
                }
                finish(std::integral_constant<int, (i & 1)>{}, t + i, i & 1 ? red1 : red0);
            }
        };
        tail_step(std::integral_constant<int, 0>{});
        tail_step(std::integral_constant<int, 1>{});
        tail_step(std::integral_constant<int, 2>{});
        tail_step(std::integral_constant<int, 3>{});
    }
    epi.end(red, threadIdx.x & 63, threadIdx.x >> 6);
}

template <int NCB, int KW, class Epi>
static void launch_gemm_one(hipStream_t s, const GemmArgs &a, dim3 grid, const Epi &epi)
{
    hipLaunchKernelGGL((gemm_kernel<NCB, KW, Epi>), grid, dim3(256), 0, s, a, epi);
}

// 64-row groups: the wavefronts split K in two and the rows in two (wavefront = (K half kh, row half rh)), so only TWO
// partial tiles have to be added per output instead of four, and each wavefront hands over just half of its
// accumulator: of the MFMA rows it computed, those of runs 8a..8a+7, a != kh, go to its partner (same rows, other
// K half) through LDS, the others stay in registers. 16 KB of LDS traffic per tile instead of 64 KB, which was the
// largest item of a tile after the MFMAs. Thanks to tile_feature() a lane ends up with 8 consecutive features
// 16 kh + 8 (lane / 32) .. of batch row 32 rh + lane % 32: the epilogues see what they saw before.
// The weights of a wavefront's K half (up to 28 k-steps) live in ONE register ring: entry kk is refilled with the
// next tile's k-step right after the two MFMAs that read it have been issued, so a whole tile is in flight ahead of
// the arithmetic. The hi and lo products accumulate separately (two dependent MFMAs on one accumulator run at half
// rate) and are added once per tile. Exchange buffers alternate, so a tile costs one barrier, and the partner's half
// and the epilogue of tile t follow the MFMAs of tile t + 1 in the same straight-line stretch.
template <int KW2, class Epi>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void gemm22_kernel(GemmArgs a, Epi epi_in)
{
    __shared__ float4 xb[2][NWAVES][2][64];
    if (a.live && *a.live == 0) return;   // uniform over the launch
    Epi epi = epi_in;   // per-thread epilogue state lives in registers
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // uniform: everything derived from it stays in scalar registers
    const int lane = threadIdx.x & 63, kh = wave & 1, rh = wave >> 1, hf = lane >> 5;
    const int ks0 = blockIdx.y * a.ksw, ks1 = min(a.KS, ks0 + a.ksw);
    const int per = (ks1 - ks0 + 1) / 2;   // <= KW2
    const int wk0 = ks0 + kh * per;
    const int nk = max(0, min(ks1, wk0 + per) - wk0);
    int bx = blockIdx.x, group = blockIdx.z;
    if (a.remap_groups > 0) {   // workgroups are dealt to the 8 XCDs round-robin: keep the groups of a tile range on one XCD
        const int xcd = bx & 7, slot = bx >> 3;
        group = slot % a.remap_groups;
        bx = (slot / a.remap_groups) * 8 + xcd;
    }
    epi.block(bx, group);
    const int m = group * 64 + rh * 32 + (lane & 31), i0 = 16 * kh + 8 * hf;
    epi.row(m, 2 * kh + hf);   // per-row inputs of the epilogue: requested first, so that they are the oldest requests in flight

    // resident activations: hi and lo halves of this wavefront's 32 rows over its k-steps (zero beyond its share)
    bf16x8 b[KW2][2];
    int koff[KW2];   // k-step of each resident slot, clamped into the matrix
#pragma unroll
    for (int kk = 0; kk < KW2; ++kk) {
        koff[kk] = min(wk0 + kk, a.KS - 1);
#pragma unroll
        for (int hl = 0; hl < 2; ++hl) {
            uint4 u = make_uint4(0, 0, 0, 0);
            if (kk < nk) u = a.pack[(((size_t)group * a.KS + wk0 + kk) * 4 + 2 * hl + rh) * 64 + lane];
            b[kk][hl] = __builtin_bit_cast(bf16x8, u);
        }
    }

    const int t0 = min(bx * a.tiles_per_wg, a.n_tiles), t1 = min(a.n_tiles, t0 + a.tiles_per_wg);
    const size_t tile_stride = (size_t)a.KS * 64;
    uint4 w[KW2];
    f32x16 acc_hi, acc_lo;
    float own[8];

    // the MFMAs of the tile held in w; with REFILL every entry is overwritten by tile tn (which must exist) once it has been read
    auto mfma_tile = [&](auto refill, int tn) {
        const uint4 *wp = a.Wt + (size_t)tn * tile_stride + lane;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc_hi[r] = 0.f; acc_lo[r] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < KW2; ++kk) {
            const bf16x8 wv = __builtin_bit_cast(bf16x8, w[kk]);
            acc_hi = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, b[kk][0], acc_hi, 0, 0, 0);
            acc_lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wv, b[kk][1], acc_lo, 0, 0, 0);
            if (decltype(refill)::value) w[kk] = wp[(size_t)koff[kk] * 64];
        }
    };
    // hi + lo; the runs of 8 MFMA rows this wavefront finishes stay in registers, the other two quads go to the partner
    auto send = [&](int buf) {
        float sum[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) sum[r] = acc_hi[r] + acc_lo[r];
#pragma unroll
        for (int e = 0; e < 8; ++e) own[e] = kh ? sum[8 + e] : sum[e];
        xb[buf][wave][0][lane] = kh ? make_float4(sum[0], sum[1], sum[2], sum[3]) : make_float4(sum[8], sum[9], sum[10], sum[11]);
        xb[buf][wave][1][lane] = kh ? make_float4(sum[4], sum[5], sum[6], sum[7]) : make_float4(sum[12], sum[13], sum[14], sum[15]);
    };
    auto finish = [&](auto par, int t, int buf) {
        const float4 p0 = xb[buf][wave ^ 1][0][lane], p1 = xb[buf][wave ^ 1][1][lane];
        const float v[8] = {own[0] + p0.x, own[1] + p0.y, own[2] + p0.z, own[3] + p0.w, own[4] + p1.x, own[5] + p1.y, own[6] + p1.z, own[7] + p1.w};
        epi.template tile<decltype(par)::value>(t, m, i0, v);
    };
    using No = std::integral_constant<bool, false>;
    using Yes = std::integral_constant<bool, true>;
    using Par0 = std::integral_constant<int, 0>;
    using Par1 = std::integral_constant<int, 1>;

    epi.begin();
    int t = t0;
    if (t0 < t1) {
        {
            const uint4 *wp = a.Wt + (size_t)t0 * tile_stride + lane;
#pragma unroll
            for (int kk = 0; kk < KW2; ++kk) w[kk] = wp[(size_t)koff[kk] * 64];
        }
        // per-row inputs: they were requested before everything else, and nothing younger is waited for here.
        // The second exchange buffer is first written after the tile loop's first barrier.
        epi.row_ready(reinterpret_cast<float *>(&xb[1][0][0][0]), rh * 32 + (lane & 31), 2 * kh + hf);
        if (t0 + 1 < t1) mfma_tile(Yes{}, t0 + 1); else mfma_tile(No{}, t0);
        // from here on: the accumulators hold tile t, the ring holds tile t + 1 (where it exists).
        // Long tile ranges: nothing conditional inside, so the compiler can wait for exactly the registers it needs.
        for (; t + 3 < t1; t += 2) {
            send(0);
            __syncthreads();
            mfma_tile(Yes{}, t + 2);
            finish(Par0{}, t, 0);
            send(1);
            __syncthreads();
            mfma_tile(Yes{}, t + 3);
            finish(Par1{}, t + 1, 1);
        }
        // up to three tiles are left
        auto tail_step = [&](auto ic) {
            constexpr int i = decltype(ic)::value;
            if (t + i < t1) {
                send(i & 1);
                __syncthreads();
                if (t + i + 2 < t1) mfma_tile(Yes{}, t + i + 2);
                else if (t + i + 1 < t1) mfma_tile(No{}, t + i + 1);
                finish(std::integral_constant<int, (i & 1)>{}, t + i, i & 1);
            }
        };
        tail_step(std::integral_constant<int, 0>{});
        tail_step(std::integral_constant<int, 1>{});
        tail_step(std::integral_constant<int, 2>{});
    }
    epi.end(reinterpret_cast<float *>(&xb[0][0][0][0]), rh * 32 + (lane & 31), 2 * kh + hf);
}

template <class Epi>
static void launch_gemm22_kw(hipStream_t s, const GemmArgs &a, dim3 grid, const Epi &epi)
{
    const int per = (a.ksw + 1) / 2;
    if (per <= 4) hipLaunchKernelGGL((gemm22_kernel<4, Epi>), grid, dim3(256), 0, s, a, epi);
    else if (per <= 8) hipLaunchKernelGGL((gemm22_kernel<8, Epi>), grid, dim3(256), 0, s, a, epi);
    else if (per <= 16) hipLaunchKernelGGL((gemm22_kernel<16, Epi>), grid, dim3(256), 0, s, a, epi);
    else hipLaunchKernelGGL((gemm22_kernel<28, Epi>), grid, dim3(256), 0, s, a, epi);
}

template <int NCB, class Epi>
static void launch_gemm_kw(hipStream_t s, const GemmArgs &a, dim3 grid, const Epi &epi)
{
    const int per = (a.ksw + NWAVES - 1) / NWAVES;
    if (per <= 2) launch_gemm_one<NCB, 2>(s, a, grid, epi);
    else if (per <= 4) launch_gemm_one<NCB, 4>(s, a, grid, epi);
    else if (per <= 8) launch_gemm_one<NCB, 8>(s, a, grid, epi);
    else launch_gemm_one<NCB, 14>(s, a, grid, epi);
}

template <class Epi>
static void launch_gemm(hipStream_t s, const GemmArgs &a, int nsplit, const Epi &epi)
{
    const int groups = (a.M + 63) / 64;
    dim3 grid((a.n_tiles + a.tiles_per_wg - 1) / a.tiles_per_wg, nsplit, groups);
    if (a.remap_groups > 0) grid = dim3((grid.x + 7) / 8 * 8 * groups, 1, 1);
    if (a.half && a.M > 32) { grid.z = 2 * groups; launch_gemm_kw<2>(s, a, grid, epi); return; }
    GemmArgs b = a;
    b.half = 0;
    if (a.M <= 32) launch_gemm_kw<2>(s, b, grid, epi);
    else if constexpr (!Epi::half_only) {   // half-only epilogues never get here: no 64-row instance of them
        // One 64-row group: weights come from HBM once and the LDS reduction is what limits a tile, so K and rows are
        // split two ways each. Several groups re-read the weights from L2, where loading every tile twice per
        // workgroup costs more than the smaller reduction saves: they keep the four-way K split.
        if (groups == 1) launch_gemm22_kw(s, b, grid, epi);
        else launch_gemm_kw<4>(s, b, grid, epi);
    }
}

int mfma_ncb(int M) { return M <= 32 ? 2 : 4; }

// split-K plan for the linear layers whose epilogue is a plain sum
// ------------------------------------------------------------------ finishing kernels of the split-K path (wide models)

// Workgroups along x share a batch row (gridDim.y rows); a thread takes the two features (j, j + dh/2) of a head that the rotation pairs up.
template <typename KT>
__global__ __launch_bounds__(256) void qkv_finish_kernel(Dims D, const float *part, int nsplit, int M, const float *bias, Rows rows, const float2 *rope,
                                                         float *q, KT *kc, KT *vc)
{
    const int m = blockIdx.y, half = D.dh / 2, N = D.qw + 2 * D.kvw, npairs = (D.Hq + 2 * D.Hkv) * half;
    if (rows.live && m >= *rows.live) return;   // padding row: nothing is appended to any cache (its q is never used)
    const int pos = rows.pos[m];
    const KvPlace at = kv_place(D, rows.slot[m], pos);
    for (int pr = blockIdx.x * blockDim.x + threadIdx.x; pr < npairs; pr += gridDim.x * blockDim.x) {
        const int hh = pr / half, j = pr % half, n1 = hh * D.dh + j, n2 = n1 + half;
        const int c1 = hh * D.dh + (j >> 4) * 32 + 2 * (j & 15), c2 = c1 + 1;   // columns of the pair in the interleaved tile order
        float y1 = bias[n1], y2 = bias[n2];
        for (int s0 = 0; s0 < nsplit; s0 += 4) {   // fixed order, four partials requested at a time
            float a1[4], a2[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float *src = part + ((size_t)min(s0 + u, nsplit - 1) * M + m) * N;
                a1[u] = src[c1]; a2[u] = src[c2];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (s0 + u < nsplit) { y1 += a1[u]; y2 += a2[u]; }
        }
        if (hh < D.Hq + D.Hkv) {
            const float2 cs = rope[(size_t)pos * half + j];
            const float o1 = y1 * cs.x - y2 * cs.y, o2 = y2 * cs.x + y1 * cs.y;
            y1 = o1; y2 = o2;
        }
        if (hh < D.Hq) {
            q[(size_t)m * D.qw + n1] = y1;
            q[(size_t)m * D.qw + n2] = y2;
        } else if (hh < D.Hq + D.Hkv) {
            KT *dst = kc + k_offset(D, at.unit, hh - D.Hq, at.pos, 0);
            EpiQkv<KT>::store1(dst + j, y1);
            EpiQkv<KT>::store1(dst + j + half, y2);
        } else {
            const int head = hh - D.Hq - D.Hkv;
            EpiQkv<KT>::store1(vc + v_offset(D, at.unit, head, at.pos, j), y1);
            EpiQkv<KT>::store1(vc + v_offset(D, at.unit, head, at.pos, j + half), y2);
        }
    }
}

// Workgroups along x share a batch row (gridDim.y rows); a thread takes 8 consecutive FFN features (gate columns
// (f/32)*64 + f%32, up columns 32 further).
__global__ __launch_bounds__(256) void swiglu_finish_kernel(const float *part, int nsplit, int M, int F, uint4 *hpack, int ncb)
{
    const int m = blockIdx.y;
    const size_t N = 2 * (size_t)((F + 31) / 32) * 32;
    for (int f8 = blockIdx.x * blockDim.x + threadIdx.x; f8 < F / 8; f8 += gridDim.x * blockDim.x) {
        const int f = f8 * 8;
        const size_t col = (size_t)(f / 32) * 64 + f % 32;
        float g[8], u[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { g[e] = 0.f; u[e] = 0.f; }
        for (int sp = 0; sp < nsplit; ++sp) {   // fixed order
            const float *src = part + ((size_t)sp * M + m) * N + col;
            const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
            const float4 c = *reinterpret_cast<const float4 *>(src + 32), d4 = *reinterpret_cast<const float4 *>(src + 36);
            g[0] += a.x; g[1] += a.y; g[2] += a.z; g[3] += a.w; g[4] += b.x; g[5] += b.y; g[6] += b.z; g[7] += b.w;
            u[0] += c.x; u[1] += c.y; u[2] += c.z; u[3] += c.w; u[4] += d4.x; u[5] += d4.y; u[6] += d4.z; u[7] += d4.w;
        }
        float h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) h[e] = g[e] * __frcp_rn(1.0f + __expf(-g[e])) * u[e];
        store_packed(hpack + (size_t)(m >> 6) * (F / 16) * ncb * 64, ncb, m & 63, f8, h);
    }
}

// One workgroup per (vocabulary slice, batch row): thread t takes columns t*8 .. t*8+7 of the slice (8 columns x 256 threads).
__global__ __launch_bounds__(256) void lmhead_finish_kernel(const float *part, int nsplit, int M, int V, float4 *slice_part, float *logits)
{
    __shared__ float s_m[256], s_s[256];
    __shared__ int s_i[256];
    const int m = blockIdx.y, v0 = blockIdx.x * LMHEAD_FINISH_COLS + threadIdx.x * 8, tid = threadIdx.x;
    float mx = -INFINITY, sum = 0.f;
    int idx = 0x7fffffff;
    if (v0 < V) {   // V % 8 == 0
        float z[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) z[e] = 0.f;
        for (int sp = 0; sp < nsplit; ++sp) {   // fixed order
            const float *src = part + ((size_t)sp * M + m) * V + v0;
            const float4 a = *reinterpret_cast<const float4 *>(src), b = *reinterpret_cast<const float4 *>(src + 4);
            z[0] += a.x; z[1] += a.y; z[2] += a.z; z[3] += a.w; z[4] += b.x; z[5] += b.y; z[6] += b.z; z[7] += b.w;
        }
        if (logits) {
            *reinterpret_cast<float4 *>(logits + (size_t)m * V + v0) = make_float4(z[0], z[1], z[2], z[3]);
            *reinterpret_cast<float4 *>(logits + (size_t)m * V + v0 + 4) = make_float4(z[4], z[5], z[6], z[7]);
        }
#pragma unroll
        for (int e = 7; e >= 0; --e)
            if (z[e] >= mx) { mx = z[e]; idx = v0 + e; }   // descending scan: the lowest index wins ties
#pragma unroll
        for (int e = 0; e < 8; ++e) sum += __expf(z[e] - mx);
    }
    s_m[tid] = mx; s_i[tid] = idx; s_s[tid] = sum;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {   // fixed tree; value first, then the lower index
        if (tid < o) {
            const float m2 = s_m[tid + o], m1 = s_m[tid];
            const int i2 = s_i[tid + o];
            const float M2 = fmaxf(m1, m2);
            const float a = m1 > -INFINITY ? s_s[tid] * __expf(m1 - M2) : 0.f, b = m2 > -INFINITY ? s_s[tid + o] * __expf(m2 - M2) : 0.f;
            if (m2 > m1 || (m2 == m1 && i2 < s_i[tid])) s_i[tid] = i2;
            s_m[tid] = M2; s_s[tid] = a + b;
        }
        __syncthreads();
    }
    if (tid == 0) slice_part[(size_t)blockIdx.x * M + m] = make_float4(s_m[0], __int_as_float(s_i[0]), s_s[0], 0.f);
}

void launch_lmhead_finish(hipStream_t s, const float *part, int nsplit, int M, int V, float *slice_part, float *logits)
{
    hipLaunchKernelGGL(lmhead_finish_kernel, dim3((V + LMHEAD_FINISH_COLS - 1) / LMHEAD_FINISH_COLS, M), dim3(256), 0, s, part, nsplit, M, V,
                       (float4 *)slice_part, logits);
}

void launch_qkv_finish(hipStream_t s, int kdt, const Dims &D, const float *part, int nsplit, const float *bias, Rows rows, const float2 *rope, float *q,
                       void *kc, void *vc)
{
    const int npairs = (D.Hq + 2 * D.Hkv) * (D.dh / 2);
    const dim3 grid((npairs + 255) / 256, rows.n);
    if (kdt == DT_F32)
        hipLaunchKernelGGL(qkv_finish_kernel<float>, grid, dim3(256), 0, s, D, part, nsplit, rows.n, bias, rows, rope, q, (float *)kc, (float *)vc);
    else
        hipLaunchKernelGGL(qkv_finish_kernel<bf16_t>, grid, dim3(256), 0, s, D, part, nsplit, rows.n, bias, rows, rope, q, (bf16_t *)kc, (bf16_t *)vc);
}

void launch_swiglu_finish(hipStream_t s, const Dims &D, const float *part, int nsplit, int M, void *hpack)
{
    hipLaunchKernelGGL(swiglu_finish_kernel, dim3((D.F / 8 + 255) / 256, M), dim3(256), 0, s, part, nsplit, M, D.F, (uint4 *)hpack, mfma_ncb(M));
}

// Tiles per workgroup, in units of `unit` tiles, for a launch that runs `copies` workgroups over every tile (row groups x
// splits): as few as possible while the whole launch is one round of at most 256 workgroups, all with the same share.
// With many 64-row groups (prefill, long catch-up segments) a workgroup therefore takes many tiles, and the activations
// it keeps in registers (229 KB for 64 rows of 896 columns) are fetched once for all of them.
static int tiles_per_workgroup(int n_tiles, int copies, int unit)
{
    const int units = (n_tiles + unit - 1) / unit;
    const int wgs_per_copy = copies >= 256 ? 1 : 256 / copies;
    return (units + wgs_per_copy - 1) / wgs_per_copy * unit;
}

// groups: 64-row groups of the launch (more of them: fewer splits are needed to fill the chip)
void plan_partial(int KS, int n_tiles, int groups, int *nsplit, int *ksw, int *tiles_per_wg)
{
    int S = (KS + NWAVES * MAXKW - 1) / (NWAVES * MAXKW);
    const int want = 128 / (n_tiles > 0 ? n_tiles * groups : 1);   // half the chip: every extra split is one more partial for the next kernel to add
    if (want > S) S = want;
    if (S > MAX_SPLITS) S = MAX_SPLITS;
    if (S > KS) S = KS;
    int w = (KS + S - 1) / S;
    S = (KS + w - 1) / w;
    *nsplit = S;
    *ksw = w;
    *tiles_per_wg = tiles_per_workgroup(n_tiles, S * groups, 1);
}

int gemm_partial_splits(int K, int N)
{
    int S, ksw, tpw;
    plan_partial(K / 16, (N + 31) / 32, 1, &S, &ksw, &tpw);   // one row group: the most splits any launch makes
    return S;
}

// floats of split-K partials a K x N layer may leave for any number of rows up to max_rows (few rows: many splits;
// many rows: only as many as K needs)
size_t gemm_partial_floats(int K, int N, int max_rows)
{
    size_t most = 0;
    for (int groups = 1; groups <= (max_rows + 63) / 64; ++groups) {
        int S, ksw, tpw;
        plan_partial(K / 16, (N + 31) / 32, groups, &S, &ksw, &tpw);
        most = std::max(most, (size_t)S * (size_t)std::min(max_rows, 64 * groups) * (size_t)N);
    }
    return most;
}

void launch_gemm_partial(hipStream_t s, const void *Wt, const void *pack, int K, int N, int M, float *part, int *nsplit_out, const int *live)
{
    GemmArgs a{};
    a.Wt = (const uint4 *)Wt; a.pack = (const uint4 *)pack; a.KS = K / 16; a.n_tiles = (N + 31) / 32; a.M = M; a.live = live;
    int S, ksw, tpw;
    plan_partial(a.KS, a.n_tiles, (M + 63) / 64, &S, &ksw, &tpw);
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
    a.tiles_per_wg = tiles_per_workgroup(a.n_tiles, rows.n > 32 ? 2 * ((rows.n + 63) / 64) : 1, 1);
    a.half = 1;
    a.live = rows.live;
    if (kdt == DT_F32) {
        EpiQkv<float> e{bias, rope, rows.slot, rows.pos, q, (float *)kc, (float *)vc, rows.n, D.Hq, D.Hkv, D.dh, kv_unit_len(D), D.qw, kv_unit_vts(D),
                        D.ptab, D.page, D.maxp, 0, 0, 0, rows.live};
        launch_gemm(s, a, 1, e);
    } else {
        EpiQkv<bf16_t> e{bias, rope, rows.slot, rows.pos, q, (bf16_t *)kc, (bf16_t *)vc, rows.n, D.Hq, D.Hkv, D.dh, kv_unit_len(D), D.qw, kv_unit_vts(D),
                         D.ptab, D.page, D.maxp, 0, 0, 0, rows.live};
        launch_gemm(s, a, 1, e);
    }
}

void launch_gemm_swiglu(hipStream_t s, const Dims &D, const void *Wt, const void *pack, int M, void *hpack, const int *live, const float *sumsq,
                        int n_ss, int ss_stride)
{
    GemmArgs a{};
    a.Wt = (const uint4 *)Wt; a.pack = (const uint4 *)pack; a.KS = D.d / 16; a.ksw = a.KS; a.n_tiles = 2 * ((D.F + 31) / 32); a.M = M; a.live = live;
    a.tiles_per_wg = tiles_per_workgroup(a.n_tiles, (M + 63) / 64, 2);   // whole gate/up pairs
    auto go = [&](auto e) {
        e.hpack = (uint4 *)hpack; e.M = M; e.F = D.F; e.ncb = mfma_ncb(M);
        e.sumsq = sumsq; e.n_ss = n_ss; e.ss_stride = ss_stride; e.eps = D.eps; e.inv_d = 1.0f / (float)D.d; e.rstd = 1.0f;
        launch_gemm(s, a, 1, e);
    };
    if (sumsq) { if (D.F % 32) go(EpiSwiglu<true, true>{}); else go(EpiSwiglu<false, true>{}); }
    else { if (D.F % 32) go(EpiSwiglu<true, false>{}); else go(EpiSwiglu<false, false>{}); }
}

int launch_gemm_oproj_residual(hipStream_t s, const Dims &D, const void *Wt, const void *pack_a, int M, float *x, const void *gain, void *pack_out,
                               float *sumsq, int ss_stride, const int *live)
{
    GemmArgs a{};
    a.Wt = (const uint4 *)Wt; a.pack = (const uint4 *)pack_a; a.KS = D.qw / 16; a.ksw = a.KS; a.n_tiles = (D.d + 31) / 32; a.M = M; a.live = live;
    a.tiles_per_wg = tiles_per_workgroup(a.n_tiles, M > 32 ? 2 * ((M + 63) / 64) : 1, 1);
    a.half = 1;
    EpiResidualNorm e{x, (const bf16_t *)gain, (uint4 *)pack_out, sumsq, M, D.d, mfma_ncb(M), ss_stride, 0, 0, 0.f};
    launch_gemm(s, a, 1, e);
    return (a.n_tiles + a.tiles_per_wg - 1) / a.tiles_per_wg;   // tile ranges = entries of sumsq per row
}

bool gemm_oproj_residual_supported(const Dims &D) { return D.qw / 16 <= NWAVES * MAXKW && (D.d + 31) / 32 <= 32; }   // one workgroup spans K; at most 32 tile ranges per row

// tiles per workgroup of the LM-head launch: the whole launch (every 64-row group over every tile) is one round of at most 256 workgroups
static int lmhead_tiles_per_wg(int n_tiles, int M)
{
    const int groups = (M + 63) / 64, per_group = groups >= 256 ? 1 : 256 / groups;
    return (n_tiles + per_group - 1) / per_group;
}

int lmhead_mfma_wgs(int V, int router_tiles, int M)
{
    const int n_tiles = (V + 31) / 32 + router_tiles;
    const int tpw = lmhead_tiles_per_wg(n_tiles, M);
    return (n_tiles + tpw - 1) / tpw;
}

void launch_gemm_lmhead(hipStream_t s, const Dims &D, const void *Wt, const void *pack, int M, float *part, float *logits, float *r1, int router_tiles,
                        const int *live)
{
    GemmArgs a{};
    a.live = live;
    const int vt = (D.V + 31) / 32;
    a.Wt = (const uint4 *)Wt; a.pack = (const uint4 *)pack; a.KS = D.d / 16; a.ksw = a.KS; a.n_tiles = vt + router_tiles; a.M = M;
    a.tiles_per_wg = lmhead_tiles_per_wg(a.n_tiles, M);
    a.remap_groups = M > 64 ? (M + 63) / 64 : 0;
    auto go = [&](auto e) {
        e.part = (float4 *)part; e.logits = logits; e.M = M; e.V = D.V; e.nwg = lmhead_mfma_wgs(D.V, router_tiles, M);
        e.r1 = r1; e.vt = router_tiles > 0 ? vt : 0x7fffffff; e.r1_stride = router_tiles * 32;
        launch_gemm(s, a, 1, e);
    };
    if (logits) { if (D.V % 32) go(EpiLmHead<true, true>{}); else go(EpiLmHead<true, false>{}); }
    else { if (D.V % 32) go(EpiLmHead<false, true>{}); else go(EpiLmHead<false, false>{}); }
}

}  // namespace tr
