// Observation-window attention on the vector ALUs (Algorithm 2, lines 2-3; eq. (2)).
//
// These kernels serve fp32 inputs and head sizes the matrix-core kernels do not cover.
// The softmax over all n keys needs each window row's max and sum before any weight can
// be summed over the window, so the keys are swept twice:
//   pass 1  per (query head, key chunk): row-wise max and sum of exp over the chunk
//   reduce  per window row: merge the chunk partials to (max, 1 / sum [/ W])
//   pass 2  per key: a_i = sum_w exp(s_wi - max_w) * inv_w
// One thread owns one key (its row stays in registers); the window queries of the head sit
// in LDS, GEN_WB rows at a time, and are read as broadcasts.
#include "common.hpp"

namespace ckv {

constexpr int GEN_THREADS = 256; // keys per workgroup of the generic attention kernels
constexpr int GEN_WB = 64;       // window rows staged in LDS at a time (longer windows take several rounds)

template <typename T> struct Vec16;
template <> struct Vec16<float> { static constexpr int N = 4; };
template <> struct Vec16<bf16_t> { static constexpr int N = 8; };

// Loads a DH-element row into fp32 registers with 16-byte loads.
template <typename T, int DH> __device__ __forceinline__ void load_row(const T *p, float (&r)[DH])
{
    constexpr int N = Vec16<T>::N;
#pragma unroll
    for (int c = 0; c < DH / N; ++c) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(p + c * N);
        if constexpr (N == 4) {
            r[c * 4 + 0] = __uint_as_float(raw.x); r[c * 4 + 1] = __uint_as_float(raw.y);
            r[c * 4 + 2] = __uint_as_float(raw.z); r[c * 4 + 3] = __uint_as_float(raw.w);
        } else {
            const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                r[c * 8 + 2 * j] = __uint_as_float(u[j] << 16);
                r[c * 8 + 2 * j + 1] = __uint_as_float(u[j] & 0xFFFF0000u);
            }
        }
    }
}

template <int DH> __device__ __forceinline__ float dot_lds(const float *q, const float (&k)[DH])
{
    float acc = 0.f;
#pragma unroll
    for (int t = 0; t < DH; t += 4) {
        const float4 qq = *reinterpret_cast<const float4 *>(q + t);
        acc = fmaf(qq.x, k[t], acc); acc = fmaf(qq.y, k[t + 1], acc);
        acc = fmaf(qq.z, k[t + 2], acc); acc = fmaf(qq.w, k[t + 3], acc);
    }
    return acc;
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

// Stages the W window queries of head (bi, h) into LDS as fp32.
template <typename T, int DH>
__device__ __forceinline__ void stage_queries(const T *q, int W, float *q_lds)
{
    for (int e = threadIdx.x; e < W * DH; e += blockDim.x) q_lds[e] = to_f32(q[e]);
}

template <typename T, int DH>
__global__ __launch_bounds__(GEN_THREADS) void attn_stats_generic_kernel(
    const T *__restrict__ q, const T *__restrict__ k, float *__restrict__ part, int H, int G, int n, int W,
    int chunks, float scale, int64_t ks0, int64_t ks1, int64_t ks2, int causal)
{
    extern __shared__ float smem[];
    float *q_lds = smem;                      // [GEN_WB][DH]
    float *red = smem + (size_t)GEN_WB * DH;  // [GEN_WB][4] wave maxima, then [GEN_WB][4] wave sums
    const int chunk = blockIdx.x, h = blockIdx.y, bi = blockIdx.z;
    const int g = h / G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int i = chunk * GEN_THREADS + threadIdx.x;
    const bool valid = i < n;
    // with the causal tail, key i is seen by window rows w >= i - (n - W) only
    const int first_w = causal ? max(0, i - (n - W)) : 0;
    float kr[DH];
    load_row<T, DH>(k + bi * ks0 + g * ks1 + (int64_t)(valid ? i : n - 1) * ks2, kr);
    for (int w0 = 0; w0 < W; w0 += GEN_WB) { // the window in rounds of GEN_WB rows
        const int wb = min(GEN_WB, W - w0);
        stage_queries<T, DH>(q + (((size_t)bi * H + h) * (size_t)W + w0) * DH, wb, q_lds);
        __syncthreads();
        for (int w = 0; w < wb; ++w) {
            const float s = (valid && w0 + w >= first_w) ? scale * dot_lds<DH>(q_lds + w * DH, kr) : -INFINITY;
            const float m = wave_max(s);
            if (lane == 0) red[w * 4 + wave] = m;
        }
        __syncthreads();
        for (int w = 0; w < wb; ++w) {
            // a chunk may hold no visible key for this row (max = -inf): its partial sum is 0
            const float m = fmaxf(fmaxf(fmaxf(red[w * 4], red[w * 4 + 1]), fmaxf(red[w * 4 + 2], red[w * 4 + 3])), -1.0e30f);
            const bool seen = valid && w0 + w >= first_w;
            const float s = seen ? scale * dot_lds<DH>(q_lds + w * DH, kr) : -INFINITY;
            const float e = wave_sum(seen ? __expf(s - m) : 0.f);
            if (lane == 0) red[GEN_WB * 4 + w * 4 + wave] = e;
        }
        __syncthreads();
        for (int w = threadIdx.x; w < wb; w += GEN_THREADS) {
            const float m = fmaxf(fmaxf(fmaxf(red[w * 4], red[w * 4 + 1]), fmaxf(red[w * 4 + 2], red[w * 4 + 3])), -1.0e30f);
            const float l = red[GEN_WB * 4 + w * 4] + red[GEN_WB * 4 + w * 4 + 1] + red[GEN_WB * 4 + w * 4 + 2] +
                            red[GEN_WB * 4 + w * 4 + 3];
            float *dst = part + ((((size_t)bi * H + h) * W + w0 + w) * (size_t)chunks + chunk) * 2;
            dst[0] = m;
            dst[1] = l;
        }
        __syncthreads(); // the next round overwrites the staged queries and the partials
    }
}

// One wave per window row: (max, sum) partials over chunks -> (max, weight) with
// weight = 1 / sum, divided by W as well when the window is averaged.
__global__ __launch_bounds__(64) void attn_stats_reduce_kernel(const float *__restrict__ part, float *__restrict__ stats,
                                                               int chunks, float post)
{
    const size_t row = blockIdx.x;
    const float *p = part + row * (size_t)chunks * 2;
    float m = -INFINITY;
    for (int c = threadIdx.x; c < chunks; c += 64) m = fmaxf(m, p[2 * c]);
    m = wave_max(m);
    float l = 0.f;
    for (int c = threadIdx.x; c < chunks; c += 64) l += p[2 * c + 1] * __expf(p[2 * c] - m);
    l = wave_sum(l);
    if (threadIdx.x == 0) {
        stats[row * 2] = m;
        stats[row * 2 + 1] = post / l;
    }
}

template <typename T, int DH>
__global__ __launch_bounds__(GEN_THREADS) void attn_colsum_generic_kernel(
    const T *__restrict__ q, const T *__restrict__ k, const float *__restrict__ stats, float *__restrict__ a_raw,
    int H, int G, int n, int W, float scale, int64_t ks0, int64_t ks1, int64_t ks2, int causal)
{
    extern __shared__ float smem[];
    float *q_lds = smem;                       // [GEN_WB][DH]
    float *st = smem + (size_t)GEN_WB * DH;    // [GEN_WB][2]
    const int chunk = blockIdx.x, h = blockIdx.y, bi = blockIdx.z;
    const int g = h / G;
    const int i = chunk * GEN_THREADS + threadIdx.x;
    const bool valid = i < n;
    float kr[DH];
    load_row<T, DH>(k + bi * ks0 + g * ks1 + (int64_t)(valid ? i : n - 1) * ks2, kr);
    const int first_w = causal ? max(0, i - (n - W)) : 0;
    float acc = 0.f;
    for (int w0 = 0; w0 < W; w0 += GEN_WB) { // the window in rounds of GEN_WB rows, rows added in ascending order
        const int wb = min(GEN_WB, W - w0);
        stage_queries<T, DH>(q + (((size_t)bi * H + h) * (size_t)W + w0) * DH, wb, q_lds);
        for (int e = threadIdx.x; e < 2 * wb; e += blockDim.x) st[e] = stats[(((size_t)bi * H + h) * (size_t)W + w0) * 2 + e];
        __syncthreads();
        for (int w = max(0, first_w - w0); w < wb; ++w) {
            const float s = scale * dot_lds<DH>(q_lds + w * DH, kr);
            acc += __expf(s - st[2 * w]) * st[2 * w + 1];
        }
        __syncthreads(); // the next round overwrites the staged queries
    }
    if (valid) a_raw[((size_t)bi * H + h) * (size_t)n + i] = acc;
}

template <typename T, int DH>
static hipError_t stats_generic_t(const Dims &d, const void *q, const void *k, float *part, int chunks, hipStream_t s)
{
    const size_t lds = ((size_t)GEN_WB * DH + (size_t)GEN_WB * 8) * sizeof(float);
    dim3 grid(chunks, d.H, d.batch);
    hipLaunchKernelGGL((attn_stats_generic_kernel<T, DH>), grid, dim3(GEN_THREADS), lds, s, (const T *)q, (const T *)k,
                       part, d.H, d.G, d.n, d.W, chunks, d.scale, d.ks[0], d.ks[1], d.ks[2], d.causal);
    return hipGetLastError();
}

template <typename T, int DH>
static hipError_t colsum_generic_t(const Dims &d, const void *q, const void *k, const float *stats, float *a_raw,
                                   hipStream_t s)
{
    const size_t lds = ((size_t)GEN_WB * DH + (size_t)GEN_WB * 2) * sizeof(float);
    dim3 grid((d.n + GEN_THREADS - 1) / GEN_THREADS, d.H, d.batch);
    hipLaunchKernelGGL((attn_colsum_generic_kernel<T, DH>), grid, dim3(GEN_THREADS), lds, s, (const T *)q,
                       (const T *)k, stats, a_raw, d.H, d.G, d.n, d.W, d.scale, d.ks[0], d.ks[1], d.ks[2], d.causal);
    return hipGetLastError();
}

int generic_attn_chunks(const Dims &d) { return (d.n + GEN_THREADS - 1) / GEN_THREADS; }

hipError_t launch_attn_stats_generic(const Dims &d, int dtype, const void *q, const void *k, float *part, int chunks,
                                     hipStream_t s)
{
    if (dtype == CKV_F32)
        return d.dh == 64 ? stats_generic_t<float, 64>(d, q, k, part, chunks, s)
                          : stats_generic_t<float, 128>(d, q, k, part, chunks, s);
    return d.dh == 64 ? stats_generic_t<bf16_t, 64>(d, q, k, part, chunks, s)
                      : stats_generic_t<bf16_t, 128>(d, q, k, part, chunks, s);
}

hipError_t launch_attn_stats_reduce(const Dims &d, const float *part, int chunks, float *stats, hipStream_t s)
{
    const size_t rows = (size_t)d.batch * d.H * d.W;
    const float post = d.window_sum ? 1.0f : 1.0f / (float)d.W;
    hipLaunchKernelGGL(attn_stats_reduce_kernel, dim3((unsigned)rows), dim3(64), 0, s, part, stats, chunks, post);
    return hipGetLastError();
}

hipError_t launch_attn_colsum_generic(const Dims &d, int dtype, const void *q, const void *k, const float *stats,
                                      float *a_raw, hipStream_t s)
{
    if (dtype == CKV_F32)
        return d.dh == 64 ? colsum_generic_t<float, 64>(d, q, k, stats, a_raw, s)
                          : colsum_generic_t<float, 128>(d, q, k, stats, a_raw, s);
    return d.dh == 64 ? colsum_generic_t<bf16_t, 64>(d, q, k, stats, a_raw, s)
                      : colsum_generic_t<bf16_t, 128>(d, q, k, stats, a_raw, s);
}

} // namespace ckv
