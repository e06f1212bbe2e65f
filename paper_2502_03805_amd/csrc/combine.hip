// Selection keys per kv head from the per-query-head scores
// (Algorithm 2 line 4: max-pool; Algorithm 1 line 3: (A + eps) * ||V W^O||_1).
//
//   abar^h_i = max{ a^h_j : |j - i| <= pool_k/2, 0 <= j < n }
//   attn[g,i] = (1/G) sum_{h in g} abar^h_i
//   crit[g,i] = (1/G) sum_{h in g} (abar^h_i + eps) * N^h_i      (= attn[g,i] when no magnitudes are given)
// Every output is computed by the same sequence of fp32 operations on its inputs, so
// entries whose pooled scores are equal get bitwise equal keys (ties stay ties).
#include "common.hpp"

namespace ckv {

constexpr int CB_THREADS = 256;
constexpr int CB_MAX_HALO = 31;

__global__ __launch_bounds__(CB_THREADS) void combine_kernel(const float *__restrict__ a_raw,
                                                             const float *__restrict__ vnorm, float *__restrict__ attn,
                                                             float *__restrict__ crit, int H, int G, int n, int radius,
                                                             float eps, int protect)
{
    __shared__ float tile[CB_THREADS + 2 * CB_MAX_HALO];
    const int g = blockIdx.y, bi = blockIdx.z;
    const int Hkv = H / G;
    const int i0 = blockIdx.x * CB_THREADS;
    const int i = i0 + threadIdx.x;
    float sum_a = 0.f, sum_c = 0.f;
    for (int j = 0; j < G; ++j) {
        const size_t row = ((size_t)bi * H + (size_t)g * G + j) * (size_t)n;
        __syncthreads();
        for (int e = threadIdx.x; e < CB_THREADS + 2 * radius; e += CB_THREADS) {
            const int src = i0 - radius + e;
            tile[e] = (src >= 0 && src < n) ? a_raw[row + src] : -INFINITY;
        }
        __syncthreads();
        float m = tile[threadIdx.x];
        for (int r = 1; r <= 2 * radius; ++r) m = fmaxf(m, tile[threadIdx.x + r]);
        if (i < n) {
            sum_a += m;
            sum_c += vnorm ? (m + eps) * vnorm[row + i] : m; // no magnitudes: crit = attn
        }
    }
    if (i < n) {
        const size_t o = ((size_t)bi * Hkv + g) * (size_t)n + i;
        const bool forced = i >= n - protect; // the window's own tokens, when they are to be kept
        attn[o] = forced ? 3.402823466e+38f : sum_a / (float)G;
        crit[o] = forced ? 3.402823466e+38f : sum_c / (float)G;
    }
}

hipError_t launch_combine(const Dims &d, const float *a_raw, const float *vnorm, float *attn, float *crit, hipStream_t s)
{
    dim3 grid((d.n + CB_THREADS - 1) / CB_THREADS, d.Hkv, d.batch);
    hipLaunchKernelGGL(combine_kernel, grid, dim3(CB_THREADS), 0, s, a_raw, vnorm, attn, crit, d.H, d.G, d.n,
                       d.pool_k / 2, d.eps, d.protect);
    return hipGetLastError();
}

} // namespace ckv
