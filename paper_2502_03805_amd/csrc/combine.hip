// Selection keys per kv head from the per-query-head scores
// (Algorithm 2 line 4: max-pool; Algorithm 1 line 3: (A + eps) * ||V W^O||_1).
//
//   abar^h_i = max{ a^h_j : |j - i| <= pool_k/2, 0 <= j < n }
//   attn[g,i] = (1/G) sum_{h in g} abar^h_i
//   crit[g,i] = (1/G) sum_{h in g} (abar^h_i + eps) * N^h_i      (= attn[g,i] when no magnitudes are given)
// Either output pointer may be null (that array is then not written).
// Every output is computed by the same sequence of fp32 operations on its inputs, so
// entries whose pooled scores are equal get bitwise equal keys (ties stay ties).
#include "common.hpp"

namespace ckv {

constexpr int CB_THREADS = 256;
constexpr int CB_MAX_HALO = 31;
constexpr int CB_HEADS = 8; // query heads of a group staged together (larger groups: several rounds)

__global__ __launch_bounds__(CB_THREADS) void combine_kernel(const float *__restrict__ a_raw,
                                                             const float *__restrict__ vnorm, float *__restrict__ attn,
                                                             float *__restrict__ crit, int H, int G, int n, int radius,
                                                             float eps)
{
    __shared__ float tile[CB_HEADS][CB_THREADS + 2 * CB_MAX_HALO];
    const int g = blockIdx.y, bi = blockIdx.z;
    const int Hkv = H / G;
    const int i0 = blockIdx.x * CB_THREADS;
    const int i = i0 + threadIdx.x;
    const int ic = min(i, n - 1); // clamped: no load sits under a branch
    float sum_a = 0.f, sum_c = 0.f;
    for (int j0 = 0; j0 < G; j0 += CB_HEADS) { // one round for groups of up to CB_HEADS heads
        const int heads = min(CB_HEADS, G - j0);
        // Every load of the round is issued before anything waits for one: per head a thread reads its own token's
        // score, one halo element (the first 2 * radius threads; the others re-read their own, so that the load
        // needs no branch) and its token's magnitude.  Positions outside the row read a clamped address and
        // count as -inf.
        const int e1 = (int)threadIdx.x < 2 * radius ? CB_THREADS + (int)threadIdx.x : (int)threadIdx.x;
        const int src0 = i0 - radius + (int)threadIdx.x, src1 = i0 - radius + e1;
        const int c0 = min(max(src0, 0), n - 1), c1 = min(max(src1, 0), n - 1);
        float x0[CB_HEADS], x1[CB_HEADS], nv[CB_HEADS];
#pragma unroll
        for (int j = 0; j < CB_HEADS; ++j) {
            x0[j] = x1[j] = nv[j] = 0.f;
            if (j < heads) { // uniform
                const size_t row = ((size_t)bi * H + (size_t)g * G + j0 + j) * (size_t)n;
                x0[j] = a_raw[row + c0];
                x1[j] = a_raw[row + c1];
                if (vnorm) nv[j] = vnorm[row + ic];
            }
        }
        __syncthreads(); // the previous round's tiles have been read
#pragma unroll
        for (int j = 0; j < CB_HEADS; ++j)
            if (j < heads) {
                tile[j][threadIdx.x] = (src0 >= 0 && src0 < n) ? x0[j] : -INFINITY;
                if ((int)threadIdx.x < 2 * radius) tile[j][e1] = (src1 >= 0 && src1 < n) ? x1[j] : -INFINITY;
            }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < CB_HEADS; ++j)
            if (j < heads) { // uniform; heads are added in ascending order, as a one-head-at-a-time loop would
                float m = tile[j][threadIdx.x];
                for (int r = 1; r <= 2 * radius; ++r) m = fmaxf(m, tile[j][threadIdx.x + r]);
                sum_a += m;
                sum_c += vnorm ? (m + eps) * nv[j] : m; // no magnitudes: crit = attn
            }
    }
    if (i < n) {
        const size_t o = ((size_t)bi * Hkv + g) * (size_t)n + i;
        if (attn) attn[o] = sum_a / (float)G;
        if (crit) crit[o] = sum_c / (float)G;
    }
}

hipError_t launch_combine(const Dims &d, const float *a_raw, const float *vnorm, float *attn, float *crit, hipStream_t s)
{
    dim3 grid((d.n + CB_THREADS - 1) / CB_THREADS, d.Hkv, d.batch);
    hipLaunchKernelGGL(combine_kernel, grid, dim3(CB_THREADS), 0, s, a_raw, vnorm, attn, crit, d.H, d.G, d.n,
                       d.pool_k / 2, d.eps);
    return hipGetLastError();
}

} // namespace ckv
