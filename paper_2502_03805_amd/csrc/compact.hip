// Gather of the selected K/V rows into the compacted cache (Algorithm 1, line 10).
// Pure data movement: each row is dh * sizeof(elem) bytes, copied as 16-byte pieces by
// consecutive lanes so that both the read of a row and the write are contiguous.
#include "common.hpp"

namespace ckv {

constexpr int CP_THREADS = 256;

__global__ __launch_bounds__(CP_THREADS) void compact_kernel(const char *__restrict__ k, const char *__restrict__ v,
                                                             const int32_t *__restrict__ idx,
                                                             const int32_t *__restrict__ count, char *__restrict__ k_out,
                                                             char *__restrict__ v_out, int Hkv, int n, int max_budget,
                                                             int row_bytes, int64_t ks0, int64_t ks1, int64_t ks2,
                                                             int64_t vs0, int64_t vs1, int64_t vs2, int esize)
{
    const int head = blockIdx.y;            // bi * Hkv + g
    const int bi = head / Hkv, g = head % Hkv;
    const int pieces = row_bytes >> 4;      // 16-byte pieces per row
    const int cnt = min(count[head], max_budget);
    const long long t = (long long)blockIdx.x * CP_THREADS + threadIdx.x;
    const int j = (int)(t / pieces), piece = (int)(t % pieces);
    if (j >= cnt) return;
    const int i = idx[(size_t)head * max_budget + j];
    if (i < 0 || i >= n) return;
    // the K piece and the V piece of the same row: one index read, two loads in flight per lane
    const uint4 kk = reinterpret_cast<const uint4 *>(k + (bi * ks0 + g * ks1 + (int64_t)i * ks2) * esize)[piece];
    const uint4 vv = reinterpret_cast<const uint4 *>(v + (bi * vs0 + g * vs1 + (int64_t)i * vs2) * esize)[piece];
    const size_t o = ((size_t)head * max_budget + j) * (size_t)row_bytes;
    reinterpret_cast<uint4 *>(k_out + o)[piece] = kk;
    reinterpret_cast<uint4 *>(v_out + o)[piece] = vv;
}

hipError_t launch_compact(const Dims &d, int dtype, const void *k, const void *v, const int32_t *idx,
                          const int32_t *count, int max_budget, void *k_out, void *v_out, hipStream_t s)
{
    const int esize = dtype == CKV_F32 ? 4 : 2;
    const int row_bytes = d.dh * esize;
    const long long threads = (long long)max_budget * (row_bytes / 16);
    dim3 grid((unsigned)((threads + CP_THREADS - 1) / CP_THREADS), d.batch * d.Hkv);
    hipLaunchKernelGGL(compact_kernel, grid, dim3(CP_THREADS), 0, s, (const char *)k, (const char *)v, idx, count,
                       (char *)k_out, (char *)v_out, d.Hkv, d.n, max_budget, row_bytes, d.ks[0], d.ks[1], d.ks[2],
                       d.vs[0], d.vs[1], d.vs[2], esize);
    return hipGetLastError();
}

} // namespace ckv
