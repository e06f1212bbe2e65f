// Per-entry L1 (or L2) magnitude of the projected value on the vector ALUs
// (Theorem 3.3; Algorithm 1, lines 2-3):  N^h_i = sum_c | sum_t V^g[i,t] * W_O^h[t,c] |.
//
// Serves fp32 inputs and head sizes the matrix-core kernel does not cover.  One thread owns
// one token row (kept in registers); the head's W_O slice is streamed through LDS in tiles
// of TC output columns and read as broadcasts.  The n x d_model products are reduced on the
// fly and never stored.
#include "common.hpp"

namespace ckv {

constexpr int VG_THREADS = 256;
constexpr int VG_TC = 32; // output columns per LDS tile

template <typename T, int DH, bool L2>
__global__ __launch_bounds__(VG_THREADS) void vproj_generic_kernel(const T *__restrict__ v, const T *__restrict__ w_t,
                                                                   float *__restrict__ vnorm, int H, int G, int n,
                                                                   int dm, int64_t vs0, int64_t vs1, int64_t vs2)
{
    __shared__ float w_lds[VG_TC * DH];
    const int h = blockIdx.y, bi = blockIdx.z, g = h / G;
    const int i = blockIdx.x * VG_THREADS + threadIdx.x;
    const bool valid = i < n;
    const T *row = v + bi * vs0 + g * vs1 + (int64_t)(valid ? i : n - 1) * vs2;
    float vr[DH];
#pragma unroll
    for (int t = 0; t < DH; ++t) vr[t] = to_f32(row[t]);
    const size_t ldw = (size_t)H * DH; // row pitch of w_t [dm, H*DH]
    float acc = 0.f;
    for (int c0 = 0; c0 < dm; c0 += VG_TC) {
        __syncthreads();
        for (int e = threadIdx.x; e < VG_TC * DH; e += VG_THREADS) {
            const int c = e / DH, t = e % DH;
            w_lds[e] = to_f32(w_t[(size_t)(c0 + c) * ldw + (size_t)h * DH + t]);
        }
        __syncthreads();
#pragma unroll 4
        for (int c = 0; c < VG_TC; ++c) {
            float p = 0.f;
#pragma unroll
            for (int t = 0; t < DH; t += 4) {
                const float4 ww = *reinterpret_cast<const float4 *>(&w_lds[c * DH + t]);
                p = fmaf(vr[t], ww.x, p); p = fmaf(vr[t + 1], ww.y, p);
                p = fmaf(vr[t + 2], ww.z, p); p = fmaf(vr[t + 3], ww.w, p);
            }
            acc += L2 ? p * p : fabsf(p);
        }
    }
    if (valid) vnorm[((size_t)bi * H + h) * (size_t)n + i] = L2 ? sqrtf(acc) : acc;
}

template <typename T, int DH>
static hipError_t vproj_generic_t(const Dims &d, const void *v, const void *w_t, float *vnorm, hipStream_t s)
{
    dim3 grid((d.n + VG_THREADS - 1) / VG_THREADS, d.H, d.batch);
    if (d.norm == CKV_NORM_L2)
        hipLaunchKernelGGL((vproj_generic_kernel<T, DH, true>), grid, dim3(VG_THREADS), 0, s, (const T *)v, (const T *)w_t,
                           vnorm, d.H, d.G, d.n, d.dm, d.vs[0], d.vs[1], d.vs[2]);
    else
        hipLaunchKernelGGL((vproj_generic_kernel<T, DH, false>), grid, dim3(VG_THREADS), 0, s, (const T *)v, (const T *)w_t,
                           vnorm, d.H, d.G, d.n, d.dm, d.vs[0], d.vs[1], d.vs[2]);
    return hipGetLastError();
}

hipError_t launch_vproj_generic(const Dims &d, int dtype, const void *v, const void *w_t, float *vnorm, hipStream_t s)
{
    if (dtype == CKV_F32)
        return d.dh == 64 ? vproj_generic_t<float, 64>(d, v, w_t, vnorm, s) : vproj_generic_t<float, 128>(d, v, w_t, vnorm, s);
    return d.dh == 64 ? vproj_generic_t<bf16_t, 64>(d, v, w_t, vnorm, s) : vproj_generic_t<bf16_t, 128>(d, v, w_t, vnorm, s);
}

// ---- W_O layout change: [H*dh, d_model] -> [d_model, H*dh] ---------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ in, T *__restrict__ out, int rows, int cols)
{
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5; // 32 x 8
    const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
    for (int j = ty; j < 32; j += 8)
        if (r0 + j < rows && c0 + tx < cols) tile[j][tx] = in[(size_t)(r0 + j) * cols + c0 + tx];
    __syncthreads();
    for (int j = ty; j < 32; j += 8)
        if (c0 + j < cols && r0 + tx < rows) out[(size_t)(c0 + j) * rows + r0 + tx] = tile[tx][j];
}

hipError_t launch_transpose_wo(const Dims &d, int dtype, const void *w_o, void *w_t, hipStream_t s)
{
    const int rows = d.H * d.dh, cols = d.dm;
    dim3 grid((cols + 31) / 32, (rows + 31) / 32);
    if (dtype == CKV_F32)
        hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, s, (const float *)w_o, (float *)w_t, rows, cols);
    else
        hipLaunchKernelGGL(transpose_kernel<bf16_t>, grid, dim3(256), 0, s, (const bf16_t *)w_o, (bf16_t *)w_t, rows, cols);
    return hipGetLastError();
}

} // namespace ckv
