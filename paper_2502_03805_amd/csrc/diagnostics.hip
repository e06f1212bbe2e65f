// Perturbation quantities of a finished selection, per (batch item, query head)
// (Definition 3.1; Theorems 3.2, 3.3, 3.5, 3.6; Assumption 3.4).
//
// With A the head's window-mean attention (unpooled, sums to 1), N_i the projected-value norm, S the
// selected set and S1 its stage-1 part:
//   sigma = sum_{S1} A_i, s = sum_S A_i, C = sum_i A_i N_i, M = min_i N_i,
//   theta (Thm 3.3), theta_hat (Thm 3.5), theta_relax (Thm 3.6) from those sums, and
//   L = || sum_i (A_i - A'_i) (V W_O)_i || with A' = A restricted to S and renormalised (Thm 3.2).
// The projection is linear, so  sum_i (A_i - A'_i) v_i W_O = (u_all - u_S / s) W_O  with the d_h-vectors
// u_all = sum_i A_i v_i and u_S = sum_{S} A_i v_i: V is read once per kv head (plus the selected rows once
// more) and W_O once per query head, instead of materialising V W_O.
//
//   sweep     128 workgroups per kv head, each over every 128th 256-token chunk: partial u_all, C, M for the
//             group's query heads
//   selected  the same over the head's index list: partial u_S and the four sums over S1 / S2; stage-1
//             membership is read from the selection's stage-2 key array
//   finish    one workgroup per query head: the 128 partials summed in double in a fixed order, the
//             d_h x d matrix-vector product, the norm of the result and the closed forms
#include "common.hpp"

namespace ckv {

constexpr int DG_THREADS = 256;
constexpr int DG_CHUNK = 256;  // == DG_THREADS: a thread stages one token of a chunk
constexpr int DG_PARTS = 128;  // workgroups (and partial sums) per head
constexpr int DG_GMAX = 8; // query heads of a group handled by one workgroup (more: blockIdx.z)
constexpr uint32_t DG_TAKEN = 0xFFFFFFFFu; // the selection's mark for stage-1 entries in its stage-2 keys

struct DiagArgs {
    const float *a_raw;   // [batch, H, n]
    const float *vnorm;   // [batch, H, n]
    const uint32_t *keys2; // [batch*Hkv, n]
    const int32_t *idx;   // [batch*Hkv, max_budget]
    const int32_t *count; // [batch*Hkv]
    const void *v;
    float *part_all;      // [batch*H][DG_PARTS][dh + 2]: u_all, C, M
    float *part_sel;      // [batch*H][DG_PARTS][dh + 4]: u_S, sigma, s2, D1, D2
    int H, Hkv, G, dh, n, max_budget;
    float a_scale;        // 1, or 1/W when the stored score is the window sum
    int64_t vs0, vs1, vs2;
};

__device__ __forceinline__ double block_sum_f64(double x, double *sh)
{
    __syncthreads();
    sh[threadIdx.x] = x;
    __syncthreads();
    for (int o = DG_THREADS / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    return sh[0];
}

__device__ __forceinline__ float block_sum_f32(float x, float *sh)
{
    __syncthreads();
    sh[threadIdx.x] = x;
    __syncthreads();
    for (int o = DG_THREADS / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    return sh[0];
}

__device__ __forceinline__ float block_min_f32(float x, float *sh)
{
    __syncthreads();
    sh[threadIdx.x] = x;
    __syncthreads();
    for (int o = DG_THREADS / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] = fminf(sh[threadIdx.x], sh[threadIdx.x + o]);
        __syncthreads();
    }
    return sh[0];
}

// 8 consecutive elements of a row as floats (rows start on 16-byte boundaries, groups of 8 stay aligned)
__device__ __forceinline__ void load8_f32(const bf16_t *p, float (&x)[8])
{
    const uint4 r = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = __uint_as_float(w[e] << 16);
        x[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
    }
}
__device__ __forceinline__ void load8_f32(const float *p, float (&x)[8])
{
    const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}

// SELECTED = false: the head's tokens.  SELECTED = true: the entries j of its index list.
// Workgroup `part` of a head takes the 256-element chunks part, part + DG_PARTS, ... and writes one partial.
template <typename T, bool SELECTED>
__global__ __launch_bounds__(DG_THREADS) void diag_partial_kernel(DiagArgs A)
{
    __shared__ float a_s[DG_GMAX][DG_CHUNK];   // A of the chunk's tokens, per query head of the group
    __shared__ int tok_s[DG_CHUNK];            // token index (-1 = skip)
    __shared__ unsigned char st1_s[DG_CHUNK];  // SELECTED: taken in stage 1
    __shared__ float red_s[DG_THREADS];
    __shared__ float u_s[DG_THREADS * 8];      // [row lanes][dh]

    const int part = blockIdx.x, head = blockIdx.y; // head = bi * Hkv + g
    const int bi = head / A.Hkv, g = head % A.Hkv;
    const int hh0 = blockIdx.z * DG_GMAX, gc = min(DG_GMAX, A.G - hh0);
    const int h0 = g * A.G + hh0;                                    // first query head handled here
    const int limit = SELECTED ? min(max(A.count[head], 0), A.max_budget) : A.n;
    const int chunks = (limit + DG_CHUNK - 1) / DG_CHUNK;

    // thread = (row lane, group of 8 columns) for the value sums: one 16-byte (bf16) or 32-byte (f32) load per row
    const int groups = A.dh >> 3, cg = threadIdx.x % groups, lane = threadIdx.x / groups, lanes = DG_THREADS / groups;
    const T *vb = reinterpret_cast<const T *>(A.v) + bi * A.vs0 + g * A.vs1 + cg * 8;
    float acc[DG_GMAX][8];
    float sc[DG_GMAX][4]; // SELECTED: sigma, s2, D1, D2; else C, min N
#pragma unroll
    for (int hh = 0; hh < DG_GMAX; ++hh) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
        sc[hh][0] = sc[hh][2] = sc[hh][3] = 0.0f;
        sc[hh][1] = SELECTED ? 0.0f : INFINITY;
    }

    for (int chunk = part; chunk < chunks; chunk += DG_PARTS) { // uniform over the workgroup
        const int j0 = chunk * DG_CHUNK;
        const int len = min(DG_CHUNK, limit - j0);
        __syncthreads(); // the previous chunk's staging is no longer read
        {
            const int jj = threadIdx.x; // DG_CHUNK == DG_THREADS
            int i = -1;
            unsigned char st1 = 0;
            if (jj < len) {
                if (SELECTED) {
                    i = A.idx[(size_t)head * A.max_budget + j0 + jj];
                    if (i < 0 || i >= A.n) i = -1;
                    else st1 = A.keys2[(size_t)head * A.n + i] == DG_TAKEN;
                } else {
                    i = j0 + jj;
                }
            }
            tok_s[jj] = i;
            st1_s[jj] = st1;
#pragma unroll
            for (int hh = 0; hh < DG_GMAX; ++hh)
                if (hh < gc) {
                    const float a = i >= 0 ? A.a_raw[((size_t)bi * A.H + h0 + hh) * A.n + i] * A.a_scale : 0.0f;
                    a_s[hh][jj] = a;
                    // scalar sums: this thread's own token
                    if (i >= 0) {
                        const float N = A.vnorm[((size_t)bi * A.H + h0 + hh) * A.n + i];
                        if (SELECTED) {
                            if (st1) { sc[hh][0] += a; sc[hh][2] += a * N; } else { sc[hh][1] += a; sc[hh][3] += a * N; }
                        } else {
                            sc[hh][0] += a * N;
                            sc[hh][1] = fminf(sc[hh][1], N);
                        }
                    }
                }
        }
        __syncthreads();
#pragma unroll 8
        for (int jj = lane; jj < len; jj += lanes) {
            const int i = tok_s[jj];
            float x[8];
            if (i >= 0) load8_f32(vb + (int64_t)i * A.vs2, x);
            else {
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = 0.0f;
            }
#pragma unroll
            for (int hh = 0; hh < DG_GMAX; ++hh)
                if (hh < gc) {
                    const float a = a_s[hh][jj];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[hh][e] += a * x[e];
                }
        }
    }

    // one partial per (query head, part): scalars, then the d_h value sums (row lanes merged through LDS)
#pragma unroll
    for (int hh = 0; hh < DG_GMAX; ++hh) {
        if (hh < gc) { // uniform over the workgroup
            const size_t slot = ((size_t)bi * A.H + h0 + hh) * DG_PARTS + part;
            float *dst = SELECTED ? A.part_sel + slot * (A.dh + 4) : A.part_all + slot * (A.dh + 2);
            const float c0 = block_sum_f32(sc[hh][0], red_s);
            if (SELECTED) {
                const float c1 = block_sum_f32(sc[hh][1], red_s);
                const float c2 = block_sum_f32(sc[hh][2], red_s);
                const float c3 = block_sum_f32(sc[hh][3], red_s);
                if (threadIdx.x == 0) { dst[A.dh] = c0; dst[A.dh + 1] = c1; dst[A.dh + 2] = c2; dst[A.dh + 3] = c3; }
            } else {
                const float mn = block_min_f32(sc[hh][1], red_s);
                if (threadIdx.x == 0) { dst[A.dh] = c0; dst[A.dh + 1] = mn; }
            }
            __syncthreads();
#pragma unroll
            for (int e = 0; e < 8; ++e) u_s[lane * A.dh + cg * 8 + e] = acc[hh][e];
            __syncthreads();
            if ((int)threadIdx.x < A.dh) {
                float sum = 0.0f;
                for (int l = 0; l < lanes; ++l) sum += u_s[l * A.dh + threadIdx.x];
                dst[threadIdx.x] = sum;
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(DG_THREADS) void diag_finish_kernel(DiagArgs A, const void *w_o, int dm, int out_in,
                                                                 int norm, float *out)
{
    __shared__ double red_s[DG_THREADS];
    __shared__ double diff_s[128];
    __shared__ double scal_s[8];
    const int bh = blockIdx.x; // bi * H + h
    const int bi = bh / A.H, h = bh % A.H, g = h / A.G;
    const int head = bi * A.Hkv + g;
    (void)head;
    const float *pa = A.part_all + (size_t)bh * DG_PARTS * (A.dh + 2);
    const float *ps = A.part_sel + (size_t)bh * DG_PARTS * (A.dh + 4);

    if (threadIdx.x < 6) {
        // 0: C  1: M  2: sigma  3: s2  4: D1  5: D2 -- each summed over the parts in ascending order
        const int q = threadIdx.x;
        double acc = q == 1 ? (double)INFINITY : 0.0;
        if (q < 2) {
            for (int c = 0; c < DG_PARTS; ++c) {
                const double x = (double)pa[(size_t)c * (A.dh + 2) + A.dh + q];
                acc = q == 1 ? fmin(acc, x) : acc + x;
            }
        } else {
            for (int c = 0; c < DG_PARTS; ++c) acc += (double)ps[(size_t)c * (A.dh + 4) + A.dh + (q - 2)];
        }
        scal_s[q] = acc;
    }
    __syncthreads();
    const double C = scal_s[0], M = scal_s[1], sigma = scal_s[2], s2 = scal_s[3], D1 = scal_s[4], D2 = scal_s[5];
    const double s = sigma + s2;
    if ((int)threadIdx.x < A.dh) {
        double ua = 0.0, us = 0.0;
        for (int c = 0; c < DG_PARTS; ++c) ua += (double)pa[(size_t)c * (A.dh + 2) + threadIdx.x];
        for (int c = 0; c < DG_PARTS; ++c) us += (double)ps[(size_t)c * (A.dh + 4) + threadIdx.x];
        diff_s[threadIdx.x] = s > 0.0 ? ua - us / s : ua;
    }
    __syncthreads();
    // y = diff W_O^h, then its norm
    const T *w = reinterpret_cast<const T *>(w_o);
    double part = 0.0;
    for (int m = threadIdx.x; m < dm; m += DG_THREADS) {
        double y = 0.0;
        if (out_in) {
            const T *row = w + (size_t)m * ((size_t)A.H * A.dh) + (size_t)h * A.dh; // 16-byte aligned: dh is a multiple of 64
            for (int c = 0; c < A.dh; c += 8) {
                float x[8];
                load8_f32(row + c, x);
#pragma unroll
                for (int e = 0; e < 8; ++e) y += diff_s[c + e] * (double)x[e];
            }
        } else {
            const T *colp = w + (size_t)h * A.dh * dm + m;
            for (int c = 0; c < A.dh; ++c) y += diff_s[c] * (double)to_f32(colp[(size_t)c * dm]);
        }
        part += norm == CKV_NORM_L2 ? y * y : fabs(y);
    }
    double L = block_sum_f64(part, red_s);
    if (norm == CKV_NORM_L2) L = sqrt(L);
    if (threadIdx.x == 0) {
        float *r = out + (size_t)bh * 8;
        const double inf = (double)INFINITY;
        r[0] = (float)sigma; r[1] = (float)s; r[2] = (float)C; r[7] = (float)M;
        r[3] = (float)(s > 0.0 ? C - (2.0 - 1.0 / s) * (D1 + D2) : C);
        if (sigma > 0.0) {
            const double C1 = C - (2.0 - 1.0 / sigma) * D1;
            r[4] = (float)(C1 - (2.0 - 1.0 / sigma) * D2);
            r[5] = (float)(C1 - M * (2.0 - 1.0 / sigma) * s2);
        } else {
            r[4] = (float)inf; r[5] = (float)inf;
        }
        r[6] = (float)L;
    }
}

size_t diagnostics_workspace_floats(const Dims &d)
{
    return (size_t)d.batch * d.H * DG_PARTS * (2 * (size_t)d.dh + 6);
}

hipError_t launch_diagnostics(const Dims &d, int dtype, int out_in, const void *v, const void *w_o, const float *a_raw,
                              const float *vnorm, const uint32_t *keys2, const int32_t *idx, const int32_t *count,
                              int max_budget, float *part, float *out, hipStream_t s)
{
    DiagArgs A;
    A.a_raw = a_raw; A.vnorm = vnorm; A.keys2 = keys2; A.idx = idx; A.count = count; A.v = v;
    A.H = d.H; A.Hkv = d.Hkv; A.G = d.G; A.dh = d.dh; A.n = d.n; A.max_budget = max_budget;
    A.part_all = part;
    A.part_sel = part + (size_t)d.batch * d.H * DG_PARTS * (d.dh + 2);
    A.a_scale = d.window_sum ? 1.0f / (float)d.W : 1.0f;
    A.vs0 = d.vs[0]; A.vs1 = d.vs[1]; A.vs2 = d.vs[2];
    const int gz = (d.G + DG_GMAX - 1) / DG_GMAX;
    dim3 block(DG_THREADS);
    if (dtype == CKV_F32) {
        hipLaunchKernelGGL((diag_partial_kernel<float, false>), dim3(DG_PARTS, d.batch * d.Hkv, gz), block, 0, s, A);
        hipLaunchKernelGGL((diag_partial_kernel<float, true>), dim3(DG_PARTS, d.batch * d.Hkv, gz), block, 0, s, A);
        hipLaunchKernelGGL(diag_finish_kernel<float>, dim3(d.batch * d.H), block, 0, s, A, w_o, d.dm, out_in, d.norm, out);
    } else {
        hipLaunchKernelGGL((diag_partial_kernel<bf16_t, false>), dim3(DG_PARTS, d.batch * d.Hkv, gz), block, 0, s, A);
        hipLaunchKernelGGL((diag_partial_kernel<bf16_t, true>), dim3(DG_PARTS, d.batch * d.Hkv, gz), block, 0, s, A);
        hipLaunchKernelGGL(diag_finish_kernel<bf16_t>, dim3(d.batch * d.H), block, 0, s, A, w_o, d.dm, out_in, d.norm, out);
    }
    return hipGetLastError();
}

} // namespace ckv
