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
//   finish    eight workgroups per query head: each sums the 128 partials in double in a fixed order, takes an
//             eighth of the d_h x d matrix-vector product and stores its share of the norm; the one that
//             draws the last ticket adds the shares in slice order and writes the closed forms
#include "common.hpp"

namespace ckv {

constexpr int DG_THREADS = 256;
constexpr int DG_WAVES = DG_THREADS / 64;
constexpr int DG_CHUNK = 256;  // == DG_THREADS: a thread stages one token of a chunk
constexpr int DG_PARTS = 128;  // workgroups (and partial sums) per head
constexpr int DG_ROWS = 8;  // value rows a lane keeps in flight
constexpr int DG_GMAX = 8; // query heads of a group handled by one workgroup (more: blockIdx.z)
constexpr int DF_SLICES = 8; // finish workgroups per query head (a single CU cannot pull W_O's slice fast enough)
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
    double *loss_part;    // [batch*H][DF_SLICES]: each finish workgroup's share of the loss norm
    uint32_t *ticket;     // [batch*H]: finish workgroups done; zeroed by the sweep kernel of the same call
    int H, Hkv, G, dh, n, max_budget;
    float a_scale;        // 1, or 1/W when the stored score is the window sum
    int64_t vs0, vs1, vs2;
};

template <int N>
__device__ __forceinline__ double block_sum_f64(double x, double *sh)
{
    __syncthreads();
    sh[threadIdx.x] = x;
    __syncthreads();
    for (int o = N / 2; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
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
// GC (1, 2, 4 or 8) is the number of query-head slots compiled in: the workgroup's gc <= GC heads fill the
// first slots, the others carry zero weights.  No global load sits under a branch (the compiler waits for such
// a load on the spot): indices are clamped into range instead and the loaded value is masked afterwards.
template <typename T, bool SELECTED, int GC>
__global__ __launch_bounds__(DG_THREADS) void diag_partial_kernel(DiagArgs A)
{
    __shared__ float a_s[GC][DG_CHUNK];        // A of the chunk's tokens, per query head of the group
    __shared__ int tok_s[DG_CHUNK];            // token index (-1 = skip)
    __shared__ float wsc_s[DG_WAVES][GC][4];   // each wave's scalar sums
    __shared__ float wu_s[DG_WAVES][GC][128];  // each wave's value sums

    const int part = blockIdx.x, head = blockIdx.y; // head = bi * Hkv + g
    const int bi = head / A.Hkv, g = head % A.Hkv;
    const int hh0 = blockIdx.z * DG_GMAX, gc = min(DG_GMAX, A.G - hh0); // 1 <= gc <= GC
    const int h0 = g * A.G + hh0;                                    // first query head handled here
    const int limit = SELECTED ? min(max(A.count[head], 0), A.max_budget) : A.n;
    const int chunks = (limit + DG_CHUNK - 1) / DG_CHUNK;
    if (!SELECTED && part == 0 && (int)threadIdx.x < gc) A.ticket[(size_t)bi * A.H + h0 + threadIdx.x] = 0u;

    // thread = (row lane, group of 8 columns) for the value sums: one 16-byte (bf16) or 32-byte (f32) load per row
    const int groups = A.dh >> 3, cg = threadIdx.x % groups, lane = threadIdx.x / groups, lanes = DG_THREADS / groups;
    const T *vb = reinterpret_cast<const T *>(A.v) + bi * A.vs0 + g * A.vs1 + cg * 8;
    float acc[GC][8];
    float sc[GC][4]; // SELECTED: sigma, s2, D1, D2; else C, min N
#pragma unroll
    for (int hh = 0; hh < GC; ++hh) {
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[hh][e] = 0.0f;
        sc[hh][0] = sc[hh][2] = sc[hh][3] = 0.0f;
        sc[hh][1] = SELECTED ? 0.0f : INFINITY;
    }
    const float *a_row[GC], *n_row[GC]; // slots past gc re-read the last head's rows
#pragma unroll
    for (int hh = 0; hh < GC; ++hh) {
        const size_t row = ((size_t)bi * A.H + h0 + min(hh, gc - 1)) * A.n;
        a_row[hh] = A.a_raw + row;
        n_row[hh] = A.vnorm + row;
    }

    for (int chunk = part; chunk < chunks; chunk += DG_PARTS) { // uniform over the workgroup
        const int j0 = chunk * DG_CHUNK;
        const int len = min(DG_CHUNK, limit - j0);
        __syncthreads(); // the previous chunk's staging is no longer read
        {
            const int jj = threadIdx.x; // DG_CHUNK == DG_THREADS: this thread stages (and sums the scalars of) one token
            int i = -1;
            if (SELECTED) {
                i = A.idx[(size_t)head * A.max_budget + min(j0 + jj, limit - 1)];
                if (jj >= len || i < 0 || i >= A.n) i = -1;
            } else if (jj < len) {
                i = j0 + jj;
            }
            const int ic = max(i, 0);
            bool st1 = false;
            if (SELECTED) st1 = A.keys2[(size_t)head * A.n + ic] == DG_TAKEN;
            float av[GC], nv[GC];
#pragma unroll
            for (int hh = 0; hh < GC; ++hh) { av[hh] = a_row[hh][ic]; nv[hh] = n_row[hh][ic]; }
            tok_s[jj] = i;
#pragma unroll
            for (int hh = 0; hh < GC; ++hh) {
                const float a = (i >= 0 && hh < gc) ? av[hh] * A.a_scale : 0.0f;
                a_s[hh][jj] = a;
                if (SELECTED) {
                    const float a1 = st1 ? a : 0.0f, a2 = st1 ? 0.0f : a;
                    sc[hh][0] += a1; sc[hh][2] += a1 * nv[hh];
                    sc[hh][1] += a2; sc[hh][3] += a2 * nv[hh];
                } else {
                    sc[hh][0] += a * nv[hh];
                    sc[hh][1] = i >= 0 ? fminf(sc[hh][1], nv[hh]) : sc[hh][1];
                }
            }
        }
        __syncthreads();
        // value sums: DG_ROWS rows per lane in flight; the staged token is -1 (and its weight 0) past the chunk's end
        for (int b0 = 0; b0 < len; b0 += lanes * DG_ROWS) {
            float x[DG_ROWS][8];
#pragma unroll
            for (int u = 0; u < DG_ROWS; ++u) {
                const int i = tok_s[b0 + u * lanes + lane]; // < DG_CHUNK: lanes * DG_ROWS divides it
                load8_f32(vb + (int64_t)max(i, 0) * A.vs2, x[u]);
            }
            __builtin_amdgcn_sched_barrier(0); // every row's load is issued before the first is consumed
#pragma unroll
            for (int u = 0; u < DG_ROWS; ++u) {
                const int jj = b0 + u * lanes + lane;
                const bool live = tok_s[jj] >= 0;
#pragma unroll
                for (int e = 0; e < 8; ++e) x[u][e] = live ? x[u][e] : 0.0f;
#pragma unroll
                for (int hh = 0; hh < GC; ++hh) {
                    const float a = a_s[hh][jj];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[hh][e] += a * x[u][e];
                }
            }
        }
    }

    // one partial per (query head, part).  Every sum is first taken inside the wave (scalars over all 64 lanes,
    // value sums over the lanes that share a column group: those lie `groups` apart), then the four waves'
    // results meet in LDS -- a single barrier for the whole epilogue.
    const int wave = threadIdx.x >> 6, wl = threadIdx.x & 63;
#pragma unroll
    for (int hh = 0; hh < GC; ++hh) {
#pragma unroll
        for (int k = 0; k < (SELECTED ? 4 : 2); ++k) {
            float x = sc[hh][k];
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const float y = __shfl_xor(x, o);
                x = (!SELECTED && k == 1) ? fminf(x, y) : x + y;
            }
            if (wl == 0) wsc_s[wave][hh][k] = x;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float x = acc[hh][e];
            for (int o = groups; o < 64; o <<= 1) x += __shfl_xor(x, o);
            if (wl < groups) wu_s[wave][hh][cg * 8 + e] = x;
        }
    }
    __syncthreads();
    for (int t = threadIdx.x; t < gc * (A.dh + 4); t += DG_THREADS) {
        const int hh = t / (A.dh + 4), c = t % (A.dh + 4);
        const size_t slot = ((size_t)bi * A.H + h0 + hh) * DG_PARTS + part;
        float *dst = SELECTED ? A.part_sel + slot * (A.dh + 4) : A.part_all + slot * (A.dh + 2);
        if (c < A.dh) {
            float x = wu_s[0][hh][c];
            for (int w = 1; w < DG_WAVES; ++w) x += wu_s[w][hh][c];
            dst[c] = x;
        } else if (c - A.dh < (SELECTED ? 4 : 2)) {
            const int k = c - A.dh;
            float x = wsc_s[0][hh][k];
            for (int w = 1; w < DG_WAVES; ++w) {
                const float y = wsc_s[w][hh][k];
                x = (!SELECTED && k == 1) ? fminf(x, y) : x + y;
            }
            dst[c] = x;
        }
    }
}

// The finish kernel has few workgroups (DF_SLICES per query head) and little to do, so every wait for memory
// shows: it runs DF_THREADS lanes and keeps many independent loads in flight in each of its three phases.  Every
// workgroup of a head sums all partials (they come from L2) and takes its own slice of W_O's rows.
constexpr int DF_THREADS = 512;

template <typename T>
__global__ __launch_bounds__(DF_THREADS) void diag_finish_kernel(DiagArgs A, const void *w_o, int dm, int out_in,
                                                                 int norm, float *out)
{
    __shared__ double red_s[DF_THREADS];
    __shared__ double grp_s[2][DF_THREADS]; // [all | selected][part group][column]
    __shared__ double diff_s[128];
    __shared__ double scal_s[8];
    const int slice = blockIdx.x, bh = blockIdx.y; // bh = bi * H + h
    const int h = bh % A.H;
    const int per = (dm + DF_SLICES - 1) / DF_SLICES, m_lo = min(slice * per, dm), m_hi = min(m_lo + per, dm);
    const float *pa = A.part_all + (size_t)bh * DG_PARTS * (A.dh + 2);
    const float *ps = A.part_sel + (size_t)bh * DG_PARTS * (A.dh + 4);
    static_assert(DG_PARTS == 128 && DF_THREADS >= 6 * 64, "six waves sum one scalar each, two parts per lane");

    // scalars, one per wave -- 0: C  1: M  2: sigma  3: s2  4: D1  5: D2
    const int q = threadIdx.x >> 6, l = threadIdx.x & 63;
    double sc = 0.0;
    if (q < 2) {
        const double x0 = (double)pa[(size_t)l * (A.dh + 2) + A.dh + q];
        const double x1 = (double)pa[(size_t)(l + 64) * (A.dh + 2) + A.dh + q];
        sc = q == 1 ? fmin(x0, x1) : x0 + x1;
    } else if (q < 6) {
        sc = (double)ps[(size_t)l * (A.dh + 4) + A.dh + (q - 2)] + (double)ps[(size_t)(l + 64) * (A.dh + 4) + A.dh + (q - 2)];
    }
    // the d_h value sums: a thread takes one column and every ngrp-th part
    const int col = threadIdx.x % A.dh, grp = threadIdx.x / A.dh, ngrp = DF_THREADS / A.dh; // 4 or 8 groups
    double ua = 0.0, us = 0.0;
#pragma unroll 16
    for (int c = grp; c < DG_PARTS; c += ngrp) ua += (double)pa[(size_t)c * (A.dh + 2) + col];
#pragma unroll 16
    for (int c = grp; c < DG_PARTS; c += ngrp) us += (double)ps[(size_t)c * (A.dh + 4) + col];
    grp_s[0][threadIdx.x] = ua;
    grp_s[1][threadIdx.x] = us;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double y = __shfl_xor(sc, o);
        sc = q == 1 ? fmin(sc, y) : sc + y;
    }
    if (q < 6 && l == 0) scal_s[q] = sc;
    __syncthreads();
    const double C = scal_s[0], M = scal_s[1], sigma = scal_s[2], s2 = scal_s[3], D1 = scal_s[4], D2 = scal_s[5];
    const double s = sigma + s2;
    if ((int)threadIdx.x < A.dh) {
        double a = 0.0, b = 0.0;
        for (int gi = 0; gi < ngrp; ++gi) { a += grp_s[0][gi * A.dh + threadIdx.x]; b += grp_s[1][gi * A.dh + threadIdx.x]; }
        diff_s[threadIdx.x] = s > 0.0 ? a - b / s : a;
    }
    __syncthreads();
    // y = diff W_O^h, then its norm
    const T *w = reinterpret_cast<const T *>(w_o);
    double part = 0.0;
    if (out_in) {
        // d_h / 8 neighbouring lanes share one row of W_O (one 16-byte piece each, so a row is read as one
        // contiguous run), multiply their eight columns and merge through the wave
        const int lpr = A.dh >> 3; // 8 or 16 lanes per row
        const int piece = threadIdx.x & (lpr - 1), rl = threadIdx.x / lpr, rows = DF_THREADS / lpr;
        // the products run in float (W_O's entries are exact there and a d_h-term dot product keeps ~1e-6
        // relative accuracy, far inside the tolerance on the loss); the sum over rows stays in double
        float dreg[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) dreg[e] = (float)diff_s[piece * 8 + e];
        const T *base = w + (size_t)h * A.dh + piece * 8; // 16-byte aligned: d_h is a multiple of 64
        const size_t ld = (size_t)A.H * A.dh;
        constexpr int U = 16; // rows in flight per lane: the loop is bound by load latency otherwise
        for (int m0 = m_lo; m0 < m_hi; m0 += rows * U) { // uniform trip count: the shuffles below need every lane
            float x[U][8];
#pragma unroll
            for (int u = 0; u < U; ++u) { // rows past the end re-read the last row (kept out of the sum below):
                const int m = min(m0 + u * rows + rl, dm - 1); // a load under a branch would be waited for at once
                load8_f32(base + (size_t)m * ld, x[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float y = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) y += dreg[e] * x[u][e];
                if (lpr == 16) y += __shfl_xor(y, 8);
                y += __shfl_xor(y, 4);
                y += __shfl_xor(y, 2);
                y += __shfl_xor(y, 1);
                if (piece == 0 && m0 + u * rows + rl < m_hi) part += norm == CKV_NORM_L2 ? (double)y * (double)y : (double)fabsf(y);
            }
        }
    } else {
        for (int m = m_lo + threadIdx.x; m < m_hi; m += DF_THREADS) {
            const T *colp = w + (size_t)h * A.dh * dm + m;
            double y = 0.0;
            for (int c = 0; c < A.dh; ++c) y += diff_s[c] * (double)to_f32(colp[(size_t)c * dm]);
            part += norm == CKV_NORM_L2 ? y * y : fabs(y);
        }
    }
    const double share = block_sum_f64<DF_THREADS>(part, red_s);
    if (threadIdx.x == 0) {
        // publish this slice's share, then draw a ticket: the workgroup that draws the last one sees every share
        // (release before the ticket, acquire after it, both at device scope; the shares are read past the L1)
        double *shares = A.loss_part + (size_t)bh * DF_SLICES;
        __hip_atomic_store(shares + slice, share, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        const uint32_t drawn = atomicAdd(A.ticket + bh, 1u);
        if (drawn != (uint32_t)(DF_SLICES - 1)) return;
        __threadfence();
        double L = 0.0;
        for (int j = 0; j < DF_SLICES; ++j) L += __hip_atomic_load(shares + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (norm == CKV_NORM_L2) L = sqrt(L);
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
    // the partials, then per query head DF_SLICES doubles and one ticket word (rounded up to an even count)
    return (size_t)d.batch * d.H * (DG_PARTS * (2 * (size_t)d.dh + 6) + 2 * DF_SLICES + 2);
}

template <typename T, int GC>
static void launch_partials_gc(dim3 grid, dim3 block, hipStream_t s, const DiagArgs &A)
{
    hipLaunchKernelGGL((diag_partial_kernel<T, false, GC>), grid, block, 0, s, A);
    hipLaunchKernelGGL((diag_partial_kernel<T, true, GC>), grid, block, 0, s, A);
}

template <typename T>
static void launch_partials(int slots, dim3 grid, dim3 block, hipStream_t s, const DiagArgs &A)
{
    switch (slots) {
    case 1: launch_partials_gc<T, 1>(grid, block, s, A); break;
    case 2: launch_partials_gc<T, 2>(grid, block, s, A); break;
    case 4: launch_partials_gc<T, 4>(grid, block, s, A); break;
    default: launch_partials_gc<T, 8>(grid, block, s, A); break;
    }
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
    float *tail = part + (size_t)d.batch * d.H * DG_PARTS * (2 * (size_t)d.dh + 6); // 8-byte aligned: an even offset
    A.loss_part = reinterpret_cast<double *>(tail);
    A.ticket = reinterpret_cast<uint32_t *>(tail + (size_t)d.batch * d.H * 2 * DF_SLICES);
    A.a_scale = d.window_sum ? 1.0f / (float)d.W : 1.0f;
    A.vs0 = d.vs[0]; A.vs1 = d.vs[1]; A.vs2 = d.vs[2];
    const int gz = (d.G + DG_GMAX - 1) / DG_GMAX;
    const int slots = d.G >= 5 ? 8 : d.G >= 3 ? 4 : d.G; // head slots compiled in: the next power of two, at most 8
    const dim3 grid(DG_PARTS, d.batch * d.Hkv, gz), block(DG_THREADS);
    if (dtype == CKV_F32) {
        launch_partials<float>(slots, grid, block, s, A);
        hipLaunchKernelGGL(diag_finish_kernel<float>, dim3(DF_SLICES, d.batch * d.H), dim3(DF_THREADS), 0, s, A, w_o, d.dm, out_in, d.norm, out);
    } else {
        launch_partials<bf16_t>(slots, grid, block, s, A);
        hipLaunchKernelGGL(diag_finish_kernel<bf16_t>, dim3(DF_SLICES, d.batch * d.H), dim3(DF_THREADS), 0, s, A, w_o, d.dm, out_in, d.norm, out);
    }
    return hipGetLastError();
}

} // namespace ckv
