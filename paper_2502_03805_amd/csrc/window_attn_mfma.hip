// Observation-window attention on the matrix cores, bf16, d_h = 128 (Algorithm 2, lines 2-3; eq. (2)).
//
// a^h_i = reduce_w softmax_i(scale * q_w . k_i) needs every window row's max and sum over all n keys
// before any weight can be summed over the window, so the keys are swept twice and the tiny logits
// (G*W rows per kv head) are recomputed on the MFMA units instead of being stored:
//   pass 1 (stats)   per key chunk: row max m and l = sum_i 2^(t_i - m) of t = logit * log2(e)
//   reduce           per row: E = log2(sum_i 2^t_i) (+ log2 W for the window mean)
//   pass 2 (colsum)  a^h_i = sum_w 2^(t_wi - E_w)
//
// Work split: one workgroup per (key chunk, kv head).  Pass 1: one WAVE per (query head of the group, block
// of 32 window rows), holding those queries as MFMA fragments in registers (rows past W are zero and masked):
// a window of more than 32 rows is spread over several waves (more waves in flight, fewer registers each; the
// row statistics need no exchange).  Pass 2: one wave per query head with all its row blocks, because a key's
// window sum runs over all of them (splitting it and adding the shares through LDS was measured slower).  Key tiles of 64 rows stream once per workgroup through LDS (direct global->LDS
// loads, double buffered, 16-byte chunks XOR-swizzled against bank conflicts) and are read by every wave.
//
// v_mfma_f32_32x32x16_bf16 operand layout: a lane holds 8 consecutive k of row (A) / column (B)
// lane % 32 at k offset 8 * (lane / 32); accumulator j is row 8*(j/4) + 4*(lane/32) + j%4, column lane%32.
//   pass 1 computes K . Q^T (lane = one query row, registers = 16 keys): row statistics stay lane-local;
//   pass 2 computes Q . K^T (lane = one key, registers = 16 query rows): the window sum is lane-local.
#include <float.h>

#include "common.hpp"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int AM_DH = 128;
constexpr int AM_TILE_KEYS = 64;
constexpr int AM_TILE_BYTES = AM_TILE_KEYS * AM_DH * 2; // 16 KiB
constexpr int AM_CHUNK_MIN = 256;                       // fewest keys per workgroup (the host picks 256, 512 or 1024)
constexpr int AM_MAX_WAVES = 16;                       // pass 1: waves per workgroup, one per (head, 32-row block)
constexpr int AM_COLSUM_WAVES = 8;                     // pass 2: waves per workgroup, one per head
constexpr float AM_LOG2E = 1.4426950408889634f;
constexpr float AM_NEG = -1.0e30f;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

struct AttnArgs {
    const bf16_t *q;
    const bf16_t *k;
    int H, G, n, W, chunks;
    int chunk_keys; // keys per workgroup, a multiple of the tile
    int qbs;        // 32-row blocks of the window: a wave owns one (query head, row block)
    int wpw;        // (head, row block) pairs per workgroup: a multiple of qbs, so a head's blocks share a workgroup
    int causal; // window row w sees keys <= n - W + w only
    float c; // scale * log2(e)
    int64_t ks0, ks1, ks2;
};

// Q fragments of one head: block qb covers window rows (qb0+qb)*32 .. +31 (zero past W).
template <int QB>
__device__ __forceinline__ void load_q_frags(const AttnArgs &A, int bi, int head, int qb0, int l32, int half,
                                             bf16x8 (&qf)[QB][8])
{
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int w = (qb0 + qb) * 32 + l32;
        const bf16_t *p = A.q + (((size_t)bi * A.H + head) * A.W + min(w, A.W - 1)) * AM_DH + half * 8;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            bf16x8 x = *reinterpret_cast<const bf16x8 *>(p + s * 16);
            if (w >= A.W) x = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            qf[qb][s] = x;
        }
    }
}

// Direct global->LDS load of one 64-key tile, shared among the nw waves of the workgroup.
// Instruction j fills LDS KiB j = keys 4j .. 4j+3; lane i writes slot i % 16 of key 4j + i / 16 and
// fetches 16-byte chunk (i % 16) ^ (key & 15) of that key row.  Rows past n-1 re-read row n-1.
// The loads are buffer loads (not flat/global ones) so that the compiler keeps exact LDS wait counts.
__device__ __forceinline__ void load_k_tile(__amdgpu_buffer_rsrc_t krsrc, int64_t ks2, int key0, int n, char *buf,
                                            int wave, int nw, int lane)
{
    for (int j = wave; j < AM_TILE_BYTES / 1024; j += nw) {
        const int key_in_tile = 4 * j + (lane >> 4);
        const int key = min(key0 + key_in_tile, n - 1);
        const uint32_t voff = (uint32_t)(((int64_t)key * ks2 + (((lane & 15) ^ (key_in_tile & 15)) * 8)) * 2);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, LDS_PTR(buf + j * 1024), 16, voff, 0, 0, 0);
    }
}

// Buffer descriptor over one kv head's keys (token stride ks2 elements; the host checks n * ks2 * 2 < 2 GiB).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_k_rsrc(const bf16_t *kbase, int64_t ks2, int n)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)kbase, 0, (int)(((int64_t)(n - 1) * ks2 + AM_DH) * 2), 0x00020000);
}

__device__ __forceinline__ void read_k_frags(const char *tile, int kb, int l32, int half, bf16x8 (&kf)[8])
{
    const char *row = tile + (kb * 32 + l32) * (AM_DH * 2);
#pragma unroll
    for (int s = 0; s < 8; ++s) kf[s] = *reinterpret_cast<const bf16x8 *>(row + (((2 * s + half) ^ (l32 & 15)) * 16));
}

__device__ __forceinline__ f32x16 zero16()
{
    return f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
}

// ---- pass 1 ---------------------------------------------------------------------------------------
template <int QB>
__global__ __launch_bounds__(64 * AM_MAX_WAVES) void attn_stats_mfma_kernel(AttnArgs A, float *__restrict__ part)
{
    __shared__ __attribute__((aligned(1024))) char lds[2 * AM_TILE_BYTES];
    const int chunk = blockIdx.x, bi = blockIdx.y / (A.H / A.G), g = blockIdx.y % (A.H / A.G);
    const int nw = blockDim.x >> 6;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int vw = blockIdx.z * A.wpw + wave;               // (query head, 32-row block of the window) of this wave
    const bool head_ok = wave < A.wpw && vw < A.G * A.qbs;
    const int head = g * A.G + (head_ok ? vw / A.qbs : 0);
    const int qb0 = head_ok ? vw % A.qbs : 0;
    const bf16_t *kbase = A.k + bi * A.ks0 + g * A.ks1;
    const __amdgpu_buffer_rsrc_t krsrc = make_k_rsrc(kbase, A.ks2, A.n);
    const int key_begin = chunk * A.chunk_keys;
    const int key_end = min(key_begin + A.chunk_keys, A.n);
    const int tiles = (key_end - key_begin + AM_TILE_KEYS - 1) / AM_TILE_KEYS;

    bf16x8 qf[QB][8];
    load_q_frags<QB>(A, bi, head, qb0, l32, half, qf);
    float m[QB], l[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { m[qb] = AM_NEG; l[qb] = 0.f; }

    load_k_tile(krsrc, A.ks2, key_begin, A.n, lds, wave, nw, lane);
    __syncthreads();
    for (int t = 0; t < tiles; ++t) {
        const char *cur = lds + (t & 1) * AM_TILE_BYTES;
        if (t + 1 < tiles)
            load_k_tile(krsrc, A.ks2, key_begin + (t + 1) * AM_TILE_KEYS, A.n, lds + ((t + 1) & 1) * AM_TILE_BYTES, wave,
                        nw, lane);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const int key0 = key_begin + t * AM_TILE_KEYS + kb * 32; // first key of this 32-key block
            if (key0 >= key_end) break;
            bf16x8 kf[8];
            read_k_frags(cur, kb, l32, half, kf);
            // blocks past the end of the keys, or (causal tail) reaching into the last W keys, need masking
            const bool ragged = key0 + 32 > A.n || (A.causal && key0 + 31 > A.n - A.W);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                f32x16 acc = zero16();
#pragma unroll
                for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[qb][s], acc, 0, 0, 0);
                // acc[j]: key key0 + 8*(j/4) + 4*half + j%4, query row l32
                // t = acc * c with c > 0, so the block maximum of t is c * max(acc); 2^(t - m) = 2^fma(acc, c, -m)
                if (ragged) {
                    const int last_seen = A.causal ? A.n - A.W + (qb0 + qb) * 32 + l32 : A.n - 1; // last key this row sees
#pragma unroll
                    for (int j = 0; j < 16; ++j) {
                        const int key = key0 + 8 * (j / 4) + 4 * half + (j % 4);
                        if (key >= A.n || key > last_seen) acc[j] = -INFINITY;
                    }
                }
                float amax = fmaxf(fmaxf(acc[0], acc[1]), acc[2]);
#pragma unroll
                for (int j = 3; j < 15; j += 2) amax = fmaxf(fmaxf(amax, acc[j]), acc[j + 1]);
                amax = fmaxf(amax, acc[15]);
                const float mn = fmaxf(m[qb], amax * A.c);
                float add = 0.f;
#pragma unroll
                for (int j = 0; j < 16; ++j) add += __builtin_amdgcn_exp2f(fmaf(acc[j], A.c, -mn));
                l[qb] = l[qb] * __builtin_amdgcn_exp2f(m[qb] - mn) + add;
                m[qb] = mn;
            }
        }
        __syncthreads();
    }
    // merge the two lanes that hold the same query row, then one (m, l) pair per row and chunk
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float mo = __shfl_xor(m[qb], 32), lo = __shfl_xor(l[qb], 32);
        const float mt = fmaxf(m[qb], mo);
        const float lt = l[qb] * __builtin_amdgcn_exp2f(m[qb] - mt) + lo * __builtin_amdgcn_exp2f(mo - mt);
        const int w = (qb0 + qb) * 32 + l32;
        if (head_ok && half == 0 && w < A.W) {
            float *dst = part + ((((size_t)bi * A.H + head) * A.W + w) * (size_t)A.chunks + chunk) * 2;
            dst[0] = mt;
            dst[1] = lt;
        }
    }
}

// One wave per window row: E = log2(sum_i 2^t_i) (+ log2 W for the mean), stored at stats[row*2].
__global__ __launch_bounds__(64) void attn_stats_reduce_log2_kernel(const float *__restrict__ part,
                                                                    float *__restrict__ stats, int chunks, float post)
{
    const size_t row = blockIdx.x;
    const float *p = part + row * (size_t)chunks * 2;
    float m = AM_NEG;
    for (int c = threadIdx.x; c < chunks; c += 64) m = fmaxf(m, p[2 * c]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    float l = 0.f;
    for (int c = threadIdx.x; c < chunks; c += 64) l += p[2 * c + 1] * exp2f(p[2 * c] - m);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) l += __shfl_xor(l, o);
    if (threadIdx.x == 0) {
        stats[row * 2] = m + log2f(l) + post;
        stats[row * 2 + 1] = 0.f;
    }
}

// ---- pass 2 ---------------------------------------------------------------------------------------
template <int QB>
__global__ __launch_bounds__(64 * AM_COLSUM_WAVES) void attn_colsum_mfma_kernel(AttnArgs A, const float *__restrict__ stats,
                                                                             float *__restrict__ a_raw)
{
    __shared__ __attribute__((aligned(1024))) char lds[2 * AM_TILE_BYTES];
    const int chunk = blockIdx.x, bi = blockIdx.y / (A.H / A.G), g = blockIdx.y % (A.H / A.G);
    const int nw = blockDim.x >> 6;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int head = g * A.G + blockIdx.z * AM_COLSUM_WAVES + wave;
    const bool head_ok = blockIdx.z * AM_COLSUM_WAVES + wave < A.G;
    const bf16_t *kbase = A.k + bi * A.ks0 + g * A.ks1;
    const __amdgpu_buffer_rsrc_t krsrc = make_k_rsrc(kbase, A.ks2, A.n);
    const int key_begin = chunk * A.chunk_keys;
    const int key_end = min(key_begin + A.chunk_keys, A.n);
    const int tiles = (key_end - key_begin + AM_TILE_KEYS - 1) / AM_TILE_KEYS;

    bf16x8 qf[QB][8];
    load_q_frags<QB>(A, bi, head_ok ? head : g * A.G, 0, l32, half, qf);
    // E of the 16 window rows a lane's accumulators belong to (+inf past W: weight 0)
    float e[QB][16];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const int w = qb * 32 + 8 * (j / 4) + 4 * half + (j % 4);
            e[qb][j] = (head_ok && w < A.W) ? stats[(((size_t)bi * A.H + head) * A.W + w) * 2] : INFINITY;
        }
    float *out = a_raw + ((size_t)bi * A.H + (head_ok ? head : g * A.G)) * (size_t)A.n;

    load_k_tile(krsrc, A.ks2, key_begin, A.n, lds, wave, nw, lane);
    __syncthreads();
    for (int t = 0; t < tiles; ++t) {
        const char *cur = lds + (t & 1) * AM_TILE_BYTES;
        if (t + 1 < tiles)
            load_k_tile(krsrc, A.ks2, key_begin + (t + 1) * AM_TILE_KEYS, A.n, lds + ((t + 1) & 1) * AM_TILE_BYTES, wave,
                        nw, lane);
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            const int key0 = key_begin + t * AM_TILE_KEYS + kb * 32;
            if (key0 >= key_end) break;
            bf16x8 kf[8];
            read_k_frags(cur, kb, l32, half, kf);
            float colsum = 0.f;
            const bool tail = A.causal && key0 + 31 > A.n - A.W; // some window rows do not see these keys
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                f32x16 acc = zero16();
#pragma unroll
                for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[qb][s], kf[s], acc, 0, 0, 0);
                // acc[j]: window row qb*32 + 8*(j/4) + 4*half + j%4, key key0 + l32
                if (tail) {
#pragma unroll
                    for (int j = 0; j < 16; ++j)
                        if (key0 + l32 > A.n - A.W + qb * 32 + 8 * (j / 4) + 4 * half + (j % 4)) acc[j] = -INFINITY;
                }
#pragma unroll
                for (int j = 0; j < 16; ++j) colsum += __builtin_amdgcn_exp2f(fmaf(acc[j], A.c, -e[qb][j]));
            }
            colsum += __shfl_xor(colsum, 32);
            const int key = key0 + l32;
            if (head_ok && half == 0 && key < A.n) out[key] = colsum;
        }
        __syncthreads();
    }
}

bool attn_mfma_supported(const Dims &d)
{
    return d.dh == AM_DH && d.W <= 96 && ((int64_t)(d.n - 1) * d.ks[2] + AM_DH) * 2 < ((int64_t)1 << 31);
}
// Keys per workgroup.  Longer chunks spread the fixed cost of a workgroup (its query fragments, the first tile's
// latency) over more keys; measured, 1024 keys win as long as the launch still has two workgroups per CU
// (Qwen 128K: both sweeps 20 % faster than with 256), 512 at Llama 32K, 256 below.
static int attn_chunk_keys(const Dims &d)
{
    const int qbs = (d.W + 31) / 32, wpw = (AM_MAX_WAVES / qbs) * qbs;
    const long long per_chunk_row = (long long)d.batch * d.Hkv * ((d.G * qbs + wpw - 1) / wpw);
    for (int keys = 1024; keys > AM_CHUNK_MIN; keys >>= 1)
        if (per_chunk_row * ((d.n + keys - 1) / keys) >= 512) return keys;
    return AM_CHUNK_MIN;
}
int mfma_attn_chunks(const Dims &d) { const int keys = attn_chunk_keys(d); return (d.n + keys - 1) / keys; }

static AttnArgs make_args(const Dims &d, const void *q, const void *k, int chunks)
{
    AttnArgs A;
    A.q = (const bf16_t *)q; A.k = (const bf16_t *)k;
    A.H = d.H; A.G = d.G; A.n = d.n; A.W = d.W; A.chunks = chunks; A.causal = d.causal;
    A.chunk_keys = attn_chunk_keys(d);
    A.qbs = (d.W + 31) / 32;
    A.wpw = (AM_MAX_WAVES / A.qbs) * A.qbs;
    A.c = d.scale * AM_LOG2E;
    A.ks0 = d.ks[0]; A.ks1 = d.ks[1]; A.ks2 = d.ks[2];
    return A;
}

hipError_t launch_attn_stats_mfma(const Dims &d, const void *q, const void *k, float *part, int chunks, hipStream_t s)
{
    const AttnArgs A = make_args(d, q, k, chunks);
    const int pairs = d.G * A.qbs, nw = pairs < A.wpw ? pairs : A.wpw;
    dim3 grid(chunks, d.batch * d.Hkv, (pairs + A.wpw - 1) / A.wpw), block(64 * nw);
    hipLaunchKernelGGL(attn_stats_mfma_kernel<1>, grid, block, 0, s, A, part);
    return hipGetLastError();
}

hipError_t launch_attn_stats_reduce_log2(const Dims &d, const float *part, int chunks, float *stats, hipStream_t s)
{
    const size_t rows = (size_t)d.batch * d.H * d.W;
    const float post = d.window_sum ? 0.0f : log2f((float)d.W);
    hipLaunchKernelGGL(attn_stats_reduce_log2_kernel, dim3((unsigned)rows), dim3(64), 0, s, part, stats, chunks, post);
    return hipGetLastError();
}

hipError_t launch_attn_colsum_mfma(const Dims &d, const void *q, const void *k, const float *stats, float *a_raw,
                                   hipStream_t s)
{
    const AttnArgs A = make_args(d, q, k, mfma_attn_chunks(d));
    const int nw = d.G < AM_COLSUM_WAVES ? d.G : AM_COLSUM_WAVES;
    dim3 grid(A.chunks, d.batch * d.Hkv, (d.G + AM_COLSUM_WAVES - 1) / AM_COLSUM_WAVES), block(64 * nw);
    const int qb = (d.W + 31) / 32;
    if (qb == 1) hipLaunchKernelGGL(attn_colsum_mfma_kernel<1>, grid, block, 0, s, A, stats, a_raw);
    else if (qb == 2) hipLaunchKernelGGL(attn_colsum_mfma_kernel<2>, grid, block, 0, s, A, stats, a_raw);
    else hipLaunchKernelGGL(attn_colsum_mfma_kernel<3>, grid, block, 0, s, A, stats, a_raw);
    return hipGetLastError();
}

} // namespace ckv
