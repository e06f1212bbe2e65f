// L2 magnitude of the projected value through the Gram matrix (bf16, d_h = 128)
// (the L2 variant of the distance the paper mentions beside its L1 default; Theorem 3.3's row norm with
// the 2-norm):   N^h_i = || v_i W_O^h ||_2 = sqrt( v_i G^h v_i^T ),   G^h = W_O^h W_O^h^T  (d_h x d_h).
//
// The shortcut is exact for the 2-norm only (for L1 the n x d_model products are needed).  It replaces the
// n x d_h x d_model contraction by n x d_h x d_h: 32 times less MFMA work at d_model = 4096.
//
//   gram_partial  G^h over a slice of the d_model columns, fp32 on the vector ALUs (W_O is a weight:
//                 this is a per-layer constant, a few GFLOP)
//   gram_finish   sums the slices and splits G into two bf16 matrices G_hi + G_lo (error ~2^-17 relative),
//                 stored [head][u][t] (G is symmetric, so a row is also a column)
//   l2 kernel     one workgroup per (row tile, kv head): the V rows stay in registers as MFMA B fragments
//                 for all G query heads of the group (V is read once); per head the two G matrices (64 KiB)
//                 are brought into LDS and  Y^T = G V^T  is accumulated with v_mfma_f32_16x16x32_bf16 over
//                 G_hi and G_lo; the epilogue multiplies by v again:  N^2_i = sum_u Y[i,u] v[i,u].
#include "common.hpp"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int GL_DH = 128;
constexpr int GL_SLICES = 4;          // d_model slices of the Gram partial sums
constexpr int GL_TILE_C = 128;        // columns of W_O staged per LDS tile in gram_partial
constexpr int GL_WAVES = 4;
constexpr int GL_RB = 6;              // 16-row blocks per wave
constexpr int GL_G_BYTES = GL_DH * GL_DH * 2; // one bf16 Gram matrix: 32 KiB

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

__device__ __forceinline__ bf16_t f32_to_bf16_rne(float x)
{
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// partial[head][slice][t][u] = sum over the slice's columns c of w_t[c][h*128+t] * w_t[c][h*128+u]
__global__ __launch_bounds__(256) void gram_partial_kernel(const bf16_t *__restrict__ w_t, float *__restrict__ partial,
                                                           int H, int dm)
{
    __shared__ __attribute__((aligned(16))) bf16_t tile[GL_TILE_C * GL_DH]; // [c][t], 32 KiB
    const int h = blockIdx.x, slice = blockIdx.y;
    const int cols = dm / GL_SLICES; // host guarantees dm % (GL_SLICES * GL_TILE_C) == 0
    const size_t ldw = (size_t)H * GL_DH;
    const int t0 = (threadIdx.x >> 4) * 8, u0 = (threadIdx.x & 15) * 8;
    float acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[i][j] = 0.f;
    for (int c0 = slice * cols; c0 < (slice + 1) * cols; c0 += GL_TILE_C) {
        __syncthreads();
        for (int e = threadIdx.x; e < GL_TILE_C * GL_DH / 8; e += 256) { // 16-byte pieces
            const int c = e >> 4, piece = e & 15;
            *reinterpret_cast<uint4 *>(&tile[c * GL_DH + piece * 8]) =
                *reinterpret_cast<const uint4 *>(w_t + (size_t)(c0 + c) * ldw + (size_t)h * GL_DH + piece * 8);
        }
        __syncthreads();
        for (int c = 0; c < GL_TILE_C; ++c) {
            float a[8], b[8];
            const uint4 ra = *reinterpret_cast<const uint4 *>(&tile[c * GL_DH + t0]);
            const uint4 rb = *reinterpret_cast<const uint4 *>(&tile[c * GL_DH + u0]);
            const uint32_t ua[4] = {ra.x, ra.y, ra.z, ra.w}, ub[4] = {rb.x, rb.y, rb.z, rb.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                a[2 * j] = __uint_as_float(ua[j] << 16); a[2 * j + 1] = __uint_as_float(ua[j] & 0xFFFF0000u);
                b[2 * j] = __uint_as_float(ub[j] << 16); b[2 * j + 1] = __uint_as_float(ub[j] & 0xFFFF0000u);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
    }
    float *dst = partial + ((size_t)h * GL_SLICES + slice) * GL_DH * GL_DH;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) dst[(t0 + i) * GL_DH + u0 + j] = acc[i][j];
}

// G = sum of the slices (fixed order), split into hi + lo bf16; gram[head][0 = hi, 1 = lo][u][t]
__global__ __launch_bounds__(256) void gram_finish_kernel(const float *__restrict__ partial, bf16_t *__restrict__ gram)
{
    const int h = blockIdx.x;
    for (int e = threadIdx.x; e < GL_DH * GL_DH; e += 256) {
        float g = 0.f;
#pragma unroll
        for (int s = 0; s < GL_SLICES; ++s) g += partial[((size_t)h * GL_SLICES + s) * GL_DH * GL_DH + e];
        const bf16_t hi = f32_to_bf16_rne(g);
        const bf16_t lo = f32_to_bf16_rne(g - bf16_to_f32(hi));
        gram[((size_t)h * 2 + 0) * GL_DH * GL_DH + e] = hi;
        gram[((size_t)h * 2 + 1) * GL_DH * GL_DH + e] = lo;
    }
}

// N^h_i for the G query heads of one kv head and one tile of 4 waves x GL_RB x 16 rows.
__global__ __launch_bounds__(256, 2) void vproj_l2_mfma_kernel(const bf16_t *__restrict__ v, const bf16_t *__restrict__ gram,
                                                               float *__restrict__ vnorm, int H, int G, int n,
                                                               int64_t vs0, int64_t vs1, int64_t vs2)
{
    __shared__ __attribute__((aligned(1024))) char lds[2 * GL_G_BYTES]; // G_hi | G_lo, 16-byte chunks XOR-swizzled
    const int Hkv = H / G;
    const int g = blockIdx.y % Hkv, bi = blockIdx.y / Hkv;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, kc = lane >> 4;
    const int row0 = (blockIdx.x * GL_WAVES + wave) * (GL_RB * 16);

    // B fragments: this wave's rows of V (token i = lane % 16 of block rb, k = t)
    bf16x8 vf[GL_RB][4];
    const bf16_t *vbase = v + bi * vs0 + g * vs1;
#pragma unroll
    for (int rb = 0; rb < GL_RB; ++rb) {
        const int row = min(row0 + rb * 16 + l16, n - 1);
        const bf16_t *p = vbase + (int64_t)row * vs2 + kc * 8;
#pragma unroll
        for (int s = 0; s < 4; ++s) vf[rb][s] = *reinterpret_cast<const bf16x8 *>(p + s * 32);
    }

    for (int hl = 0; hl < G; ++hl) {
        const int h = g * G + hl;
        // G_hi and G_lo of this head: 64 KiB = 64 direct loads of 1 KiB, 16 per wave.  Row u of a matrix is
        // 256 B = 16 chunks; chunk q is stored at slot q ^ (u & 15).
        __syncthreads(); // every wave is done with the previous head's matrices
        {
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
                (void *)(gram + (size_t)h * 2 * GL_DH * GL_DH), 0, 2 * GL_G_BYTES, 0x00020000);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int kib = j * GL_WAVES + wave;            // KiB index inside the 64 KiB: rows 4*kib .. 4*kib+3
                const int urow = (kib * 4 + (lane >> 4)) & (GL_DH - 1);
                const uint32_t voff = (uint32_t)(kib * 1024 + (lane >> 4) * 256 + (((lane & 15) ^ (urow & 15)) * 16));
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(lds + kib * 1024), 16, voff, 0, 0, 0);
            }
        }
        __syncthreads();

        float nsq[GL_RB];
#pragma unroll
        for (int rb = 0; rb < GL_RB; ++rb) nsq[rb] = 0.f;
#pragma unroll 1
        for (int ub = 0; ub < GL_DH / 16; ++ub) {
            // A fragments: rows u = 16*ub + lane%16 of G_hi / G_lo, k = t
            bf16x8 ghi[4], glo[4];
            const char *rowp = lds + (ub * 16 + l16) * 256;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int slot = ((4 * s + kc) ^ l16) * 16;
                ghi[s] = *reinterpret_cast<const bf16x8 *>(rowp + slot);
                glo[s] = *reinterpret_cast<const bf16x8 *>(rowp + GL_G_BYTES + slot);
            }
#pragma unroll
            for (int rb = 0; rb < GL_RB; ++rb) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(glo[s], vf[rb][s], acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ghi[s], vf[rb][s], acc, 0, 0, 0);
                }
                // acc[j] = Y[i][u] for token i = rb*16 + lane%16, u = 16*ub + 4*kc + j; multiply by v[i][u]
                const int row = min(row0 + rb * 16 + l16, n - 1);
                const uint2 raw = *reinterpret_cast<const uint2 *>(vbase + (int64_t)row * vs2 + ub * 16 + kc * 4);
                nsq[rb] = fmaf(acc[0], __uint_as_float(raw.x << 16), nsq[rb]);
                nsq[rb] = fmaf(acc[1], __uint_as_float(raw.x & 0xFFFF0000u), nsq[rb]);
                nsq[rb] = fmaf(acc[2], __uint_as_float(raw.y << 16), nsq[rb]);
                nsq[rb] = fmaf(acc[3], __uint_as_float(raw.y & 0xFFFF0000u), nsq[rb]);
            }
        }
        // merge the four k-chunk lanes of a token, then one value per token
        float *out = vnorm + ((size_t)bi * H + h) * (size_t)n;
#pragma unroll
        for (int rb = 0; rb < GL_RB; ++rb) {
            float x = nsq[rb];
            x += __shfl_xor(x, 16);
            x += __shfl_xor(x, 32);
            const int row = row0 + rb * 16 + l16;
            if (kc == 0 && row < n) out[row] = sqrtf(fmaxf(x, 0.f));
        }
    }
}

bool vproj_l2_mfma_supported(const Dims &d) { return d.dh == GL_DH && d.dm % (GL_SLICES * GL_TILE_C) == 0; }

size_t vproj_l2_gram_bytes(const Dims &d) { return (size_t)d.H * 2 * GL_DH * GL_DH * 2; }

// partial sums of the Gram slices, followed by room for the Gram matrices themselves
size_t vproj_l2_workspace_bytes(const Dims &d)
{
    return (size_t)d.H * GL_SLICES * GL_DH * GL_DH * 4 + vproj_l2_gram_bytes(d);
}

hipError_t launch_gram(const Dims &d, const void *w_t, void *gram_out, void *partial_scratch, hipStream_t s)
{
    float *partial = (float *)partial_scratch;
    hipLaunchKernelGGL(gram_partial_kernel, dim3(d.H, GL_SLICES), dim3(256), 0, s, (const bf16_t *)w_t, partial, d.H, d.dm);
    hipLaunchKernelGGL(gram_finish_kernel, dim3(d.H), dim3(256), 0, s, partial, (bf16_t *)gram_out);
    return hipGetLastError();
}

hipError_t launch_vproj_l2_mfma(const Dims &d, const void *v, const void *gram, float *vnorm, hipStream_t s)
{
    const int rows_per_wg = GL_WAVES * GL_RB * 16;
    dim3 grid((d.n + rows_per_wg - 1) / rows_per_wg, d.batch * d.Hkv);
    hipLaunchKernelGGL(vproj_l2_mfma_kernel, grid, dim3(256), 0, s, (const bf16_t *)v, (const bf16_t *)gram, vnorm, d.H,
                       d.G, d.n, d.vs[0], d.vs[1], d.vs[2]);
    return hipGetLastError();
}

} // namespace ckv
