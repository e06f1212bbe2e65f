// L2 magnitude of the projected value through the Gram matrix (bf16, d_h = 128)
// (the L2 variant of the distance the paper mentions beside its L1 default; Theorem 3.3's row norm with
// the 2-norm):   N^h_i = || v_i W_O^h ||_2 = sqrt( v_i G^h v_i^T ),   G^h = W_O^h W_O^h^T  (d_h x d_h).
//
// The shortcut is exact for the 2-norm only (for L1 the n x d_model products are needed).  It replaces the
// n x d_h x d_model contraction by n x d_h x d_h: 32 times less MFMA work at d_model = 4096.
//
//   gram_partial  G^h over a slice of the d_model columns, fp32 on the vector ALUs (W_O is a weight:
//                 this is a per-layer constant, a few GFLOP)
//   gram_finish   sums the slices, folds the symmetric G onto its lower block triangle (32 x 32 blocks: those
//                 below the diagonal doubled, those above dropped -- the quadratic form is unchanged and
//                 12 of the 32 block products fall away) and splits it into two bf16 matrices G_hi + G_lo
//                 (error ~2^-17 relative), stored [head][u][t]
//   l2 kernel     one workgroup per (group of row tiles, kv head): a tile's V rows stay in registers as MFMA
//                 B fragments for all G query heads of the group (V is read once); per head the two G
//                 matrices (64 KiB) stream through a double-buffered LDS and  Y^T = G V^T  is accumulated
//                 with v_mfma_f32_16x16x32_bf16 over G_hi and G_lo; the epilogue multiplies by v again:
//                 N^2_i = sum_u Y[i,u] v[i,u].
#include "common.hpp"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int GL_DH = 128;
constexpr int GL_SLICES = 4;          // d_model slices of the Gram partial sums
constexpr int GL_TILE_C = 128;        // columns of W_O staged per LDS tile in gram_partial
constexpr int GL_WAVES = 8;            // one workgroup of 8 waves per CU
constexpr int GL_THREADS = GL_WAVES * 64;
constexpr int GL_RB = 4;              // 16-row blocks per wave and row tile
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

// G = sum of the slices (fixed order), folded onto its lower block triangle, split into hi + lo bf16;
// gram[head][0 = hi, 1 = lo][u][t]
__global__ __launch_bounds__(256) void gram_finish_kernel(const float *__restrict__ partial, bf16_t *__restrict__ gram)
{
    const int h = blockIdx.x;
    for (int e = threadIdx.x; e < GL_DH * GL_DH; e += 256) {
        float g = 0.f;
#pragma unroll
        for (int s = 0; s < GL_SLICES; ++s) g += partial[((size_t)h * GL_SLICES + s) * GL_DH * GL_DH + e];
        // G is symmetric, so v G v^T = sum over the 32 x 32 blocks (bu, bt) on and below the diagonal, the ones
        // below it counted twice: the kernel reads those blocks only (20 of the 32 block products)
        const int bu = e >> 12, bt = (e & (GL_DH - 1)) >> 5; // e = u * 128 + t
        g = bt < bu ? 2.f * g : bt == bu ? g : 0.f;
        const bf16_t hi = f32_to_bf16_rne(g);
        const bf16_t lo = f32_to_bf16_rne(g - bf16_to_f32(hi));
        gram[((size_t)h * 2 + 0) * GL_DH * GL_DH + e] = hi;
        gram[((size_t)h * 2 + 1) * GL_DH * GL_DH + e] = lo;
    }
}

// N^h_i for the G query heads of one kv head and `passes` row tiles of 8 waves x GL_RB x 16 rows.
//
// One workgroup of 8 waves per CU.  The work of a workgroup is a sequence of steps (row tile, query head);
// a step needs that head's two Gram matrices (64 KiB) in LDS.  The matrices are double buffered (128 KiB):
// the loads of step k + 1 are issued before the MFMAs of step k and are waited for after them, so one barrier
// per step is the only synchronisation and the L2 latency of the matrices hides behind 160 MFMAs per wave.
// A row tile's V fragments stay in registers for its G steps.
__global__ __launch_bounds__(GL_THREADS) void vproj_l2_mfma_kernel(const bf16_t *__restrict__ v,
                                                                    const bf16_t *__restrict__ gram,
                                                                    float *__restrict__ vnorm, int H, int G, int n,
                                                                    int64_t vs0, int64_t vs1, int64_t vs2, int passes)
{
    __shared__ __attribute__((aligned(1024))) char lds[2 * 2 * GL_G_BYTES]; // 2 buffers x (G_hi | G_lo), XOR-swizzled
    const int Hkv = H / G;
    const int g = blockIdx.y % Hkv, bi = blockIdx.y / Hkv;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, kc = lane >> 4;
    const int rows_per_pass = GL_WAVES * GL_RB * 16;
    const int tile_row0 = blockIdx.x * passes * rows_per_pass;
    // row tiles that start inside the head (a uniform count: all waves take the same number of barriers)
    const int my_passes = min(passes, (n - tile_row0 + rows_per_pass - 1) / rows_per_pass);
    const int steps = my_passes * G;
    const bf16_t *vbase = v + bi * vs0 + g * vs1;

    // 64 KiB of one head = 64 direct loads of 1 KiB, 8 per wave.  Row u of a matrix is 256 B = 16 chunks;
    // chunk q is stored at slot q ^ f(u), f(u) = 4 * ((u / 8) % 4) + u % 4: the 16 rows that one MFMA A operand
    // reads together (see below) have 16 different f, so their 16-byte reads fall on different banks.
    auto issue_gram = [&](int step, int buf) {
        const int h = g * G + step % G;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(gram + (size_t)h * 2 * GL_DH * GL_DH), 0, 2 * GL_G_BYTES, 0x00020000);
#pragma unroll
        for (int j = 0; j < 64 / GL_WAVES; ++j) {
            const int kib = j * GL_WAVES + wave;            // KiB index inside the 64 KiB: rows 4*kib .. 4*kib+3
            const int urow = (kib * 4 + (lane >> 4)) & (GL_DH - 1);
            const int f = ((urow >> 3) & 3) * 4 + (urow & 3);
            const uint32_t voff = (uint32_t)(kib * 1024 + (lane >> 4) * 256 + (((lane & 15) ^ f) * 16));
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(lds + buf * 2 * GL_G_BYTES + kib * 1024), 16, voff, 0, 0, 0);
        }
    };
    // B fragments: this wave's rows of V (token i = lane % 16 of block rb, k = t)
    auto load_v = [&](int pass, bf16x8 (&dst)[GL_RB][4]) {
        const int row0 = tile_row0 + (pass * GL_WAVES + wave) * (GL_RB * 16);
#pragma unroll
        for (int rb = 0; rb < GL_RB; ++rb) {
            const int row = min(row0 + rb * 16 + l16, n - 1);
            const bf16_t *p = vbase + (int64_t)row * vs2 + kc * 8;
#pragma unroll
            for (int s = 0; s < 4; ++s) dst[rb][s] = *reinterpret_cast<const bf16x8 *>(p + s * 32);
        }
    };

    if (steps <= 0) return; // uniform over the workgroup
    bf16x8 vf[GL_RB][4];
    issue_gram(0, 0);
    load_v(0, vf);
    __syncthreads(); // waits for the direct loads of this wave, then for every wave

#pragma unroll 1
    for (int step = 0; step < steps; ++step) {
        const int pass = step / G, hl = step - pass * G, buf = step & 1;
        if (step + 1 < steps) issue_gram(step + 1, buf ^ 1); // that buffer was last read in step - 1
        const char *gl = lds + buf * 2 * GL_G_BYTES;
        const int row0 = tile_row0 + (pass * GL_WAVES + wave) * (GL_RB * 16);

        float nsq[GL_RB];
#pragma unroll
        for (int rb = 0; rb < GL_RB; ++rb) nsq[rb] = 0.f;
        // The 16 rows u of G that one MFMA takes as its A operand are chosen so that the product's epilogue factor
        // v[i][u] is already in the lane's registers: accumulator value j of lane (i, kc) belongs to A row
        // m = 4 * kc + j, and that row is u(m) = 32 * sp + 8 * (m / 4) + 4 * half + m % 4 = 32 * sp + 8 * kc + 4 * half + j,
        // i.e. element 4 * half + j of the lane's own fragment vf[rb][sp].  (sp, half) = (ub / 2, ub % 2) covers all rows.
        const int a_row = 8 * (l16 >> 2) + (l16 & 3);          // + 32 * sp + 4 * half
        const int a_f = 4 * (l16 >> 2) + (l16 & 3);            // f(u) of that row: bits 3-4 and 0-1 of u
        // fragments of 16 rows of G_hi (0-3) and G_lo (4-7); read one ub ahead of their use
        bf16x8 gf[2][8];
        // (rows of block sp meet the k-chunks s <= sp only: the stored matrices are block lower triangular)
        auto read_g = [&](int ub, bf16x8 (&dst)[8]) {
            const char *rowp = gl + (32 * (ub >> 1) + 4 * (ub & 1) + a_row) * 256;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                if (s > (ub >> 1)) continue; // static: the loop over ub is unrolled
                const int slot = ((4 * s + kc) ^ a_f) * 16;
                dst[s] = *reinterpret_cast<const bf16x8 *>(rowp + slot);
                dst[4 + s] = *reinterpret_cast<const bf16x8 *>(rowp + GL_G_BYTES + slot);
            }
        };
        read_g(0, gf[0]);
#pragma unroll
        for (int ub = 0; ub < GL_DH / 16; ++ub) {
            const int sp = ub >> 1, half = ub & 1, cur = ub & 1;
            if (ub + 1 < GL_DH / 16) read_g(ub + 1, gf[cur ^ 1]);
            // GL_RB independent accumulator chains taken in turns
            f32x4 acc[GL_RB];
#pragma unroll
            for (int rb = 0; rb < GL_RB; ++rb) acc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s <= sp; ++s) {
#pragma unroll
                for (int rb = 0; rb < GL_RB; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gf[cur][4 + s], vf[rb][s], acc[rb], 0, 0, 0);
#pragma unroll
                for (int rb = 0; rb < GL_RB; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gf[cur][s], vf[rb][s], acc[rb], 0, 0, 0);
            }
#pragma unroll
            for (int rb = 0; rb < GL_RB; ++rb) {
                typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
                const u32x4 w = __builtin_bit_cast(u32x4, vf[rb][sp]);
                const uint32_t w0 = w[2 * half], w1 = w[2 * half + 1];
                nsq[rb] = fmaf(acc[rb][0], __uint_as_float(w0 << 16), nsq[rb]);
                nsq[rb] = fmaf(acc[rb][1], __uint_as_float(w0 & 0xFFFF0000u), nsq[rb]);
                nsq[rb] = fmaf(acc[rb][2], __uint_as_float(w1 << 16), nsq[rb]);
                nsq[rb] = fmaf(acc[rb][3], __uint_as_float(w1 & 0xFFFF0000u), nsq[rb]);
            }
            __builtin_amdgcn_sched_barrier(0); // keep the read-ahead distance at one ub (registers)
        }
        // merge the four k-chunk lanes of a token, then one value per token
        float *out = vnorm + ((size_t)bi * H + g * G + hl) * (size_t)n;
#pragma unroll
        for (int rb = 0; rb < GL_RB; ++rb) {
            float x = nsq[rb];
            x += __shfl_xor(x, 16);
            x += __shfl_xor(x, 32);
            const int row = row0 + rb * 16 + l16;
            if (kc == 0 && row < n) out[row] = sqrtf(fmaxf(x, 0.f));
        }
        // the next row tile's fragments replace this one's after its last step (they are waited for with the barrier)
        if (hl == G - 1 && pass + 1 < my_passes) load_v(pass + 1, vf);
        __syncthreads(); // the next step's matrices have landed (own loads waited first) and this buffer is free
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
    // row tiles per workgroup: aim at one workgroup per CU (256) for the whole launch, so that every CU streams
    // the Gram matrices the same number of times and the launch has no partial last round
    const int rows_per_pass = GL_WAVES * GL_RB * 16;
    const long long total_rows = (long long)d.batch * d.Hkv * d.n;
    int passes = (int)((total_rows + 128ll * rows_per_pass) / (256ll * rows_per_pass));
    passes = passes < 1 ? 1 : passes > 64 ? 64 : passes;
    const int rows_per_wg = passes * rows_per_pass;
    dim3 grid((d.n + rows_per_wg - 1) / rows_per_wg, d.batch * d.Hkv);
    hipLaunchKernelGGL(vproj_l2_mfma_kernel, grid, dim3(GL_THREADS), 0, s, (const bf16_t *)v, (const bf16_t *)gram, vnorm,
                       d.H, d.G, d.n, d.vs[0], d.vs[1], d.vs[2], passes);
    return hipGetLastError();
}

} // namespace ckv
