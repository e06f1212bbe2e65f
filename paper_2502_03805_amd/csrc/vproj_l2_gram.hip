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
//   l2 kernel     one workgroup per (query head, range of rows) with the head's two G matrices (64 KiB) resident in
//                 LDS; V rows stream through registers as MFMA B fragments,  Y^T = G V^T  is accumulated with
//                 v_mfma_f32_16x16x32_bf16 over G_hi and G_lo, and the epilogue multiplies by v again:
//                 N^2_i = sum_u Y[i,u] v[i,u].
#include <type_traits>

#include "common.hpp"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int GL_DH = 128;
constexpr int GL_SLICES = 4;          // d_model slices of the Gram partial sums
constexpr int GL_TILE_C = 128;        // columns of W_O staged per LDS tile in gram_partial
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

// N^h_i for HEADS query heads of a kv group and one range of rows, with the heads' Gram matrices resident in LDS.
//
// One workgroup of 4 * HEADS waves per (HEADS query heads, range of rows): two 4-wave workgroups per CU with one
// head each, or one 8-wave workgroup with two.  The heads' G_hi | G_lo (64 KiB each) are fetched once, at the
// start; after the one barrier that follows, every wave is on its own: it walks its blocks of GR_RB x 16 rows,
// requests the next block's V fragments (global -> registers) before it starts on the current one, and runs the
// block through the workgroup's heads, reading the Gram fragments it needs from LDS.  No barrier and no Gram
// traffic in the loop.  V is read once per workgroup of a kv group; the workgroups that work on the same rows are
// neighbours in launch order on one XCD (workgroup L of a 1-D grid runs on XCD L % 8), so the later readers of a
// row find it in that XCD's L2.  Two heads per workgroup halve the V traffic (6 % faster with four heads per
// group); with an odd number of heads the workgroup that is left with one head would idle half of the time
// (measured 6 % slower with five), so such groups take one head per workgroup.
constexpr int GR_RB = 4;
constexpr int GR_BLOCK_ROWS = GR_RB * 16;

template <int HEADS>
__global__ __launch_bounds__(HEADS * 256, HEADS == 1 ? 2 : 1) void vproj_l2_resident_kernel(const bf16_t *__restrict__ v,
                                                                             const bf16_t *__restrict__ gram,
                                                                             float *__restrict__ vnorm, int H, int G, int n,
                                                                             int64_t vs0, int64_t vs1, int64_t vs2, int pairs,
                                                                             int ranges, int rows_per_range)
{
    constexpr int GR_HEADS = HEADS, GR_WAVES = 4 * HEADS;
    __shared__ __attribute__((aligned(1024))) char lds[GR_HEADS * 2 * GL_G_BYTES]; // per head: G_hi | G_lo, XOR-swizzled
    const int Hkv = H / G, hgroups = G / GR_HEADS; // (the launcher takes HEADS = 2 for even G only)
    const int L = blockIdx.x, xcd = L & 7;
    int r = L >> 3;
    const int hl = (r % hgroups) * GR_HEADS;                 // first head of this workgroup inside its kv group
    r /= hgroups;
    const int range = r % ranges;
    const int pair = (r / ranges) * 8 + xcd;
    if (pair >= pairs) return; // uniform over the workgroup
    const int bi = pair / Hkv, g = pair % Hkv, h = g * G + hl;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l16 = lane & 15, kc = lane >> 4;
    const int row_begin = range * rows_per_range;            // a multiple of GR_BLOCK_ROWS
    const int row_end = min(n, row_begin + rows_per_range);
    if (row_begin >= row_end) return;                        // uniform over the workgroup
    const int nblk = (row_end - row_begin + GR_BLOCK_ROWS - 1) / GR_BLOCK_ROWS;
    const bf16_t *vbase = v + bi * vs0 + g * vs1;

    for (int hh = 0; hh < GR_HEADS; ++hh) {   // a head's 64 KiB: 64 direct loads of 1 KiB; row u of a matrix is 256 B = 16 chunks;
        // chunk q sits at slot q ^ f(u), f(u) = 4 * ((u / 8) % 4) + u % 4: the 16 rows that one MFMA A operand reads
        // together (see below) have 16 different f, so their 16-byte reads fall on different banks
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            (void *)(gram + (size_t)(h + hh) * 2 * GL_DH * GL_DH), 0, 2 * GL_G_BYTES, 0x00020000);
#pragma unroll
        for (int j = 0; j < 64 / GR_WAVES; ++j) {
            const int kib = j * GR_WAVES + wave;
            const int urow = (kib * 4 + (lane >> 4)) & (GL_DH - 1);
            const int f = ((urow >> 3) & 3) * 4 + (urow & 3);
            const uint32_t voff = (uint32_t)(kib * 1024 + (lane >> 4) * 256 + (((lane & 15) ^ f) * 16));
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, LDS_PTR(lds + hh * 2 * GL_G_BYTES + kib * 1024), 16, voff, 0, 0, 0);
        }
    }
    // V rows through a buffer descriptor over this kv head's rows (the host checks that they span less than 2 GiB, so
    // 32-bit byte offsets do).  Rows past n - 1 re-read row n - 1 (never stored): the clamp is in the lane's
    // offset, because the descriptor's range check does not see the scalar offset.
    const __amdgpu_buffer_rsrc_t vrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void *)vbase, 0, (int)(((int64_t)(n - 1) * vs2 + GL_DH) * 2), 0x00020000);
    const uint32_t row_bytes = (uint32_t)(vs2 * 2);
    // a block's V fragments in two halves: k-chunks 0-1 (the row's first 128 bytes) and 2-3 (its second)
    auto load_v_half = [&](int blk, int hf, bf16x8 (&dst)[GR_RB][2]) {
        const int row0 = row_begin + blk * GR_BLOCK_ROWS;
#pragma unroll
        for (int rb = 0; rb < GR_RB; ++rb) {
            const uint32_t voff = (uint32_t)min(row0 + rb * 16 + l16, n - 1) * row_bytes + (uint32_t)(kc * 16 + hf * 128);
#pragma unroll
            for (int s = 0; s < 2; ++s)
                dst[rb][s] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(vrsrc, voff + s * 64, 0, 0));
        }
    };
    // Registers: the first halves of two blocks (the current one and the wave's next, requested a block ahead) and
    // the second half of the current block only, requested when the block starts: the block-lower-triangular
    // Gram matrix needs k-chunks 2-3 from its fifth 16-row slab on, 48 MFMAs into the block.
    bf16x8 va[2][GR_RB][2], vb[GR_RB][2];
    if (wave < nblk) load_v_half(wave, 0, va[0]);
    __syncthreads(); // the Gram matrices have landed (every wave waits for its own loads first)
    if (wave >= nblk) return; // after the only barrier

    // The 16 rows u of G that one MFMA takes as its A operand are chosen so that the product's epilogue factor
    // v[i][u] is already in the lane's registers: accumulator value j of lane (i, kc) belongs to A row
    // m = 4 * kc + j, and that row is u(m) = 32 * sp + 8 * (m / 4) + 4 * half + m % 4 = 32 * sp + 8 * kc + 4 * half + j,
    // i.e. element 4 * half + j of the lane's own V fragment of k-chunk sp.  (sp, half) = (ub / 2, ub % 2) covers all rows.
    const int a_row = 8 * (l16 >> 2) + (l16 & 3);          // + 32 * sp + 4 * half
    const int a_f = 4 * (l16 >> 2) + (l16 & 3);            // f(u) of that row: bits 3-4 and 0-1 of u
    float *out = vnorm + ((size_t)bi * H + h) * (size_t)n;

    // One block of rows from register set CUR; the other set receives the wave's next block meanwhile.
    auto block_step = [&](auto cur_c, int blk) {
        constexpr int CUR = decltype(cur_c)::value;
        load_v_half(blk, 1, vb);
        load_v_half(blk + GR_WAVES, 0, va[CUR ^ 1]); // unconditional (clamped rows): the wait counts stay exact
        // the block's fragments serve every head of the workgroup, one after the other
#pragma unroll 1
        for (int hh = 0; hh < GR_HEADS; ++hh) {
        const char *gl = lds + hh * 2 * GL_G_BYTES;
        float nsq[GR_RB];
#pragma unroll
        for (int rb = 0; rb < GR_RB; ++rb) nsq[rb] = 0.f;
        // fragments of 16 rows of G_hi (0-3) and G_lo (4-7) for one ub; the next ub's are requested into the same
        // registers as soon as this ub's MFMAs are issued and arrive under its epilogue and the other wave's work
        bf16x8 gf[8];
        auto read_g = [&](int ub) {
            const char *rowp = gl + (32 * (ub >> 1) + 4 * (ub & 1) + a_row) * 256;
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                if (s > (ub >> 1)) continue; // (rows of block sp meet the k-chunks s <= sp only)
                const int slot = ((4 * s + kc) ^ a_f) * 16;
                gf[s] = *reinterpret_cast<const bf16x8 *>(rowp + slot);
                gf[4 + s] = *reinterpret_cast<const bf16x8 *>(rowp + GL_G_BYTES + slot);
            }
        };
        read_g(0);
#pragma unroll
        for (int ub = 0; ub < GL_DH / 16; ++ub) {
            const int sp = ub >> 1, half = ub & 1;
            f32x4 acc[GR_RB];
#pragma unroll
            for (int rb = 0; rb < GR_RB; ++rb) acc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s <= sp; ++s) {
#pragma unroll
                for (int rb = 0; rb < GR_RB; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gf[4 + s], s < 2 ? va[CUR][rb][s] : vb[rb][s - 2], acc[rb], 0, 0, 0);
#pragma unroll
                for (int rb = 0; rb < GR_RB; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gf[s], s < 2 ? va[CUR][rb][s] : vb[rb][s - 2], acc[rb], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (ub + 1 < GL_DH / 16) read_g(ub + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int rb = 0; rb < GR_RB; ++rb) {
                typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
                const u32x4 w = __builtin_bit_cast(u32x4, sp < 2 ? va[CUR][rb][sp] : vb[rb][sp - 2]);
                const uint32_t w0 = w[2 * half], w1 = w[2 * half + 1];
                nsq[rb] = fmaf(acc[rb][0], __uint_as_float(w0 << 16), nsq[rb]);
                nsq[rb] = fmaf(acc[rb][1], __uint_as_float(w0 & 0xFFFF0000u), nsq[rb]);
                nsq[rb] = fmaf(acc[rb][2], __uint_as_float(w1 << 16), nsq[rb]);
                nsq[rb] = fmaf(acc[rb][3], __uint_as_float(w1 & 0xFFFF0000u), nsq[rb]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        const int row0 = row_begin + blk * GR_BLOCK_ROWS;
#pragma unroll
        for (int rb = 0; rb < GR_RB; ++rb) {
            float x = nsq[rb];
            x += __shfl_xor(x, 16);
            x += __shfl_xor(x, 32);
            const int row = row0 + rb * 16 + l16;
            if (kc == 0 && row < row_end) out[(size_t)hh * n + row] = sqrtf(fmaxf(x, 0.f));
        }
        }
    };
    for (int blk = wave; blk < nblk; blk += 2 * GR_WAVES) {
        block_step(std::integral_constant<int, 0>{}, blk);
        if (blk + GR_WAVES < nblk) block_step(std::integral_constant<int, 1>{}, blk + GR_WAVES);
    }
}

bool vproj_l2_mfma_supported(const Dims &d)
{
    // (the V rows of one kv head are addressed through a buffer descriptor with 32-bit byte offsets)
    return d.dh == GL_DH && d.dm % (GL_SLICES * GL_TILE_C) == 0 &&
           (((int64_t)(d.n - 1) * d.vs[2] + GL_DH) * 2) < ((int64_t)1 << 31);
}

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
    // heads per workgroup: two where the group's heads pair up, else one
    const int heads = d.G % 2 == 0 ? 2 : 1, waves = 4 * heads;
    // ranges of rows per workgroup of heads: eight waves per CU over the whole launch where the context allows it,
    // so that every workgroup is resident from the start (a kv group's workgroups then walk the same rows side by side)
    const int pairs = d.batch * d.Hkv;
    const int per_range = 8 * ((pairs + 7) / 8) * (d.G / heads);
    int ranges = (512 / heads) / per_range;
    const int most = (d.n + waves * GR_BLOCK_ROWS - 1) / (waves * GR_BLOCK_ROWS); // a block per wave at least
    ranges = ranges > most ? most : ranges;
    ranges = ranges < 1 ? 1 : ranges;
    int rows_per_range = (d.n + ranges - 1) / ranges;
    rows_per_range = (rows_per_range + GR_BLOCK_ROWS - 1) / GR_BLOCK_ROWS * GR_BLOCK_ROWS;
    const dim3 grid((unsigned)(per_range * ranges)), block(waves * 64);
    if (heads == 2)
        hipLaunchKernelGGL(vproj_l2_resident_kernel<2>, grid, block, 0, s, (const bf16_t *)v, (const bf16_t *)gram, vnorm,
                           d.H, d.G, d.n, d.vs[0], d.vs[1], d.vs[2], pairs, ranges, rows_per_range);
    else
        hipLaunchKernelGGL(vproj_l2_resident_kernel<1>, grid, block, 0, s, (const bf16_t *)v, (const bf16_t *)gram, vnorm,
                           d.H, d.G, d.n, d.vs[0], d.vs[1], d.vs[2], pairs, ranges, rows_per_range);
    return hipGetLastError();
}

} // namespace ckv
