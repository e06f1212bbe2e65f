// Per-entry L1 magnitude of the projected value on the matrix cores (bf16 in, fp32 accumulate)
// (Theorem 3.3; Algorithm 1, lines 2-3):  N^h_i = sum_c | sum_t V^g[i,t] * W_O^h[t,c] |.
//
// This is a dense n x d_h by d_h x d_model contraction per query head whose n x d_model result is
// only needed as a row-wise sum of magnitudes, so the products live in MFMA accumulators, are
// folded into per-row partial sums by the epilogue and never reach memory.
//
// Tiling (d_h = 128):
//   * workgroup = 4 waves, two workgroups per CU; wave w owns R blocks of 32 token rows whose V
//     fragments (MFMA A operand, 8 k-steps of 16) stay in registers for the whole kernel: V is
//     read once.
//   * the head's W_O slice, stored output-major ([d_model][H*d_h]: the 128 inner-dimension values
//     of an output column are contiguous), streams through LDS in tiles of TN columns, double
//     buffered, with direct global->LDS loads (no staging registers).  A wave-level direct load
//     fills 1 KiB of consecutive LDS, so the tile is unpadded [TN][256 B]; bank conflicts of the
//     fragment reads are avoided by storing 16-byte chunk q of column c at slot q ^ (c & 15).
//   * v_mfma_f32_32x32x16_bf16: a lane holds 8 consecutive k of row/column (lane % 32) at k offset
//     8 * (lane / 32); accumulator register j of a lane is row 8*(j/4) + 4*(lane/32) + j%4,
//     column lane % 32.
//   * software pipeline per 32-column block: for each row block a chain of 8 dependent MFMAs into
//     one accumulator set, while the previous column block's set is drained with sum += |acc| (abs
//     is a source modifier: one VALU op per product, two per MFMA) and the next block's B fragments
//     are fetched from LDS.  sched_barrier fences keep this order through the compiler's scheduler.
#include "common.hpp"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int VM_THREADS = 256;
constexpr int VM_WAVES = 4;
constexpr int VM_DH = 128;
constexpr int VM_TN = 128;                 // W_O columns per LDS tile
constexpr int VM_COL_BYTES = VM_DH * 2;    // 256 B per column, 16 chunks of 16 B
constexpr int VM_TILE_BYTES = VM_TN * VM_COL_BYTES;
constexpr int VM_CB = VM_TN / 32;          // 32-column blocks per tile
constexpr int VM_LOADS = VM_TILE_BYTES / 1024 / VM_WAVES; // direct loads per wave per tile

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void *)(p))

template <int R>
__global__ __launch_bounds__(VM_THREADS, 2) void vproj_mfma_kernel(const bf16_t *__restrict__ v,
                                                                   const bf16_t *__restrict__ w_t,
                                                                   float *__restrict__ vnorm, int H, int G, int n,
                                                                   int dm, int64_t vs0, int64_t vs1, int64_t vs2)
{
    __shared__ __attribute__((aligned(1024))) char lds[2 * VM_TILE_BYTES];
    const int h = blockIdx.y, bi = blockIdx.z, g = h / G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int row0 = (blockIdx.x * VM_WAVES + wave) * (R * 32);

    // A fragments: rows of V, resident in registers
    bf16x8 a[R][8];
    const bf16_t *vbase = v + bi * vs0 + g * vs1;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int row = min(row0 + r * 32 + l32, n - 1);
        const bf16_t *p = vbase + (int64_t)row * vs2 + half * 8;
#pragma unroll
        for (int s = 0; s < 8; ++s) a[r][s] = *reinterpret_cast<const bf16x8 *>(p + s * 16);
    }

    float sum[R][16];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < 16; ++j) sum[r][j] = 0.f;

    // Direct loads: instruction j of wave w fills LDS KiB m = j * 4 + w of the tile = columns 4m .. 4m+3;
    // lane i writes slot i % 16 of column 4m + i / 16 and therefore fetches chunk (i % 16) ^ (column & 15).
    // The loads are buffer loads (not flat/global ones): the compiler then keeps exact LDS wait counts.
    const size_t ldw = (size_t)H * VM_DH; // elements between consecutive output columns
    const int ld_col = wave * 4 + (lane >> 4);                       // column of this lane for j = 0
    const uint32_t ld_voff = (uint32_t)(((size_t)h * VM_DH + (size_t)ld_col * ldw + (size_t)(((lane & 15) ^ (ld_col & 15)) * 8)) * 2);
    // (columns advance by 16 per instruction, which leaves column & 15 and thus the chunk unchanged)
    const int tiles = dm / VM_TN; // host guarantees dm % VM_TN == 0 and the whole matrix < 4 GiB
    const __amdgpu_buffer_rsrc_t w_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)w_t, 0, (int)((size_t)dm * ldw * 2), 0x00020000);

    auto issue_load = [&](int tile, int j, char *buf) {
        const uint32_t soff = (uint32_t)(((size_t)tile * VM_TN + (size_t)j * 16) * ldw * 2);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, LDS_PTR(buf + (j * 4 + wave) * 1024), 16, ld_voff, soff, 0, 0);
    };

#pragma unroll
    for (int j = 0; j < VM_LOADS; ++j) issue_load(0, j, lds);

    // per-lane byte offsets of the 8 B fragments inside a 32-column block
    int boff[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) boff[s] = l32 * VM_COL_BYTES + (((2 * s + half) ^ (l32 & 15)) * 16);

    f32x16 acc[2][R];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[p][r][j] = 0.f;

    __syncthreads();
    bf16x8 b[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) b[s] = *reinterpret_cast<const bf16x8 *>(lds + boff[s]);

    for (int t = 0; t < tiles; ++t) {
        const char *cur = lds + (t & 1) * VM_TILE_BYTES;
        char *nxt = lds + ((t + 1) & 1) * VM_TILE_BYTES;
        const int tn = min(t + 1, tiles - 1); // the last iteration re-fetches its own tile into the idle buffer
#pragma unroll
        for (int cb = 0; cb < VM_CB; ++cb) {
            const int pp = cb & 1;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                // one accumulator chain at a time: 8 dependent MFMAs issue back to back at full rate,
                // whereas two chains taken in turns stall on each other
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    if (r == 0 && (s & 3) == 2) issue_load(tn, cb * 2 + (s >> 2), nxt);
                    if (s == 0) {
                        const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        acc[pp][r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r][s], b[s], z, 0, 0, 0);
                    } else {
                        acc[pp][r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r][s], b[s], acc[pp][r], 0, 0, 0);
                    }
                    // after its last use in this block, refill the fragment slot for the next block
                    if (r == R - 1 && cb + 1 < VM_CB)
                        b[s] = *reinterpret_cast<const bf16x8 *>(cur + (cb + 1) * 32 * VM_COL_BYTES + boff[s]);
                    // drain the same row block's accumulators of the previous column block (complete
                    // since R * 8 MFMAs ago): sum += |acc|, two values per MFMA
                    sum[r][2 * s] += fabsf(acc[pp ^ 1][r][2 * s]);
                    sum[r][2 * s + 1] += fabsf(acc[pp ^ 1][r][2 * s + 1]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < 8; ++s) b[s] = *reinterpret_cast<const bf16x8 *>(nxt + boff[s]);
    }
    // the last column block is still in acc[(VM_CB - 1) & 1]
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int j = 0; j < 16; ++j) sum[r][j] += fabsf(acc[(VM_CB - 1) & 1][r][j]);

    // merge the 32 column classes (lanes with equal lane / 32) of every row sum
    float *out = vnorm + ((size_t)bi * H + h) * (size_t)n;
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            float x = sum[r][j];
#pragma unroll
            for (int o = 16; o > 0; o >>= 1) x += __shfl_xor(x, o);
            sum[r][j] = x;
        }
        if (l32 == 0) {
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const int row = row0 + r * 32 + 8 * (j / 4) + 4 * half + (j % 4);
                if (row < n) out[row] = sum[r][j];
            }
        }
    }
}

bool vproj_mfma_supported(const Dims &d)
{
    return d.dh == VM_DH && d.dm % VM_TN == 0 && (size_t)d.dm * d.H * d.dh * 2 < ((size_t)1 << 31);
}

hipError_t launch_vproj_mfma(const Dims &d, const void *v, const void *w_t, float *vnorm, hipStream_t s)
{
    constexpr int R = 2;
    const int rows_per_wg = VM_WAVES * R * 32;
    dim3 grid((d.n + rows_per_wg - 1) / rows_per_wg, d.H, d.batch);
    hipLaunchKernelGGL((vproj_mfma_kernel<R>), grid, dim3(VM_THREADS), 0, s, (const bf16_t *)v, (const bf16_t *)w_t,
                       vnorm, d.H, d.G, d.n, d.dm, d.vs[0], d.vs[1], d.vs[2]);
    return hipGetLastError();
}

} // namespace ckv
