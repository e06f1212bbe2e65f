// Per-entry L1 magnitude of the projected value on the matrix cores (bf16 in, fp32 accumulate)
// (Theorem 3.3; Algorithm 1, lines 2-3):  N^h_i = sum_c | sum_t V^g[i,t] * W_O^h[t,c] |.
//
// This is a dense n x d_h by d_h x d_model contraction per query head whose n x d_model result is
// only needed as a row-wise sum of magnitudes, so the products live in MFMA accumulators, are
// folded into per-row partial sums by the epilogue and never reach memory.
//
// Tiling (d_h = 128):
//   workgroup = 4 waves; wave w owns R blocks of 32 token rows; their V fragments (the MFMA A
//   operand, 8 k-steps of 16) stay in registers for the whole kernel: V is read once.
//   The head's W_O slice, stored output-major ([d_model][H*d_h], so the 128 inner-dimension
//   values of one output column are contiguous), streams through LDS in tiles of TN columns,
//   double buffered; each wave reads the B fragments of a 32-column block once and reuses them
//   for its R row blocks.
//   v_mfma_f32_32x32x16_bf16: a lane holds 8 consecutive k of row/column (lane % 32), k offset
//   8 * (lane / 32); accumulator register j of a lane is row 8*(j/4) + 4*(lane/32) + j%4,
//   column lane % 32.  The epilogue adds |acc[j]| into 16 per-lane row sums per block; lanes
//   are merged once at the end.
#include "common.hpp"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int VM_THREADS = 256;
constexpr int VM_WAVES = 4;
constexpr int VM_DH = 128;
constexpr int VM_TN = 128;                  // W_O columns per LDS tile
constexpr int VM_ROW_BYTES = VM_DH * 2 + 16; // padded LDS pitch of one column's 128 bf16
constexpr int VM_TILE_BYTES = VM_TN * VM_ROW_BYTES;

template <int R>
__global__ __launch_bounds__(VM_THREADS) void vproj_mfma_kernel(const bf16_t *__restrict__ v,
                                                                const bf16_t *__restrict__ w_t,
                                                                float *__restrict__ vnorm, int H, int G, int n, int dm,
                                                                int64_t vs0, int64_t vs1, int64_t vs2)
{
    __shared__ __attribute__((aligned(16))) char lds[2 * VM_TILE_BYTES];
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

    // global -> LDS staging: thread t moves 16 bytes of column (t / 16 + 16 * j), j = 0..7
    const size_t ldw = (size_t)H * VM_DH;
    const bf16_t *wsrc = w_t + (size_t)h * VM_DH + (size_t)(threadIdx.x >> 4) * ldw + (threadIdx.x & 15) * 8;
    const int lds_dst = (threadIdx.x >> 4) * VM_ROW_BYTES + (threadIdx.x & 15) * 16;
    uint4 stage[VM_TN / 16];
    const int tiles = dm / VM_TN; // host guarantees dm % VM_TN == 0

#pragma unroll
    for (int j = 0; j < VM_TN / 16; ++j) stage[j] = *reinterpret_cast<const uint4 *>(wsrc + (size_t)(16 * j) * ldw);
#pragma unroll
    for (int j = 0; j < VM_TN / 16; ++j) *reinterpret_cast<uint4 *>(lds + lds_dst + 16 * j * VM_ROW_BYTES) = stage[j];
    __syncthreads();

    for (int t = 0; t < tiles; ++t) {
        const char *cur = lds + (t & 1) * VM_TILE_BYTES;
        char *nxt = lds + ((t + 1) & 1) * VM_TILE_BYTES;
        const bool more = t + 1 < tiles;
        if (more) {
            const bf16_t *src = wsrc + (size_t)(t + 1) * VM_TN * ldw;
#pragma unroll
            for (int j = 0; j < VM_TN / 16; ++j) stage[j] = *reinterpret_cast<const uint4 *>(src + (size_t)(16 * j) * ldw);
        }
#pragma unroll
        for (int cb = 0; cb < VM_TN / 32; ++cb) {
            bf16x8 b[8];
            const char *bp = cur + (cb * 32 + l32) * VM_ROW_BYTES + half * 16;
#pragma unroll
            for (int s = 0; s < 8; ++s) b[s] = *reinterpret_cast<const bf16x8 *>(bp + s * 32);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 8; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[r][s], b[s], acc, 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 16; ++j) sum[r][j] += fabsf(acc[j]);
            }
        }
        if (more) {
#pragma unroll
            for (int j = 0; j < VM_TN / 16; ++j)
                *reinterpret_cast<uint4 *>(nxt + lds_dst + 16 * j * VM_ROW_BYTES) = stage[j];
        }
        __syncthreads();
    }

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

bool vproj_mfma_supported(const Dims &d) { return d.dh == VM_DH && d.dm % VM_TN == 0; }

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
