// Per-entry L1 magnitude of the projected value on the matrix cores (bf16 in, fp32 accumulate)
// (Theorem 3.3; Algorithm 1, lines 2-3):  N^h_i = sum_c | sum_t V^g[i,t] * W_O^h[t,c] |.
//
// This is a dense n x d_h by d_h x d_model contraction per query head whose n x d_model result is
// only needed as a row-wise sum of magnitudes, so the products live in MFMA accumulators, are
// folded into per-row partial sums by the epilogue and never reach memory.
//
// Tiling (written for d_h = 128; d_h = 64 runs the same kernel with two k-steps per chain and 256-column tiles):
//   * workgroup = 4 waves, two workgroups per CU; wave w owns RB blocks of 16 token rows whose V
//     fragments (4 k-steps of 32) stay in registers for the whole kernel: V is read once per
//     workgroup.  The product is taken transposed, (W_O^h)^T V^T: the streamed W_O fragment is the
//     MFMA A operand, shared by RB consecutive MFMAs, and the resident V fragments are B operands
//     (measured 1.3 % faster than the other way round; the fragment layouts are the same).
//   * the head's W_O slice, stored output-major ([d_model][H*d_h]: the 128 inner-dimension values
//     of an output column are contiguous), streams through LDS in tiles of TN columns, double
//     buffered, with direct buffer->LDS loads (no staging registers).  A wave-level direct load
//     fills 1 KiB of consecutive LDS, so the tile is unpadded [TN][256 B]; bank conflicts of the
//     fragment reads are avoided by storing 16-byte chunk q of column c at slot q ^ (c & 15).
//   * v_mfma_f32_16x16x32_bf16: a lane holds 8 consecutive k of row (A) / column (B) lane % 16 at
//     k offset 8 * (lane / 16); accumulator register v of a lane is row 4*(lane/16) + v, column
//     lane % 16, i.e. here output column 4*(lane/16) + v of token lane % 16.  This shape sustains a markedly higher rate than 32x32x16 on this part when the
//     operands are real (toggling) data, i.e. when the chip is power limited.
//   * software pipeline per 16-column block: 4 k-steps x RB row blocks of MFMAs into one accumulator
//     set while the previous block's set is drained with sum += |acc| (abs is a source modifier:
//     one VALU op per product, one per MFMA) and the next block's W_O fragments are fetched from LDS.
//     sched_barrier fences keep this order through the compiler's scheduler.
#include <type_traits>

#include "common.hpp"

namespace ckv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int VM_THREADS = 256;
constexpr int VM_WAVES = 4;
constexpr int VM_TILE_BYTES = 32768;       // one LDS tile of W_O columns
constexpr int VM_LOADS = VM_TILE_BYTES / 1024 / VM_WAVES; // direct loads per wave per tile

template <int DH>
struct VGeo {
    static constexpr int KS = DH / 32;                 // k-steps of one 16x16x32 MFMA chain
    static constexpr int COL_BYTES = DH * 2;           // one W_O column of the head: 16 or 8 chunks of 16 B
    static constexpr int CPR = COL_BYTES / 16;         // chunks per column
    static constexpr int TN = VM_TILE_BYTES / COL_BYTES; // W_O columns per LDS tile (128 or 256)
    static constexpr int CB = TN / 16;                 // 16-column blocks per tile
    static constexpr int CPK = 1024 / COL_BYTES;       // columns per KiB (one direct load of a wave)
    static constexpr int LPC = KS / 2;                 // direct loads issued per column block (first half of a tile)
};

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

template <int DH, int RB>
__global__ __launch_bounds__(VM_THREADS, 2) void vproj_mfma_kernel(const bf16_t *__restrict__ v,
                                                                   const bf16_t *__restrict__ w_t,
                                                                   float *__restrict__ vnorm, int H, int G, int n,
                                                                   int dm, int64_t vs0, int64_t vs1, int64_t vs2,
                                                                   int row_tiles, int heads, int pair)
{
    using geo = VGeo<DH>;
    constexpr int VM_KS = geo::KS, VM_CB = geo::CB, VM_TN = geo::TN, VM_COL_BYTES = geo::COL_BYTES, VM_DH = DH;
    static_assert(VM_LOADS * 2 == VM_CB * geo::LPC, "the next tile's loads go out during the first half of a tile");
    __shared__ __attribute__((aligned(1024))) char lds[2 * VM_TILE_BYTES];
    // XCD-aware work mapping.  Workgroups of a 1-D grid are handed to the 8 XCDs round-robin (workgroup L
    // runs on XCD L % 8) and every XCD has its own 4 MiB L2.  An XCD gets consecutive (batch item, query head)
    // pairs, i.e. heads of one kv group, and walks them two at a time: the two heads take turns on every row
    // tile, so the second one finds the tile's V rows in that L2, and the workgroups resident on the XCD stream
    // the same two 1 MiB W_O slices, which stay in L2 as well.  (Four heads in turn were measured slower: their
    // four slices evict each other.  Measured against one head at a time: same speed, half the L2 misses -- as
    // long as two slices leave room in L2: at d_model 5120 (2 x 1.25 MiB) pairing was 13 % slower, so the host
    // pairs heads only up to d_model 4096.)
    const int xcd = blockIdx.x & 7, k_in_xcd = blockIdx.x >> 3;
    const int hpx = (heads + 7) >> 3;                    // heads per XCD
    // pair = 1: two heads take turns on a row tile; pair = 0: one head at a time (its slice alone in L2)
    const int member = pair ? (k_in_xcd & 1) : 0, pt = pair ? (k_in_xcd >> 1) : k_in_xcd;
    const int in_xcd = (pair ? 2 : 1) * (pt / row_tiles) + member;
    const int hb = xcd * hpx + in_xcd;                   // batch * H + head
    if (in_xcd >= hpx || hb >= heads) return;
    const int tile_x = pt % row_tiles;
    const int h = hb % H, bi = hb / H, g = h / G;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6); // wave-uniform, kept in a scalar register
    const int l16 = lane & 15, kc = lane >> 4;
    const int row0 = (tile_x * VM_WAVES + wave) * (RB * 16);

    // V fragments (16 token rows x 32 k each), resident in registers
    bf16x8 a[RB][VM_KS];
    const bf16_t *vbase = v + bi * vs0 + g * vs1;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const int row = min(row0 + rb * 16 + l16, n - 1);
        const bf16_t *p = vbase + (int64_t)row * vs2 + kc * 8;
#pragma unroll
        for (int s = 0; s < VM_KS; ++s) a[rb][s] = *reinterpret_cast<const bf16x8 *>(p + s * 32);
    }

    float sum[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < 4; ++j) sum[rb][j] = 0.f;

    // Direct loads: instruction j of wave w fills LDS KiB m = j * 4 + w of the tile = columns CPK*m .. (CPK = 4 at
    // d_h 128); lane i writes slot i % CPR of column CPK*m + i / CPR and therefore fetches chunk
    // (i % CPR) ^ (column & (CPR-1)).
    // They are buffer loads (not flat/global ones): the compiler then keeps exact LDS wait counts.
    const size_t ldw = (size_t)H * VM_DH; // elements between consecutive output columns
    const int ld_col = wave * geo::CPK + lane / geo::CPR;                // column of this lane for j = 0
    const uint32_t ld_voff = (uint32_t)(((size_t)h * VM_DH + (size_t)ld_col * ldw +
                                         (size_t)(((lane % geo::CPR) ^ (ld_col & (geo::CPR - 1))) * 8)) * 2);
    // (columns advance by 4 * CPK per instruction, a multiple of CPR, which leaves the chunk unchanged)
    const int tiles = dm / VM_TN; // host guarantees dm % VM_TN == 0 and the whole matrix < 2 GiB
    const __amdgpu_buffer_rsrc_t w_rsrc =
        __builtin_amdgcn_make_buffer_rsrc((void *)w_t, 0, (int)((size_t)dm * ldw * 2), 0x00020000);

    auto issue_load = [&](int tile, int j, char *buf) {
        const uint32_t soff = (uint32_t)(((size_t)tile * VM_TN + (size_t)j * 4 * geo::CPK) * ldw * 2);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(w_rsrc, LDS_PTR(buf + (j * 4 + wave) * 1024), 16, ld_voff, soff, 0, 0);
    };

#pragma unroll
    for (int j = 0; j < VM_LOADS; ++j) issue_load(0, j, lds);

    // per-lane byte offsets of the 4 W_O fragments inside a 16-column block
    int boff[VM_KS];
#pragma unroll
    for (int s = 0; s < VM_KS; ++s) boff[s] = l16 * VM_COL_BYTES + (((4 * s + kc) ^ (l16 & (geo::CPR - 1))) * 16);

    f32x4 acc[2][RB];
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) acc[p][rb] = f32x4{0.f, 0.f, 0.f, 0.f};

    __syncthreads();
    bf16x8 b[VM_KS];
#pragma unroll
    for (int s = 0; s < VM_KS; ++s) b[s] = *reinterpret_cast<const bf16x8 *>(lds + boff[s]);

    // One tile.  BUF (which LDS buffer holds it) is a compile-time constant so that every fragment
    // read is "per-lane offset register + immediate": the tile loop below is unrolled by two.
    auto tile_step = [&](auto buf_c, int t) {
        constexpr int BUF = decltype(buf_c)::value;
        const char *cur = lds + BUF * VM_TILE_BYTES;
        char *nxt = lds + (BUF ^ 1) * VM_TILE_BYTES;
        const int tn = min(t + 1, tiles - 1); // the last iteration re-fetches its own tile into the idle buffer
#pragma unroll
        for (int cb = 0; cb < VM_CB; ++cb) {
            const int pp = cb & 1;
#pragma unroll
            for (int s = 0; s < VM_KS; ++s) {
#pragma unroll
                for (int rb = 0; rb < RB; ++rb) {
                    // the next tile's loads go out early in this tile (its buffer is idle since the last barrier),
                    // so that they have landed long before the barrier at the end
                    if (cb < VM_CB / 2 && (s & 1) && rb == 0) issue_load(tn, geo::LPC * cb + (s >> 1), nxt);
                    // RB independent accumulator chains, taken in turns (a chain's next link is RB MFMAs later)
                    if (s == 0)
                        acc[pp][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[s], a[rb][s], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
                    else
                        acc[pp][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(b[s], a[rb][s], acc[pp][rb], 0, 0, 0);
                    // after its last use in this block, refill the fragment slot for the next block
                    if (rb == RB - 1 && cb + 1 < VM_CB)
                        b[s] = *reinterpret_cast<const bf16x8 *>(cur + (cb + 1) * 16 * VM_COL_BYTES + boff[s]);
                    // drain the previous column block's accumulators (complete since >= RB MFMAs): 4 / KS values per MFMA
#pragma unroll
                    for (int v = 0; v < 4 / VM_KS; ++v) sum[rb][s * (4 / VM_KS) + v] += fabsf(acc[pp ^ 1][rb][s * (4 / VM_KS) + v]);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < VM_KS; ++s) b[s] = *reinterpret_cast<const bf16x8 *>(nxt + boff[s]);
    };
    for (int t = 0; t < tiles; t += 2) {
        tile_step(std::integral_constant<int, 0>{}, t);
        if (t + 1 < tiles) tile_step(std::integral_constant<int, 1>{}, t + 1);
    }
    // the last column block is still in acc[(VM_CB - 1) & 1]
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < 4; ++j) sum[rb][j] += fabsf(acc[(VM_CB - 1) & 1][rb][j]);

    // accumulator value j of lane (l16, kc) is output column 4 * kc + j of token l16: merge the four values and
    // the four lanes of a token
    float *out = vnorm + ((size_t)bi * H + h) * (size_t)n;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        float x = (sum[rb][0] + sum[rb][1]) + (sum[rb][2] + sum[rb][3]);
        x += __shfl_xor(x, 16);
        x += __shfl_xor(x, 32);
        const int row = row0 + rb * 16 + l16;
        if (kc == 0 && row < n) out[row] = x;
    }
}

bool vproj_mfma_supported(const Dims &d)
{
    return (d.dh == 128 || d.dh == 64) && d.dm % (VM_TILE_BYTES / (d.dh * 2)) == 0 &&
           (size_t)d.dm * d.H * d.dh * 2 < ((size_t)1 << 31) &&
           ((long long)d.batch * d.H + 8) * (d.n / 64 + 2) < (1ll << 31);
}

template <int DH, int RB>
static void launch_rb(const Dims &d, const void *v, const void *w_t, float *vnorm, hipStream_t s)
{
    const int rows_per_wg = VM_WAVES * RB * 16;
    const int row_tiles = (d.n + rows_per_wg - 1) / rows_per_wg;
    const int heads = d.batch * d.H;
    const int pair = (size_t)2 * DH * d.dm * 2 <= ((size_t)2 << 20) ? 1 : 0; // two slices within 2 MiB
    const int hpx = (heads + 7) / 8;
    const long long wgs = 8ll * (pair ? 2 * ((hpx + 1) / 2) : hpx) * row_tiles; // 8 XCDs x heads (in pairs) x row tiles
    hipLaunchKernelGGL((vproj_mfma_kernel<DH, RB>), dim3((unsigned)wgs), dim3(VM_THREADS), 0, s, (const bf16_t *)v,
                       (const bf16_t *)w_t, vnorm, d.H, d.G, d.n, d.dm, d.vs[0], d.vs[1], d.vs[2], row_tiles, heads, pair);
}

hipError_t launch_vproj_mfma(const Dims &d, const void *v, const void *w_t, float *vnorm, hipStream_t s)
{
    // 7 row blocks per wave stream W_O 14 % less often than 6, but the workgroups are longer; measured, that wins
    // once the launch has many rounds of workgroups (1.4 % at 128K) and loses on short launches (2 % at 32K)
    const long long wgs7 = (long long)d.batch * d.H * ((d.n + VM_WAVES * 7 * 16 - 1) / (VM_WAVES * 7 * 16));
    if (d.dh == 64) launch_rb<64, 6>(d, v, w_t, vnorm, s);
    else if (wgs7 >= 4096) launch_rb<128, 7>(d, v, w_t, vnorm, s);
    else launch_rb<128, 6>(d, v, w_t, vnorm, s);
    return hipGetLastError();
}

} // namespace ckv
