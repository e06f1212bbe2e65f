// Observation-window attention on the matrix cores with wave-private key streams, bf16, d_h = 64 or 128
// (Algorithm 2, lines 2-3; eq. (2)).  Same mathematics and the same two sweeps as window_attn_mfma.hip
// (pass 1: per-range row max and sum of 2^(t - m); reduce; pass 2: a^h_i = sum_w 2^(t_wi - E_w)); used for the
// shapes whose row blocks do not fit that file's one-wave-per-head layout (groups of more than four 32-row
// blocks, windows up to 128 rows, d_h = 64), where it measured 6 % faster on the 5:1 group with a 64-row window.
//
// Work split: every WAVE is on its own.  It owns every ranges-th 32-key block of one kv head and up to four
// blocks of 32 window rows (whole query heads of the group), whose queries it keeps as MFMA fragments in
// registers for its whole life.  Its keys stream through a wave-private ring of two 32-key blocks in LDS,
// filled by direct global->LDS loads (16-byte chunks, XOR-swizzled against bank conflicts) that are requested
// two blocks ahead; a block's key fragments are read into registers once and serve every row block of the wave.
// Nothing is shared between waves, so there is no barrier anywhere: a wave only ever waits for its own loads.
// Inside a key block the MFMAs of row block r+1 are issued before the exponentials of row block r, so that the
// matrix pipe works under the vector work.  A group with more row blocks than one wave holds is spread over
// several workgroups that are placed on the same XCD (workgroup L of a 1-D grid runs on XCD L % 8), where the
// second reader of a key finds it in L2.
//
// v_mfma_f32_32x32x16_bf16 operand layout: a lane holds 8 consecutive k of row (A) / column (B)
// lane % 32 at k offset 8 * (lane / 32); accumulator j is row 8*(j/4) + 4*(lane/32) + j%4, column lane%32.
//   pass 1 computes K . Q^T (lane = one query row, registers = 16 keys): row statistics stay lane-local;
//   pass 2 computes Q . K^T (lane = one key, registers = 16 query rows): the window sum is lane-local.  The
//   16 rows' constants -E_w / c are the accumulator's initial value (read from a small wave-private table in
//   LDS, the same address for all lanes of a half wave), so that acc * c is already t - E.
#include <float.h>
#include <type_traits>

#include "common.hpp"

namespace ckv {
namespace { // everything up to the launchers is private to this file (the shared-tile file has its own AttnArgs etc.)

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int AM_WAVES = 4;           // waves per workgroup, each with its own key range
constexpr int AM_BLOCK_KEYS = 32;     // keys per MFMA block
constexpr int AM_MAX_QB = 4;          // 32-row blocks of window queries a wave keeps in registers
constexpr int AM_MIN_KPW = 128;       // fewest keys per wave (sizes the per-range partials)
constexpr float AM_LOG2E = 1.4426950408889634f;
constexpr float AM_NEG = -1.0e30f;

#define LDS_PTR(p) ((__attribute__((address_space(3))) void *)(p))

struct AttnArgs {
    const bf16_t *q;
    const bf16_t *k;
    int H, G, n, W;
    int ranges;   // waves per (kv head, group of query heads): wave r takes key blocks r, r + ranges, ...;
                  // the per-wave partials of pass 1 are [row][ranges][2]
    int qbs;      // 32-row blocks of the window
    int hpw;      // query heads per wave (hpw * qbs <= AM_MAX_QB)
    int groups;   // ceil(G / hpw): workgroups over the same keys
    int xc8;      // ceil(workgroups along the keys / 8)
    int causal;   // window row w sees keys <= n - W + w only
    float c;      // scale * log2(e)
    int64_t ks0, ks1, ks2;
};

// s_waitcnt with only the vector-memory counter set: wait until at most N of this wave's loads are outstanding
// (gfx9 encoding: vmcnt in bits 3:0 and 15:14; the export and LDS counters stay at "do not wait").
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(15 | (3 << 14) | (7 << 4) | (0 << 8)); }

template <int DH>
struct Geo {
    static constexpr int KS = DH / 16;                        // k-steps of one 32x32x16 MFMA chain
    static constexpr int ROW_BYTES = DH * 2;
    static constexpr int CPR = ROW_BYTES / 16;                // 16-byte chunks per key row
    static constexpr int BLOCK_BYTES = AM_BLOCK_KEYS * ROW_BYTES;
    static constexpr int LOADS = BLOCK_BYTES / 1024;          // direct loads (1 KiB each) per key block
    static constexpr int ROWS_PER_LOAD = 1024 / ROW_BYTES;
};

// Q fragments of row block rb of this wave: head h0 + rb / qbs, window rows (rb % qbs) * 32 .. +31 (zero past W).
template <int DH, int QB>
__device__ __forceinline__ void load_q_frags(const AttnArgs &A, int bi, int head0, int nrb, int l32, int half,
                                             bf16x8 (&qf)[QB][Geo<DH>::KS])
{
#pragma unroll
    for (int rb = 0; rb < QB; ++rb) {
        const int rbc = min(rb, nrb - 1);
        const int head = head0 + rbc / A.qbs;
        const int w = (rbc % A.qbs) * 32 + l32;
        const bf16_t *p = A.q + (((size_t)bi * A.H + head) * A.W + min(w, A.W - 1)) * DH + half * 8;
        // every load is unconditional (clamped address); rows past W and unused row blocks are zeroed by a mask
        const uint32_t keep = (w < A.W && rb < nrb) ? 0xFFFFFFFFu : 0u;
#pragma unroll
        for (int s = 0; s < Geo<DH>::KS; ++s) {
            uint4 x = *reinterpret_cast<const uint4 *>(p + s * 16);
            x.x &= keep; x.y &= keep; x.z &= keep; x.w &= keep;
            qf[rb][s] = __builtin_bit_cast(bf16x8, x);
        }
    }
}

// Direct global->LDS load of one 32-key block into a wave-private slot.  Instruction j fills KiB j of the slot
// = keys j*ROWS_PER_LOAD ..; lane i writes chunk slot i % CPR of key j*RPL + i / CPR and fetches 16-byte chunk
// (i % CPR) ^ (key & (CPR-1)) of that key row.  Rows past n-1 re-read row n-1 (masked by the caller).
// Buffer loads (not flat/global ones): their completion is counted by vmcnt alone.
template <int DH>
__device__ __forceinline__ void load_k_block(__amdgpu_buffer_rsrc_t krsrc, int64_t ks2, int key0, int n, char *slot, int lane)
{
    using g = Geo<DH>;
#pragma unroll
    for (int j = 0; j < g::LOADS; ++j) {
        const int key_in_block = j * g::ROWS_PER_LOAD + lane / g::CPR;
        const int key = min(key0 + key_in_block, n - 1);
        const uint32_t voff = (uint32_t)(((int64_t)key * ks2 + (((lane % g::CPR) ^ (key_in_block & (g::CPR - 1))) * 8)) * 2);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, LDS_PTR(slot + j * 1024), 16, voff, 0, 0, 0);
    }
}

// Buffer descriptor over one kv head's keys (token stride ks2 elements; the host checks n * ks2 * 2 < 2 GiB).
template <int DH>
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_k_rsrc(const bf16_t *kbase, int64_t ks2, int n)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)kbase, 0, (int)(((int64_t)(n - 1) * ks2 + DH) * 2), 0x00020000);
}

template <int DH>
__device__ __forceinline__ void read_k_frags(const char *slot, int l32, int half, bf16x8 (&kf)[Geo<DH>::KS])
{
    using g = Geo<DH>;
    const char *row = slot + l32 * g::ROW_BYTES;
#pragma unroll
    for (int s = 0; s < g::KS; ++s)
        kf[s] = *reinterpret_cast<const bf16x8 *>(row + (((2 * s + half) ^ (l32 & (g::CPR - 1))) * 16));
}

__device__ __forceinline__ f32x16 zero16()
{
    return f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
}

// Which (batch item, kv head, group of heads, key range) this wave works on; false if it has nothing to do.
struct WaveJob {
    int bi, g, head0, nrb, range, nblk;
};
__device__ __forceinline__ bool wave_job(const AttnArgs &A, int wave, WaveJob &J)
{
    // workgroups that read the same keys (the groups of heads) sit on one XCD, next to each other in launch order
    const int L = blockIdx.x, xcd = L & 7;
    int r = L >> 3;
    const int group = r % A.groups;
    r /= A.groups;
    const int wg_chunk = (r % A.xc8) * 8 + xcd;
    const int bh = r / A.xc8, Hkv = A.H / A.G;
    J.bi = bh / Hkv;
    J.g = bh % Hkv;
    // wave `range` of the head takes key blocks range, range + ranges, range + 2 * ranges, ...: at any time the
    // resident waves read one contiguous stretch of the keys, which is what the memory system serves fastest
    J.range = wg_chunk * AM_WAVES + wave;
    const int blocks = (A.n + AM_BLOCK_KEYS - 1) / AM_BLOCK_KEYS;
    J.nblk = J.range < blocks ? (blocks - J.range + A.ranges - 1) / A.ranges : 0;
    const int h_in_group = group * A.hpw;
    J.head0 = J.g * A.G + h_in_group;
    J.nrb = min(A.hpw, A.G - h_in_group) * A.qbs;
    return J.nblk > 0 && J.range < A.ranges;
}

// ---- pass 1 ---------------------------------------------------------------------------------------
template <int DH, int QB>
__global__ __launch_bounds__(64 * AM_WAVES, 2) void attn_stats_wave_kernel(AttnArgs A, float *__restrict__ part)
{
    using g = Geo<DH>;
    __shared__ __attribute__((aligned(1024))) char lds[AM_WAVES][2][g::BLOCK_BYTES];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    WaveJob J;
    if (!wave_job(A, wave, J)) return; // no barrier in this kernel: a wave may leave at any time
    const bf16_t *kbase = A.k + J.bi * A.ks0 + J.g * A.ks1;
    const __amdgpu_buffer_rsrc_t krsrc = make_k_rsrc<DH>(kbase, A.ks2, A.n);
    const int nblk = J.nblk;
    const int stride_keys = A.ranges * AM_BLOCK_KEYS; // keys between two blocks of this wave
    const int key_first = J.range * AM_BLOCK_KEYS;
    char *slot0 = lds[wave][0], *slot1 = lds[wave][1];

    load_k_block<DH>(krsrc, A.ks2, key_first, A.n, slot0, lane);
    if (nblk > 1) load_k_block<DH>(krsrc, A.ks2, key_first + stride_keys, A.n, slot1, lane);

    bf16x8 qf[QB][g::KS];
    load_q_frags<DH, QB>(A, J.bi, J.head0, J.nrb, l32, half, qf);
    float m[QB], l[QB];
#pragma unroll
    for (int rb = 0; rb < QB; ++rb) { m[rb] = AM_NEG; l[rb] = 0.f; }

    // One key block: its fragments from the ring slot, the slot refilled two blocks ahead, then per row block the
    // MFMA chain and the running max / sum of its 16 logits per lane (t = acc * c, c > 0).  MASKED blocks reach
    // past the last key or (causal tail) into the last W keys; they are the last few of the last ranges only.
    auto key_block = [&](int kb, auto masked_c) {
        constexpr bool MASKED = decltype(masked_c)::value;
        const char *cur = (kb & 1) ? slot1 : slot0;
        const int key0 = key_first + kb * stride_keys;
        // this block's loads have landed once at most the next block's are outstanding
        if (kb + 1 < nblk) wait_vmcnt<g::LOADS>(); else wait_vmcnt<0>();
        bf16x8 kf[g::KS];
        read_k_frags<DH>(cur, l32, half, kf);
        wait_lgkmcnt0(); // the fragments are in registers: the slot may be refilled
        if (kb + 2 < nblk) load_k_block<DH>(krsrc, A.ks2, key0 + 2 * stride_keys, A.n, (char *)cur, lane);
        auto chain = [&](int rb) {
            f32x16 a = zero16();
#pragma unroll
            for (int s = 0; s < g::KS; ++s) a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[rb][s], a, 0, 0, 0);
            return a;
        };
        auto fold = [&](f32x16 acc, int rb) {
            if (MASKED) {
                // last key this lane's query row sees
                const int last_seen = A.causal ? A.n - A.W + (rb % A.qbs) * 32 + l32 : A.n - 1;
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
            const float mn = fmaxf(m[rb], amax * A.c);
            float add = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) add += __builtin_amdgcn_exp2f(fmaf(acc[j], A.c, -mn));
            l[rb] = l[rb] * __builtin_amdgcn_exp2f(m[rb] - mn) + add;
            m[rb] = mn;
        };
        // the exponentials of row block r run while the matrix pipe works on row block r + 1
        f32x16 acc[2];
        acc[0] = chain(0);
#pragma unroll
        for (int rb = 1; rb < QB; ++rb) {
            acc[rb & 1] = chain(rb);
            fold(acc[(rb - 1) & 1], rb - 1);
        }
        fold(acc[(QB - 1) & 1], QB - 1);
    };
    // blocks that lie wholly inside the keys every row of the window sees need no masking
    const int clean_end = A.causal ? min(A.n, A.n - A.W + 1) : A.n;
    for (int kb = 0; kb < nblk; ++kb) {
        if (key_first + kb * stride_keys + AM_BLOCK_KEYS <= clean_end) key_block(kb, std::false_type{});
        else key_block(kb, std::true_type{});
    }
    // merge the two lanes that hold the same query row, then one (m, l) pair per row and key range
#pragma unroll
    for (int rb = 0; rb < QB; ++rb) {
        const float mo = __shfl_xor(m[rb], 32), lo = __shfl_xor(l[rb], 32);
        const float mt = fmaxf(m[rb], mo);
        const float lt = l[rb] * __builtin_amdgcn_exp2f(m[rb] - mt) + lo * __builtin_amdgcn_exp2f(mo - mt);
        const int head = J.head0 + rb / A.qbs;
        const int w = (rb % A.qbs) * 32 + l32;
        if (rb < J.nrb && half == 0 && w < A.W) {
            float *dst = part + ((((size_t)J.bi * A.H + head) * A.W + w) * (size_t)A.ranges + J.range) * 2;
            dst[0] = mt;
            dst[1] = lt;
        }
    }
}

// ---- pass 2 ---------------------------------------------------------------------------------------
template <int DH, int QB>
__global__ __launch_bounds__(64 * AM_WAVES, 2) void attn_colsum_wave_kernel(AttnArgs A, const float *__restrict__ stats,
                                                                        float *__restrict__ a_raw)
{
    using g = Geo<DH>;
    __shared__ __attribute__((aligned(1024))) char lds[AM_WAVES][2][g::BLOCK_BYTES];
    // per wave and row block: -E_w / c of the block's 32 window rows, ordered [half][16] as a lane's accumulators are
    __shared__ __attribute__((aligned(16))) float etab[AM_WAVES][QB][2][16];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    WaveJob J;
    if (!wave_job(A, wave, J)) return; // no barrier in this kernel
    const bf16_t *kbase = A.k + J.bi * A.ks0 + J.g * A.ks1;
    const __amdgpu_buffer_rsrc_t krsrc = make_k_rsrc<DH>(kbase, A.ks2, A.n);
    const int nblk = J.nblk;
    const int stride_keys = A.ranges * AM_BLOCK_KEYS; // keys between two blocks of this wave
    const int key_first = J.range * AM_BLOCK_KEYS;
    char *slot0 = lds[wave][0], *slot1 = lds[wave][1];

    load_k_block<DH>(krsrc, A.ks2, key_first, A.n, slot0, lane);
    if (nblk > 1) load_k_block<DH>(krsrc, A.ks2, key_first + stride_keys, A.n, slot1, lane);

    bf16x8 qf[QB][g::KS];
    load_q_frags<DH, QB>(A, J.bi, J.head0, J.nrb, l32, half, qf);
    // table entry (rb, hf, j) belongs to window row 8*(j/4) + 4*hf + j%4 of the block; rows past W get -inf
    // (weight 0).  Lane t < 32 writes entry (hf = t / 16, j = t % 16) of every row block.
    const float inv_c = 1.0f / A.c;
    if (lane < 32) {
        const int hf = lane >> 4, j = lane & 15;
#pragma unroll
        for (int rb = 0; rb < QB; ++rb) {
            const int rbc = min(rb, J.nrb - 1);
            const int head = J.head0 + rbc / A.qbs;
            const int w = (rbc % A.qbs) * 32 + 8 * (j / 4) + 4 * hf + (j % 4);
            float e = -INFINITY;
            if (w < A.W) e = -stats[(((size_t)J.bi * A.H + head) * A.W + w) * 2] * inv_c;
            etab[wave][rb][hf][j] = e;
        }
    }
    // (the table is read by the wave that wrote it: program order and the LDS counter keep it coherent)

    auto key_block = [&](int kb, auto masked_c) {
        constexpr bool MASKED = decltype(masked_c)::value; // (causal tail) some window rows do not see these keys
        const char *cur = (kb & 1) ? slot1 : slot0;
        const int key0 = key_first + kb * stride_keys;
        if (kb + 1 < nblk) wait_vmcnt<g::LOADS>(); else wait_vmcnt<0>();
        bf16x8 kf[g::KS];
        read_k_frags<DH>(cur, l32, half, kf);
        wait_lgkmcnt0();
        if (kb + 2 < nblk) load_k_block<DH>(krsrc, A.ks2, key0 + 2 * stride_keys, A.n, (char *)cur, lane);
        const int key = key0 + l32;
        auto chain = [&](int rb) {
            // accumulators start at -E_w / c
            const f32x4 *t = reinterpret_cast<const f32x4 *>(&etab[wave][rb][half][0]);
            const f32x4 t0 = t[0], t1 = t[1], t2 = t[2], t3 = t[3];
            f32x16 a = f32x16{t0[0], t0[1], t0[2], t0[3], t1[0], t1[1], t1[2], t1[3],
                              t2[0], t2[1], t2[2], t2[3], t3[0], t3[1], t3[2], t3[3]};
#pragma unroll
            for (int s = 0; s < g::KS; ++s) a = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[rb][s], kf[s], a, 0, 0, 0);
            return a;
        };
        auto weights = [&](f32x16 acc, int rb) {
            if (MASKED) {
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (key > A.n - A.W + (rb % A.qbs) * 32 + 8 * (j / 4) + 4 * half + (j % 4)) acc[j] = -INFINITY;
            }
            float s = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) s += __builtin_amdgcn_exp2f(acc[j] * A.c);
            return s;
        };
        // a head's window sum runs over its qbs row blocks; the wave's heads one after the other
        auto finish_head = [&](float colsum, int rb) {
            colsum += __shfl_xor(colsum, 32);
            if (rb < J.nrb && half == 0 && key < A.n)
                a_raw[((size_t)J.bi * A.H + J.head0 + rb / A.qbs) * (size_t)A.n + key] = colsum;
        };
        f32x16 acc[2];
        float colsum = 0.f;
        acc[0] = chain(0);
#pragma unroll
        for (int rb = 1; rb < QB; ++rb) {
            acc[rb & 1] = chain(rb);
            colsum += weights(acc[(rb - 1) & 1], rb - 1);
            if (rb % A.qbs == 0) { // row block rb-1 was the last of its head
                finish_head(colsum, rb - 1);
                colsum = 0.f;
            }
        }
        colsum += weights(acc[(QB - 1) & 1], QB - 1);
        finish_head(colsum, QB - 1);
    };
    const int clean_end = A.causal ? min(A.n, A.n - A.W + 1) : (1 << 30);
    for (int kb = 0; kb < nblk; ++kb) {
        if (key_first + kb * stride_keys + AM_BLOCK_KEYS <= clean_end) key_block(kb, std::false_type{});
        else key_block(kb, std::true_type{});
    }
}

} // namespace

bool attn_wave_supported(const Dims &d)
{
    return (d.dh == 64 || d.dh == 128) && d.W <= 32 * AM_MAX_QB &&
           ((int64_t)(d.n - 1) * d.ks[2] + d.dh) * 2 < ((int64_t)1 << 31);
}

// Keys per wave (it sets the number of waves per head).  Many keys spread a wave's fixed cost (its query fragments:
// up to 32 KiB) over more key blocks; few give the chip enough waves (it holds 8 per CU, 2048 in all).  Measured
// on the 5:1 group with a 64-row window at a 128K context: 1024 keys per wave is the best (512 and 2048 are 4-7 %
// slower, 256 is 14 % slower), so: 1024, halved while that leaves less than one full round of waves.
static int attn_kpw(const Dims &d, int groups)
{
    const long long per_range = (long long)d.batch * d.Hkv * groups;
    int kpw = 1024;
    while (kpw > AM_MIN_KPW && per_range * ((d.n + kpw - 1) / kpw) < 2048) kpw >>= 1;
    return kpw;
}

static AttnArgs make_args(const Dims &d, const void *q, const void *k)
{
    AttnArgs A;
    A.q = (const bf16_t *)q; A.k = (const bf16_t *)k;
    A.H = d.H; A.G = d.G; A.n = d.n; A.W = d.W; A.causal = d.causal;
    A.qbs = (d.W + 31) / 32;
    // Heads per wave: every wave runs all of its hpw * qbs row blocks (a last group with fewer heads works on zero
    // queries for the rest), so hpw is the choice with the least wave work in all, a key block's own cost (its
    // loads and fragment reads) counted like one row block's; ties go to the larger hpw (measured on the 5:1 group
    // with a 64-row window: two heads per wave 1.5 % faster than one).
    A.hpw = 1;
    {
        const int most = AM_MAX_QB / A.qbs < d.G ? AM_MAX_QB / A.qbs : d.G;
        int best = 1 << 30;
        for (int h = 1; h <= (most > 0 ? most : 1); ++h) {
            const int cost = ((d.G + h - 1) / h) * (1 + h * A.qbs);
            if (cost <= best) { best = cost; A.hpw = h; }
        }
    }
    A.groups = (d.G + A.hpw - 1) / A.hpw;
    const int kpw = attn_kpw(d, A.groups);
    A.ranges = (d.n + kpw - 1) / kpw;
    A.xc8 = ((A.ranges + AM_WAVES - 1) / AM_WAVES + 7) / 8;
    A.c = d.scale * AM_LOG2E;
    A.ks0 = d.ks[0]; A.ks1 = d.ks[1]; A.ks2 = d.ks[2];
    return A;
}
int wave_attn_chunks(const Dims &d) { return make_args(d, nullptr, nullptr).ranges; }

template <int DH>
static void launch_sweep(const AttnArgs &A, const Dims &d, bool stats_pass, float *part, const float *stats, float *a_raw,
                         hipStream_t s)
{
    const dim3 grid((unsigned)(8 * A.groups * A.xc8 * d.batch * d.Hkv)), block(64 * AM_WAVES);
    const int qb = A.hpw * A.qbs;
#define CKV_SWEEP(QB)                                                                                             \
    if (stats_pass) hipLaunchKernelGGL((attn_stats_wave_kernel<DH, QB>), grid, block, 0, s, A, part);              \
    else hipLaunchKernelGGL((attn_colsum_wave_kernel<DH, QB>), grid, block, 0, s, A, stats, a_raw)
    if (qb == 1) { CKV_SWEEP(1); }
    else if (qb == 2) { CKV_SWEEP(2); }
    else if (qb == 3) { CKV_SWEEP(3); }
    else { CKV_SWEEP(4); }
#undef CKV_SWEEP
}

hipError_t launch_attn_stats_wave(const Dims &d, const void *q, const void *k, float *part, int chunks, hipStream_t s)
{
    const AttnArgs A = make_args(d, q, k);
    if (chunks != A.ranges) return hipErrorInvalidValue;
    if (d.dh == 64) launch_sweep<64>(A, d, true, part, nullptr, nullptr, s);
    else launch_sweep<128>(A, d, true, part, nullptr, nullptr, s);
    return hipGetLastError();
}

hipError_t launch_attn_colsum_wave(const Dims &d, const void *q, const void *k, const float *stats, float *a_raw,
                                   hipStream_t s)
{
    const AttnArgs A = make_args(d, q, k);
    if (d.dh == 64) launch_sweep<64>(A, d, false, nullptr, stats, a_raw, s);
    else launch_sweep<128>(A, d, false, nullptr, stats, a_raw, s);
    return hipGetLastError();
}

} // namespace ckv
