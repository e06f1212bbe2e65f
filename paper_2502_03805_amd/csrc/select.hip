// Budget split and the two Top-k stages (Algorithm 1, lines 4-9).
//
//   b' = floor(alpha * B), b'' = B - b'
//   S1 = the b' largest attn;  S2 = the b'' largest crit among entries outside S1
//   idx = S1 u S2 in ascending token order
// With a kept observation window (protect = W > 0) the last min(W, B) entries are part of the result as they
// are, and the two stages run on entries 0 .. n-W-1 with the budget that is left (B above is then that rest).
// Top-k is an exact order statistic: a most-significant-digit radix select on an order-preserving
// 32-bit image of the float keys (digits of 11, 11 and 10 bits).  Equal keys are taken in ascending
// token order: after the last digit the threshold key tau and the number r of entries equal to tau that
// still fit are known, and the r-th tie is located with ordered prefix counts.
//
// A head's n keys are cut into slices of 2048 tokens, one 256-thread workgroup per (slice, head), so the
// whole chip works on a layer's few heads.  Workgroups only meet at kernel boundaries:
//   zero      clear the digit histograms
//   hist 1.0  digit-0 histogram of attn            (LDS histogram per slice, flushed with integer atomics)
//   hist 1.1  find digit 0, digit-1 histogram of the entries that match it
//   hist 1.2  find digit 1, digit-2 histogram (each slice also keeps its own copy)
//   mark      find digit 2 -> tau1, r1; stage-1 membership (ties ranked through the slices' own digit-2
//             histograms: the ties of a slice are its count at digit 2 of tau1), stage-2 keys written
//             (stage-1 entries carry a reserved key), digit-0 histogram of stage 2
//   hist 2.1, hist 2.2  (each slice also counts its entries above the digit just decided; 2.2 keeps the slice's
//             digit-2 counts as suffix sums)
//   write     find digit 2 -> tau2, r2; ordered write of S1 u S2: what earlier slices contribute is read from
//             their per-slice counts; -1 tail; count
// Every decision is integer arithmetic on exact counts, so the result does not depend on scheduling.
#include "common.hpp"

namespace ckv {

constexpr int SEL_THREADS = 256;
constexpr int SEL_PER_THREAD = 8;
constexpr int SEL_SLICE = SEL_THREADS * SEL_PER_THREAD; // tokens per workgroup
constexpr int SEL_BINS = 2048;
constexpr uint32_t SEL_TAKEN = 0xFFFFFFFFu; // image of no finite float: marks stage-1 entries
constexpr int DSHIFT0 = 21, DSHIFT1 = 10;
constexpr uint32_t DMASK0 = 0x7FFu, DMASK1 = 0x7FFu, DMASK2 = 0x3FFu;

// per-head state words
enum { ST_D0 = 0, ST_A0, ST_D1, ST_A1, ST_TAU, ST_R, ST_WORDS = 8 };

struct SelArgs {
    const uint32_t *attn; // float bits
    const uint32_t *crit;
    const int32_t *budget;
    uint32_t *keys2;   // [heads][n]
    uint32_t *hist;    // [heads][2 stages][3 passes][SEL_BINS]
    uint32_t *state;   // [heads][2 stages][ST_WORDS]
    uint32_t *slices;  // [heads][3][n_slices]: stage-1 members; stage-2 entries above the threshold at digit 0; at digit 1
    uint32_t *slice_suf; // [heads][n_slices][1025]: each slice's digit-2 suffix counts of stage 2
    uint32_t *slice_hist; // [heads][n_slices][1024]: each slice's digit-2 histogram of stage 1
    int32_t *idx;
    int32_t *count;
    double alpha;
    int n, max_budget, n_slices;
    int n_rank; // entries 0 .. n_rank-1 compete in the two stages (n minus the kept window)
};

// Monotone map float -> uint32 (larger float, larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t order_key(uint32_t u)
{
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// B: entries the head keeps in all; kept: how many of them are the kept window's (the last `kept` entries);
// b1, b2: the two stages' shares of the rest
__device__ __forceinline__ void head_budget(const SelArgs &A, int head, int &B, int &b1, int &b2, int &kept)
{
    B = max(0, min(A.budget[head], min(A.n, A.max_budget)));
    kept = min(A.n - A.n_rank, B);
    const int rest = B - kept;
    b1 = (int)floor(A.alpha * (double)rest);
    b2 = rest - b1;
}

struct SelShared {
    uint32_t hist[SEL_BINS];
    uint32_t wave_tot[SEL_THREADS / 64];
    uint32_t digit, above;
};

// Exclusive prefix sum over the workgroup in thread order; total in `total`.
__device__ __forceinline__ uint32_t block_exclusive_scan(SelShared &sh, uint32_t x, uint32_t &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    __syncthreads(); // wave_tot may still be read by a previous scan
    if (lane == 63) sh.wave_tot[wave] = incl;
    __syncthreads();
    uint32_t base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < SEL_THREADS / 64; ++w) {
        const uint32_t t = sh.wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    total = tot;
    return base + incl - x;
}

__device__ __forceinline__ uint32_t block_sum(SelShared &sh, uint32_t x)
{
    uint32_t total;
    (void)block_exclusive_scan(sh, x, total);
    return total;
}

// The thread's 8 consecutive words starting at token i0; words at or beyond n read as 0.
__device__ __forceinline__ void load8(const uint32_t *base, int i0, int n, bool vec_ok, uint32_t (&out)[8])
{
    if (vec_ok && i0 + 7 < n) {
        const uint4 a = *reinterpret_cast<const uint4 *>(base + i0);
        const uint4 b = *reinterpret_cast<const uint4 *>(base + i0 + 4);
        out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
        out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) out[j] = (i0 + j < n) ? base[i0 + j] : 0u;
    }
}

// Largest digit d of a global histogram with  #(digit > d) < remaining <= #(digit >= d); also #(digit > d).
__device__ void find_digit(SelShared &sh, const uint32_t *ghist, int nbins, uint32_t remaining, uint32_t &digit,
                           uint32_t &above)
{
    constexpr int PER = SEL_BINS / SEL_THREADS; // 8 bins per thread, descending order
    uint32_t h[PER], local = 0;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int bin = nbins - 1 - (threadIdx.x * PER + j);
        h[j] = bin >= 0 ? ghist[bin] : 0u;
        local += h[j];
    }
    if (threadIdx.x == 0) { sh.digit = 0u; sh.above = 0u; }
    uint32_t total;
    uint32_t run = block_exclusive_scan(sh, local, total);
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        if (run < remaining && remaining <= run + h[j]) {
            sh.digit = (uint32_t)(nbins - 1 - (threadIdx.x * PER + j));
            sh.above = run;
        }
        run += h[j];
    }
    __syncthreads();
    digit = sh.digit;
    above = sh.above;
    __syncthreads();
}

__global__ __launch_bounds__(256) void select_zero_kernel(uint32_t *p, size_t words)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < words) p[i] = 0u;
}

// Histogram of one digit over a slice.  STAGE 0 reads attn floats, STAGE 1 the stage-2 key array.
// PASS 0 histograms digit 0 of every entry; PASS 1 / 2 first decode the previous digit(s) of the threshold.
template <int STAGE, int PASS>
__global__ __launch_bounds__(SEL_THREADS) void select_hist_kernel(SelArgs A)
{
    __shared__ SelShared sh;
    const int slice = blockIdx.x, head = blockIdx.y;
    int B, b1, b2, kept;
    head_budget(A, head, B, b1, b2, kept);
    const uint32_t want = STAGE == 0 ? (uint32_t)b1 : (uint32_t)b2;
    if (want == 0) return;
    uint32_t *hist = A.hist + ((size_t)head * 2 + STAGE) * 3 * SEL_BINS;
    uint32_t *st = A.state + ((size_t)head * 2 + STAGE) * ST_WORDS;
    uint32_t prefix = 0u, pmask = 0u;
    if (PASS == 1) {
        uint32_t d0, a0;
        find_digit(sh, hist, 2048, want, d0, a0);
        if (slice == 0 && threadIdx.x == 0) { st[ST_D0] = d0; st[ST_A0] = a0; }
        prefix = d0 << DSHIFT0; pmask = DMASK0 << DSHIFT0;
    } else if (PASS == 2) {
        const uint32_t d0 = st[ST_D0], a0 = st[ST_A0];
        uint32_t d1, a1;
        find_digit(sh, hist + SEL_BINS, 2048, want - a0, d1, a1);
        if (slice == 0 && threadIdx.x == 0) { st[ST_D1] = d1; st[ST_A1] = a1; }
        prefix = (d0 << DSHIFT0) | (d1 << DSHIFT1);
        pmask = (DMASK0 << DSHIFT0) | (DMASK1 << DSHIFT1);
    }
    const int shift = PASS == 0 ? DSHIFT0 : PASS == 1 ? DSHIFT1 : 0;
    const uint32_t mask = PASS == 2 ? DMASK2 : DMASK0;

    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) sh.hist[b] = 0u;
    __syncthreads();
    const uint32_t *src = (STAGE == 0 ? A.attn : A.keys2) + (size_t)head * A.n;
    const bool vec_ok = (A.n & 3) == 0;
    const int i0 = slice * SEL_SLICE + threadIdx.x * SEL_PER_THREAD;
    uint32_t w[8];
    load8(src, i0, A.n, vec_ok, w);
    // runs of equal digits inside a thread's 8 tokens are merged into one atomic
    uint32_t run_digit = 0u, run_len = 0u, n_above = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t key = STAGE == 0 ? order_key(w[j]) : w[j];
        const bool on = (i0 + j < A.n_rank) && key != SEL_TAKEN && (key & pmask) == prefix;
        if (STAGE == 1 && PASS >= 1) {
            // stage 2: entries that beat the threshold at the digit this kernel has just decided (and agree with it
            // on the digit before): the ordered write adds these per-slice counts up instead of counting again
            constexpr uint32_t M0 = DMASK0 << DSHIFT0;
            const bool above = (i0 + j < A.n_rank) && key != SEL_TAKEN && (key & pmask) > prefix &&
                               (PASS == 1 || (key & M0) == (prefix & M0));
            n_above += above ? 1u : 0u;
        }
        const uint32_t d = (key >> shift) & mask;
        if (on && run_len && d == run_digit) {
            ++run_len;
        } else {
            if (run_len) atomicAdd(&sh.hist[run_digit], run_len);
            run_digit = d;
            run_len = on ? 1u : 0u;
        }
    }
    if (run_len) atomicAdd(&sh.hist[run_digit], run_len);
    __syncthreads();
    uint32_t *dst = hist + PASS * SEL_BINS;
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) {
        const uint32_t c = sh.hist[b];
        if (c) atomicAdd(&dst[b], c);
    }
    if (STAGE == 0 && PASS == 2) { // the slice's own counts: the mark kernel reads its ties from here
        uint32_t *mine = A.slice_hist + ((size_t)head * A.n_slices + slice) * 1024;
        for (int b = threadIdx.x; b < 1024; b += SEL_THREADS) mine[b] = sh.hist[b];
    }
    if (STAGE == 1 && PASS >= 1) {
        uint32_t *sl = A.slices + (size_t)head * 3 * A.n_slices;
        const uint32_t tot = block_sum(sh, n_above);
        if (threadIdx.x == 0) sl[PASS * A.n_slices + slice] = tot;
    }
    if (STAGE == 1 && PASS == 2) {
        // the slice's digit-2 counts as suffix sums: suf[b] = entries of the slice (with the threshold's first two
        // digits) whose digit 2 is >= b; suf[1024] = 0.  The write kernel reads suf[d2 + 1] and suf[d2].
        static_assert(SEL_THREADS * 4 == 1024, "four bins per thread");
        uint32_t h[4], local = 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j) { h[j] = sh.hist[threadIdx.x * 4 + j]; local += h[j]; }
        uint32_t total;
        uint32_t below = block_exclusive_scan(sh, local, total); // entries in bins before this thread's
        uint32_t *suf = A.slice_suf + ((size_t)head * A.n_slices + slice) * 1025;
#pragma unroll
        for (int j = 0; j < 4; ++j) { suf[threadIdx.x * 4 + j] = total - below; below += h[j]; }
        if (threadIdx.x == 0) suf[1024] = 0u;
    }
}

// Stage-1 membership, stage-2 keys, digit-0 histogram of stage 2.
__global__ __launch_bounds__(SEL_THREADS) void select_mark_kernel(SelArgs A)
{
    __shared__ SelShared sh;
    const int slice = blockIdx.x, head = blockIdx.y;
    int B, b1, b2, kept;
    head_budget(A, head, B, b1, b2, kept);
    uint32_t *st1 = A.state + ((size_t)head * 2 + 0) * ST_WORDS;
    uint32_t tau1 = 0u, r1 = 0u, before = 0u;
    if (b1 > 0) { // uniform over the workgroup
        // last digit of the stage-1 threshold, decided redundantly by every workgroup
        const uint32_t d0 = st1[ST_D0], a0 = st1[ST_A0], d1 = st1[ST_D1], a1 = st1[ST_A1];
        uint32_t d2, a2;
        find_digit(sh, A.hist + ((size_t)head * 2 + 0) * 3 * SEL_BINS + 2 * SEL_BINS, 1024, (uint32_t)b1 - a0 - a1, d2, a2);
        tau1 = (d0 << DSHIFT0) | (d1 << DSHIFT1) | d2;
        r1 = (uint32_t)b1 - a0 - a1 - a2;
        if (slice == 0 && threadIdx.x == 0) { st1[ST_TAU] = tau1; st1[ST_R] = r1; }
        // ties of stage 1 in earlier slices: their counts at digit d2 (only entries with the threshold's first two
        // digits were counted there)
        const uint32_t *sh2 = A.slice_hist + (size_t)head * A.n_slices * 1024 + d2;
        for (int s = threadIdx.x; s < slice; s += SEL_THREADS) before += sh2[(size_t)s * 1024];
        before = block_sum(sh, before);
    }

    const bool vec_ok = (A.n & 3) == 0;
    const int i0 = slice * SEL_SLICE + threadIdx.x * SEL_PER_THREAD;
    uint32_t a[8], c[8];
    load8(A.attn + (size_t)head * A.n, i0, A.n, vec_ok, a);
    load8(A.crit + (size_t)head * A.n, i0, A.n, vec_ok, c);
    bool gt[8], tie[8];
    uint32_t n_tie = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t key = order_key(a[j]);
        const bool valid = i0 + j < A.n_rank;
        gt[j] = b1 > 0 && valid && key > tau1;
        tie[j] = b1 > 0 && valid && key == tau1;
        n_tie += tie[j] ? 1u : 0u;
    }
    uint32_t tot;
    uint32_t rank = before + block_exclusive_scan(sh, n_tie, tot);
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) sh.hist[b] = 0u;
    __syncthreads();
    uint32_t key2[8];
    uint32_t run_digit = 0u, run_len = 0u, n_taken = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        bool taken = gt[j] || (i0 + j >= A.n - kept && i0 + j < A.n); // the kept window carries the stage-1 mark
        if (tie[j]) { taken = rank < r1; ++rank; }
        n_taken += taken ? 1u : 0u;
        key2[j] = taken ? SEL_TAKEN : order_key(c[j]);
        const bool on = b2 > 0 && (i0 + j < A.n_rank) && !taken;
        const uint32_t d = (key2[j] >> DSHIFT0) & DMASK0;
        if (on && run_len && d == run_digit) {
            ++run_len;
        } else {
            if (run_len) atomicAdd(&sh.hist[run_digit], run_len);
            run_digit = d;
            run_len = on ? 1u : 0u;
        }
    }
    if (run_len) atomicAdd(&sh.hist[run_digit], run_len);
    uint32_t *k2 = A.keys2 + (size_t)head * A.n;
    if (vec_ok && i0 + 7 < A.n) {
        *reinterpret_cast<uint4 *>(k2 + i0) = make_uint4(key2[0], key2[1], key2[2], key2[3]);
        *reinterpret_cast<uint4 *>(k2 + i0 + 4) = make_uint4(key2[4], key2[5], key2[6], key2[7]);
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (i0 + j < A.n) k2[i0 + j] = key2[j];
    }
    __syncthreads();
    if (b2 > 0) {
        uint32_t *dst = A.hist + ((size_t)head * 2 + 1) * 3 * SEL_BINS;
        for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) {
            const uint32_t cnt = sh.hist[b];
            if (cnt) atomicAdd(&dst[b], cnt);
        }
    }
    const uint32_t taken_here = block_sum(sh, n_taken);
    if (threadIdx.x == 0) A.slices[(size_t)head * 3 * A.n_slices + slice] = taken_here;
}

// Ordered write of S1 u S2.
__global__ __launch_bounds__(SEL_THREADS) void select_write_kernel(SelArgs A)
{
    __shared__ SelShared sh;
    const int slice = blockIdx.x, head = blockIdx.y;
    int B, b1, b2, kept;
    head_budget(A, head, B, b1, b2, kept);
    uint32_t *st2 = A.state + ((size_t)head * 2 + 1) * ST_WORDS;
    uint32_t tau2 = 0u, r2 = 0u, d2 = 0u;
    if (b2 > 0) { // uniform over the workgroup: last digit of the stage-2 threshold
        const uint32_t d0 = st2[ST_D0], a0 = st2[ST_A0], d1 = st2[ST_D1], a1 = st2[ST_A1];
        uint32_t a2;
        find_digit(sh, A.hist + ((size_t)head * 2 + 1) * 3 * SEL_BINS + 2 * SEL_BINS, 1024, (uint32_t)b2 - a0 - a1, d2, a2);
        tau2 = (d0 << DSHIFT0) | (d1 << DSHIFT1) | d2;
        r2 = (uint32_t)b2 - a0 - a1 - a2;
        if (slice == 0 && threadIdx.x == 0) { st2[ST_TAU] = tau2; st2[ST_R] = r2; }
    }
    const uint32_t *taken_cnt = A.slices + (size_t)head * 3 * A.n_slices;
    const uint32_t *above0 = taken_cnt + A.n_slices, *above1 = above0 + A.n_slices;
    const uint32_t *suf = A.slice_suf + (size_t)head * A.n_slices * 1025;
    // entries written and stage-2 ties seen by earlier slices: slice s' contributes its stage-1 members, its
    // stage-2 keys above tau2 (counted digit by digit by the histogram kernels) and
    // clamp(r2 - ties before s', 0, ties of s')
    uint32_t out_base = 0u, tie_base = 0u, carry = 0u;
    for (int c0 = 0; c0 < slice; c0 += SEL_THREADS) {
        const int s = c0 + threadIdx.x;
        uint32_t t = 0u, sel_s = 0u;
        if (s < slice) {
            sel_s = taken_cnt[s];
            if (b2 > 0) {
                const uint32_t ge = suf[(size_t)s * 1025 + d2], gt2 = suf[(size_t)s * 1025 + d2 + 1];
                t = ge - gt2;
                sel_s += above0[s] + above1[s] + gt2;
            }
        }
        uint32_t tot;
        const uint32_t tb = carry + block_exclusive_scan(sh, t, tot);
        uint32_t mine = 0u;
        if (s < slice) mine = sel_s + min(r2 > tb ? r2 - tb : 0u, t);
        out_base += block_sum(sh, mine);
        carry += tot;
    }
    tie_base = carry;

    const bool vec_ok = (A.n & 3) == 0;
    const int i0 = slice * SEL_SLICE + threadIdx.x * SEL_PER_THREAD;
    uint32_t key[8];
    load8(A.keys2 + (size_t)head * A.n, i0, A.n, vec_ok, key);
    bool sel[8], tie[8];
    uint32_t n_tie = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const bool valid = i0 + j < A.n_rank; // window entries outside the budget carry ordinary keys: not ranked
        const bool taken = i0 + j < A.n && key[j] == SEL_TAKEN;
        sel[j] = taken || (b2 > 0 && valid && key[j] > tau2);
        tie[j] = b2 > 0 && valid && key[j] == tau2;
        n_tie += tie[j] ? 1u : 0u;
    }
    uint32_t tot;
    uint32_t rank = tie_base + block_exclusive_scan(sh, n_tie, tot);
    uint32_t n_sel = 0u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        if (tie[j]) { sel[j] = rank < r2; ++rank; }
        n_sel += sel[j] ? 1u : 0u;
    }
    uint32_t pos = out_base + block_exclusive_scan(sh, n_sel, tot);
    int32_t *out = A.idx + (size_t)head * A.max_budget;
#pragma unroll
    for (int j = 0; j < 8; ++j)
        if (sel[j]) {
            if (pos < (uint32_t)A.max_budget) out[pos] = i0 + j;
            ++pos;
        }
    // unused tail and the count, spread over the slices
    for (int j = B + slice * SEL_THREADS + (int)threadIdx.x; j < A.max_budget; j += A.n_slices * SEL_THREADS) out[j] = -1;
    if (slice == 0 && threadIdx.x == 0) A.count[head] = B;
}

size_t select_workspace_words(int heads, int n)
{
    const size_t n_slices = (size_t)(n + SEL_SLICE - 1) / SEL_SLICE;
    return (size_t)heads * (2 * 3 * SEL_BINS + 2 * ST_WORDS) + (size_t)heads * 3 * n_slices + (size_t)heads * n_slices * (1024 + 1025);
}

static SelArgs make_sel_args(int heads, int n, int protect, const float *attn, const float *crit, const int32_t *budget,
                             float alpha, int max_budget, int32_t *idx, int32_t *count, uint32_t *keys2, uint32_t *scratch)
{
    SelArgs A;
    A.attn = reinterpret_cast<const uint32_t *>(attn);
    A.crit = reinterpret_cast<const uint32_t *>(crit);
    A.budget = budget;
    A.keys2 = keys2;
    A.hist = scratch;
    A.state = scratch + (size_t)heads * 2 * 3 * SEL_BINS;
    A.slices = A.state + (size_t)heads * 2 * ST_WORDS;
    A.idx = idx; A.count = count;
    A.alpha = (double)alpha;
    A.n = n; A.max_budget = max_budget;
    A.n_rank = n - protect;
    A.n_slices = (n + SEL_SLICE - 1) / SEL_SLICE;
    A.slice_hist = A.slices + (size_t)heads * 3 * A.n_slices;
    A.slice_suf = A.slice_hist + (size_t)heads * A.n_slices * 1024;
    return A;
}

// First half of the selection: the three digit histograms of stage 1.  It reads attn only (not crit), so it can
// run while the projected-value magnitudes are still being computed.
hipError_t launch_select_stage1_hist(int heads, int n, int protect, const float *attn, const int32_t *budget, float alpha,
                                     int max_budget, uint32_t *keys2, uint32_t *scratch, hipStream_t s)
{
    const SelArgs A = make_sel_args(heads, n, protect, attn, attn, budget, alpha, max_budget, nullptr, nullptr, keys2, scratch);
    const size_t zero_words = (size_t)heads * (2 * 3 * SEL_BINS + 2 * ST_WORDS);
    dim3 grid(A.n_slices, heads), block(SEL_THREADS);
    hipLaunchKernelGGL(select_zero_kernel, dim3((unsigned)((zero_words + 255) / 256)), dim3(256), 0, s, scratch, zero_words);
    hipLaunchKernelGGL((select_hist_kernel<0, 0>), grid, block, 0, s, A);
    hipLaunchKernelGGL((select_hist_kernel<0, 1>), grid, block, 0, s, A);
    hipLaunchKernelGGL((select_hist_kernel<0, 2>), grid, block, 0, s, A);
    return hipGetLastError();
}

// Second half: stage-1 membership and stage-2 keys, the two remaining histograms of stage 2, the ordered write.
hipError_t launch_select_finish(int heads, int n, int protect, const float *attn, const float *crit, const int32_t *budget,
                                float alpha, int max_budget, int32_t *idx, int32_t *count, uint32_t *keys2,
                                uint32_t *scratch, hipStream_t s)
{
    const SelArgs A = make_sel_args(heads, n, protect, attn, crit, budget, alpha, max_budget, idx, count, keys2, scratch);
    dim3 grid(A.n_slices, heads), block(SEL_THREADS);
    hipLaunchKernelGGL(select_mark_kernel, grid, block, 0, s, A);
    hipLaunchKernelGGL((select_hist_kernel<1, 1>), grid, block, 0, s, A);
    hipLaunchKernelGGL((select_hist_kernel<1, 2>), grid, block, 0, s, A);
    hipLaunchKernelGGL(select_write_kernel, grid, block, 0, s, A);
    return hipGetLastError();
}

// heads rows of n keys each (a row is one (batch item, kv head), or one whole batch item for the allocation)
hipError_t launch_select_rows(int heads, int n, int protect, const float *attn, const float *crit,
                              const int32_t *budget, float alpha, int max_budget, int32_t *idx, int32_t *count,
                              uint32_t *keys2, uint32_t *scratch, hipStream_t s)
{
    hipError_t e = launch_select_stage1_hist(heads, n, protect, attn, budget, alpha, max_budget, keys2, scratch, s);
    if (e != hipSuccess) return e;
    return launch_select_finish(heads, n, protect, attn, crit, budget, alpha, max_budget, idx, count, keys2, scratch, s);
}

hipError_t launch_select(const Dims &d, const float *attn, const float *crit, const int32_t *budget, float alpha,
                         int max_budget, int32_t *idx, int32_t *count, uint32_t *keys2, uint32_t *scratch,
                         hipStream_t s)
{
    return launch_select_rows(d.batch * d.Hkv, d.n, d.protect, attn, crit, budget, alpha, max_budget, idx, count, keys2,
                              scratch, s);
}

// ---- budget allocation across the kv heads of a batch item (Algorithm 2, line 1) -------------------------
// The P entries with the largest pooled score among all Hkv * n entries of a batch item are found with the
// same selection kernels (one row of Hkv * n keys per batch item, attention only); a head's share is the
// number of those entries it owns, located by binary search in the ascending index list.
__global__ void allocate_fill_kernel(int32_t *pool_budget, int batch, int P)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < batch) pool_budget[i] = P;
}

__global__ void allocate_count_kernel(const int32_t *__restrict__ idx, int P, int Hkv, int n, int floor_each,
                                      int32_t *__restrict__ budget_out)
{
    const int bi = blockIdx.x, g = threadIdx.x;
    if (g >= Hkv) return;
    const int32_t *row = idx + (size_t)bi * P;
    auto lower_bound = [&](long long key) { // first position whose index is >= key
        int lo = 0, hi = P;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if ((long long)row[mid] < key) lo = mid + 1; else hi = mid;
        }
        return lo;
    };
    const int owned = lower_bound((long long)(g + 1) * n) - lower_bound((long long)g * n);
    budget_out[bi * Hkv + g] = min(n, floor_each + owned);
}

hipError_t launch_allocate(const Dims &d, const float *attn, int total, float floor_frac, int32_t *budget_out,
                           uint32_t *keys2, uint32_t *scratch, int32_t *tmp, hipStream_t s)
{
    const int floor_each = (int)floor((double)floor_frac * (double)total / (double)d.Hkv);
    const int P = (int)min((long long)total - (long long)d.Hkv * floor_each, (long long)d.Hkv * d.n);
    int32_t *pool_budget = tmp;                 // [batch]
    int32_t *pool_count = tmp + d.batch;        // [batch]
    int32_t *pool_idx = tmp + 2 * d.batch;      // [batch][P]
    if (P > 0) {
        hipLaunchKernelGGL(allocate_fill_kernel, dim3((d.batch + 63) / 64), dim3(64), 0, s, pool_budget, d.batch, P);
        hipError_t e = launch_select_rows(d.batch, d.Hkv * d.n, 0, attn, attn, pool_budget, 1.0f, P, pool_idx, pool_count,
                                          keys2, scratch, s);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(allocate_count_kernel, dim3(d.batch), dim3(((d.Hkv + 63) / 64) * 64), 0, s, pool_idx, P, d.Hkv, d.n,
                       floor_each, budget_out);
    return hipGetLastError();
}

} // namespace ckv
