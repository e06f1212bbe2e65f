// Budget split and the two Top-k stages (Algorithm 1, lines 4-9), one workgroup per (batch, kv head).
//
//   b' = floor(alpha * B), b'' = B - b'
//   S1 = the b' largest attn;  S2 = the b'' largest crit among entries outside S1
//   idx = S1 u S2 in ascending token order
// Top-k is an exact order statistic, found by a most-significant-digit radix select on an
// order-preserving 32-bit image of the float keys (digits of 11, 11 and 10 bits, histograms
// in LDS).  Equal keys are taken in ascending token order: the threshold key tau and the
// number r of entries equal to tau that still fit are known after the last digit, and the
// r-th tie is located with an ordered prefix count over the tokens.
// Stage 1 membership is materialised once as the stage-2 key array (taken entries carry a
// reserved key), which the final ordered write reads back.
#include "common.hpp"

namespace ckv {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;
constexpr int SEL_PER_IT = SEL_THREADS * 4;
constexpr int SEL_BINS = 2048;
constexpr uint32_t SEL_TAKEN = 0xFFFFFFFFu; // image of no finite float: marks stage-1 entries

// Monotone map float -> uint32 (larger float, larger key); -0 and +0 share a key.
__device__ __forceinline__ uint32_t order_key(uint32_t u)
{
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct SelShared {
    uint32_t hist[SEL_BINS];
    uint32_t wave_tot[SEL_WAVES];
    uint32_t digit, above;
};

// Exclusive prefix sum of x over the workgroup in thread order; total in `total`.
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
    for (int w = 0; w < SEL_WAVES; ++w) {
        const uint32_t t = sh.wave_tot[w];
        if (w < wave) base += t;
        tot += t;
    }
    total = tot;
    return base + incl - x;
}

// 4 consecutive 32-bit words starting at i0 (a multiple of 4); words at or beyond n read as 0.
__device__ __forceinline__ void load4(const uint32_t *base, int i0, int n, bool vec_ok, uint32_t (&out)[4])
{
    if (vec_ok && i0 + 3 < n) {
        const uint4 r = *reinterpret_cast<const uint4 *>(base + i0);
        out[0] = r.x; out[1] = r.y; out[2] = r.z; out[3] = r.w;
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) out[j] = (i0 + j < n) ? base[i0 + j] : 0u;
    }
}

// Histogram update; the two most frequent digits of a wave are merged into one atomic each,
// which keeps narrow key distributions from serialising on a handful of bins.
__device__ __forceinline__ void hist_add(uint32_t *hist, bool active, uint32_t digit)
{
#pragma unroll
    for (int round = 0; round < 2; ++round) {
        const unsigned long long act = __ballot(active);
        if (act == 0ull) return;
        const int leader = __ffsll((long long)act) - 1;
        const uint32_t ld = __shfl(digit, leader);
        const bool same = active && digit == ld;
        const unsigned long long grp = __ballot(same);
        if ((int)(threadIdx.x & 63) == leader) atomicAdd(&hist[ld], (uint32_t)__popcll(grp));
        if (same) active = false;
    }
    if (active) atomicAdd(&hist[digit], 1u);
}

// One digit of the radix select: histogram of digit (key >> shift) & mask over the entries whose
// higher digits equal `prefix`.  FROM_FLOAT: src holds floats; otherwise order keys where
// SEL_TAKEN entries are skipped.
template <bool FROM_FLOAT>
__device__ void radix_hist(SelShared &sh, const uint32_t *src, int n, bool vec_ok, int shift, uint32_t mask,
                           uint32_t prefix_mask, uint32_t prefix)
{
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) sh.hist[b] = 0u;
    __syncthreads();
    for (int base = 0; base < n; base += SEL_PER_IT) {
        const int i0 = base + threadIdx.x * 4;
        uint32_t w[4];
        load4(src, i0, n, vec_ok, w);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t key = FROM_FLOAT ? order_key(w[j]) : w[j];
            const bool on = (i0 + j < n) && key != SEL_TAKEN && (key & prefix_mask) == prefix;
            hist_add(sh.hist, on, (key >> shift) & mask);
        }
    }
    __syncthreads();
}

// Largest digit d with  #(digit > d) < remaining <= #(digit >= d).  Returns d and #(digit > d).
__device__ void find_digit(SelShared &sh, int nbins, uint32_t remaining, uint32_t &digit, uint32_t &above)
{
    const int rb = 2 * threadIdx.x; // bins in descending order, two per thread
    const int b0 = nbins - 1 - rb, b1 = b0 - 1;
    const uint32_t h0 = rb < nbins ? sh.hist[b0] : 0u;
    const uint32_t h1 = rb + 1 < nbins ? sh.hist[b1] : 0u;
    if (threadIdx.x == 0) { sh.digit = 0u; sh.above = 0u; }
    uint32_t total;
    const uint32_t excl = block_exclusive_scan(sh, h0 + h1, total);
    if (excl < remaining && remaining <= excl + h0) { sh.digit = (uint32_t)b0; sh.above = excl; }
    else if (excl + h0 < remaining && remaining <= excl + h0 + h1) { sh.digit = (uint32_t)b1; sh.above = excl + h0; }
    __syncthreads();
    digit = sh.digit;
    above = sh.above;
    __syncthreads();
}

constexpr int DSHIFT0 = 21, DSHIFT1 = 10, DSHIFT2 = 0;
constexpr uint32_t DMASK0 = 0x7FFu, DMASK1 = 0x7FFu, DMASK2 = 0x3FFu;

__global__ __launch_bounds__(SEL_THREADS) void select_kernel(const float *__restrict__ attn, const float *__restrict__ crit,
                                                             const int32_t *__restrict__ budget, double alpha, int n,
                                                             int max_budget, int32_t *__restrict__ idx,
                                                             int32_t *__restrict__ count, uint32_t *__restrict__ keys2)
{
    __shared__ SelShared sh;
    const int head = blockIdx.x;
    const uint32_t *a_src = reinterpret_cast<const uint32_t *>(attn) + (size_t)head * n;
    const uint32_t *c_src = reinterpret_cast<const uint32_t *>(crit) + (size_t)head * n;
    uint32_t *k2 = keys2 + (size_t)head * n;
    int32_t *out = idx + (size_t)head * max_budget;
    const bool vec_ok = (n & 3) == 0; // every head's row then starts on a 16-byte boundary

    int B = budget[head];
    B = max(0, min(B, min(n, max_budget)));
    const int b1 = (int)floor(alpha * (double)B);
    const int b2 = B - b1;

    // ---- stage 1: threshold of the b' largest attn ------------------------------------------------
    uint32_t tau1 = 0u, r1 = 0u;
    if (b1 > 0) {
        uint32_t remaining = (uint32_t)b1, digit, above, prefix = 0u, pmask = 0u;
        radix_hist<true>(sh, a_src, n, vec_ok, DSHIFT0, DMASK0, pmask, prefix);
        find_digit(sh, 2048, remaining, digit, above);
        remaining -= above; prefix |= digit << DSHIFT0; pmask |= DMASK0 << DSHIFT0;
        radix_hist<true>(sh, a_src, n, vec_ok, DSHIFT1, DMASK1, pmask, prefix);
        find_digit(sh, 2048, remaining, digit, above);
        remaining -= above; prefix |= digit << DSHIFT1; pmask |= DMASK1 << DSHIFT1;
        radix_hist<true>(sh, a_src, n, vec_ok, DSHIFT2, DMASK2, pmask, prefix);
        find_digit(sh, 1024, remaining, digit, above);
        remaining -= above; prefix |= digit;
        tau1 = prefix; r1 = remaining;
    }

    // ---- mark stage-1 entries, write stage-2 keys, first digit histogram of stage 2 ---------------
    for (int b = threadIdx.x; b < SEL_BINS; b += SEL_THREADS) sh.hist[b] = 0u;
    __syncthreads();
    uint32_t tie_seen = 0u;
    for (int base = 0; base < n; base += SEL_PER_IT) {
        const int i0 = base + threadIdx.x * 4;
        uint32_t a[4], c[4];
        load4(a_src, i0, n, vec_ok, a);
        load4(c_src, i0, n, vec_ok, c);
        bool gt[4], tie[4];
        uint32_t n_tie = 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t key = order_key(a[j]);
            const bool valid = i0 + j < n;
            gt[j] = b1 > 0 && valid && key > tau1;
            tie[j] = b1 > 0 && valid && key == tau1;
            n_tie += tie[j] ? 1u : 0u;
        }
        uint32_t rank = tie_seen, tot = 0u;
        if (__syncthreads_or((int)n_tie)) rank += block_exclusive_scan(sh, n_tie, tot);
        tie_seen += tot;
        uint32_t key2[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            bool taken = gt[j];
            if (tie[j]) { taken = rank < r1; ++rank; }
            key2[j] = taken ? SEL_TAKEN : order_key(c[j]);
            const bool on = (i0 + j < n) && !taken;
            if (b2 > 0) hist_add(sh.hist, on, (key2[j] >> DSHIFT0) & DMASK0);
        }
        if (vec_ok && i0 + 3 < n) {
            *reinterpret_cast<uint4 *>(k2 + i0) = make_uint4(key2[0], key2[1], key2[2], key2[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (i0 + j < n) k2[i0 + j] = key2[j];
        }
    }
    __syncthreads(); // histogram complete; keys2 written by this workgroup only and re-read after this barrier

    // ---- stage 2: threshold of the b'' largest crit among the remaining entries -------------------
    uint32_t tau2 = 0u, r2 = 0u;
    if (b2 > 0) {
        uint32_t remaining = (uint32_t)b2, digit, above, prefix = 0u, pmask = 0u;
        find_digit(sh, 2048, remaining, digit, above);
        remaining -= above; prefix |= digit << DSHIFT0; pmask |= DMASK0 << DSHIFT0;
        radix_hist<false>(sh, k2, n, vec_ok, DSHIFT1, DMASK1, pmask, prefix);
        find_digit(sh, 2048, remaining, digit, above);
        remaining -= above; prefix |= digit << DSHIFT1; pmask |= DMASK1 << DSHIFT1;
        radix_hist<false>(sh, k2, n, vec_ok, DSHIFT2, DMASK2, pmask, prefix);
        find_digit(sh, 1024, remaining, digit, above);
        remaining -= above; prefix |= digit;
        tau2 = prefix; r2 = remaining;
    }

    // ---- ordered write of S1 u S2 ------------------------------------------------------------------
    uint32_t out_base = 0u;
    tie_seen = 0u;
    for (int base = 0; base < n; base += SEL_PER_IT) {
        const int i0 = base + threadIdx.x * 4;
        uint32_t key[4];
        load4(k2, i0, n, vec_ok, key);
        bool sel[4], tie[4];
        uint32_t n_tie = 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool valid = i0 + j < n;
            const bool taken = valid && key[j] == SEL_TAKEN;
            sel[j] = taken || (b2 > 0 && valid && key[j] > tau2);
            tie[j] = b2 > 0 && valid && key[j] == tau2; // tau2 is a finite float's image, never SEL_TAKEN
            n_tie += tie[j] ? 1u : 0u;
        }
        uint32_t rank = tie_seen, tot = 0u;
        if (__syncthreads_or((int)n_tie)) rank += block_exclusive_scan(sh, n_tie, tot);
        tie_seen += tot;
        uint32_t n_sel = 0u;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (tie[j]) { sel[j] = rank < r2; ++rank; }
            n_sel += sel[j] ? 1u : 0u;
        }
        uint32_t tot_sel;
        uint32_t pos = out_base + block_exclusive_scan(sh, n_sel, tot_sel);
        out_base += tot_sel;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (sel[j]) {
                if (pos < (uint32_t)max_budget) out[pos] = i0 + j;
                ++pos;
            }
    }
    for (int j = B + (int)threadIdx.x; j < max_budget; j += SEL_THREADS) out[j] = -1;
    if (threadIdx.x == 0) count[head] = B;
}

hipError_t launch_select(const Dims &d, const float *attn, const float *crit, const int32_t *budget, float alpha,
                         int max_budget, int32_t *idx, int32_t *count, uint32_t *keys2, hipStream_t s)
{
    hipLaunchKernelGGL(select_kernel, dim3(d.batch * d.Hkv), dim3(SEL_THREADS), 0, s, attn, crit, budget, (double)alpha,
                       d.n, max_budget, idx, count, keys2);
    return hipGetLastError();
}

} // namespace ckv
