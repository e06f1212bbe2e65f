// Internal declarations shared by the host dispatch and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "criticalkv.h"

namespace ckv {

// bf16 storage type: raw 16 bits; conversion to float is a shift (exact).
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_to_f32(x); }

// Problem sizes resolved from the descriptor (strides filled in).
struct Dims {
    int batch, H, Hkv, G, dh, dm, n, W, pool_k;
    int window_sum;
    int norm; // CKV_NORM_L1 or CKV_NORM_L2
    int causal;  // window row w sees keys <= n - W + w only
    int protect; // trailing entries the selection keeps as they are (0 or W)
    float scale, eps;
    int64_t ks[3], vs[3];
};

// Workspace carving for criticalkv_score / criticalkv_select (byte offsets, 256-aligned).
struct Workspace {
    size_t a_raw;      // [batch, H, n] f32: window score per query head before pooling
    size_t vnorm;      // [batch, H, n] f32: projected-value norm (when the caller passes none)
    size_t stats_part; // [batch, H, W, chunks, 2] f32: per-chunk (max, sum of exp)
    size_t stats;      // [batch, H, W, 2] f32: per-row (max + log sum, unused)
    size_t w_t;        // [d_model, H*dh] copy of W_O in output-major layout (when given canonical)
    size_t sel_keys;   // [batch*Hkv, n] u32: stage-2 keys with stage-1 entries marked
    size_t l2_scratch; // Gram partial sums and the split bf16 Gram matrices (L2 norm only)
    size_t diag_part;  // per-chunk partial sums of the perturbation diagnostics
    size_t alloc_tmp;  // budget allocation: pool budgets, counts and the pooled index list
    size_t sel_scratch; // digit histograms, per-head state, per-slice counts of the selection kernels
    size_t total;
    int max_chunks;    // capacity of stats_part per window row
};

constexpr int ATTN_MIN_CHUNK = 128; // fewest keys any attention kernel gives one workgroup (sizes stats_part)
int generic_attn_chunks(const Dims &d);
int mfma_attn_chunks(const Dims &d);
bool attn_mfma_supported(const Dims &d);  // shapes the matrix-core attention kernels cover (shared key tiles)
bool attn_wave_supported(const Dims &d);  // shapes the wave-private matrix-core attention kernels cover
int wave_attn_chunks(const Dims &d);
bool vproj_mfma_supported(const Dims &d); // shapes the matrix-core projection kernel covers

Workspace carve_workspace(const Dims &d, int dtype, int max_budget);

// ---- kernel launchers (each returns hipGetLastError after its launches) -------------------------
// window attention, pass 1: per (row, key chunk) running max and sum of exp
hipError_t launch_attn_stats_generic(const Dims &d, int dtype, const void *q, const void *k, float *part,
                                     int chunks, hipStream_t s);
// reduce chunk partials to one (max, 1/sum) pair per window row
hipError_t launch_attn_stats_reduce(const Dims &d, const float *part, int chunks, float *stats, hipStream_t s);
// window attention, pass 2: a_raw[b,h,i] = reduce_w exp(s - max_w) / sum_w
hipError_t launch_attn_colsum_generic(const Dims &d, int dtype, const void *q, const void *k, const float *stats,
                                      float *a_raw, hipStream_t s);
hipError_t launch_attn_stats_mfma(const Dims &d, const void *q, const void *k, float *part, int chunks,
                                  hipStream_t s);
// matrix-core path: partials are in the log2 domain; per row E = log2(sum 2^t) (+ log2 W for the mean)
hipError_t launch_attn_stats_reduce_log2(const Dims &d, const float *part, int chunks, float *stats, hipStream_t s);
hipError_t launch_attn_colsum_mfma(const Dims &d, const void *q, const void *k, const float *stats, float *a_raw,
                                   hipStream_t s);
// the same two sweeps with wave-private key streams (larger groups and windows, d_h = 64); same partial layout
hipError_t launch_attn_stats_wave(const Dims &d, const void *q, const void *k, float *part, int chunks, hipStream_t s);
hipError_t launch_attn_colsum_wave(const Dims &d, const void *q, const void *k, const float *stats, float *a_raw,
                                   hipStream_t s);
// projected-value L1 norm; w_t is [d_model, H*dh]
hipError_t launch_vproj_generic(const Dims &d, int dtype, const void *v, const void *w_t, float *vnorm,
                                hipStream_t s);
hipError_t launch_vproj_mfma(const Dims &d, const void *v, const void *w_t, float *vnorm, hipStream_t s);
// L2 norm through the Gram matrix W_O^h W_O^h^T (bf16, d_h = 128)
bool vproj_l2_mfma_supported(const Dims &d);
size_t vproj_l2_workspace_bytes(const Dims &d);
size_t vproj_l2_gram_bytes(const Dims &d); // the split bf16 Gram matrices alone
// gram: the prepared Gram matrices; when null they are computed from w_t into scratch first
hipError_t launch_gram(const Dims &d, const void *w_t, void *gram_out, void *partial_scratch, hipStream_t s);
hipError_t launch_vproj_l2_mfma(const Dims &d, const void *v, const void *gram, float *vnorm, hipStream_t s);
// [H*dh, d_model] -> [d_model, H*dh]
hipError_t launch_transpose_wo(const Dims &d, int dtype, const void *w_o, void *w_t, hipStream_t s);
// pool + eps + product + group mean; crit may be null (only the pooled attention is written)
hipError_t launch_combine(const Dims &d, const float *a_raw, const float *vnorm, float *attn, float *crit,
                          hipStream_t s);
size_t select_workspace_words(int heads, int n); // u32 words of histogram / state / per-slice scratch
hipError_t launch_select(const Dims &d, const float *attn, const float *crit, const int32_t *budget, float alpha,
                         int max_budget, int32_t *idx, int32_t *count, uint32_t *keys2, uint32_t *scratch,
                         hipStream_t s);
// the selection in two halves: stage 1's digit histograms need attn only (they can run beside the projection),
// the rest needs crit as well
hipError_t launch_select_stage1_hist(int heads, int n, int protect, const float *attn, const int32_t *budget, float alpha,
                                     int max_budget, uint32_t *keys2, uint32_t *scratch, hipStream_t s);
hipError_t launch_select_finish(int heads, int n, int protect, const float *attn, const float *crit, const int32_t *budget,
                                float alpha, int max_budget, int32_t *idx, int32_t *count, uint32_t *keys2,
                                uint32_t *scratch, hipStream_t s);
// per-head budgets from a per-batch-item total; tmp holds 2 * batch + batch * total int32
hipError_t launch_allocate(const Dims &d, const float *attn, int total, float floor_frac, int32_t *budget_out,
                           uint32_t *keys2, uint32_t *scratch, int32_t *tmp, hipStream_t s);
// perturbation quantities of a finished selection; part holds diagnostics_workspace_floats(d) floats
size_t diagnostics_workspace_floats(const Dims &d);
hipError_t launch_diagnostics(const Dims &d, int dtype, int out_in, const void *v, const void *w_o, const float *a_raw,
                              const float *vnorm, const uint32_t *keys2, const int32_t *idx, const int32_t *count,
                              int max_budget, float *part, float *out, hipStream_t s);
hipError_t launch_compact(const Dims &d, int dtype, const void *k, const void *v, const int32_t *idx,
                          const int32_t *count, int max_budget, void *k_out, void *v_out, hipStream_t s);

} // namespace ckv
