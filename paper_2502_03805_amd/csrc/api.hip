// Host side of the C ABI: argument validation, workspace carving, kernel dispatch.
// Nothing here computes any part of the pass; every step runs in the gfx950 kernels.
#include <math.h>
#include <algorithm>
#include <mutex>

#include "common.hpp"

namespace ckv {

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static size_t elem_size(int dtype) { return dtype == CKV_F32 ? 4 : 2; }

// Validates the descriptor and resolves defaults.  No HIP call.
static int resolve(const ckv_layer_desc *desc, Dims *out)
{
    if (!desc) return CKV_E_INVALID_ARG;
    const ckv_layer_desc &c = *desc;
    if (c.batch < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.n_ctx < 1 || c.d_model < 1) return CKV_E_INVALID_ARG;
    if (c.n_q_heads % c.n_kv_heads) return CKV_E_INVALID_ARG;
    if (c.window < 1 || c.window > c.n_ctx) return CKV_E_INVALID_ARG;
    if (c.pool_kernel < 1 || (c.pool_kernel % 2) == 0) return CKV_E_INVALID_ARG;
    if (c.dtype != CKV_BF16 && c.dtype != CKV_F32) return CKV_E_INVALID_ARG;
    if (c.window_reduce != CKV_MEAN && c.window_reduce != CKV_SUM) return CKV_E_INVALID_ARG;
    if (c.flags & ~(CKV_WO_OUT_IN | CKV_NO_MFMA | CKV_WO_IS_GRAM | CKV_CAUSAL_TAIL | CKV_PROTECT_WINDOW | CKV_ATTN_ONLY))
        return CKV_E_INVALID_ARG;
    if ((c.flags & CKV_WO_IS_GRAM) && (c.norm != CKV_NORM_L2 || (c.flags & CKV_NO_MFMA))) return CKV_E_INVALID_ARG;
    if (!(c.softmax_scale >= 0.0f) || !isfinite(c.softmax_scale)) return CKV_E_INVALID_ARG;
    if (!(c.eps >= 0.0f) || !isfinite(c.eps)) return CKV_E_INVALID_ARG;
    if (c.head_dim != 64 && c.head_dim != 128) return CKV_E_UNSUPPORTED;
    if (c.d_model % 32) return CKV_E_UNSUPPORTED;
    if (c.norm != CKV_NORM_L1 && c.norm != CKV_NORM_L2) return CKV_E_INVALID_ARG;
    if (c.pool_kernel > 63) return CKV_E_UNSUPPORTED;
    // index arithmetic inside the kernels is 64-bit for tensors and 32-bit for per-head token indices
    if ((int64_t)c.batch * c.n_q_heads * c.window > (int64_t)1 << 24) return CKV_E_UNSUPPORTED;
    if ((int64_t)c.batch * c.n_q_heads > 65535) return CKV_E_UNSUPPORTED;

    Dims d;
    d.batch = c.batch; d.H = c.n_q_heads; d.Hkv = c.n_kv_heads; d.G = d.H / d.Hkv;
    d.dh = c.head_dim; d.dm = c.d_model; d.n = c.n_ctx; d.W = c.window; d.pool_k = c.pool_kernel;
    d.window_sum = c.window_reduce == CKV_SUM;
    d.norm = c.norm;
    d.causal = (c.flags & CKV_CAUSAL_TAIL) ? 1 : 0;
    d.protect = (c.flags & CKV_PROTECT_WINDOW) ? c.window : 0;
    d.scale = c.softmax_scale > 0.0f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
    d.eps = c.eps;
    const int64_t contiguous[3] = {(int64_t)d.Hkv * d.n * d.dh, (int64_t)d.n * d.dh, (int64_t)d.dh};
    const int64_t *src[2] = {c.k_stride, c.v_stride};
    int64_t *dst[2] = {d.ks, d.vs};
    for (int t = 0; t < 2; ++t) {
        const bool all_zero = src[t][0] == 0 && src[t][1] == 0 && src[t][2] == 0;
        for (int j = 0; j < 3; ++j) dst[t][j] = all_zero ? contiguous[j] : src[t][j];
        if (dst[t][2] < d.dh || dst[t][0] < 0 || dst[t][1] < 0) return CKV_E_INVALID_ARG;
        // vector loads of 16 bytes need rows that start on a 16-byte boundary
        const int64_t per16 = 16 / (int64_t)elem_size(c.dtype);
        if (dst[t][0] % per16 || dst[t][1] % per16 || dst[t][2] % per16) return CKV_E_UNSUPPORTED;
    }
    *out = d;
    return CKV_OK;
}

Workspace carve_workspace(const Dims &d, int dtype, int max_budget)
{
    Workspace w;
    size_t off = 0;
    const size_t per_head = (size_t)d.batch * d.H * d.n;
    w.max_chunks = (d.n + ATTN_MIN_CHUNK - 1) / ATTN_MIN_CHUNK;
    w.a_raw = off; off = align256(off + per_head * 4);
    w.vnorm = off; off = align256(off + per_head * 4);
    w.stats_part = off; off = align256(off + (size_t)d.batch * d.H * d.W * w.max_chunks * 2 * 4);
    w.stats = off; off = align256(off + (size_t)d.batch * d.H * d.W * 2 * 4);
    // (reserved whether or not this call re-lays the projection out: every call on a layer sees the same offsets)
    w.w_t = off; off = align256(off + (size_t)d.H * d.dh * d.dm * elem_size(dtype));
    w.l2_scratch = off; if (d.norm == CKV_NORM_L2 && d.dh == 128) off = align256(off + vproj_l2_workspace_bytes(d));
    w.sel_keys = off; off = align256(off + (size_t)d.batch * d.Hkv * d.n * 4);
    w.sel_scratch = off; off = align256(off + select_workspace_words(d.batch * d.Hkv, d.n) * 4);
    w.diag_part = off; off = align256(off + diagnostics_workspace_floats(d) * 4);
    // last, so that the offsets above do not depend on max_budget
    w.alloc_tmp = off; off = align256(off + ((size_t)2 * d.batch + (size_t)d.batch * d.Hkv * (max_budget > 0 ? max_budget : 0)) * 4);
    w.total = off;
    return w;
}

// kernels read rows with 16-byte vector loads
static bool misaligned16(const void *p) { return ((uintptr_t)p & 15) != 0; }

static bool mfma_allowed(const ckv_layer_desc *desc)
{
    return desc->dtype == CKV_BF16 && !(desc->flags & CKV_NO_MFMA);
}

} // namespace ckv

// Scratch of criticalkv_select_noalloc: one copy per GPU, part of the loaded code object.  In host code this
// name is only a handle for hipGetSymbolAddress; the device address is looked up once per device below.
static __device__ __align__(256) unsigned char ckv_static_scratch[CKV_STATIC_SCRATCH_BYTES];

namespace ckv {

constexpr int MAX_DEVICES = 64;
static void *g_static_scratch[MAX_DEVICES];
static std::mutex g_static_scratch_mutex;

// Device address of the static scratch buffer on the current device (nullptr on failure).
static void *static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_static_scratch_mutex);
    if (!g_static_scratch[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(ckv_static_scratch)) != hipSuccess) return nullptr;
        g_static_scratch[dev] = p;
    }
    return g_static_scratch[dev];
}

} // namespace ckv

using namespace ckv;

extern "C" {

size_t criticalkv_workspace_bytes(const ckv_layer_desc *desc, int32_t max_budget)
{
    Dims d;
    if (resolve(desc, &d) != CKV_OK || max_budget < 0) return 0;
    // sized for either w_o layout and either norm so that one allocation serves every call on this layer
    d.norm = CKV_NORM_L2;
    return carve_workspace(d, desc->dtype, max_budget).total;
}

static void mark(void *const *ev, int slot, hipStream_t s)
{
    if (ev && ev[slot]) (void)hipEventRecord((hipEvent_t)ev[slot], s);
}

// What a score call works with once its arguments are validated: sizes, the carved workspace, the kernels chosen.
struct ScorePlan {
    Dims d;
    Workspace ws;
    char *base;
    float *a_raw, *vnorm, *part, *stats;
    const void *w_t; // the projection in output-major layout (the caller's, or the workspace copy)
    bool attn_only, have_gram, need_wt, tile_a, wave_a, mfma_v, l2_mfma;
    int chunks;
    hipStream_t s;
};

// Validation and workspace carving of criticalkv_score.  No HIP call.
static int score_plan(const ckv_layer_desc *desc, const void *q_win, const void *k, const void *v, const void *w_o,
                      float *attn, float *crit, float *vnorm_opt, void *workspace, size_t workspace_bytes,
                      void *hip_stream, ScorePlan *out)
{
    ScorePlan p;
    int rc = resolve(desc, &p.d);
    if (rc != CKV_OK) return rc;
    const Dims &d = p.d;
    p.attn_only = desc->flags & CKV_ATTN_ONLY;
    if (!q_win || !k || !attn || !crit || (!p.attn_only && (!v || !w_o))) return CKV_E_INVALID_ARG;
    if (p.attn_only && vnorm_opt) return CKV_E_INVALID_ARG; // no magnitudes are computed in this mode
    if (misaligned16(q_win) || misaligned16(k) || misaligned16(v) || misaligned16(w_o) || misaligned16(attn) ||
        misaligned16(crit) || misaligned16(vnorm_opt))
        return CKV_E_INVALID_ARG;
    p.have_gram = desc->flags & CKV_WO_IS_GRAM;
    if (p.have_gram && !(mfma_allowed(desc) && vproj_l2_mfma_supported(d))) return CKV_E_UNSUPPORTED;
    p.need_wt = !p.attn_only && !p.have_gram && !(desc->flags & CKV_WO_OUT_IN);
    p.ws = carve_workspace(d, desc->dtype, 0);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < p.ws.total) return CKV_E_WORKSPACE;
    p.s = (hipStream_t)hip_stream;
    p.base = (char *)workspace;
    p.a_raw = (float *)(p.base + p.ws.a_raw);
    p.vnorm = p.attn_only ? nullptr : vnorm_opt ? vnorm_opt : (float *)(p.base + p.ws.vnorm);
    p.part = (float *)(p.base + p.ws.stats_part);
    p.stats = (float *)(p.base + p.ws.stats);
    p.w_t = p.need_wt ? (const void *)(p.base + p.ws.w_t) : w_o;
    // matrix-core attention: one wave per query head over shared key tiles where a kv group has at most four
    // 32-row blocks of window queries (the 4:1 group with a 32-row window), wave-private key streams otherwise
    const int row_blocks = d.G * ((d.W + 31) / 32);
    p.tile_a = mfma_allowed(desc) && attn_mfma_supported(d) && (row_blocks <= 4 || !attn_wave_supported(d));
    p.wave_a = mfma_allowed(desc) && !p.tile_a && attn_wave_supported(d);
    p.mfma_v = mfma_allowed(desc) && vproj_mfma_supported(d);
    p.l2_mfma = d.norm == CKV_NORM_L2 && mfma_allowed(desc) && vproj_l2_mfma_supported(d);
    p.chunks = p.tile_a ? mfma_attn_chunks(d) : p.wave_a ? wave_attn_chunks(d) : generic_attn_chunks(d);
    if (p.chunks > p.ws.max_chunks) return CKV_E_WORKSPACE;
    *out = p;
    return CKV_OK;
}

// Layout change of a canonical W_O (nothing when the caller hands over the output-major form).
static int score_layout(const ScorePlan &p, const ckv_layer_desc *desc, const void *w_o, void *const *ev)
{
    mark(ev, 2 * CKV_STAGE_WO_LAYOUT, p.s);
    if (p.need_wt && launch_transpose_wo(p.d, desc->dtype, w_o, p.base + p.ws.w_t, p.s) != hipSuccess) return CKV_E_HIP;
    mark(ev, 2 * CKV_STAGE_WO_LAYOUT + 1, p.s);
    return CKV_OK;
}

// The two key sweeps: a_raw (per query head, before pooling).
static int score_attention(const ScorePlan &p, const ckv_layer_desc *desc, const void *q_win, const void *k,
                           void *const *ev)
{
    const Dims &d = p.d;
    hipStream_t s = p.s;
    hipError_t e;
    mark(ev, 2 * CKV_STAGE_ATTN_STATS, s);
    e = p.tile_a ? launch_attn_stats_mfma(d, q_win, k, p.part, p.chunks, s)
        : p.wave_a ? launch_attn_stats_wave(d, q_win, k, p.part, p.chunks, s)
                   : launch_attn_stats_generic(d, desc->dtype, q_win, k, p.part, p.chunks, s);
    if (e != hipSuccess) return CKV_E_HIP;
    e = (p.tile_a || p.wave_a) ? launch_attn_stats_reduce_log2(d, p.part, p.chunks, p.stats, s)
                               : launch_attn_stats_reduce(d, p.part, p.chunks, p.stats, s);
    if (e != hipSuccess) return CKV_E_HIP;
    mark(ev, 2 * CKV_STAGE_ATTN_STATS + 1, s);
    mark(ev, 2 * CKV_STAGE_ATTN_COLSUM, s);
    e = p.tile_a ? launch_attn_colsum_mfma(d, q_win, k, p.stats, p.a_raw, s)
        : p.wave_a ? launch_attn_colsum_wave(d, q_win, k, p.stats, p.a_raw, s)
                   : launch_attn_colsum_generic(d, desc->dtype, q_win, k, p.stats, p.a_raw, s);
    if (e != hipSuccess) return CKV_E_HIP;
    mark(ev, 2 * CKV_STAGE_ATTN_COLSUM + 1, s);
    return CKV_OK;
}

// The projected-value magnitudes (nothing in the attention-only mode).
static int score_magnitudes(const ScorePlan &p, const ckv_layer_desc *desc, const void *v, const void *w_o, void *const *ev)
{
    const Dims &d = p.d;
    hipStream_t s = p.s;
    hipError_t e = hipSuccess;
    mark(ev, 2 * CKV_STAGE_VPROJ, s);
    if (p.attn_only) {
        // combine then writes crit = attn
    } else if (p.l2_mfma) {
        const void *gram = w_o; // prepared by the caller, or computed here from the projection
        if (!p.have_gram) {
            char *scratch = p.base + p.ws.l2_scratch;
            void *g = scratch + vproj_l2_workspace_bytes(d) - vproj_l2_gram_bytes(d);
            e = launch_gram(d, p.w_t, g, scratch, s);
            if (e != hipSuccess) return CKV_E_HIP;
            gram = g;
        }
        e = launch_vproj_l2_mfma(d, v, gram, p.vnorm, s);
    } else if (d.norm == CKV_NORM_L1 && p.mfma_v)
        e = launch_vproj_mfma(d, v, p.w_t, p.vnorm, s);
    else
        e = launch_vproj_generic(d, desc->dtype, v, p.w_t, p.vnorm, s);
    if (e != hipSuccess) return CKV_E_HIP;
    mark(ev, 2 * CKV_STAGE_VPROJ + 1, s);
    return CKV_OK;
}

static int score_impl(const ckv_layer_desc *desc, const void *q_win, const void *k, const void *v, const void *w_o,
                      float *attn, float *crit, float *vnorm_opt, void *workspace, size_t workspace_bytes,
                      void *hip_stream, void *const *ev)
{
    ScorePlan p;
    int rc = score_plan(desc, q_win, k, v, w_o, attn, crit, vnorm_opt, workspace, workspace_bytes, hip_stream, &p);
    if (rc != CKV_OK) return rc;
    // The magnitudes go first: the projection is compute bound and hardly touches HBM, so whatever the caller's
    // previous kernel left to be written back (the gather of the layer before writes hundreds of MiB) drains under
    // it, and the two key sweeps, which live on HBM bandwidth, find the memory system quiet (a streaming read right
    // after a large write runs at 3.3 instead of 5.2 TB/s on this part).
    if ((rc = score_layout(p, desc, w_o, ev)) != CKV_OK) return rc;
    if ((rc = score_magnitudes(p, desc, v, w_o, ev)) != CKV_OK) return rc;
    if ((rc = score_attention(p, desc, q_win, k, ev)) != CKV_OK) return rc;
    mark(ev, 2 * CKV_STAGE_COMBINE, p.s);
    if (launch_combine(p.d, p.a_raw, p.vnorm, attn, crit, p.s) != hipSuccess) return CKV_E_HIP;
    mark(ev, 2 * CKV_STAGE_COMBINE + 1, p.s);
    return CKV_OK;
}

int criticalkv_score(const ckv_layer_desc *desc, const void *q_win, const void *k, const void *v, const void *w_o,
                     float *attn, float *crit, float *vnorm_opt, void *workspace, size_t workspace_bytes,
                     void *hip_stream)
{
    return score_impl(desc, q_win, k, v, w_o, attn, crit, vnorm_opt, workspace, workspace_bytes, hip_stream, nullptr);
}

int criticalkv_score_profiled(const ckv_layer_desc *desc, const void *q_win, const void *k, const void *v,
                              const void *w_o, float *attn, float *crit, float *vnorm_opt, void *workspace,
                              size_t workspace_bytes, void *hip_stream, void *const *stage_events)
{
    return score_impl(desc, q_win, k, v, w_o, attn, crit, vnorm_opt, workspace, workspace_bytes, hip_stream,
                      stage_events);
}

size_t criticalkv_gram_bytes(const ckv_layer_desc *desc)
{
    Dims d;
    if (resolve(desc, &d) != CKV_OK || desc->dtype != CKV_BF16 || !vproj_l2_mfma_supported(d)) return 0;
    return vproj_l2_gram_bytes(d);
}

int criticalkv_prepare_gram(const ckv_layer_desc *desc, const void *w_o, void *gram_out, void *workspace,
                            size_t workspace_bytes, void *hip_stream)
{
    Dims d;
    int rc = resolve(desc, &d);
    if (rc != CKV_OK) return rc;
    if (!w_o || !gram_out || (desc->flags & CKV_WO_IS_GRAM)) return CKV_E_INVALID_ARG;
    if (misaligned16(w_o) || misaligned16(gram_out)) return CKV_E_INVALID_ARG;
    if (desc->dtype != CKV_BF16 || !vproj_l2_mfma_supported(d)) return CKV_E_UNSUPPORTED;
    d.norm = CKV_NORM_L2; // the carve below must contain the Gram scratch whatever norm the descriptor names
    const bool need_wt = !(desc->flags & CKV_WO_OUT_IN);
    const Workspace ws = carve_workspace(d, desc->dtype, 0);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < ws.total) return CKV_E_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    char *base = (char *)workspace;
    const void *w_t = w_o;
    if (need_wt) {
        if (launch_transpose_wo(d, desc->dtype, w_o, base + ws.w_t, s) != hipSuccess) return CKV_E_HIP;
        w_t = base + ws.w_t;
    }
    return launch_gram(d, w_t, gram_out, base + ws.l2_scratch, s) == hipSuccess ? CKV_OK : CKV_E_HIP;
}

int criticalkv_select(const ckv_layer_desc *desc, const float *attn, const float *crit, const int32_t *budget,
                      float alpha, int32_t max_budget, int32_t *idx, int32_t *count, void *workspace,
                      size_t workspace_bytes, void *hip_stream)
{
    Dims d;
    int rc = resolve(desc, &d);
    if (rc != CKV_OK) return rc;
    if (!attn || !crit || !budget || !idx || !count) return CKV_E_INVALID_ARG;
    if (misaligned16(attn) || misaligned16(crit)) return CKV_E_INVALID_ARG;
    if (!(alpha >= 0.0f) || !(alpha <= 1.0f)) return CKV_E_INVALID_ARG;
    if (max_budget < 1 || max_budget > d.n) return CKV_E_INVALID_ARG;
    const Workspace ws = carve_workspace(d, desc->dtype, 0);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < ws.total) return CKV_E_WORKSPACE;
    uint32_t *keys2 = (uint32_t *)((char *)workspace + ws.sel_keys);
    uint32_t *scratch = (uint32_t *)((char *)workspace + ws.sel_scratch);
    hipError_t e = launch_select(d, attn, crit, budget, alpha, max_budget, idx, count, keys2, scratch,
                                 (hipStream_t)hip_stream);
    return e == hipSuccess ? CKV_OK : CKV_E_HIP;
}

int criticalkv_select_noalloc(const ckv_layer_desc *desc, const float *attn, const float *crit, const int32_t *budget,
                              float alpha, int32_t max_budget, int32_t *idx, int32_t *count, void *hip_stream)
{
    Dims d;
    int rc = resolve(desc, &d);
    if (rc != CKV_OK) return rc;
    if (!attn || !crit || !budget || !idx || !count) return CKV_E_INVALID_ARG;
    if (misaligned16(attn) || misaligned16(crit)) return CKV_E_INVALID_ARG;
    if (!(alpha >= 0.0f) || !(alpha <= 1.0f)) return CKV_E_INVALID_ARG;
    if (max_budget < 1 || max_budget > d.n) return CKV_E_INVALID_ARG;
    // the two pieces criticalkv_select carves from a workspace, laid out back to back in the static buffer
    const size_t keys_bytes = align256((size_t)d.batch * d.Hkv * d.n * 4);
    const size_t scratch_bytes = align256(select_workspace_words(d.batch * d.Hkv, d.n) * 4);
    if (keys_bytes + scratch_bytes > CKV_STATIC_SCRATCH_BYTES) return CKV_E_STATIC_LIMIT;
    char *base = (char *)static_scratch_ptr();
    if (!base) return CKV_E_HIP;
    // (the selection's first kernel clears the histograms and the per-head state it accumulates into; every
    // other word of the buffer is written before it is read, so what the previous call left does not matter)
    hipError_t e = launch_select(d, attn, crit, budget, alpha, max_budget, idx, count, (uint32_t *)base,
                                 (uint32_t *)(base + keys_bytes), (hipStream_t)hip_stream);
    return e == hipSuccess ? CKV_OK : CKV_E_HIP;
}

size_t criticalkv_prepared_wo_bytes(const ckv_layer_desc *desc)
{
    Dims d;
    if (resolve(desc, &d) != CKV_OK) return 0;
    return (size_t)d.H * d.dh * d.dm * elem_size(desc->dtype);
}

int criticalkv_prepare_wo(const ckv_layer_desc *desc, const void *w_o, void *w_out, void *hip_stream)
{
    Dims d;
    int rc = resolve(desc, &d);
    if (rc != CKV_OK) return rc;
    if (!w_o || !w_out || w_o == w_out || misaligned16(w_o) || misaligned16(w_out)) return CKV_E_INVALID_ARG;
    if (desc->flags & (CKV_WO_OUT_IN | CKV_WO_IS_GRAM)) return CKV_E_INVALID_ARG;
    return launch_transpose_wo(d, desc->dtype, w_o, w_out, (hipStream_t)hip_stream) == hipSuccess ? CKV_OK : CKV_E_HIP;
}

int criticalkv_allocate(const ckv_layer_desc *desc, const float *attn, int32_t total_budget, float floor_frac,
                        int32_t *budget, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Dims d;
    int rc = resolve(desc, &d);
    if (rc != CKV_OK) return rc;
    if (!attn || !budget || misaligned16(attn)) return CKV_E_INVALID_ARG;
    if (total_budget < 0 || !(floor_frac >= 0.0f) || !(floor_frac <= 1.0f)) return CKV_E_INVALID_ARG;
    if ((int64_t)d.Hkv * d.n > (int64_t)INT32_MAX) return CKV_E_UNSUPPORTED;
    if ((int64_t)total_budget > (int64_t)d.Hkv * d.n) return CKV_E_INVALID_ARG;
    const int floor_each = (int)floor((double)floor_frac * (double)total_budget / (double)d.Hkv);
    const int64_t pool = std::min<int64_t>((int64_t)total_budget - (int64_t)d.Hkv * floor_each, (int64_t)d.Hkv * d.n);
    const int per_head = (int)((pool + d.Hkv - 1) / d.Hkv);
    const Workspace ws = carve_workspace(d, desc->dtype, per_head);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < ws.total) return CKV_E_WORKSPACE;
    uint32_t *keys2 = (uint32_t *)((char *)workspace + ws.sel_keys);
    uint32_t *scratch = (uint32_t *)((char *)workspace + ws.sel_scratch);
    int32_t *tmp = (int32_t *)((char *)workspace + ws.alloc_tmp);
    hipError_t e = launch_allocate(d, attn, total_budget, floor_frac, budget, keys2, scratch, tmp, (hipStream_t)hip_stream);
    return e == hipSuccess ? CKV_OK : CKV_E_HIP;
}

int criticalkv_diagnostics(const ckv_layer_desc *desc, const void *v, const void *w_o, const float *vnorm_opt,
                           const int32_t *idx, const int32_t *count, int32_t max_budget, float *out, void *workspace,
                           size_t workspace_bytes, void *hip_stream)
{
    Dims d;
    int rc = resolve(desc, &d);
    if (rc != CKV_OK) return rc;
    if (!v || !w_o || !idx || !count || !out) return CKV_E_INVALID_ARG;
    if (misaligned16(v) || misaligned16(w_o) || misaligned16(vnorm_opt)) return CKV_E_INVALID_ARG;
    if (desc->flags & (CKV_ATTN_ONLY | CKV_WO_IS_GRAM)) return CKV_E_INVALID_ARG; // needs the magnitudes and W_O itself
    if (max_budget < 1 || max_budget > d.n) return CKV_E_INVALID_ARG;
    const Workspace ws = carve_workspace(d, desc->dtype, 0); // the layout criticalkv_select used
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < ws.total) return CKV_E_WORKSPACE;
    char *base = (char *)workspace;
    const float *vnorm = vnorm_opt ? vnorm_opt : (const float *)(base + ws.vnorm);
    hipError_t e = launch_diagnostics(d, desc->dtype, (desc->flags & CKV_WO_OUT_IN) ? 1 : 0, v, w_o,
                                      (const float *)(base + ws.a_raw), vnorm, (const uint32_t *)(base + ws.sel_keys),
                                      idx, count, max_budget, (float *)(base + ws.diag_part), out,
                                      (hipStream_t)hip_stream);
    return e == hipSuccess ? CKV_OK : CKV_E_HIP;
}

int criticalkv_compact(const ckv_layer_desc *desc, const void *k, const void *v, const int32_t *idx,
                       const int32_t *count, int32_t max_budget, void *k_out, void *v_out, void *hip_stream)
{
    Dims d;
    int rc = resolve(desc, &d);
    if (rc != CKV_OK) return rc;
    if (!k || !v || !idx || !count || !k_out || !v_out) return CKV_E_INVALID_ARG;
    if (misaligned16(k) || misaligned16(v) || misaligned16(k_out) || misaligned16(v_out)) return CKV_E_INVALID_ARG;
    if (max_budget < 1 || max_budget > d.n) return CKV_E_INVALID_ARG;
    hipError_t e = launch_compact(d, desc->dtype, k, v, idx, count, max_budget, k_out, v_out, (hipStream_t)hip_stream);
    return e == hipSuccess ? CKV_OK : CKV_E_HIP;
}

const char *criticalkv_strerror(int code)
{
    switch (code) {
    case CKV_OK: return "success";
    case CKV_E_INVALID_ARG: return "invalid argument (null pointer, shape or parameter out of range)";
    case CKV_E_UNSUPPORTED: return "unsupported configuration (head_dim, d_model, norm, strides or sizes)";
    case CKV_E_WORKSPACE: return "workspace missing, not 256-byte aligned or too small";
    case CKV_E_HIP: return "a HIP kernel launch failed";
    case CKV_E_STATIC_LIMIT: return "the layer needs more scratch than the static buffer of the no-allocation entry point holds";
    default: return "unknown error code";
    }
}

} // extern "C"
