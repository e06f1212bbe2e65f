/*
 * criticalkv.h - C ABI of the per-layer KV-cache selection pass on AMD MI355X (gfx950).
 *
 * The pass is the prefill-time "score -> select -> compact" step of
 * perturbation-constrained KV-cache eviction:
 *   score   : observation-window attention (Algorithm 2, lines 2-4) and the
 *             per-entry L1 magnitude of the value projected through its head's
 *             slice of W^O (Theorem 3.3; Algorithm 1, lines 2-3)
 *   select  : budget split b' = b*alpha, b'' = b - b' and the two Top-k stages
 *             (Algorithm 1, lines 4-9)
 *   compact : the selected K/V rows gathered into the new cache
 *             (Algorithm 1, line 10; Definition 3.1)
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers (HIP global memory) unless a
 *     parameter says "host".  Tensors are row-major with the last dimension
 *     contiguous.  The descriptor is a host struct and is read during the call.
 *     Floating-point tensors (inputs and outputs) must start on a 16-byte
 *     boundary (CKV_E_INVALID_ARG otherwise): rows are moved with vector accesses.
 *   - Ownership: the caller owns every buffer.  The library allocates nothing,
 *     frees nothing and keeps no pointer after a call returns; temporary device
 *     memory is the caller's `workspace` (size from criticalkv_workspace_bytes,
 *     256-byte aligned).  Inputs are never modified.  Outputs must not alias
 *     inputs or the workspace.
 *   - Execution: work is enqueued on `hip_stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns without waiting.
 *     score -> select -> compact on one stream need no host synchronisation.
 *     Two calls that share a workspace must be ordered on one stream.
 *   - Errors: 0 on success, a negative CKV_E_* code otherwise.  Arguments are
 *     validated before any HIP call, so CKV_E_INVALID_ARG / CKV_E_UNSUPPORTED /
 *     CKV_E_WORKSPACE are returned without touching a device.  No exception
 *     crosses this boundary.  Non-finite input values give undefined scores.
 */
#ifndef CRITICALKV_H
#define CRITICALKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CKV_API __attribute__((visibility("default")))

/* error codes */
#define CKV_OK 0
#define CKV_E_INVALID_ARG (-1) /* null pointer, shape or parameter out of range            */
#define CKV_E_UNSUPPORTED (-2) /* valid request this build has no kernel for               */
#define CKV_E_WORKSPACE (-3)   /* workspace missing, misaligned or too small               */
#define CKV_E_HIP (-4)         /* a HIP launch failed (hipGetLastError was not hipSuccess) */
#define CKV_E_STATIC_LIMIT (-5) /* criticalkv_select_noalloc: the layer needs more scratch than the
                                   library's static buffer holds (CKV_STATIC_SCRATCH_BYTES)         */

/* ckv_layer_desc.dtype: element type of q_win, k, v, w_o and of k_out, v_out */
#define CKV_BF16 0
#define CKV_F32 1

/* ckv_layer_desc.norm: norm applied to each row of V W^O.  The paper's results use L1; it reports the L2
   distance as giving similar quality.  For L2 the bf16 d_h = 128 path uses the exact identity
   ||v W||_2^2 = v (W W^T) v^T (a d_h x d_h Gram matrix per head instead of the d_h x d_model slice). */
#define CKV_NORM_L1 1
#define CKV_NORM_L2 2

/* ckv_layer_desc.window_reduce: how the W window rows are merged (Algorithm 2 line 3 takes the mean) */
#define CKV_MEAN 0
#define CKV_SUM 1

/* ckv_layer_desc.flags */
#define CKV_WO_OUT_IN 1u /* w_o is stored [d_model, H*d_h] (the layout of a linear layer's weight:
                            output feature major); without it w_o is [H*d_h, d_model], head h = rows
                            h*d_h .. (h+1)*d_h-1, i.e. the paper's d_h x d slice per head (Section 3.1) */
#define CKV_NO_MFMA 2u   /* run the plain vector-ALU kernels even where a matrix-core kernel exists
                            (same results up to fp32 rounding order; for validation)               */
#define CKV_CAUSAL_TAIL 8u /* the window queries are the last W tokens of the prompt and attend causally:
                            window row w (position n-W+w) sees keys 0 .. n-W+w only (chunked prefill);
                            without it every window row sees all n keys (the algorithm as printed)    */
#define CKV_PROTECT_WINDOW 16u /* criticalkv_select keeps the window's own tokens: the last min(W, B) entries
                            are part of every selection, and Algorithm 1 runs on entries 0 .. n-W-1 alone
                            with the rest of the budget, B - min(W, B) (so b' = floor(alpha * rest)).
                            The scores written by criticalkv_score are not changed by this flag.       */
#define CKV_ATTN_ONLY 32u /* baseline: skip the projected-value magnitude; crit is set equal to attn, so the
                            selection is attention-only Top-B for every alpha (Algorithm 2's regular
                            selection).  w_o and v are not read by criticalkv_score (may be NULL).      */
#define CKV_WO_IS_GRAM 4u /* CKV_NORM_L2 only: the w_o argument of criticalkv_score is the per-layer
                            constant written by criticalkv_prepare_gram, not the projection itself  */

/*
 * One attention layer.  Notation of the paper: n cached entries per head, window of n' = `window`
 * queries, per-head output-projection slice W^O of shape d_h x d.  Grouped-query attention:
 * query head h reads kv head h / (n_q_heads / n_kv_heads).
 */
typedef struct ckv_layer_desc {
    int32_t batch;         /* >= 1                                                            */
    int32_t n_q_heads;     /* H, multiple of n_kv_heads                                       */
    int32_t n_kv_heads;    /* Hkv                                                             */
    int32_t head_dim;      /* d_h: 64 or 128                                                  */
    int32_t d_model;       /* d: columns of W^O, multiple of 32                               */
    int32_t n_ctx;         /* n >= 1 cached entries per head                                  */
    int32_t window;        /* n' = W observation-window queries, 1 <= W <= n                  */
    int32_t pool_kernel;   /* odd max-pool width over the token axis, 1 = no pooling          */
    int32_t dtype;         /* CKV_BF16 or CKV_F32                                             */
    int32_t norm;          /* CKV_NORM_L1 or CKV_NORM_L2                                      */
    int32_t window_reduce; /* CKV_MEAN or CKV_SUM                                             */
    uint32_t flags;        /* CKV_WO_OUT_IN | CKV_NO_MFMA | CKV_WO_IS_GRAM | CKV_CAUSAL_TAIL | ... */
    float softmax_scale;   /* logit scale; 0 selects 1/sqrt(head_dim) (eq. 2)                 */
    float eps;             /* added to the pooled score before the product (paper: 1e-4)      */
    int64_t k_stride[3];   /* element strides of k for (batch, kv head, token); all 0 =       */
    int64_t v_stride[3];   /*   contiguous [batch, Hkv, n, d_h].  The last dim has stride 1.  */
} ckv_layer_desc;

/*
 * Bytes of workspace that criticalkv_score, criticalkv_select and criticalkv_allocate need for this
 * layer, criticalkv_diagnostics included (the largest of them; compact needs none).  max_budget only sizes criticalkv_allocate's list.  Returns 0 if the descriptor is invalid.
 * Host-only computation.
 */
CKV_API size_t criticalkv_workspace_bytes(const ckv_layer_desc *desc, int32_t max_budget);

/*
 * Scores of every cached entry (Algorithm 2 lines 2-4; Algorithm 1 lines 2-3).
 *
 * Per batch item bi, query head h with kv head g = h / G, G = H / Hkv:
 *   p_{w,.}   = softmax_i(scale * q_win[bi,h,w,:] . k[bi,g,i,:])   over all n keys, no mask
 *   a^h_i     = mean_w p_{w,i}          (sum_w with CKV_SUM)
 *   abar^h_i  = max{ a^h_j : |j - i| <= pool_kernel/2, 0 <= j < n }
 *   N^h_i     = sum_c | sum_t v[bi,g,i,t] * W^O[h*d_h + t, c] |      (CKV_NORM_L2: sqrt of the sum of squares)
 * and, per kv head (group means; with G = 1 exactly the paper's A and (A + eps) * ||V W^O||_1):
 *   attn[bi,g,i] = (1/G) sum_{h in g} abar^h_i
 *   crit[bi,g,i] = (1/G) sum_{h in g} (abar^h_i + eps) * N^h_i
 *
 * in : q_win [batch, H, W, d_h]   the last W query states of the prompt
 *      k, v  [batch, Hkv, n, d_h] (or strided per the descriptor)
 *      w_o   [H*d_h, d_model]     (or [d_model, H*d_h] with CKV_WO_OUT_IN)
 * out: attn, crit [batch, Hkv, n] float32
 *      vnorm_opt  [batch, H, n]   float32, N^h_i; may be NULL
 * bf16 inputs are multiplied exactly and accumulated in float32.
 */
CKV_API int criticalkv_score(const ckv_layer_desc *desc, const void *q_win, const void *k, const void *v,
                             const void *w_o, float *attn, float *crit, float *vnorm_opt, void *workspace,
                             size_t workspace_bytes, void *hip_stream);

/*
 * L2 variant: the per-layer constant G^h = W^O_h W^O_h^T (d_h x d_h per query head), which depends on the
 * pretrained projection only and can be prepared once per layer and reused for every prompt.
 * criticalkv_gram_bytes: size of gram_out (0 if the layer has no Gram-matrix path: bf16, d_h = 128,
 * d_model a multiple of 512).  criticalkv_prepare_gram writes it (device memory, opaque layout: two bf16
 * matrices per head whose sum is G to ~2^-17 relative); w_o as for criticalkv_score (layout per
 * CKV_WO_OUT_IN), workspace as for criticalkv_score.  Pass gram_out as `w_o` to criticalkv_score together
 * with CKV_NORM_L2 and CKV_WO_IS_GRAM; without that flag criticalkv_score computes G itself on every call.
 */
CKV_API size_t criticalkv_gram_bytes(const ckv_layer_desc *desc);
CKV_API int criticalkv_prepare_gram(const ckv_layer_desc *desc, const void *w_o, void *gram_out, void *workspace,
                                    size_t workspace_bytes, void *hip_stream);

/*
 * criticalkv_score with per-stage timing marks, for benchmarks and profiles (the scores are the same).
 * stage_events is a HOST array of 2 * CKV_N_SCORE_STAGES hipEvent_t (as void*) created by the caller with
 * timing enabled; entry 2*s is recorded on the stream before stage s, entry 2*s+1 after it.  NULL entries
 * (or a NULL array) are skipped.  The caller reads the events after synchronising.  The stages are issued in the
 * order layout, projection, first sweep, second sweep, combine (the projection hardly touches HBM, so a previous
 * kernel's pending write-backs drain under it and not under the bandwidth-bound sweeps).
 */
#define CKV_STAGE_WO_LAYOUT 0   /* layout change of a canonical w_o (empty with CKV_WO_OUT_IN) */
#define CKV_STAGE_ATTN_STATS 1  /* first key sweep: row max and sum of exp                      */
#define CKV_STAGE_ATTN_COLSUM 2 /* second key sweep: window-reduced softmax weights             */
#define CKV_STAGE_VPROJ 3       /* ||V W^O||_1 per entry                                        */
#define CKV_STAGE_COMBINE 4     /* pooling, eps, product, group mean                            */
#define CKV_N_SCORE_STAGES 5
CKV_API int criticalkv_score_profiled(const ckv_layer_desc *desc, const void *q_win, const void *k, const void *v,
                                      const void *w_o, float *attn, float *crit, float *vnorm_opt, void *workspace,
                                      size_t workspace_bytes, void *hip_stream, void *const *stage_events);

/*
 * Two-stage selection per (batch item, kv head) (Algorithm 1 lines 4-9).
 *
 *   B   = clamp(budget[bi,g], 0, min(n, max_budget))
 *   b'  = floor(alpha * B) (in double), b'' = B - b'
 *   S1  = the b' entries with the largest attn
 *   S2  = the b'' entries with the largest crit among entries not in S1
 * Equal keys: the lower token index is taken first.  Keys are compared as IEEE floats
 * (-0 equals +0); NaN keys give an undefined selection.
 * With CKV_PROTECT_WINDOW the result is  {last min(W, B) entries}  u  {the two stages run on entries
 * 0 .. n-W-1 with budget B - min(W, B)}.
 *
 * in : attn, crit [batch, Hkv, n] float32 (normally criticalkv_score's outputs)
 *      budget     [batch, Hkv]    int32, DEVICE memory
 *      alpha      in [0, 1]; 1 = attention-only Top-B (Algorithm 2's regular selection)
 * out: idx   [batch, Hkv, max_budget] int32: S1 u S2 in ascending token order, tail filled with -1
 *      count [batch, Hkv]             int32: B
 */
CKV_API int criticalkv_select(const ckv_layer_desc *desc, const float *attn, const float *crit,
                              const int32_t *budget, float alpha, int32_t max_budget, int32_t *idx,
                              int32_t *count, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * criticalkv_select for callers that cannot allocate or pass device scratch memory (code under HIP graph
 * capture that owns no workspace, tight serving loops, harnesses that forbid hipMalloc): same arguments and
 * results as criticalkv_select without the workspace; the kernels' scratch (stage-2 keys, digit histograms,
 * per-slice counts) lives in a static device buffer of CKV_STATIC_SCRATCH_BYTES inside the library, one copy
 * per GPU, held until the process ends.  The call allocates and frees nothing and enqueues only kernels.
 * A layer that needs more scratch than the buffer holds is refused with CKV_E_STATIC_LIMIT (the buffer
 * covers batch * Hkv * n <= 2^20 entries with up to 64 (batch item, kv head) pairs, e.g. every 32K-128K
 * layer shape of 8 kv heads).  Every call on a GPU shares that GPU's buffer: two calls that overlap in time
 * on one GPU (different streams, different threads) race; order them on one stream or with events.
 * criticalkv_diagnostics cannot follow this call (it reads a caller workspace).
 */
#define CKV_STATIC_SCRATCH_BYTES ((size_t)12 << 20)
CKV_API int criticalkv_select_noalloc(const ckv_layer_desc *desc, const float *attn, const float *crit,
                                      const int32_t *budget, float alpha, int32_t max_budget, int32_t *idx,
                                      int32_t *count, void *hip_stream);

/*
 * Output-major copy of a canonical projection, prepared once per layer: w_o [H*d_h, d_model] ->
 * w_out [d_model, H*d_h] (criticalkv_prepared_wo_bytes bytes, device, 16-byte aligned).  Pass w_out to
 * criticalkv_score together with CKV_WO_OUT_IN; without this step criticalkv_score re-lays a canonical
 * w_o out on every call (Section 3.1's d_h x d slice per head is the canonical form; the output-major form
 * is what the projection kernel streams).  desc->flags must not carry CKV_WO_OUT_IN or CKV_WO_IS_GRAM.
 */
CKV_API size_t criticalkv_prepared_wo_bytes(const ckv_layer_desc *desc);
CKV_API int criticalkv_prepare_wo(const ckv_layer_desc *desc, const void *w_o, void *w_out, void *hip_stream);

/*
 * Per-head budgets from a per-batch-item total (the allocation step of Algorithm 2 line 1).
 *
 * The paper names this step and cites adaptive allocation methods without defining one; the rule here is
 * this library's own, in the spirit of those methods:
 *   f  = floor(floor_frac * total_budget / Hkv) (in double)     every head's floor
 *   P  = total_budget - Hkv * f                                  slots handed out by score
 *   T  = the P entries with the largest attn among all Hkv * n entries of the batch item
 *        (equal scores: the lower kv head, then the lower token, first)
 *   budget[bi,g] = min(n, f + #{entries of T owned by head g})
 * floor_frac = 1 gives the uniform split, floor_frac = 0 a purely score-driven one.
 *
 * in : attn [batch, Hkv, n] float32 contiguous (criticalkv_score's pooled attention output), DEVICE
 *      total_budget in [0, Hkv * n], floor_frac in [0, 1]
 * out: budget [batch, Hkv] int32, DEVICE; feed it to criticalkv_select
 * workspace: criticalkv_workspace_bytes(desc, max_budget) bytes with Hkv * max_budget >= P always
 *      suffice; too few bytes give CKV_E_WORKSPACE.  Hkv * n must fit an int32 (CKV_E_UNSUPPORTED).
 */
CKV_API int criticalkv_allocate(const ckv_layer_desc *desc, const float *attn, int32_t total_budget,
                                float floor_frac, int32_t *budget, void *workspace, size_t workspace_bytes,
                                void *hip_stream);

/*
 * Perturbation quantities of a finished selection, per (batch item, query head)
 * (Definition 3.1; Theorems 3.2, 3.3, 3.5, 3.6; Assumption 3.4): what the paper's analysis plots.
 *
 * For query head h (kv head g = h / G): A = the head's window-mean attention over the n entries, before
 * pooling (it sums to 1; the theorems are stated for one query's distribution, the window mean takes its
 * place); P_i = v[bi,g,i,:] W^O_h; N_i = ||P_i|| in the descriptor's norm; S = idx[bi,g,0..count) and
 * S1 the part of it taken in stage 1.
 *   out[bi,h,CKV_DIAG_SIGMA]       sigma = sum_{S1} A_i                     (Assumption 3.4 asks > 0.5)
 *   out[bi,h,CKV_DIAG_S]           s     = sum_{S} A_i
 *   out[bi,h,CKV_DIAG_C]           C     = sum_i A_i N_i
 *   out[bi,h,CKV_DIAG_THETA]       C - (2 - 1/s) sum_{S} A_i N_i                              (Thm 3.3)
 *   out[bi,h,CKV_DIAG_THETA_HAT]   C' - (2 - 1/sigma) sum_{S\S1} A_i N_i,
 *                                  C' = C - (2 - 1/sigma) sum_{S1} A_i N_i                    (Thm 3.5)
 *   out[bi,h,CKV_DIAG_THETA_RELAX] C' - M (2 - 1/sigma) sum_{S\S1} A_i                        (Thm 3.6)
 *   out[bi,h,CKV_DIAG_L]           || sum_i (A_i - A'_i) P_i ||, A' = A on S renormalised     (Def. 3.1, Thm 3.2)
 *   out[bi,h,CKV_DIAG_M]           M = min_i N_i
 * S empty: L = ||sum_i A_i P_i|| and theta = C.  S1 empty: theta_hat = theta_relax = +inf.
 *
 * STATE: reads what criticalkv_score and then criticalkv_select left in `workspace` for this descriptor
 * (the unpooled scores, the magnitudes, the stage-1 marks).  Call it after those two, with the same
 * descriptor and workspace and no other call on that workspace in between; anything else gives
 * undefined values (never a fault).  The descriptor must not carry CKV_ATTN_ONLY or CKV_WO_IS_GRAM.
 *
 * in : v, idx, count, max_budget as given to / returned by the two calls; w_o the projection itself in
 *      the layout the descriptor names; vnorm_opt the pointer criticalkv_score was given (NULL if none)
 * out: out [batch, H, CKV_N_DIAG] float32, DEVICE
 */
#define CKV_DIAG_SIGMA 0
#define CKV_DIAG_S 1
#define CKV_DIAG_C 2
#define CKV_DIAG_THETA 3
#define CKV_DIAG_THETA_HAT 4
#define CKV_DIAG_THETA_RELAX 5
#define CKV_DIAG_L 6
#define CKV_DIAG_M 7
#define CKV_N_DIAG 8
CKV_API int criticalkv_diagnostics(const ckv_layer_desc *desc, const void *v, const void *w_o,
                                   const float *vnorm_opt, const int32_t *idx, const int32_t *count,
                                   int32_t max_budget, float *out, void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/*
 * Compacted cache (Algorithm 1 line 10):  k_out[bi,g,j,:] = k[bi,g,idx[bi,g,j],:] for j < count[bi,g],
 * likewise v_out.  Rows j >= count[bi,g] are left untouched.  Bit-exact copies in the input dtype.
 *
 * in : k, v [batch, Hkv, n, d_h] (or strided per the descriptor); idx, count from criticalkv_select
 * out: k_out, v_out [batch, Hkv, max_budget, d_h] contiguous
 * An index outside [0, n) is skipped (its output row is left untouched).
 */
CKV_API int criticalkv_compact(const ckv_layer_desc *desc, const void *k, const void *v, const int32_t *idx,
                               const int32_t *count, int32_t max_budget, void *k_out, void *v_out,
                               void *hip_stream);

/*
 * Measurement aids, no part of the pass: what the device sustains for the two resources the pass is priced against.
 * Benchmarks report them beside their roofline fractions (the published peaks assume clocks and access patterns
 * that real data and real kernels do not reach).
 *   criticalkv_probe_mfma_bf16: a register-only loop of bf16 matrix-core instructions (16x16x32, seven accumulator
 *     chains per wave, two 4-wave workgroups per CU: the launch geometry of the projection kernel) whose operands
 *     are taken from `operands` (device, 1 MiB, 16-byte aligned; random values toggle the multipliers as real data
 *     does, zeros do not).  *flop_out (host, may be NULL) receives the floating-point operations of the launch.
 *   criticalkv_probe_hbm_read: a plain streaming read of `bytes` bytes at `buf` (device, 16-byte aligned).
 * `sink` is a device word that is never written (it keeps the work alive).  Both enqueue one kernel on the stream
 * and return; the caller times them.
 */
CKV_API int criticalkv_probe_mfma_bf16(const void *operands, int32_t iters, double *flop_out, float *sink,
                                       void *hip_stream);
CKV_API int criticalkv_probe_hbm_read(const void *buf, size_t bytes, uint32_t *sink, void *hip_stream);

/* Static, NUL-terminated description of an error code. */
CKV_API const char *criticalkv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* CRITICALKV_H */
