"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the same seeded inputs.

Scores: within 2e-3 relative.  Index sets: identical up to swaps inside the 2e-3 band around the
stage thresholds (counted and printed).  Compaction: bit-exact.
"""
import numpy as np
import pytest

from helpers import (assert_compaction_exact, assert_scores_close, cfg_desc, compare_selection, run_gpu_pass,
                     to_device)  # noqa: F401
from oracle import cpu_oracle as O
from workload import CONFIGS, budget_from_fraction, make_layer, reduced

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2502_03805_amd as pkg
    pkg.load()  # fails loudly if the HIP library is not built
    return pkg


def oracle_pass(cfg, t, budget=None, alpha=None, window_sum=False, scale=None):
    return O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget if budget is None else budget,
                       cfg.alpha if alpha is None else alpha, pool_kernel=cfg.pool_kernel, eps=cfg.eps,
                       window_sum=window_sum, scale=scale)


def check_full(P, cfg, t, *, flags=0, wo_out_in=False, budget=None, alpha=None, label=""):
    budget = cfg.budget if budget is None else budget
    alpha = cfg.alpha if alpha is None else alpha
    ref = oracle_pass(cfg, t, budget, alpha)
    res = run_gpu_pass(P, cfg, t, budget, alpha, flags=flags, wo_out_in=wo_out_in)
    e_v = assert_scores_close(res.vnorm, ref.vnorm, "vnorm")
    e_a = assert_scores_close(res.attn, ref.attn, "attn")
    e_c = assert_scores_close(res.crit, ref.crit, "crit")
    swaps = compare_selection(res.idx, res.count, ref, budget, alpha)
    assert_compaction_exact(res, t, budget)
    print(f"[{label or cfg.name}] max rel err vnorm {e_v[0]:.2e} attn {e_a[0]:.2e} crit {e_c[0]:.2e}; swapped indices {swaps}")
    return res, ref, swaps


# ------------------------------------------------------------------------------------------------ whole pass
@pytest.mark.parametrize("wo_out_in", [False, True])
def test_tiny_fp32_config(P, wo_out_in):
    cfg = CONFIGS["tiny"]
    t = make_layer(cfg)
    check_full(P, cfg, t, wo_out_in=wo_out_in)


@pytest.mark.parametrize("flags_name", ["mfma", "valu"])
@pytest.mark.parametrize("n", [4096, 4133, 257])
def test_llama_shape_reduced_context(P, n, flags_name):
    cfg = reduced(CONFIGS["llama32k"], n, d_model=1024)
    t = make_layer(cfg)
    flags = P.CKV_NO_MFMA if flags_name == "valu" else 0
    check_full(P, cfg, t, flags=flags, wo_out_in=True, label=f"llama n={n} {flags_name}")


def test_llama_shape_canonical_wo_layout_and_full_d_model(P):
    cfg = reduced(CONFIGS["llama32k"], 1500)
    t = make_layer(cfg)
    check_full(P, cfg, t, wo_out_in=False, label="llama n=1500 d_model=4096 canonical W_O")


def test_qwen_shape_reduced_context(P):
    cfg = reduced(CONFIGS["qwen128k"], 3000, d_model=1280)
    t = make_layer(cfg)
    for frac, alpha in [(0.1, 0.25), (0.2, 0.5), (0.4, 0.75)]:
        check_full(P, cfg, t, wo_out_in=True, budget=int(round(frac * cfg.n_ctx)), alpha=alpha,
                   label=f"qwen n=3000 B={frac} alpha={alpha}")


def test_batch_and_head_dim_64(P):
    cfg = reduced(CONFIGS["llama32k"], 700, d_model=256, batch=3, head_dim=64, n_q_heads=6, n_kv_heads=3, window=5,
                  pool_kernel=3)
    t = make_layer(cfg)
    check_full(P, cfg, t, wo_out_in=True, label="b3 dh64 bf16")
    cfg32 = cfg.with_(dtype="f32")
    t = make_layer(cfg32)
    check_full(P, cfg32, t, wo_out_in=False, label="b3 dh64 f32")


@pytest.mark.parametrize("case", ["llama_gram", "llama_valu", "qwen_gram", "tiny_f32", "dh64_bf16", "g16_gram", "mha_batch2_gram",
                                  "twelve_kv_pairs_gram", "short_context_gram"])
def test_l2_norm_variant(P, case):
    """L2 distance variant: N = ||v W_O^h||_2.  The bf16 d_h = 128 path goes through the Gram matrix
    (exact for the 2-norm); the oracle evaluates the definition (all d_model products) in float64."""
    flags, wo = 0, True
    if case == "llama_gram":
        cfg = reduced(CONFIGS["llama32k"], 4133, d_model=1024)
    elif case == "llama_valu":
        cfg = reduced(CONFIGS["llama32k"], 1500, d_model=512)
        flags = P.CKV_NO_MFMA
    elif case == "qwen_gram":
        cfg = reduced(CONFIGS["qwen128k"], 3000, d_model=2560)
    elif case == "tiny_f32":
        cfg, wo = CONFIGS["tiny"], False
    elif case == "g16_gram":
        cfg = reduced(CONFIGS["llama32k"], 2100, d_model=512, n_q_heads=16, n_kv_heads=1)
    elif case == "mha_batch2_gram":
        cfg = reduced(CONFIGS["llama32k"], 1300, d_model=512, n_q_heads=3, n_kv_heads=3, batch=2)
    elif case == "twelve_kv_pairs_gram":   # more (batch item, kv head) pairs than XCDs: the pair index wraps
        cfg = reduced(CONFIGS["llama32k"], 900, d_model=512, n_q_heads=8, n_kv_heads=4, batch=3)
    elif case == "short_context_gram":     # fewer 64-row blocks than waves in a workgroup
        cfg = reduced(CONFIGS["llama32k"], 130, d_model=512, n_q_heads=4, n_kv_heads=2, window=16)
    else:
        cfg = reduced(CONFIGS["llama32k"], 700, d_model=256, head_dim=64, n_q_heads=6, n_kv_heads=3, window=5)
    t = make_layer(cfg)
    ref = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget, cfg.alpha, pool_kernel=cfg.pool_kernel,
                      eps=cfg.eps, norm=2)
    res = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, flags=flags, wo_out_in=wo, norm=P.CKV_NORM_L2)
    e_v = assert_scores_close(res.vnorm, ref.vnorm, "vnorm (L2)")
    e_c = assert_scores_close(res.crit, ref.crit, "crit (L2)")
    swaps = compare_selection(res.idx, res.count, ref, cfg.budget, cfg.alpha)
    assert_compaction_exact(res, t, cfg.budget)
    # sanity: the L2 and L1 norms differ (the flag is honoured)
    ref1 = O.projected_value_norm(t["v"], t["w_o"], cfg.n_q_heads, norm=1)
    assert np.all(ref.vnorm < ref1)
    print(f"[L2 {case}] max rel err vnorm {e_v[0]:.2e} crit {e_c[0]:.2e}; swapped indices {swaps}")


def test_l2_with_prepared_gram_matches_inline_gram(P):
    """criticalkv_prepare_gram once, then criticalkv_score with CKV_WO_IS_GRAM: identical scores."""
    import torch
    cfg = reduced(CONFIGS["llama32k"], 2500, d_model=1024)
    t = make_layer(cfg)
    inline = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, wo_out_in=True, norm=P.CKV_NORM_L2)
    for wo_out_in in (True, False):
        desc = cfg_desc(P, cfg, flags=P.CKV_WO_OUT_IN if wo_out_in else 0, norm=P.CKV_NORM_L2)
        dev = to_device(cfg, t, wo_out_in)
        ws = torch.empty(P.workspace_bytes(desc, cfg.budget), dtype=torch.uint8, device="cuda")
        gram = torch.empty(P.gram_bytes(desc), dtype=torch.uint8, device="cuda")
        P.criticalkv_prepare_gram(desc, dev["w_o"], gram, workspace=ws)
        desc_g = cfg_desc(P, cfg, flags=P.CKV_WO_IS_GRAM, norm=P.CKV_NORM_L2)
        dev["w_o"] = gram
        res = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, flags=P.CKV_WO_IS_GRAM, norm=P.CKV_NORM_L2, dev=dev)
        assert np.array_equal(res.vnorm, inline.vnorm) and np.array_equal(res.crit, inline.crit)
        assert np.array_equal(res.idx, inline.idx)


@pytest.mark.parametrize("path", ["mfma", "valu", "f32"])
@pytest.mark.parametrize("n", [1000, 257, 70])
def test_causal_tail_and_protected_window(P, path, n):
    """Chunked-prefill mode: causal mask inside the window and the window's own tokens always kept."""
    if path == "f32":
        cfg = CONFIGS["tiny"].with_(n_ctx=n, budget=max(12, n // 8), window=8)
    else:
        cfg = reduced(CONFIGS["llama32k"], n, d_model=256, budget=max(40, n // 5))
    t = make_layer(cfg)
    flags = P.CKV_CAUSAL_TAIL | P.CKV_PROTECT_WINDOW | (P.CKV_NO_MFMA if path == "valu" else 0)
    ref = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget, cfg.alpha, pool_kernel=cfg.pool_kernel,
                      eps=cfg.eps, causal_tail=True, protect_window=True)
    res = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, flags=flags, wo_out_in=(path != "f32"))
    W = cfg.window
    # the flag changes the selection only: the scores are the plain ones
    assert_scores_close(res.attn, ref.attn, "attn (causal tail)")
    assert_scores_close(res.crit, ref.crit, "crit (causal tail)")
    compare_selection(res.idx, res.count, ref, cfg.budget, cfg.alpha)
    for g in range(cfg.n_kv_heads):
        assert res.idx[0, g, -W:].tolist() == list(range(n - W, n)), "window tokens must be kept"
    # exactly the oracle's sets on the GPU's own keys, for budgets around the window size and every split
    for B in sorted({0, 1, W - 1, W, W + 1, cfg.budget, n - 1, n} & set(range(n + 1))):
        for alpha in (0.0, 0.5, 1.0):
            got, cnt, _ = run_select(P, res.attn, res.crit, B, alpha, flags=P.CKV_PROTECT_WINDOW, window=W)
            want, wcnt, _ = O.select(res.attn.astype(np.float64), res.crit.astype(np.float64), B, np.float32(alpha),
                                     protect_last=W, max_budget=got.shape[-1])
            assert np.array_equal(cnt, wcnt) and np.array_equal(got, want), (B, alpha)
    # each flag alone
    ref_c = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget, cfg.alpha, pool_kernel=cfg.pool_kernel,
                        eps=cfg.eps, causal_tail=True)
    res_c = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, flags=flags & ~P.CKV_PROTECT_WINDOW, wo_out_in=(path != "f32"))
    assert_scores_close(res_c.attn, ref_c.attn, "attn (causal only)")
    compare_selection(res_c.idx, res_c.count, ref_c, cfg.budget, cfg.alpha)


def test_chunked_prefill_loop_matches_oracle_loop(P):
    """Three chunks of a prompt with eviction after each: the GPU host loop and the same loop over the oracle
    keep the same entries and end with the same cache."""
    import torch
    from paper_2502_03805_amd.chunked import chunked_prefill_evict
    base = reduced(CONFIGS["llama32k"], 3 * 700, d_model=256)
    t = make_layer(base)
    chunk, budget, alpha = 700, 500, 0.5
    qs = [make_layer(base.with_(n_ctx=64), seed_offset=10 + c)["q_win"] for c in range(3)]
    ks = [t["k"][:, :, c * chunk:(c + 1) * chunk] for c in range(3)]
    vs = [t["v"][:, :, c * chunk:(c + 1) * chunk] for c in range(3)]
    # oracle loop
    kc = vc = None
    kept_ref = []
    for c in range(3):
        k_all = ks[c] if kc is None else np.concatenate([kc, ks[c]], axis=2)
        v_all = vs[c] if vc is None else np.concatenate([vc, vs[c]], axis=2)
        r = O.full_pass(qs[c], k_all, v_all, t["w_o"], budget, alpha, pool_kernel=base.pool_kernel, eps=base.eps,
                        causal_tail=True, protect_window=True)
        kc, vc = r.k_out, r.v_out
        kept_ref.append(r.idx)
    # GPU loop
    dev = to_device(base, t, True)
    tb = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda", torch.bfloat16)
    mk = lambda n: cfg_desc(P, base.with_(n_ctx=n), flags=P.CKV_WO_OUT_IN | P.CKV_CAUSAL_TAIL | P.CKV_PROTECT_WINDOW)
    k_cache, v_cache, kept = chunked_prefill_evict(mk, [tb(q) for q in qs], [tb(k) for k in ks], [tb(v) for v in vs],
                                                   dev["w_o"], budget, alpha)
    torch.cuda.synchronize()
    for c in range(3):
        assert np.array_equal(kept[c].cpu().numpy(), kept_ref[c]), f"chunk {c}: kept sets differ"
    assert np.array_equal(k_cache.float().cpu().numpy(), kc) and np.array_equal(v_cache.float().cpu().numpy(), vc)


def test_attention_only_baseline_mode(P):
    """CKV_ATTN_ONLY: no projected magnitude; crit == attn and the selection is attention-only Top-B
    (Algorithm 2's regular selection) for every alpha."""
    import torch
    cfg = reduced(CONFIGS["llama32k"], 3000, d_model=256)
    t = make_layer(cfg)
    a = O.maxpool1d(O.window_attention(t["q_win"], t["k"]), cfg.pool_kernel)
    attn_ref, _ = O.group_keys(a, np.zeros_like(a), cfg.n_kv_heads, cfg.eps)
    desc = cfg_desc(P, cfg, flags=P.CKV_ATTN_ONLY)
    dev = to_device(cfg, t, False)
    b, Hkv, n = cfg.batch, cfg.n_kv_heads, cfg.n_ctx
    ws = torch.empty(P.workspace_bytes(desc, cfg.budget), dtype=torch.uint8, device="cuda")
    attn = torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda")
    crit = torch.empty_like(attn)
    P.criticalkv_score(desc, dev["q_win"], dev["k"], None, None, attn, crit, None, workspace=ws)
    idx = torch.empty((b, Hkv, cfg.budget), dtype=torch.int32, device="cuda")
    count = torch.empty((b, Hkv), dtype=torch.int32, device="cuda")
    bud = torch.full((b, Hkv), cfg.budget, dtype=torch.int32, device="cuda")
    got = {}
    for alpha in (0.0, 0.5, 1.0):
        P.criticalkv_select(desc, attn, crit, bud, alpha, cfg.budget, idx, count, workspace=ws)
        torch.cuda.synchronize()
        got[alpha] = idx.cpu().numpy().copy()
    assert torch.equal(attn, crit)
    assert_scores_close(attn.cpu().numpy(), attn_ref, "attn (attention-only)")
    a32 = attn.cpu().numpy().astype(np.float64)
    ref_idx, _, _ = O.select(a32, a32, cfg.budget, 1.0)
    for alpha in got:
        assert np.array_equal(got[alpha], ref_idx)


def test_window_sum_and_explicit_scale(P):
    cfg = reduced(CONFIGS["llama32k"], 900, d_model=256)
    t = make_layer(cfg)
    ref = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget, cfg.alpha, pool_kernel=cfg.pool_kernel,
                      eps=cfg.eps, window_sum=True, scale=0.05)
    res = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, wo_out_in=True, window_reduce=P.CKV_SUM, softmax_scale=0.05)
    assert_scores_close(res.attn, ref.attn, "attn(sum)")
    assert_scores_close(res.crit, ref.crit, "crit(sum)")
    compare_selection(res.idx, res.count, ref, cfg.budget, cfg.alpha)


def test_per_head_budgets_and_special_alphas(P):
    cfg = reduced(CONFIGS["llama32k"], 1024, d_model=256)
    t = make_layer(cfg)
    budget = np.array([[0, 1, 2, 100, 511, 1023, 1024, 37]], dtype=np.int32)
    for alpha in (0.0, 0.3, 1.0):
        ref = oracle_pass(cfg, t, budget, np.float32(alpha))
        res = run_gpu_pass(P, cfg, t, budget, alpha, wo_out_in=True, max_budget=1024)
        compare_selection(res.idx, res.count, ref, budget, alpha)
        assert_compaction_exact(res, t, budget)
    # alpha = 1 is attention-only Top-B (Algorithm 2, regular selection); B = n keeps everything
    assert res.idx[0, 6].tolist() == list(range(1024))


@pytest.mark.parametrize("norm", [1, 2])
def test_strided_kv_views(P, norm):
    """K and V living inside a larger [batch, n, Hkv, 2*d_h] buffer (token-major, padded rows), for both norms
    (the L2 kernel addresses the V rows through a buffer descriptor of its own)."""
    import torch
    cfg = reduced(CONFIGS["llama32k"], 640, d_model=256 if norm == 1 else 512)
    t = make_layer(cfg)
    ref = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget, cfg.alpha, pool_kernel=cfg.pool_kernel,
                      eps=cfg.eps, norm=norm)
    b, Hkv, n, dh = cfg.batch, cfg.n_kv_heads, cfg.n_ctx, cfg.head_dim
    big_k = torch.zeros((b, n, Hkv, 2 * dh), dtype=torch.bfloat16, device="cuda")
    big_v = torch.zeros_like(big_k)
    big_k[..., :dh] = torch.from_numpy(t["k"]).permute(0, 2, 1, 3).to(torch.bfloat16)
    big_v[..., dh:] = torch.from_numpy(t["v"]).permute(0, 2, 1, 3).to(torch.bfloat16)
    kview = big_k[..., :dh].permute(0, 2, 1, 3)   # [b, Hkv, n, dh] view
    vview = big_v[..., dh:].permute(0, 2, 1, 3)
    desc = cfg_desc(P, cfg, flags=P.CKV_WO_OUT_IN, k_stride=tuple(kview.stride()[:3]), v_stride=tuple(vview.stride()[:3]),
                    norm=P.CKV_NORM_L1 if norm == 1 else P.CKV_NORM_L2)
    dev = to_device(cfg, t, True)
    ws = torch.empty(P.workspace_bytes(desc, cfg.budget), dtype=torch.uint8, device="cuda")
    attn = torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda")
    crit = torch.empty_like(attn)
    idx = torch.empty((b, Hkv, cfg.budget), dtype=torch.int32, device="cuda")
    count = torch.empty((b, Hkv), dtype=torch.int32, device="cuda")
    k_out = torch.zeros((b, Hkv, cfg.budget, dh), dtype=torch.bfloat16, device="cuda")
    v_out = torch.zeros_like(k_out)
    bud = torch.full((b, Hkv), cfg.budget, dtype=torch.int32, device="cuda")

    class View:  # hands the view's own data pointer to the binding
        def __init__(self, x): self.x = x
        def data_ptr(self): return self.x.data_ptr()

    P.criticalkv_score(desc, dev["q_win"], View(kview), View(vview), dev["w_o"], attn, crit, None, workspace=ws)
    P.criticalkv_select(desc, attn, crit, bud, cfg.alpha, cfg.budget, idx, count, workspace=ws)
    P.criticalkv_compact(desc, View(kview), View(vview), idx, count, cfg.budget, k_out, v_out)
    torch.cuda.synchronize()
    assert_scores_close(attn.cpu().numpy(), ref.attn, "attn(strided)")
    assert_scores_close(crit.cpu().numpy(), ref.crit, "crit(strided)")
    compare_selection(idx.cpu().numpy(), count.cpu().numpy(), ref, cfg.budget, cfg.alpha)
    sel = idx.cpu().numpy()
    for g in range(Hkv):
        assert np.array_equal(k_out[0, g].float().cpu().numpy(), t["k"][0, g, sel[0, g]])
        assert np.array_equal(v_out[0, g].float().cpu().numpy(), t["v"][0, g, sel[0, g]])


# ------------------------------------------------------------------------------------------------ select alone
def run_select(P, attn, crit, budget, alpha, max_budget=None, flags=0, window=1):
    import torch
    b, Hkv, n = attn.shape
    desc = P.make_desc(batch=b, n_q_heads=Hkv, n_kv_heads=Hkv, head_dim=128, d_model=128, n_ctx=n, window=window,
                       pool_kernel=1, dtype=P.CKV_BF16, flags=flags)
    budget = np.broadcast_to(np.asarray(budget, dtype=np.int32), (b, Hkv)).copy()
    mb = max_budget or max(1, int(budget.max()))
    ws = torch.empty(P.workspace_bytes(desc, mb), dtype=torch.uint8, device="cuda")
    idx = torch.full((b, Hkv, mb), -7, dtype=torch.int32, device="cuda")
    count = torch.full((b, Hkv), -7, dtype=torch.int32, device="cuda")
    P.criticalkv_select(desc, torch.from_numpy(attn).cuda(), torch.from_numpy(crit).cuda(),
                        torch.from_numpy(budget).cuda(), alpha, mb, idx, count, workspace=ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), count.cpu().numpy(), budget


def assert_select_exact(P, attn, crit, budget, alpha, max_budget=None):
    """Same float32 keys on both sides: the index sets must be identical, ties included."""
    attn = np.ascontiguousarray(attn, dtype=np.float32)
    crit = np.ascontiguousarray(crit, dtype=np.float32)
    idx, count, budget = run_select(P, attn, crit, budget, alpha, max_budget)
    ref_idx, ref_count, _ = O.select(attn.astype(np.float64), crit.astype(np.float64), budget, np.float32(alpha),
                                     max_budget=idx.shape[-1])
    assert np.array_equal(count, ref_count)
    assert np.array_equal(idx, ref_idx)


@pytest.mark.parametrize("n", [1, 3, 4, 5, 1000, 2047, 2048, 2049, 4096, 4097, 12289, 40000])
def test_select_exact_on_random_keys(P, n):
    r = np.random.Generator(np.random.PCG64(n))
    attn = r.random((2, 3, n), dtype=np.float32)
    crit = r.lognormal(0, 2, (2, 3, n)).astype(np.float32)
    budget = r.integers(0, n + 1, (2, 3))
    for alpha in (0.5, 0.25, 0.0, 1.0):
        assert_select_exact(P, attn, crit, budget, alpha, max_budget=n)


def test_select_exact_with_heavy_ties(P):
    r = np.random.Generator(np.random.PCG64(5))
    n = 9000
    # few distinct values: thresholds fall inside large tie groups in both stages
    attn = r.integers(0, 6, (1, 4, n)).astype(np.float32) / 8
    crit = r.integers(0, 4, (1, 4, n)).astype(np.float32)
    for B in (1, 17, 4500, 8999, 9000):
        for alpha in (0.5, 0.1, 0.9):
            assert_select_exact(P, attn, crit, B, alpha)
    # all keys equal: the selection is the first B tokens
    ones = np.ones((1, 2, n), dtype=np.float32)
    idx, count, _ = run_select(P, ones, ones, 1234, 0.5)
    assert idx[0, 0].tolist() == list(range(1234)) and count.tolist() == [[1234, 1234]]
    # pooled scores replicate values over neighbours (the structural source of ties)
    base = r.random((1, 2, n)).astype(np.float64)
    pooled = O.maxpool1d(base, 7).astype(np.float32)
    assert_select_exact(P, pooled, pooled * r.integers(1, 3, (1, 2, n)).astype(np.float32), 3000, 0.5)


def test_select_signed_zero_and_negative_keys(P):
    n = 64
    attn = np.linspace(-1, 1, n, dtype=np.float32)[None, None]
    crit = np.zeros((1, 1, n), dtype=np.float32)
    crit[0, 0, ::2] = -0.0   # -0 and +0 compare equal: ties resolved by index
    crit[0, 0, 5] = -3.0
    for B in (10, 40, 64):
        assert_select_exact(P, attn, crit, B, 0.5)
        assert_select_exact(P, -attn, crit, B, 0.25)


def test_select_infinities_denormals_and_extreme_magnitudes(P):
    """Keys at the ends of the float range (both infinities, the largest and smallest normals, denormals) keep
    their IEEE order in the radix image."""
    r = np.random.Generator(np.random.PCG64(31))
    n = 5000
    specials = np.array([np.inf, -np.inf, 3.4028235e38, -3.4028235e38, 1.1754944e-38, -1.1754944e-38, 1e-45, -1e-45,
                         1e-40, 0.0, -0.0, 1.0, -1.0], dtype=np.float32)
    attn = r.choice(specials, (1, 3, n)).astype(np.float32)
    crit = (r.standard_normal((1, 3, n)) * 10.0 ** r.integers(-44, 38, (1, 3, n))).astype(np.float32)
    crit[0, :, ::97] = np.inf
    crit[0, :, 5::101] = -np.inf
    for B in (1, 600, 2500, n):
        for alpha in (0.5, 0.0, 1.0):
            assert_select_exact(P, attn, crit, B, alpha)
            assert_select_exact(P, crit, attn, B, alpha)


def test_budget_is_clamped_to_n_and_max_budget(P):
    n = 100
    r = np.random.Generator(np.random.PCG64(9))
    attn = r.random((1, 2, n), dtype=np.float32)
    idx, count, _ = run_select(P, attn, attn, np.array([[500, -3]]), 0.5, max_budget=60)
    assert count.tolist() == [[60, 0]]
    assert np.all(idx[0, 1] == -1) and np.all(idx[0, 0] >= 0)


# ------------------------------------------------------------------------------------------------ allocation
def run_allocate(P, attn, total, floor_frac):
    import torch
    b, Hkv, n = attn.shape
    desc = P.make_desc(batch=b, n_q_heads=Hkv, n_kv_heads=Hkv, head_dim=128, d_model=128, n_ctx=n, window=1,
                       pool_kernel=1, dtype=P.CKV_BF16)
    ws = torch.empty(P.workspace_bytes(desc, -(-total // Hkv)), dtype=torch.uint8, device="cuda")
    budget = torch.full((b, Hkv), -7, dtype=torch.int32, device="cuda")
    P.criticalkv_allocate(desc, torch.from_numpy(np.ascontiguousarray(attn, dtype=np.float32)).cuda(), total, floor_frac,
                          budget, workspace=ws)
    torch.cuda.synchronize()
    return budget.cpu().numpy()


@pytest.mark.parametrize("n", [5, 1000, 4097, 40000])
def test_allocate_exact_against_oracle(P, n):
    """Same float32 scores on both sides: budgets are integers and must be identical."""
    r = np.random.Generator(np.random.PCG64(77 + n))
    Hkv = 8
    # heads of different concentration, as in a real layer: some heads own most of the pooled top scores
    attn = (r.random((2, Hkv, n)) ** r.integers(1, 9, (2, Hkv, 1))).astype(np.float32)
    for total in (0, 1, Hkv, n, 3 * n + 1, Hkv * n):
        for floor_frac in (0.0, 0.2, 0.5, 1.0):
            got = run_allocate(P, attn, total, floor_frac)
            ref = O.allocate(attn.astype(np.float64), total, np.float32(floor_frac))
            assert np.array_equal(got, ref), (n, total, floor_frac, got, ref)
            assert got.sum(axis=1).max() <= total


def test_allocate_ties_and_pooled_scores(P):
    r = np.random.Generator(np.random.PCG64(3))
    n, Hkv = 6000, 4
    few = r.integers(0, 5, (1, Hkv, n)).astype(np.float32)          # the threshold falls inside a large tie group
    pooled = O.maxpool1d(r.random((1, Hkv, n)), 7).astype(np.float32)
    same = np.broadcast_to(r.random((1, 1, n)).astype(np.float32), (1, Hkv, n)).copy()  # identical heads
    for attn in (few, pooled, same):
        for total in (7, 2 * n, 3 * n + 5):
            for floor_frac in (0.0, 0.25):
                got = run_allocate(P, attn, total, floor_frac)
                ref = O.allocate(attn.astype(np.float64), total, np.float32(floor_frac))
                assert np.array_equal(got, ref), (total, floor_frac, got, ref)


def test_allocate_then_select_on_llama_shape(P):
    """Scores from the GPU path, allocation on both sides from their own scores, then the two-stage selection
    with the allocated budgets; the budgets may differ only through scores inside the 2e-3 band."""
    import torch
    cfg = reduced(CONFIGS["llama32k"], 4133)
    t = make_layer(cfg)
    total = cfg.n_kv_heads * cfg.budget
    ref = O.score(t["q_win"], t["k"], t["v"], t["w_o"], pool_kernel=cfg.pool_kernel, eps=cfg.eps)
    ff = np.float32(0.2)
    ref_budget = O.allocate(ref.attn, total, ff)
    res = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha)
    got_on_gpu_scores = run_allocate(P, res.attn, total, ff)
    assert np.array_equal(got_on_gpu_scores, O.allocate(res.attn.astype(np.float64), total, ff))
    # slots may move between heads only through entries whose score lies in the 2e-3 band around the pooled threshold
    floor_each = int(np.floor(float(ff) * total / cfg.n_kv_heads))
    pool = total - cfg.n_kv_heads * floor_each
    tau = np.sort(ref.attn.reshape(-1))[::-1][pool - 1]
    band = int((np.abs(ref.attn - tau) <= 2e-3 * tau).sum())
    moved = int(np.abs(got_on_gpu_scores - ref_budget).sum())
    print(f"[allocate llama 4133] budgets {got_on_gpu_scores.tolist()} oracle {ref_budget.tolist()} moved slots {moved} "
          f"(entries in the band: {band})")
    assert got_on_gpu_scores.sum() == total and moved <= 2 * band
    assert got_on_gpu_scores.min() >= floor_each and got_on_gpu_scores.std() > 0
    res2 = run_gpu_pass(P, cfg, t, got_on_gpu_scores, cfg.alpha)
    ref2 = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], got_on_gpu_scores, cfg.alpha, pool_kernel=cfg.pool_kernel,
                       eps=cfg.eps)
    compare_selection(res2.idx, res2.count, ref2, got_on_gpu_scores, cfg.alpha)
    assert np.array_equal(res2.count, got_on_gpu_scores)


# ------------------------------------------------------------------------------------------------ diagnostics
DIAG_TOL = 2e-3


def run_diagnostics(P, cfg, t, budget, alpha, *, flags=0, wo_out_in=False, norm=1, window_reduce=None, own_vnorm=False,
                    crit_is_attn=False):
    """score -> select -> diagnostics through the C ABI; returns (out [b,H,8], idx, count)."""
    import torch
    if wo_out_in:
        flags |= P.CKV_WO_OUT_IN
    desc = cfg_desc(P, cfg, flags=flags, norm=norm, window_reduce=window_reduce)
    dev = to_device(cfg, t, wo_out_in)
    b, H, Hkv, n = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_ctx
    budget = np.broadcast_to(np.asarray(budget, dtype=np.int32), (b, Hkv)).copy()
    mb = max(1, int(budget.max()))
    ws = torch.empty(P.workspace_bytes(desc, mb), dtype=torch.uint8, device="cuda")
    attn = torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda")
    crit = torch.empty_like(attn)
    vnorm = torch.empty((b, H, n), dtype=torch.float32, device="cuda") if own_vnorm else None
    idx = torch.empty((b, Hkv, mb), dtype=torch.int32, device="cuda")
    count = torch.empty((b, Hkv), dtype=torch.int32, device="cuda")
    out = torch.full((b, H, 8), -7.0, dtype=torch.float32, device="cuda")
    P.criticalkv_score(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], attn, crit, vnorm, workspace=ws)
    P.criticalkv_select(desc, attn, attn if crit_is_attn else crit, torch.from_numpy(budget).cuda(), alpha, mb, idx, count,
                        workspace=ws)
    P.criticalkv_diagnostics(desc, dev["v"], dev["w_o"], vnorm, idx, count, mb, out, workspace=ws)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), idx.cpu().numpy(), count.cpu().numpy()


def oracle_diagnostics(cfg, t, budget, alpha, norm=1, window_sum=False, crit_is_attn=False):
    r = O.score(t["q_win"], t["k"], t["v"], t["w_o"], pool_kernel=cfg.pool_kernel, eps=cfg.eps, norm=norm)
    mb = max(1, int(np.max(budget)))  # the index list the GPU side allocates has at least one slot
    idx, count, _, st1 = O.select(r.attn, r.attn if crit_is_attn else r.crit, budget, alpha, max_budget=mb, with_stage1=True)
    return O.diagnostics(r.a_head, t["v"], t["w_o"], idx, count, st1, norm), idx


def assert_diagnostics_close(got, ref, label):
    """Every field is a sum of terms bounded by C (or a plain sum of A), so the error is measured against
    max(|ref|, 1e-3 C); infinities must match exactly."""
    f = {name: j for j, name in enumerate(O.DIAG_FIELDS)}
    assert np.array_equal(np.isinf(got), np.isinf(ref)), label
    fin = np.isfinite(ref)
    scale = np.maximum(np.abs(ref), 1e-3 * ref[..., f["C"]][..., None])
    for name in ("sigma", "s"):
        scale[..., f[name]] = np.maximum(np.abs(ref[..., f[name]]), 1e-3)
    rel = np.where(fin, np.abs(np.where(fin, got, 0) - np.where(fin, ref, 0)) / scale, 0.0)
    worst = {name: float(rel[..., j].max()) for name, j in f.items()}
    print(f"[diagnostics {label}] max scaled error per field: " + " ".join(f"{k}={v:.1e}" for k, v in worst.items()))
    assert rel.max() <= DIAG_TOL, (label, worst)
    return worst


@pytest.mark.parametrize("case", ["tiny_f32", "llama_mfma", "llama_valu_outin", "qwen", "dh64_batch2", "l2", "own_vnorm"])
def test_diagnostics_against_oracle(P, case):
    kw, norm = {}, 1
    if case == "tiny_f32":
        cfg = CONFIGS["tiny"]
    elif case == "qwen":
        cfg = reduced(CONFIGS["qwen128k"], 3000, d_model=512)
    elif case == "dh64_batch2":
        cfg = reduced(CONFIGS["llama32k"], 1500, d_model=256, head_dim=64, batch=2)
    else:
        cfg = reduced(CONFIGS["llama32k"], 4133, d_model=512)
    if case == "llama_valu_outin":
        kw = dict(flags=P.CKV_NO_MFMA, wo_out_in=True)
    if case == "l2":
        norm = 2
    if case == "own_vnorm":
        kw = dict(own_vnorm=True)
    t = make_layer(cfg)
    got, idx, _ = run_diagnostics(P, cfg, t, cfg.budget, cfg.alpha, norm=norm, **kw)
    ref, ref_idx = oracle_diagnostics(cfg, t, cfg.budget, cfg.alpha, norm=norm)
    assert np.array_equal(idx, ref_idx)      # no swaps on these inputs, so both sides describe the same sets
    assert_diagnostics_close(got, ref, case)
    f = {name: j for j, name in enumerate(O.DIAG_FIELDS)}
    assert np.all(got[..., f["L"]] <= got[..., f["theta"]] * (1 + 1e-4))
    assert np.all(got[..., f["theta"]] <= got[..., f["theta_hat"]] * (1 + 1e-4))


def test_diagnostics_special_budgets_and_baseline_selection(P):
    cfg = reduced(CONFIGS["llama32k"], 2100, d_model=256)
    t = make_layer(cfg)
    n = cfg.n_ctx
    # per-head budgets with an empty head and a full head; alpha = 0 leaves stage 1 empty, alpha = 1 stage 2
    budgets = np.array([[0, 1, 7, 500, 1024, 1025, n - 1, n]])
    for alpha in (0.5, 0.0, 1.0):
        got, idx, _ = run_diagnostics(P, cfg, t, budgets, alpha)
        ref, ref_idx = oracle_diagnostics(cfg, t, budgets, alpha)
        assert np.array_equal(idx, ref_idx)
        assert_diagnostics_close(got, ref, f"budgets alpha={alpha}")
    # the attention-only baseline with the same split (stage 2 ranked by attention): its relaxed bound
    got, idx, _ = run_diagnostics(P, cfg, t, cfg.budget, 0.5, crit_is_attn=True)
    ref, ref_idx = oracle_diagnostics(cfg, t, cfg.budget, 0.5, crit_is_attn=True)
    assert np.array_equal(idx, ref_idx)
    assert_diagnostics_close(got, ref, "attention-only selection")


# ------------------------------------------------------------------------------------------------ odd shapes
ODD_SHAPES = {
    "g16_w40_dm128": dict(base="llama32k", n_q_heads=16, n_kv_heads=1, n_ctx=700, window=40, d_model=128, pool_kernel=1,
                          budget=150),
    "mha_w96_batch2": dict(base="llama32k", n_q_heads=3, n_kv_heads=3, n_ctx=300, window=96, d_model=256, batch=2, budget=120),
    "g12_two_wave_groups": dict(base="llama32k", n_q_heads=24, n_kv_heads=2, n_ctx=400, window=8, d_model=128, budget=77),
    "n_equals_window_bf16": dict(base="llama32k", n_q_heads=8, n_kv_heads=2, n_ctx=32, window=32, d_model=128, budget=9, pool_kernel=3),
    "single_entry_bf16": dict(base="llama32k", n_q_heads=4, n_kv_heads=2, n_ctx=1, window=1, d_model=128, budget=1, pool_kernel=1),
    "single_entry_f32": dict(base="tiny", n_q_heads=2, n_kv_heads=2, n_ctx=1, window=1, d_model=32, budget=1, pool_kernel=1),
    "n_equals_window_f32": dict(base="tiny", n_q_heads=4, n_kv_heads=2, n_ctx=5, window=5, d_model=64, budget=2, pool_kernel=5),
    "g7_w64": dict(base="llama32k", n_q_heads=28, n_kv_heads=4, n_ctx=1000, window=64, d_model=384, budget=333),
    "f32_dh64_g3_w1_dm32": dict(base="tiny", n_q_heads=6, n_kv_heads=2, n_ctx=257, window=1, d_model=32, pool_kernel=3,
                                budget=40),
    "bf16_dh64_g2": dict(base="llama32k", n_q_heads=4, n_kv_heads=2, head_dim=64, n_ctx=515, window=16, d_model=96, budget=100),
    # windows past what the matrix-core sweeps hold in registers (vector-ALU sweeps, the window staged in rounds)
    "w200_bf16": dict(base="llama32k", n_q_heads=4, n_kv_heads=2, n_ctx=600, window=200, d_model=128, budget=100),
    "w_equals_n_300_f32": dict(base="tiny", n_q_heads=2, n_kv_heads=1, n_ctx=300, window=300, d_model=64, budget=50),
    # wave-private matrix-core sweeps: 128-row window (four row blocks per head), 100-row window, d_h = 64 with a 5:1 group
    "w128_g2_wave": dict(base="llama32k", n_q_heads=4, n_kv_heads=2, n_ctx=900, window=128, d_model=128, budget=200),
    "w100_mha_wave": dict(base="llama32k", n_q_heads=2, n_kv_heads=2, n_ctx=333, window=100, d_model=128, budget=60),
    "dh64_g5_w64_wave": dict(base="llama32k", n_q_heads=10, n_kv_heads=2, head_dim=64, n_ctx=1100, window=64, d_model=128, budget=300),
}


@pytest.mark.parametrize("shape", sorted(ODD_SHAPES))
def test_odd_shapes_every_entry_point(P, shape):
    """Group sizes 1, 2, 3, 5, 7, 12 and 16, windows 1 to 300 (= n), the smallest d_model, both dtypes and head sizes,
    every attention code path: whole pass, allocation and diagnostics against the oracle."""
    kw = dict(ODD_SHAPES[shape])
    cfg = CONFIGS[kw.pop("base")].with_(**kw)
    t = make_layer(cfg)
    res, ref, _ = check_full(P, cfg, t, label=shape)
    total = cfg.n_kv_heads * cfg.budget
    got_b = run_allocate(P, res.attn, total, np.float32(0.3))
    assert np.array_equal(got_b, O.allocate(res.attn.astype(np.float64), total, np.float32(0.3)))
    got, idx, _ = run_diagnostics(P, cfg, t, cfg.budget, cfg.alpha)
    ref_d, ref_idx = oracle_diagnostics(cfg, t, cfg.budget, cfg.alpha)
    assert np.array_equal(idx, ref_idx)
    assert_diagnostics_close(got, ref_d, shape)


# ------------------------------------------------------------------------------------------------ full-size
def _kv_subset(cfg, t, kv_heads):
    """The sub-layer made of the given kv heads: their query heads, keys, values and rows of W_O."""
    G, dh = cfg.n_q_heads // cfg.n_kv_heads, cfg.head_dim
    qh = np.concatenate([np.arange(g * G, (g + 1) * G) for g in kv_heads])
    rows = np.concatenate([np.arange(h * dh, (h + 1) * dh) for h in qh])
    return {"q_win": t["q_win"][:, qh], "k": t["k"][:, kv_heads], "v": t["v"][:, kv_heads], "w_o": t["w_o"][rows]}, qh


def _full_size_check(P, cfg, t, sweeps=None, layer_label="", kv_heads=None):
    """Full BASELINE shape in the launch configuration the benchmark times (output-major W_O), against the
    float64 oracle run in full on every token (of every kv head, or of the listed ones where a whole layer is
    more than the host can afford): all three scores element by element; the GPU's selection against the
    ORACLE's own selection from the oracle's own scores, differences allowed only inside the 2e-3 band around the
    oracle's stage thresholds and counted; then the same selection against the oracle's sort on the GPU's own
    float32 keys, where it must be identical; compaction bit-exact.  Returns the number of swapped indices."""
    import torch
    res = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, wo_out_in=True)
    if kv_heads is None:
        sub, gs, qh = t, np.arange(cfg.n_kv_heads), np.arange(cfg.n_q_heads)
    else:
        gs = np.asarray(kv_heads)
        sub, qh = _kv_subset(cfg, t, gs)
    ref = O.score(sub["q_win"], sub["k"], sub["v"], sub["w_o"], pool_kernel=cfg.pool_kernel, eps=cfg.eps)
    e_v = assert_scores_close(res.vnorm[:, qh], ref.vnorm, "vnorm (all tokens)")
    e_a = assert_scores_close(res.attn[:, gs], ref.attn, "attn (all tokens)")
    e_c = assert_scores_close(res.crit[:, gs], ref.crit, "crit (all tokens)")
    gpu_attn64, gpu_crit64 = res.attn.astype(np.float64), res.crit.astype(np.float64)
    total_swaps = 0
    for k, (B, alpha) in enumerate([(cfg.budget, cfg.alpha)] + list(sweeps or [])):
        if k == 0:
            idx, count = res.idx, res.count
        else:
            idx, count, _ = run_select(P, res.attn, res.crit, B, alpha)
        # (1) the pass against the oracle's pass: the oracle ranks its own float64 scores
        ref.idx, ref.count, ref.tau = O.select(ref.attn, ref.crit, B, np.float32(alpha), max_budget=idx.shape[-1])
        swaps = compare_selection(idx[:, gs], count[:, gs], ref, B, alpha)
        total_swaps += swaps
        # (2) the selection kernels alone: identical keys on both sides, identical sets
        own_idx, own_count, _ = O.select(gpu_attn64, gpu_crit64, B, np.float32(alpha), max_budget=idx.shape[-1])
        assert np.array_equal(count, own_count) and np.array_equal(idx, own_idx), (B, alpha)
        print(f"[{cfg.name}{layer_label} full] B {B} alpha {alpha}: swaps {swaps} against the oracle's selection on "
              f"{len(gs) * cfg.batch} heads x {cfg.n_ctx} tokens; identical on the GPU's own keys")
    assert_compaction_exact(res, t, cfg.budget)
    # the two-stage result must differ from attention-only Top-B on this workload (stage 2 is exercised)
    top_idx, _, _ = O.select(gpu_attn64, gpu_crit64, cfg.budget, 1.0)
    assert not np.array_equal(top_idx, res.idx)
    print(f"[{cfg.name}{layer_label} full] all {cfg.n_ctx} tokens of {len(gs)} kv heads: max / median rel err "
          f"vnorm {e_v[0]:.2e} / {e_v[1]:.2e} attn {e_a[0]:.2e} / {e_a[1]:.2e} crit {e_c[0]:.2e} / {e_c[1]:.2e}; "
          f"swaps {total_swaps}")
    # adaptive budgets over the whole layer: one row of Hkv * n keys per batch item, exact on the GPU's own keys
    total = cfg.n_kv_heads * cfg.budget
    for ff in (np.float32(0.2), np.float32(0.0)):
        got_b = run_allocate(P, res.attn, total, ff)
        assert np.array_equal(got_b, O.allocate(gpu_attn64, total, ff)), ff
    print(f"[{cfg.name}{layer_label} full] allocated budgets (floor 0): {got_b.tolist()}")
    del res
    torch.cuda.empty_cache()
    return total_swaps


def test_full_size_llama32k(P):
    cfg = CONFIGS["llama32k"]
    _full_size_check(P, cfg, make_layer(cfg))


def test_full_size_diagnostics_one_kv_group_llama32k(P):
    """Full shape on the GPU; the oracle computes the last kv head's group alone (its queries, keys, values and
    W_O rows), which is the part of the output one can afford to check one by one."""
    cfg = CONFIGS["llama32k"]
    t = make_layer(cfg)
    got, idx, _ = run_diagnostics(P, cfg, t, cfg.budget, cfg.alpha, wo_out_in=True)
    G = cfg.n_q_heads // cfg.n_kv_heads
    g = cfg.n_kv_heads - 1
    hs = slice(g * G, (g + 1) * G)
    sub = {"q_win": t["q_win"][:, hs], "k": t["k"][:, g:g + 1], "v": t["v"][:, g:g + 1],
           "w_o": t["w_o"][g * G * cfg.head_dim:(g + 1) * G * cfg.head_dim]}
    ref, ref_idx = oracle_diagnostics(cfg, sub, cfg.budget, cfg.alpha)
    assert np.array_equal(idx[:, g:g + 1], ref_idx)
    assert_diagnostics_close(got[:, hs], ref, "llama32k full, last kv group")
    f = {name: j for j, name in enumerate(O.DIAG_FIELDS)}
    assert np.all(got[..., f["L"]] <= got[..., f["theta"]]) and np.all(got[..., f["theta"]] <= got[..., f["theta_hat"]] * (1 + 1e-5))
    print(f"[llama32k full] heads with sigma > 0.5: {(got[..., f['sigma']] > 0.5).mean():.3f}; mean L {got[..., f['L']].mean():.4f} "
          f"theta_hat {got[..., f['theta_hat']].mean():.4f} theta_relax {got[..., f['theta_relax']].mean():.4f}")


@pytest.mark.parametrize("name", ["llama32k", "llama128k"])
def test_full_size_l2_with_prepared_gram(P, name):
    """The launch configuration `bench.py --norm l2` times (several row tiles per workgroup): every token's
    magnitude and criticality against the oracle's definition (all d_model products in float64), the selection
    against the oracle's own under the tie rule, and exactly on the GPU's own keys."""
    import torch
    cfg = CONFIGS[name]
    t = make_layer(cfg)
    prep = cfg_desc(P, cfg, flags=P.CKV_WO_OUT_IN, norm=P.CKV_NORM_L2)
    dev = to_device(cfg, t, True)
    ws = torch.empty(P.workspace_bytes(prep, cfg.budget), dtype=torch.uint8, device="cuda")
    gram = torch.empty(P.gram_bytes(prep), dtype=torch.uint8, device="cuda")
    P.criticalkv_prepare_gram(prep, dev["w_o"], gram, workspace=ws)
    dev["w_o"] = gram
    del ws
    res = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, flags=P.CKV_WO_IS_GRAM, norm=P.CKV_NORM_L2, dev=dev)
    ref = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget, cfg.alpha, pool_kernel=cfg.pool_kernel,
                      eps=cfg.eps, norm=2)
    e_v = assert_scores_close(res.vnorm, ref.vnorm, "vnorm L2 (all tokens)")
    e_c = assert_scores_close(res.crit, ref.crit, "crit L2 (all tokens)")
    swaps = compare_selection(res.idx, res.count, ref, cfg.budget, cfg.alpha)
    own_idx, own_count, _ = O.select(res.attn.astype(np.float64), res.crit.astype(np.float64), cfg.budget, np.float32(cfg.alpha))
    assert np.array_equal(res.count, own_count) and np.array_equal(res.idx, own_idx)
    assert_compaction_exact(res, t, cfg.budget)
    print(f"[{name} L2 full] all tokens: max rel err vnorm {e_v[0]:.2e} crit {e_c[0]:.2e}; swaps {swaps} against the "
          f"oracle's selection")
    del res, dev
    torch.cuda.empty_cache()


def test_full_size_llama128k(P):
    cfg = CONFIGS["llama128k"]
    _full_size_check(P, cfg, make_layer(cfg))


def test_full_size_qwen128k_with_budget_and_alpha_sweep(P):
    cfg = CONFIGS["qwen128k"]
    sweeps = [(B, a) for B in (13107, 26214, 52429) for a in (0.25, 0.5, 0.75)]
    _full_size_check(P, cfg, make_layer(cfg), sweeps=sweeps)


def test_full_size_one_million_tokens_ragged(P):
    """A context far beyond the workloads' (1,000,003 entries per head: 64-bit offsets, 2 GiB buffer descriptors,
    thousands of key chunks and selection slices, a ragged last tile everywhere), checked like the other full
    sizes; the oracle covers every token of the first and the last kv head (a quarter of the layer: the whole
    of it is 34 TFLOP in float64 on the host).  Selection and allocation (one row of 8 million keys) on the GPU's
    own keys and the compaction are compared on all heads."""
    n = 1000003
    cfg = CONFIGS["llama128k"].with_(n_ctx=n, budget=budget_from_fraction(0.2, n))
    _full_size_check(P, cfg, make_layer(cfg), kv_heads=[0, cfg.n_kv_heads - 1])


@pytest.mark.parametrize("layer", [0, 15, 31])
def test_full_size_mistral_prefill_layer(P, layer):
    """One layer of the 32-layer batch-4 prefill workload (independent seeds per layer)."""
    cfg = CONFIGS["mistral_prefill"]
    _full_size_check(P, cfg, make_layer(cfg, layer=layer), layer_label=f" layer {layer}")


# ------------------------------------------------------------------------------------------------ runtime plumbing
def test_pass_replays_from_a_hip_graph(P):
    """score -> select -> compact captured once and replayed with new input values in the same buffers; eager
    work and synchronisations sit between the replays, and every replay must equal the eager result bit for bit
    (the pass enqueues kernels only: no memset nodes, no host synchronisation, no allocation)."""
    import torch
    cfg = reduced(CONFIGS["llama32k"], 4133, d_model=512)
    desc = cfg_desc(P, cfg, flags=P.CKV_WO_OUT_IN)
    b, H, Hkv, n, dh, B = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_ctx, cfg.head_dim, cfg.budget
    layers = [to_device(cfg, make_layer(cfg, layer=0, seed_offset=s), True) for s in range(3)]
    buf = {k: torch.empty_like(v) for k, v in layers[0].items()}

    def outputs():
        return dict(attn=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
                    crit=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
                    idx=torch.empty((b, Hkv, B), dtype=torch.int32, device="cuda"),
                    count=torch.empty((b, Hkv), dtype=torch.int32, device="cuda"),
                    k_out=torch.zeros((b, Hkv, B, dh), dtype=torch.bfloat16, device="cuda"),
                    v_out=torch.zeros((b, Hkv, B, dh), dtype=torch.bfloat16, device="cuda"),
                    ws=torch.empty(P.workspace_bytes(desc, B), dtype=torch.uint8, device="cuda"))
    budget = torch.full((b, Hkv), B, dtype=torch.int32, device="cuda")

    def one_pass(o, stream):
        P.criticalkv_score(desc, buf["q_win"], buf["k"], buf["v"], buf["w_o"], o["attn"], o["crit"], None, workspace=o["ws"],
                           stream=stream)
        P.criticalkv_select(desc, o["attn"], o["crit"], budget, cfg.alpha, B, o["idx"], o["count"], workspace=o["ws"],
                            stream=stream)
        P.criticalkv_compact(desc, buf["k"], buf["v"], o["idx"], o["count"], B, o["k_out"], o["v_out"], stream=stream)

    eager, replayed = outputs(), outputs()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for k in buf:
            buf[k].copy_(layers[0][k])
        one_pass(replayed, st)            # warm-up outside the capture
        st.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            one_pass(replayed, torch.cuda.current_stream())
        for r in (1, 2, 0, 1):
            for k in buf:
                buf[k].copy_(layers[r][k])
            one_pass(eager, st)           # the program's own eager work between replays
            st.synchronize()
            for t in ("idx", "k_out", "v_out", "attn", "crit"):
                replayed[t].fill_(0)      # a replay must rewrite everything it owns
            g.replay()
            torch.cuda.synchronize()
            for t in ("attn", "crit", "idx", "count", "k_out", "v_out"):
                assert torch.equal(eager[t], replayed[t]), (r, t)
    ref = O.full_pass(*(make_layer(cfg, layer=0, seed_offset=1)[k] for k in ("q_win", "k", "v", "w_o")), B, cfg.alpha,
                      pool_kernel=cfg.pool_kernel, eps=cfg.eps)
    compare_selection(replayed["idx"].cpu().numpy(), replayed["count"].cpu().numpy(), ref, B, cfg.alpha)


def test_default_path_is_bitwise_repeatable(P):
    """Three runs of the whole pass on the same inputs (fresh workspaces and outputs each time, other work in
    between) give identical scores, index sets and compacted rows: every cross-workgroup decision is made on
    integer counts, every floating-point sum has a fixed order."""
    for cfg, wo in ((reduced(CONFIGS["llama32k"], 20011, d_model=1024), True),
                    (reduced(CONFIGS["qwen128k"], 6007, d_model=512), True), (CONFIGS["tiny"], False)):
        t = make_layer(cfg)
        runs = []
        for r in range(3):
            runs.append(run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, wo_out_in=wo))
            if r == 0:  # unrelated work on the device between the runs
                other = reduced(CONFIGS["llama32k"], 1037, d_model=256)
                run_gpu_pass(P, other, make_layer(other), other.budget, other.alpha, wo_out_in=True)
        for r in runs[1:]:
            for name in ("attn", "crit", "vnorm", "idx", "count", "k_out", "v_out"):
                assert np.array_equal(getattr(runs[0], name), getattr(r, name)), (cfg.name, name)


def test_prepared_projection_layout_matches_the_per_call_one(P):
    """criticalkv_prepare_wo once, then criticalkv_score with CKV_WO_OUT_IN on the prepared copy: bit for bit the
    scores that criticalkv_score gives when it is handed the canonical projection and re-lays it out itself."""
    import torch
    for cfg in (reduced(CONFIGS["llama32k"], 2100, d_model=1024), CONFIGS["tiny"]):
        t = make_layer(cfg)
        canon = cfg_desc(P, cfg)
        dev = to_device(cfg, t, False)
        prepared = torch.empty(P.prepared_wo_bytes(canon), dtype=torch.uint8, device="cuda")
        P.criticalkv_prepare_wo(canon, dev["w_o"], prepared)
        torch.cuda.synchronize()
        assert torch.equal(prepared.view(dev["w_o"].dtype).view(cfg.d_model, -1), dev["w_o"].t().contiguous())
        per_call = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, wo_out_in=False)
        dev2 = dict(dev, w_o=prepared)
        once = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, flags=P.CKV_WO_OUT_IN, dev=dev2)
        for name in ("attn", "crit", "vnorm", "idx"):
            assert np.array_equal(getattr(per_call, name), getattr(once, name)), name


def test_measurement_probes_run(P):
    """The two measurement aids enqueue one kernel each and report plausible work (no timing asserted here)."""
    import torch
    ops = torch.randn(1 << 19, dtype=torch.float32, device="cuda").to(torch.bfloat16)
    sink = torch.zeros(16, dtype=torch.float32, device="cuda")
    flop = P.criticalkv_probe_mfma_bf16(ops, 10, sink)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert flop == 2 * cus * 4 * 10 * (4 * 4 * 7) * 2 * 16 * 16 * 32
    buf = torch.zeros(1 << 24, dtype=torch.uint8, device="cuda")
    isink = torch.zeros(16, dtype=torch.int32, device="cuda")
    P.criticalkv_probe_hbm_read(buf, buf.numel(), isink)
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0 and int(isink.abs().sum()) == 0
    with pytest.raises(P.CriticalKVError):
        P.criticalkv_probe_mfma_bf16(ops, 0, sink)


def test_single_hip_runtime_and_side_stream(P):
    """The library must run in PyTorch's HIP runtime (one libamdhip64 mapped) and honour a non-default stream."""
    import torch
    mapped = {line.split()[-1] for line in open("/proc/self/maps") if "libamdhip64" in line}
    assert len(mapped) == 1, mapped
    loaded = [line.split()[-1] for line in open("/proc/self/maps") if "libcriticalkv.so" in line]
    assert loaded, "the HIP extension is not loaded"
    cfg = reduced(CONFIGS["llama32k"], 2048, d_model=512)
    t = make_layer(cfg)
    ref = oracle_pass(cfg, t)
    side = torch.cuda.Stream()
    assert side.cuda_stream != 0
    with torch.cuda.stream(side):
        res = run_gpu_pass(P, cfg, t, cfg.budget, cfg.alpha, wo_out_in=True)
    assert_scores_close(res.crit, ref.crit, "crit(side stream)")
    compare_selection(res.idx, res.count, ref, cfg.budget, cfg.alpha)


def test_two_streams_with_their_own_workspaces_run_concurrently(P):
    """No state is shared between calls: two layers issued on two streams at once (each with its own workspace and
    outputs, several passes deep) give bit for bit what they give one after the other."""
    import torch
    cfg = reduced(CONFIGS["llama32k"], 6100, d_model=1024)
    desc = cfg_desc(P, cfg, flags=P.CKV_WO_OUT_IN)
    b, H, Hkv, n, dh, B = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_ctx, cfg.head_dim, cfg.budget
    layers = [to_device(cfg, make_layer(cfg, layer=0, seed_offset=s), True) for s in range(2)]
    budget = torch.full((b, Hkv), B, dtype=torch.int32, device="cuda")

    def outputs():
        return dict(attn=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
                    crit=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
                    idx=torch.empty((b, Hkv, B), dtype=torch.int32, device="cuda"),
                    count=torch.empty((b, Hkv), dtype=torch.int32, device="cuda"),
                    k_out=torch.zeros((b, Hkv, B, dh), dtype=torch.bfloat16, device="cuda"),
                    v_out=torch.zeros((b, Hkv, B, dh), dtype=torch.bfloat16, device="cuda"),
                    diag=torch.empty((b, H, 8), dtype=torch.float32, device="cuda"),
                    ws=torch.empty(P.workspace_bytes(desc, B), dtype=torch.uint8, device="cuda"))

    def one_pass(dev, o, stream):
        P.criticalkv_score(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], o["attn"], o["crit"], None, workspace=o["ws"],
                           stream=stream)
        P.criticalkv_select(desc, o["attn"], o["crit"], budget, cfg.alpha, B, o["idx"], o["count"], workspace=o["ws"],
                            stream=stream)
        P.criticalkv_compact(desc, dev["k"], dev["v"], o["idx"], o["count"], B, o["k_out"], o["v_out"], stream=stream)
        P.criticalkv_diagnostics(desc, dev["v"], dev["w_o"], None, o["idx"], o["count"], B, o["diag"], workspace=o["ws"],
                                 stream=stream)

    serial = [outputs(), outputs()]
    for dev, o in zip(layers, serial):
        one_pass(dev, o, torch.cuda.current_stream())
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    both = [outputs(), outputs()]
    for _ in range(4):                      # several passes in flight on each stream
        for dev, o, st in zip(layers, both, streams):
            one_pass(dev, o, st)
    torch.cuda.synchronize()
    for o_ser, o_con in zip(serial, both):
        for name in ("attn", "crit", "idx", "count", "k_out", "v_out", "diag"):
            assert torch.equal(o_ser[name], o_con[name]), name
    assert not torch.equal(serial[0]["idx"], serial[1]["idx"])


def test_profiled_score_records_every_stage_and_changes_nothing(P):
    """criticalkv_score_profiled: same outputs as criticalkv_score; every stage's pair of events is recorded in
    order on the launch stream (elapsed times non-negative, the projection the longest at this shape)."""
    import ctypes
    import torch
    cfg = reduced(CONFIGS["llama32k"], 8200, d_model=1024)
    t = make_layer(cfg)
    desc = cfg_desc(P, cfg)                       # canonical W_O: the layout stage does real work
    dev = to_device(cfg, t, False)
    b, H, Hkv, n = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_ctx
    ws = torch.empty(P.workspace_bytes(desc, cfg.budget), dtype=torch.uint8, device="cuda")
    out = [dict(attn=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda"),
                crit=torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda")) for _ in range(2)]
    P.criticalkv_score(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], out[0]["attn"], out[0]["crit"], None, workspace=ws)
    events = [torch.cuda.Event(enable_timing=True) for _ in range(2 * len(P.STAGES))]
    for e in events:
        e.record()                                # creates the underlying hipEvent_t
    torch.cuda.synchronize()
    arr = (ctypes.c_void_p * len(events))(*[e.cuda_event for e in events])
    P.criticalkv_score_profiled(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], out[1]["attn"], out[1]["crit"], None,
                                workspace=ws, stage_events=arr)
    torch.cuda.synchronize()
    assert torch.equal(out[0]["attn"], out[1]["attn"]) and torch.equal(out[0]["crit"], out[1]["crit"])
    ms = {name: events[2 * i].elapsed_time(events[2 * i + 1]) for i, name in enumerate(P.STAGES)}
    assert all(v >= 0.0 for v in ms.values()), ms
    assert ms["vproj"] == max(ms.values()) and ms["wo_layout"] > 0.0, ms
    # the stages follow each other on the stream in the order the library issues them: the projection before
    # the two key sweeps
    order = [P.STAGES.index(name) for name in ("wo_layout", "vproj", "attn_stats", "attn_colsum", "combine")]
    for a, b in zip(order, order[1:]):
        assert events[2 * a + 1].elapsed_time(events[2 * b]) >= 0.0, (P.STAGES[a], P.STAGES[b])
    # a NULL entry is skipped: only the projection marked
    arr2 = (ctypes.c_void_p * len(events))()
    v = P.STAGES.index("vproj")
    arr2[2 * v], arr2[2 * v + 1] = events[2 * v].cuda_event, events[2 * v + 1].cuda_event
    P.criticalkv_score_profiled(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], out[1]["attn"], out[1]["crit"], None,
                                workspace=ws, stage_events=arr2)
    torch.cuda.synchronize()
    assert events[2 * v].elapsed_time(events[2 * v + 1]) > 0.0
    print(f"[profiled score, n {n}] " + " ".join(f"{k}={v:.4f}ms" for k, v in ms.items()))


# (the seeds past 39 are draws with W = n under a kept window, or a zero budget, found on a wider one-off run;
# seeds from 1000 on draw long windows, 100 to 256 rows)
@pytest.mark.parametrize("seed", list(range(40)) + [54, 57, 71, 113, 146, 181] + list(range(1000, 1012)))
def test_random_valid_shapes_whole_pass(P, seed):
    """Seeded draws over the descriptor's valid range (group size, window, pool width, context with ragged tails,
    d_model, budget, alpha, W_O layout, norm, the prefill flags): whole pass against the oracle."""
    r = np.random.Generator(np.random.PCG64(9000 + seed))
    bf16 = bool(r.integers(0, 2))
    dh = 128 if bf16 and r.random() < 0.7 else 64
    Hkv = int(r.integers(1, 4))
    G = int(r.choice([1, 2, 3, 4, 5, 8]))
    n = int(r.choice([r.integers(1, 64), r.integers(64, 700), r.integers(700, 5000)]))
    W = int(min(n, r.choice([1, 2, 7, 16, 32, 33, 64, 96] if seed < 1000 else [100, 128, 129, 160, 200, 224, 255, 256])))
    dm = int(r.choice([32, 96, 128, 256, 384, 512, 640]))
    if bf16 and dh == 128 and r.random() < 0.5:
        dm = int(r.choice([128, 256, 512, 1024]))         # shapes the matrix-core projection covers
    pool = int(r.choice([1, 3, 5, 7, 13]))
    batch = int(r.integers(1, 3))
    budget = int(r.integers(0, n + 1))
    alpha = float(r.choice([0.0, 0.25, 0.5, 0.5, 0.75, 1.0]))
    norm = int(r.choice([1, 1, 2]))
    wo_out_in = bool(r.integers(0, 2))
    causal = bool(r.integers(0, 2))
    protect = causal and bool(r.integers(0, 2))
    base = CONFIGS["llama32k" if bf16 else "tiny"]
    cfg = base.with_(batch=batch, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=dh, d_model=dm, n_ctx=n, window=W,
                     pool_kernel=pool, budget=budget, alpha=alpha, n_sinks=min(base.n_sinks, n))
    t = make_layer(cfg, seed_offset=seed)
    flags = (P.CKV_CAUSAL_TAIL if causal else 0) | (P.CKV_PROTECT_WINDOW if protect else 0)
    ref = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], budget, alpha, pool_kernel=pool, eps=cfg.eps, norm=norm,
                      causal_tail=causal, protect_window=protect)
    res = run_gpu_pass(P, cfg, t, budget, alpha, flags=flags, wo_out_in=wo_out_in, norm=norm)
    label = (f"seed {seed}: {'bf16' if bf16 else 'f32'} dh{dh} H{G * Hkv}/{Hkv} n{n} W{W} dm{dm} pool{pool} b{batch} "
             f"B{budget} a{alpha} norm{norm} {'out_in ' if wo_out_in else ''}{'causal ' if causal else ''}{'protect' if protect else ''}")
    e_v = assert_scores_close(res.vnorm, ref.vnorm, "vnorm " + label)
    e_a = assert_scores_close(res.attn, ref.attn, "attn " + label)
    e_c = assert_scores_close(res.crit, ref.crit, "crit " + label)
    swaps = compare_selection(res.idx, res.count, ref, budget, alpha)
    assert_compaction_exact(res, t, budget)
    print(f"[{label}] err vnorm {e_v[0]:.1e} attn {e_a[0]:.1e} crit {e_c[0]:.1e} swaps {swaps}")
    # the calls beside the pass on the same draw: allocation on the GPU's own scores (exact), diagnostics
    total = int(r.integers(0, Hkv * n + 1))
    ff = np.float32(r.choice([0.0, 0.3, 1.0]))
    assert np.array_equal(run_allocate(P, res.attn, total, ff), O.allocate(res.attn.astype(np.float64), total, ff))
    if not causal and swaps == 0:
        got, idx, _ = run_diagnostics(P, cfg, t, budget, alpha, wo_out_in=wo_out_in, norm=norm)
        ref_d, ref_idx = oracle_diagnostics(cfg, t, budget, alpha, norm=norm)
        assert np.array_equal(idx, ref_idx)
        assert_diagnostics_close(got, ref_d, label)
