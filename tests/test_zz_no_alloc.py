"""criticalkv_select_noalloc (static device scratch, no workspace argument) against criticalkv_select.

Collected last on purpose (file name): a failure here must not hide the parity tests.  Runs alone in a fresh
process as well as after the other tests: it needs nothing they leave behind."""
import numpy as np
import pytest

from workload import CONFIGS, make_layer, reduced

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2502_03805_amd as pkg
    pkg.load()
    return pkg


def _both(P, desc, attn, crit, budget, alpha, max_budget):
    import torch
    b, Hkv, n = attn.shape
    ws = torch.empty(P.workspace_bytes(desc, max_budget), dtype=torch.uint8, device="cuda")
    out = []
    for name in ("workspace", "static"):
        idx = torch.full((b, Hkv, max_budget), -7, dtype=torch.int32, device="cuda")
        count = torch.full((b, Hkv), -7, dtype=torch.int32, device="cuda")
        if name == "workspace":
            P.criticalkv_select(desc, attn, crit, budget, alpha, max_budget, idx, count, workspace=ws)
        else:
            P.criticalkv_select_noalloc(desc, attn, crit, budget, alpha, max_budget, idx, count)
        torch.cuda.synchronize()
        out.append((idx.cpu().numpy(), count.cpu().numpy()))
    return out


def test_select_noalloc_matches_select_on_two_calls_in_a_row(P):
    """Two calls in a row on the same GPU, the second with a smaller input (the static buffer still holds the
    first call's histograms, counts and keys): index sets and counts identical to criticalkv_select's, which
    the parity tests compare with the oracle.  Scores come from the real scoring kernels (pooled scores carry
    exact ties)."""
    import torch
    from paper_2502_03805_amd.marshal import cfg_desc, to_device
    for n, flags in ((20011, 0), (4133, 0), (4133, P.CKV_PROTECT_WINDOW), (300, 0)):
        cfg = reduced(CONFIGS["llama32k"], n, d_model=256)
        t = make_layer(cfg)
        desc = cfg_desc(cfg, flags=P.CKV_WO_OUT_IN | flags)
        dev = to_device(cfg, t, True)
        b, Hkv = cfg.batch, cfg.n_kv_heads
        ws = torch.empty(P.workspace_bytes(desc, n), dtype=torch.uint8, device="cuda")
        attn = torch.empty((b, Hkv, n), dtype=torch.float32, device="cuda")
        crit = torch.empty_like(attn)
        P.criticalkv_score(desc, dev["q_win"], dev["k"], dev["v"], dev["w_o"], attn, crit, None, workspace=ws)
        r = np.random.Generator(np.random.PCG64(n))
        for alpha in (0.5, 0.0, 1.0):
            budget = torch.from_numpy(r.integers(0, n + 1, (b, Hkv)).astype(np.int32)).cuda()
            (i0, c0), (i1, c1) = _both(P, desc, attn, crit, budget, alpha, n)
            assert np.array_equal(c0, c1) and np.array_equal(i0, i1), (n, alpha)
            assert np.array_equal(c1, budget.cpu().numpy())


def test_select_noalloc_full_size_and_limit(P):
    """The largest layer shapes of the workloads fit the static buffer; a larger one is refused with its own
    error code before anything is launched."""
    import torch
    r = np.random.Generator(np.random.PCG64(11))
    for b, Hkv, n in ((1, 8, 131072), (4, 8, 32768)):
        desc = P.make_desc(batch=b, n_q_heads=Hkv, n_kv_heads=Hkv, head_dim=128, d_model=128, n_ctx=n, window=1,
                           pool_kernel=1, dtype=P.CKV_BF16)
        attn = torch.from_numpy(r.random((b, Hkv, n), dtype=np.float32)).cuda()
        crit = torch.from_numpy(r.lognormal(0, 2, (b, Hkv, n)).astype(np.float32)).cuda()
        B = n * 2 // 5
        budget = torch.full((b, Hkv), B, dtype=torch.int32, device="cuda")
        (i0, c0), (i1, c1) = _both(P, desc, attn, crit, budget, 0.5, B)
        assert np.array_equal(c0, c1) and np.array_equal(i0, i1)
    big = P.make_desc(batch=1, n_q_heads=8, n_kv_heads=8, head_dim=128, d_model=128, n_ctx=1 << 19, window=1,
                      pool_kernel=1, dtype=P.CKV_BF16)
    x = torch.zeros(16, dtype=torch.float32, device="cuda")
    with pytest.raises(P.CriticalKVError) as e:
        P.criticalkv_select_noalloc(big, x, x, x, 0.5, 10, x, x)
    assert e.value.code == P.CKV_E_STATIC_LIMIT
