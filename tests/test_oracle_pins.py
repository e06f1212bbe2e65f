"""Pins of the float64 CPU oracle against things the paper and the mathematics fix.

None of these tests touches the GPU path.  Each pins one oracle routine to something
other than itself: a library routine on a special case, a closed form, an invariant,
brute-force enumeration of the paper's bounds (Theorems 3.2, 3.3, 3.5, 3.6), or a
hand-worked fixture.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import cpu_oracle as O
from oracle.numpy_transcription import pass_numpy
from workload import CONFIGS, make_layer

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


# ----------------------------------------------------------------------------- window attention
def test_window_attention_single_row_is_textbook_softmax():
    r = rng(1)
    H, Hkv, n, dh = 3, 3, 37, 16
    q = r.standard_normal((1, H, 1, dh)).astype(np.float32)
    k = r.standard_normal((1, Hkv, n, dh)).astype(np.float32)
    a = O.window_attention(q, k)
    for h in range(H):
        logits = (q[0, h, 0].astype(np.float64) @ k[0, h].astype(np.float64).T) / np.sqrt(dh)
        np.testing.assert_allclose(a[0, h], scipy.special.softmax(logits), rtol=1e-13, atol=0)


def test_window_attention_is_mean_of_row_softmaxes_and_sums_to_one():
    r = rng(2)
    H, Hkv, n, dh, W = 4, 2, 53, 8, 5
    q = r.standard_normal((2, H, W, dh)).astype(np.float32)
    k = r.standard_normal((2, Hkv, n, dh)).astype(np.float32)
    a_mean = O.window_attention(q, k)
    a_sum = O.window_attention(q, k, window_sum=True)
    np.testing.assert_allclose(a_mean.sum(-1), 1.0, rtol=1e-13)
    np.testing.assert_allclose(a_sum, a_mean * W, rtol=1e-13)
    # grouped-query mapping: query head h reads kv head h // G
    G = H // Hkv
    for bi in range(2):
        for h in range(H):
            logits = q[bi, h].astype(np.float64) @ k[bi, h // G].astype(np.float64).T / np.sqrt(dh)
            ref = scipy.special.softmax(logits, axis=1).mean(axis=0)
            np.testing.assert_allclose(a_mean[bi, h], ref, rtol=1e-12)


def test_window_attention_scale_and_shift_invariance():
    r = rng(3)
    n, dh, W = 41, 8, 3
    q = r.standard_normal((1, 1, W, dh)).astype(np.float32)
    k = r.standard_normal((1, 1, n, dh)).astype(np.float32)
    # explicit scale is honoured: scale s on q equals softmax_scale s
    a1 = O.window_attention(q * np.float32(0.5), k, scale=1.0)
    a2 = O.window_attention(q, k, scale=0.5)
    np.testing.assert_allclose(a1, a2, rtol=1e-12)
    # adding the same vector u to every key shifts each row's logits by a constant: A unchanged
    u = r.standard_normal(dh).astype(np.float32)
    k64 = k.astype(np.float64) + u.astype(np.float64)
    k_shift = k64.astype(np.float32)
    if np.array_equal(k_shift.astype(np.float64), k64):  # only exact if representable; otherwise use loose tol
        tol = 1e-12
    else:
        tol = 1e-5
    a3 = O.window_attention(q, k_shift, scale=0.5)
    np.testing.assert_allclose(a3, a2, rtol=tol)


def test_causal_tail_matches_explicitly_masked_softmax():
    r = rng(5)
    H, Hkv, n, dh, W = 4, 2, 29, 8, 6
    q = r.standard_normal((1, H, W, dh)).astype(np.float32)
    k = r.standard_normal((1, Hkv, n, dh)).astype(np.float32)
    a = O.window_attention(q, k, causal_tail=True)
    for h in range(H):
        logits = q[0, h].astype(np.float64) @ k[0, h // 2].astype(np.float64).T / np.sqrt(dh)   # [W, n]
        pos = n - W + np.arange(W)[:, None]
        masked = np.where(np.arange(n)[None, :] <= pos, logits, -np.inf)
        ref = scipy.special.softmax(masked, axis=1).mean(axis=0)
        np.testing.assert_allclose(a[0, h], ref, rtol=1e-12, atol=1e-300)
    # the last key is visible to the last window row only: its weight is at most 1/W
    assert np.all(a[0, :, -1] <= 1.0 / W + 1e-15) and np.all(a[0, :, -1] > 0)
    # without the flag nothing is masked; W = n, W = 1 corner cases run
    full = O.window_attention(q, k)
    assert not np.allclose(full, a)
    one = O.window_attention(q[:, :, :1], k, causal_tail=True)
    np.testing.assert_allclose(one, O.window_attention(q[:, :, :1], k), rtol=1e-13)


def _best_subset(candidates, size, key):
    """Brute force: the subset of `candidates` of the given size with the largest key sum (keys distinct, so it is
    unique); enumerates every subset."""
    best, best_sum = None, -np.inf
    for sub in itertools.combinations(candidates, size):
        tot = float(sum(key[i] for i in sub))
        if tot > best_sum:
            best, best_sum = sub, tot
    return set(best)


@pytest.mark.parametrize("seed", range(4))
def test_protected_window_by_brute_force_enumeration(seed):
    """Kept window: S = (last min(W, B) entries) u (Algorithm 1 on the entries before the window with what is left
    of the budget).  Checked without any sort or sentinel: each stage's Top-k is found by enumerating every subset
    of the competing entries and taking the one with the largest key sum."""
    r = rng(100 + seed)
    n = int(r.integers(6, 13))
    attn = r.permutation(n).astype(np.float64) / 64.0 + 0.01          # distinct keys
    crit = attn * r.permutation(n).astype(np.float64) + r.permutation(n) / 1024.0
    assert len(set(crit.tolist())) == n
    for W in (1, 2, 3, n // 2, n):
        for B in range(0, n + 1):
            for alpha in (0.0, 0.3, 0.5, 1.0):
                idx, flag, tau = O.select_head(attn, crit, B, alpha, protect_last=W)
                kept_window = set(range(n - min(W, B), n))
                prefix = list(range(n - W))
                left = B - len(kept_window)
                b1 = int(np.floor(alpha * left))
                s1 = _best_subset(prefix, b1, attn)
                s2 = _best_subset([i for i in prefix if i not in s1], left - b1, crit)
                assert set(idx.tolist()) == kept_window | s1 | s2, (n, W, B, alpha)
                assert np.all(np.diff(idx) > 0) and len(idx) == B
                # the flag marks what was fixed before stage 2: stage 1 and the kept window
                assert set(idx[flag].tolist()) == kept_window | s1
                if b1 > 0:
                    assert tau[0] == min(attn[i] for i in s1)
                if left - b1 > 0:
                    assert tau[1] == min(crit[i] for i in s2)


def test_protected_window_hand_worked_fixture_and_properties():
    # the hand-worked head of tests/golden/two_stage_hand_example.txt with its last two entries as the window
    A = N = None
    cases = []
    with open(os.path.join(GOLDEN, "two_stage_hand_example.txt")) as f:
        for line in f:
            t = line.split()
            if t[:1] == ["A"]:
                A = np.array([float(x) for x in t[1:]])
            elif t[:1] == ["N"]:
                N = np.array([float(x) for x in t[1:]])
            elif t[:1] == ["window_case"]:
                kv = dict(x.split("=") for x in t[1:4])
                cases.append((int(kv["W"]), int(kv["b"]), float(kv["alpha"]), [int(x) for x in t[5:]]))
    assert len(cases) >= 5
    for W, B, alpha, expect in cases:
        idx, _, _ = O.select_head(A, A * N, B, alpha, protect_last=W)
        assert idx.tolist() == expect, (W, B, alpha)
    # properties on a grouped layer: the scores themselves are not touched, W = 0 is the plain algorithm,
    # the window is a subset of every selection whose budget covers it
    r = rng(6)
    b, H, Hkv, n, W = 1, 4, 2, 40, 5
    abar, Nn = r.random((b, H, n)), r.random((b, H, n))
    attn, crit = O.group_keys(abar, Nn, Hkv, 1e-4)
    for B in (W, W + 3, 20):
        for alpha in (0.0, 0.5, 1.0):
            idx, count, _ = O.select(attn, crit, B, alpha, protect_last=W)
            plain, _, _ = O.select(attn[..., :n - W], crit[..., :n - W], B - W, alpha, max_budget=B)
            for g in range(Hkv):
                assert idx[0, g].tolist() == plain[0, g, :B - W].tolist() + list(range(n - W, n))
    idx0, _, _ = O.select(attn, crit, 7, 0.5, protect_last=0)
    idx1, _, _ = O.select(attn, crit, 7, 0.5)
    assert np.array_equal(idx0, idx1)
    # a budget below the window keeps the most recent tokens
    idx, _, _ = O.select(attn, crit, 3, 0.5, protect_last=W)
    assert idx[0, 0].tolist() == [n - 3, n - 2, n - 1]


def test_theorem_3_2_masked_softmax_identity():
    """A' = (N . A) / sum(N A) equals the softmax with -inf on the evicted logits (Theorem 3.2)."""
    r = rng(4)
    n, dh = 12, 8
    q = r.standard_normal((1, 1, 1, dh)).astype(np.float32)
    k = r.standard_normal((1, 1, n, dh)).astype(np.float32)
    A = O.window_attention(q, k)[0, 0]
    logits = q[0, 0, 0].astype(np.float64) @ k[0, 0].astype(np.float64).T / np.sqrt(dh)
    for b in (1, 5, 11):
        for keep in itertools.islice(itertools.combinations(range(n), b), 40):
            mask = np.zeros(n)
            mask[list(keep)] = 1
            masked_logits = np.where(mask > 0, logits, -np.inf)
            A_direct = scipy.special.softmax(masked_logits)
            A_thm = mask * A / (mask * A).sum()
            np.testing.assert_allclose(A_thm, A_direct, rtol=1e-12, atol=1e-300)


# ----------------------------------------------------------------------------- pooling
@pytest.mark.parametrize("kernel", [1, 3, 5, 7, 9])
@pytest.mark.parametrize("n", [1, 2, 6, 64, 101])
def test_maxpool_matches_library_routine(kernel, n):
    x = rng(10 + n).standard_normal((3, n))
    got = O.maxpool1d(x, kernel)
    ref = torch.nn.functional.max_pool1d(torch.from_numpy(x)[None], kernel, stride=1, padding=kernel // 2)[0].numpy()
    np.testing.assert_array_equal(got, ref)
    if kernel == 1:
        np.testing.assert_array_equal(got, x)


# ----------------------------------------------------------------------------- projected value norm
def test_projected_norm_matches_dgemm_and_head_slices():
    r = rng(20)
    b, H, Hkv, n, dh, dm = 2, 6, 2, 19, 8, 24
    v = r.standard_normal((b, Hkv, n, dh)).astype(np.float32)
    w = r.standard_normal((H * dh, dm)).astype(np.float32)
    N1 = O.projected_value_norm(v, w, H, norm=1)
    N2 = O.projected_value_norm(v, w, H, norm=2)
    G = H // Hkv
    for bi in range(b):
        for h in range(H):
            P = v[bi, h // G].astype(np.float64) @ w[h * dh:(h + 1) * dh].astype(np.float64)
            np.testing.assert_allclose(N1[bi, h], np.abs(P).sum(1), rtol=1e-13)
            np.testing.assert_allclose(N2[bi, h], np.sqrt((P * P).sum(1)), rtol=1e-13)


def test_projected_norm_closed_forms():
    r = rng(21)
    n, dh, dm = 33, 8, 20
    v = r.standard_normal((1, 1, n, dh)).astype(np.float32)
    w = np.zeros((dh, dm), dtype=np.float32)
    w[np.arange(dh), np.arange(dh)] = 1.0                      # W_O = [I | 0]
    N = O.projected_value_norm(v, w, 1)
    np.testing.assert_allclose(N[0, 0], np.abs(v[0, 0].astype(np.float64)).sum(1), rtol=1e-14)
    # a single column equal to a vector u: N_i = |v_i . u|  (sign cancellation inside a column matters)
    u = r.standard_normal(dh).astype(np.float32)
    w1 = np.zeros((dh, dm), dtype=np.float32)
    w1[:, 3] = u
    N = O.projected_value_norm(v, w1, 1)
    np.testing.assert_allclose(N[0, 0], np.abs(v[0, 0].astype(np.float64) @ u.astype(np.float64)), rtol=1e-12, atol=1e-15)
    # homogeneity: scaling W_O by 4 (exact in binary) scales N by 4
    w2 = r.standard_normal((dh, dm)).astype(np.float32)
    np.testing.assert_allclose(O.projected_value_norm(v, 4 * w2, 1), 4 * O.projected_value_norm(v, w2, 1), rtol=1e-15)


# ----------------------------------------------------------------------------- keys
def test_group_keys_single_head_is_paper_formula_and_group_mean():
    r = rng(30)
    b, H, Hkv, n = 2, 6, 3, 17
    abar = r.random((b, H, n))
    N = r.random((b, H, n)) * 10
    eps = 1e-4
    attn, crit = O.group_keys(abar, N, H, eps)                 # G = 1
    np.testing.assert_array_equal(attn, abar)
    np.testing.assert_allclose(crit, (abar + eps) * N, rtol=1e-15)
    attn, crit = O.group_keys(abar, N, Hkv, eps)               # G = 2
    np.testing.assert_allclose(attn, abar.reshape(b, Hkv, 2, n).mean(2), rtol=1e-15)
    np.testing.assert_allclose(crit, ((abar + eps) * N).reshape(b, Hkv, 2, n).mean(2), rtol=1e-15)


# ----------------------------------------------------------------------------- two-stage selection
def _check_invariants(idx, flag, n, B, alpha):
    b1 = int(np.floor(alpha * B))
    assert idx.shape == (B,)
    assert np.all(np.diff(idx) > 0), "indices strictly ascending (hence distinct)"
    assert B == 0 or (idx[0] >= 0 and idx[-1] < n)
    assert int(flag.sum()) == b1


def test_hand_worked_fixture():
    A = N = None
    cases = []
    with open(os.path.join(GOLDEN, "two_stage_hand_example.txt")) as f:
        for line in f:
            t = line.split()
            if not t or t[0].startswith("#"):
                continue
            if t[0] == "A":
                A = np.array([float(x) for x in t[1:]])
            elif t[0] == "N":
                N = np.array([float(x) for x in t[1:]])
            elif t[0] == "case":
                cases.append((int(t[1].split("=")[1]), float(t[2].split("=")[1]), [int(x) for x in t[4:]]))
    assert A.sum() == 1.0 and len(cases) >= 6
    _, crit = O.group_keys(A[None, None], N[None, None], 1, 0.0)
    for B, alpha, expect in cases:
        idx, flag, _ = O.select_head(A, crit[0, 0], B, alpha)
        assert idx.tolist() == expect, (B, alpha)
        _check_invariants(idx, flag, len(A), B, alpha)


def theta_closed(A, Vn, mask):
    """Theorem 3.3: C - (2 - 1/sum(N A)) sum(N A ||V_i||_1)."""
    s = (mask * A).sum()
    C = (A * Vn).sum()
    return C - (2.0 - 1.0 / s) * (mask * A * Vn).sum()


def theta_hat(A, Vn, m1, m2):
    """Theorem 3.5."""
    sigma = (m1 * A).sum()
    C = (A * Vn).sum()
    Cp = C - (2 - 1 / sigma) * (m1 * A * Vn).sum()
    return Cp - (2 - 1 / sigma) * (m2 * A * Vn).sum()


def theta_relax(A, Vn, m1, m2):
    """Theorem 3.6."""
    sigma = (m1 * A).sum()
    C = (A * Vn).sum()
    Cp = C - (2 - 1 / sigma) * (m1 * A * Vn).sum()
    return Cp - Vn.min() * (2 - 1 / sigma) * (m2 * A).sum()


def _tiny_head(seed, n=10, dh=4, dm=6, peaked=True):
    r = rng(seed)
    q = r.standard_normal((1, 1, 1, dh)).astype(np.float32) * (3.0 if peaked else 1.0)
    k = r.standard_normal((1, 1, n, dh)).astype(np.float32)
    v = (r.standard_normal((1, 1, n, dh)) * r.lognormal(0, 1.0, size=(1, 1, n, 1))).astype(np.float32)
    w = r.standard_normal((dh, dm)).astype(np.float32)
    return q, k, v, w


@pytest.mark.parametrize("seed", range(6))
def test_theorem_3_3_bound_by_brute_force(seed):
    """For every mask of size b: L = ||(A - A') V W_O||_1 <= theta, and the closed form equals
    sum_i |A_i - A'_i| ||V_i||_1 with A' from the actual masked softmax."""
    n, b = 9, 4
    q, k, v, w = _tiny_head(seed, n=n)
    A = O.window_attention(q, k)[0, 0]
    Vn = O.projected_value_norm(v, w, 1)[0, 0]
    P = v[0, 0].astype(np.float64) @ w.astype(np.float64)
    logits = q[0, 0, 0].astype(np.float64) @ k[0, 0].astype(np.float64).T / np.sqrt(q.shape[-1])
    o_full = scipy.special.softmax(logits) @ P
    for keep in itertools.combinations(range(n), b):
        mask = np.zeros(n)
        mask[list(keep)] = 1
        A_masked = scipy.special.softmax(np.where(mask > 0, logits, -np.inf))
        L = np.abs(o_full - A_masked @ P).sum()
        th_direct = (np.abs(A - A_masked) * Vn).sum()
        th_closed = theta_closed(A, Vn, mask)
        assert L <= th_direct * (1 + 1e-12) + 1e-15
        np.testing.assert_allclose(th_closed, th_direct, rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("B,alpha", [(4, 0.5), (6, 0.5), (5, 0.25), (6, 0.75)])
def test_theorem_3_5_stage_two_minimises_theta_hat(seed, B, alpha):
    """Given the oracle's stage-1 set, its stage-2 set attains the minimum of theta_hat over all
    completions (eps = 0); and theta <= theta_hat whenever sigma > 0.5."""
    n = 10
    q, k, v, w = _tiny_head(100 + seed, n=n)
    A = O.window_attention(q, k)[0, 0]
    Vn = O.projected_value_norm(v, w, 1)[0, 0]
    _, crit = O.group_keys(A[None, None], Vn[None, None], 1, 0.0)
    idx, flag, _ = O.select_head(A, crit[0, 0], B, alpha)
    _check_invariants(idx, flag, n, B, alpha)
    b1 = int(np.floor(alpha * B))
    b2 = B - b1
    s1 = idx[flag]
    s2 = idx[~flag]
    # stage 1 is the attention Top-b'
    assert set(s1.tolist()) == set(np.argsort(-A, kind="stable")[:b1].tolist())
    m1 = np.zeros(n)
    m1[s1] = 1
    m2 = np.zeros(n)
    m2[s2] = 1
    sigma = (m1 * A).sum()
    if b1 == 0 or sigma <= 0.5:
        pytest.skip("Assumption 3.4 does not hold for this draw")
    mine = theta_hat(A, Vn, m1, m2)
    rest = [i for i in range(n) if m1[i] == 0]
    best = np.inf
    for comp in itertools.combinations(rest, b2):
        mm = np.zeros(n)
        mm[list(comp)] = 1
        th = theta_hat(A, Vn, m1, mm)
        best = min(best, th)
        assert theta_closed(A, Vn, m1 + mm) <= th + 1e-12       # theta <= theta_hat for every completion
    assert mine <= best + 1e-12


@pytest.mark.parametrize("seed", range(6))
def test_theorem_3_6_attention_only_minimises_relaxed_bound(seed):
    """alpha = 1 in stage 2's place: attention-only Top-k attains min theta_hat_relax; and the oracle with
    alpha = 1 returns exactly the attention Top-B (Algorithm 2, regular selection)."""
    n, B = 10, 6
    q, k, v, w = _tiny_head(200 + seed, n=n)
    A = O.window_attention(q, k)[0, 0]
    Vn = O.projected_value_norm(v, w, 1)[0, 0]
    _, crit = O.group_keys(A[None, None], Vn[None, None], 1, 1e-4)
    idx, flag, _ = O.select_head(A, crit[0, 0], B, 1.0)
    top = np.sort(np.argsort(-A, kind="stable")[:B])
    assert idx.tolist() == top.tolist() and flag.all()
    b1 = 3
    order = np.argsort(-A, kind="stable")
    m1 = np.zeros(n)
    m1[order[:b1]] = 1
    if (m1 * A).sum() <= 0.5:
        pytest.skip("Assumption 3.4 does not hold for this draw")
    m2 = np.zeros(n)
    m2[order[b1:B]] = 1
    mine = theta_relax(A, Vn, m1, m2)
    rest = [i for i in range(n) if m1[i] == 0]
    for comp in itertools.combinations(rest, B - b1):
        mm = np.zeros(n)
        mm[list(comp)] = 1
        assert mine <= theta_relax(A, Vn, m1, mm) + 1e-12
        assert theta_hat(A, Vn, m1, mm) <= theta_relax(A, Vn, m1, mm) + 1e-12


def test_selection_special_cases_and_ties():
    r = rng(40)
    n = 50
    A = r.random(n)
    A /= A.sum()
    Vn = r.lognormal(0, 1, n)
    _, crit = O.group_keys(A[None, None], Vn[None, None], 1, 1e-4)
    crit = crit[0, 0]
    # alpha = 0: pure Top-B of the criticality
    idx, flag, _ = O.select_head(A, crit, 12, 0.0)
    assert idx.tolist() == sorted(np.argsort(-crit, kind="stable")[:12].tolist()) and not flag.any()
    # B = n: identity; B = 0: empty
    idx, flag, _ = O.select_head(A, crit, n, 0.5)
    assert idx.tolist() == list(range(n))
    idx, flag, tau = O.select_head(A, crit, 0, 0.5)
    assert idx.size == 0 and np.isnan(tau).all()
    # uniform projected norm: result is attention-only Top-B for every alpha
    _, crit_u = O.group_keys(A[None, None], np.full((1, 1, n), 3.5), 1, 1e-4)
    top = sorted(np.argsort(-A, kind="stable")[:11].tolist())
    for alpha in (0.0, 0.25, 0.5, 0.9, 1.0):
        idx, flag, _ = O.select_head(A, crit_u[0, 0], 11, alpha)
        assert idx.tolist() == top
        _check_invariants(idx, flag, n, 11, alpha)
    # ties: the lower index wins in both stages
    A_t = np.array([0.1, 0.2, 0.2, 0.2, 0.1, 0.1, 0.1])
    c_t = np.array([5.0, 1.0, 1.0, 1.0, 7.0, 7.0, 7.0])
    idx, flag, tau = O.select_head(A_t, c_t, 4, 0.5)           # stage 1: {1,2}; stage 2 over rest: 7,7 -> {4,5}
    assert idx.tolist() == [1, 2, 4, 5] and flag.tolist() == [True, True, False, False]
    assert tau.tolist() == [0.2, 7.0]
    # stage 2 never re-takes a stage-1 entry even if it has the largest criticality
    A2 = np.array([0.7, 0.1, 0.1, 0.1])
    c2 = np.array([100.0, 1.0, 3.0, 2.0])
    idx, flag, _ = O.select_head(A2, c2, 2, 0.5)
    assert idx.tolist() == [0, 2]
    # rounding of b' = floor(alpha * B)
    for B, alpha, b1 in [(7, 0.5, 3), (5, 0.25, 1), (3, 0.75, 2), (1, 0.5, 0), (6554, 0.5, 3277)]:
        nn = max(B, 10)
        a = rng(B).random(nn)
        idx, flag, _ = O.select_head(a, a, B, alpha)
        assert int(flag.sum()) == b1 and idx.size == B


def test_select_batch_layout_and_compaction_bytes():
    r = rng(50)
    b, Hkv, n, dh = 2, 3, 40, 8
    attn = r.random((b, Hkv, n))
    crit = r.random((b, Hkv, n))
    budget = np.array([[5, 0, 40], [7, 12, 1]], dtype=np.int32)
    idx, count, tau = O.select(attn, crit, budget, 0.5, max_budget=40)
    assert np.array_equal(count, budget)
    src = r.standard_normal((b, Hkv, n, dh)).astype(np.float32)
    out = O.compact(src, idx, count)
    for bi in range(b):
        for g in range(Hkv):
            B = budget[bi, g]
            one, flag, _ = O.select_head(attn[bi, g], crit[bi, g], int(B), 0.5)
            assert idx[bi, g, :B].tolist() == one.tolist()
            assert np.all(idx[bi, g, B:] == -1)
            assert out[bi, g, :B].tobytes() == src[bi, g, one].tobytes()
            assert not out[bi, g, B:].any()


def test_budget_allocation_against_brute_force_and_closed_cases():
    r = rng(60)
    b, Hkv, n = 2, 4, 30
    attn = r.random((b, Hkv, n)) * np.array([1.0, 2.0, 0.5, 1.5])[None, :, None]
    for total, ff in [(40, 0.0), (40, 0.25), (41, 0.5), (120, 0.0), (0, 0.3), (17, 1.0)]:
        got = O.allocate(attn, total, ff)
        f = int(np.floor(ff * total / Hkv))
        P = total - Hkv * f
        for bi in range(b):
            flat = attn[bi].reshape(-1)
            order = np.lexsort((np.arange(flat.size), -flat))[:P]
            ref = np.minimum(n, f + np.bincount(order // n, minlength=Hkv))
            assert got[bi].tolist() == ref.tolist()
            if ref.max() < n:
                assert got[bi].sum() == total
    # uniform split when the floor takes everything; all to the dominant head when its scores dominate
    assert O.allocate(attn, 40, 1.0).tolist() == [[10] * 4] * 2
    dom = attn.copy()
    dom[:, 2] += 10.0
    assert O.allocate(dom, 20, 0.0)[0].tolist() == [0, 0, 20, 0]
    assert O.allocate(dom, 50, 0.0)[0, 2] == n            # capped at n, the rest spills to the other heads
    # identical heads: ties go to the lower head first
    same = np.tile(r.random((1, 1, n)), (1, Hkv, 1))
    assert O.allocate(same, 6, 0.0)[0].tolist() == [2, 2, 1, 1]
    with pytest.raises(RuntimeError):
        O.allocate(attn, Hkv * n + 1, 0.0)


# ------------------------------------------------------------------------------------------------ diagnostics
def _diag(A, v, w, keep1, keep2, norm=1):
    """One head through the oracle's diagnostics: A [n], v [n,dh], w [dh,dm], index lists of the two stages."""
    n = len(A)
    sel = sorted(list(keep1) + list(keep2))
    mb = max(1, len(sel))
    idx = np.full((1, 1, mb), -1, dtype=np.int32)
    idx[0, 0, :len(sel)] = sel
    st1 = np.zeros((1, 1, mb), dtype=np.uint8)
    st1[0, 0, :len(sel)] = [i in set(keep1) for i in sel]
    out = O.diagnostics(np.asarray(A, dtype=np.float64)[None, None], np.asarray(v, dtype=np.float32)[None, None],
                        np.asarray(w, dtype=np.float32), idx, np.array([[len(sel)]], dtype=np.int32), st1, norm)
    return dict(zip(O.DIAG_FIELDS, out[0, 0]))


def test_diagnostics_hand_worked_fixture():
    rows = {}
    for line in open(os.path.join(GOLDEN, "perturbation_hand_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        rows[key] = [float(x) for x in vals]
    A, N = np.array(rows["A"]), np.array(rows["N"])
    k1, k2 = [int(x) for x in rows["stage1"]], [int(x) for x in rows["stage2"]]
    layouts = {"orthogonal": (np.diag(N), np.eye(3)), "parallel": (N[:, None], np.ones((1, 1)))}
    for name, (v, w) in layouts.items():
        for norm in (1, 2):
            d = _diag(A, v, w, k1, k2, norm)
            for f in ("sigma", "s", "C", "M", "theta", "theta_hat", "theta_relax"):
                np.testing.assert_allclose(d[f], rows[f][0], rtol=1e-12, err_msg=f"{name} {f}")
            np.testing.assert_allclose(d["L"], rows[f"L{norm}_{name}"][0], rtol=1e-7, err_msg=f"{name} L{norm}")


@pytest.mark.parametrize("seed", range(5))
def test_diagnostics_L_is_the_masked_softmax_perturbation(seed):
    """One window query: L equals ||o - o_hat||_1 with o_hat from the softmax over the kept logits only
    (the additive -inf mask of section 3.1), for every subset; theta equals sum_i |A_i - A'_i| N_i, the
    quantity the proof of Theorem 3.3 bounds L with."""
    n, b = 8, 3
    q, k, v, w = _tiny_head(300 + seed, n=n)
    A = O.window_attention(q, k)[0, 0]
    Vn = O.projected_value_norm(v, w, 1)[0, 0]
    P = v[0, 0].astype(np.float64) @ w.astype(np.float64)
    logits = q[0, 0, 0].astype(np.float64) @ k[0, 0].astype(np.float64).T / np.sqrt(q.shape[-1])
    o_full = scipy.special.softmax(logits) @ P
    for keep in itertools.combinations(range(n), b):
        masked = scipy.special.softmax(np.where(np.isin(np.arange(n), keep), logits, -np.inf))
        d = _diag(A, v[0, 0], w, keep[:1], keep[1:])
        np.testing.assert_allclose(d["L"], np.abs(o_full - masked @ P).sum(), rtol=1e-9, atol=1e-13)
        np.testing.assert_allclose(d["theta"], (np.abs(A - masked) * Vn).sum(), rtol=1e-9, atol=1e-13)
        np.testing.assert_allclose(d["sigma"], A[keep[0]], rtol=1e-12)
        np.testing.assert_allclose(d["s"], A[list(keep)].sum(), rtol=1e-12)
        np.testing.assert_allclose(d["C"], A @ Vn, rtol=1e-12)
        assert d["M"] == Vn.min()
        assert d["L"] <= d["theta"] * (1 + 1e-12) <= d["theta_hat"] * (1 + 1e-11)
        if d["sigma"] >= 0.5:
            assert d["theta_hat"] <= d["theta_relax"] * (1 + 1e-12)
        # L2: the Euclidean norm of the same difference vector
        d2 = _diag(A, v[0, 0], w, keep[:1], keep[1:], norm=2)
        np.testing.assert_allclose(d2["L"], np.sqrt(((o_full - masked @ P) ** 2).sum()), rtol=1e-9, atol=1e-13)


def test_diagnostics_closed_cases():
    r = rng(17)
    n, dh, dm = 12, 4, 5
    A = r.random(n)
    A /= A.sum()
    v = r.standard_normal((n, dh))
    w = r.standard_normal((dh, dm))
    everything = _diag(A, v, w, range(0, 5), range(5, n))
    assert abs(everything["L"]) < 1e-12 and abs(everything["theta"]) < 1e-12 and abs(everything["s"] - 1) < 1e-12
    # stage 2 empty: s = sigma, so theta_hat collapses onto theta (and so does the relaxed bound)
    only1 = _diag(A, v, w, [1, 4, 7], [])
    np.testing.assert_allclose(only1["theta_hat"], only1["theta"], rtol=1e-12)
    np.testing.assert_allclose(only1["theta_relax"], only1["theta"], rtol=1e-12)
    # nothing kept: the pruned output is zero
    P = np.float32(v).astype(np.float64) @ np.float32(w).astype(np.float64)
    none = _diag(A, v, w, [], [])
    np.testing.assert_allclose(none["L"], np.abs(A @ P).sum(), rtol=1e-12)
    np.testing.assert_allclose(none["theta"], none["C"], rtol=1e-15)
    assert none["sigma"] == 0 and np.isinf(none["theta_hat"]) and np.isinf(none["theta_relax"])
    # stage 1 empty only
    no1 = _diag(A, v, w, [], [2, 3])
    assert np.isinf(no1["theta_hat"]) and np.isfinite(no1["theta"]) and no1["L"] <= no1["theta"]
    # identical projected values: any selection reproduces the output exactly
    same = _diag(A, np.tile(v[:1], (n, 1)), w, [0], [5, 6])
    assert same["L"] < 1e-12 * same["C"]
    # equal magnitudes N_i = 1 (signed unit vectors through the identity): the relaxed bound is not relaxed
    signs = np.eye(dh)[r.integers(0, dh, n)] * r.choice([-1.0, 1.0], (n, 1))
    eq = _diag(A, signs, np.eye(dh), [int(np.argmax(A))], [2, 3] if int(np.argmax(A)) not in (2, 3) else [4, 5])
    np.testing.assert_allclose(eq["theta_relax"], eq["theta_hat"], rtol=1e-12)
    assert eq["M"] == 1.0


def test_diagnostics_head_layout_and_chain_on_tiny_config():
    """GQA layout: query head h reads kv head h / G, its own W_O slice and its own A; and on the synthetic
    workload the chain L <= theta <= theta_hat (<= theta_relax when sigma >= 0.5) holds for every head."""
    cfg = CONFIGS["tiny"]
    t = make_layer(cfg)
    r = O.score(t["q_win"], t["k"], t["v"], t["w_o"], pool_kernel=cfg.pool_kernel, eps=cfg.eps)
    idx, count, _, st1 = O.select(r.attn, r.crit, cfg.budget, cfg.alpha, with_stage1=True)
    out = O.diagnostics(r.a_head, t["v"], t["w_o"], idx, count, st1)
    b, H, Hkv, dh = cfg.batch, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G = H // Hkv
    assert out.shape == (b, H, 8)
    for bi in range(b):
        for h in range(H):
            g = h // G
            c = int(count[bi, g])
            sel = idx[bi, g, :c]
            one = _diag(r.a_head[bi, h], t["v"][bi, g], t["w_o"][h * dh:(h + 1) * dh], sel[st1[bi, g, :c] > 0],
                        sel[st1[bi, g, :c] == 0])
            np.testing.assert_allclose(out[bi, h], [one[f] for f in O.DIAG_FIELDS], rtol=1e-12)
            d = dict(zip(O.DIAG_FIELDS, out[bi, h]))
            np.testing.assert_allclose(d["C"], r.a_head[bi, h] @ r.vnorm[bi, h], rtol=1e-12)
            assert d["L"] <= d["theta"] * (1 + 1e-12) <= d["theta_hat"] * (1 + 1e-11)
            if d["sigma"] >= 0.5:
                assert d["theta_hat"] <= d["theta_relax"] * (1 + 1e-12)
    assert (st1.sum(axis=-1) == int(np.floor(cfg.alpha * cfg.budget))).all()


def test_bad_arguments_are_rejected():
    a = np.ones(4)
    with pytest.raises(RuntimeError):
        O.select_head(a, a, 5, 0.5)
    with pytest.raises(RuntimeError):
        O.select_head(a, a, 2, 1.5)
    with pytest.raises(RuntimeError):
        O.maxpool1d(np.ones((1, 4)), 4)


# ----------------------------------------------------------------------------- whole pass, second opinion
def test_numpy_transcription_agrees_on_tiny_config():
    cfg = CONFIGS["tiny"]
    t = make_layer(cfg)
    res = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget, cfg.alpha, pool_kernel=cfg.pool_kernel,
                      eps=cfg.eps)
    attn, crit, sets = pass_numpy(t["q_win"][0], t["k"][0], t["v"][0], t["w_o"], cfg.budget, cfg.alpha,
                                  cfg.pool_kernel, cfg.eps)
    np.testing.assert_allclose(res.attn[0], attn, rtol=1e-12)
    np.testing.assert_allclose(res.crit[0], crit, rtol=1e-12)
    for g in range(cfg.n_kv_heads):
        assert res.count[0, g] == cfg.budget
        assert res.idx[0, g, :cfg.budget].tolist() == sets[g].tolist()
    # the synthetic workload must actually exercise stage 2: it differs from attention-only Top-B
    idx_a, _, _ = O.select(res.attn, res.crit, cfg.budget, 1.0)
    assert any(set(idx_a[0, g].tolist()) != set(res.idx[0, g].tolist()) for g in range(cfg.n_kv_heads))


def test_numpy_transcription_agrees_on_gqa_bf16_shape():
    cfg = CONFIGS["llama32k"].with_(n_ctx=300, budget=60, d_model=96, n_q_heads=8, n_kv_heads=2, head_dim=16,
                                    window=4)
    t = make_layer(cfg)
    res = O.full_pass(t["q_win"], t["k"], t["v"], t["w_o"], cfg.budget, cfg.alpha, pool_kernel=cfg.pool_kernel)
    attn, crit, sets = pass_numpy(t["q_win"][0], t["k"][0], t["v"][0], t["w_o"], cfg.budget, cfg.alpha,
                                  cfg.pool_kernel)
    np.testing.assert_allclose(res.attn[0], attn, rtol=1e-12)
    np.testing.assert_allclose(res.crit[0], crit, rtol=1e-12)
    for g in range(cfg.n_kv_heads):
        assert res.idx[0, g].tolist() == sets[g].tolist()
