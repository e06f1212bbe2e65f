"""The acceptance rules that compare a result with the float64 oracle (test infrastructure, not product code).

Used by the tests and by the benchmark's cpu_baseline leg, which reports the same figures beside the timing:
  * scores within a relative tolerance of the oracle's (2e-3: bf16 inputs, fp32 accumulation);
  * selected index sets identical, except for swaps between entries whose ORACLE key lies within that
    tolerance of the oracle's stage threshold (the smallest key the oracle took in stage 1 or in stage 2);
    every swapped index is counted.
No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np

REL_TOL = 2e-3


def score_errors(got: np.ndarray, ref: np.ndarray):
    """max and median relative error with the floor 1e-7 * max|ref| on the denominator (attention tails
    reach denormals, where a relative error means nothing)."""
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    denom = np.maximum(np.abs(ref), 1e-7 * np.abs(ref).max())
    rel = np.abs(got - ref) / denom
    return float(rel.max()), float(np.median(rel))


def assert_scores_close(got, ref, what, tol=REL_TOL):
    mx, med = score_errors(got, ref)
    assert mx <= tol, f"{what}: max relative error {mx:.3e} > {tol} (median {med:.3e})"
    return mx, med


def compare_selection(idx_got, count_got, oracle, budget, alpha, tol=REL_TOL):
    """Set comparison per (batch, kv head) under the tie rule.  `oracle` carries idx, tau, attn, crit of the
    oracle's own pass.  Returns the total number of swapped indices (entries in exactly one of the two sets);
    raises AssertionError on any difference outside the tolerance band."""
    b, Hkv, _ = idx_got.shape
    budget = np.broadcast_to(np.asarray(budget, dtype=np.int64), (b, Hkv))
    swaps = 0
    for bi in range(b):
        for g in range(Hkv):
            B = int(budget[bi, g])
            assert int(count_got[bi, g]) == B, f"count[{bi},{g}] = {count_got[bi, g]} != budget {B}"
            got = idx_got[bi, g, :B]
            assert np.all(idx_got[bi, g, B:] == -1), "tail must be -1"
            assert np.all(np.diff(got) > 0), "indices must be strictly ascending"
            ref = oracle.idx[bi, g, :B]
            if np.array_equal(got, ref):
                continue
            diff = np.setxor1d(got, ref)
            tau1, tau2 = oracle.tau[bi, g]
            a = oracle.attn[bi, g, diff]
            c = oracle.crit[bi, g, diff]
            near1 = np.abs(a - tau1) <= tol * abs(tau1) if np.isfinite(tau1) else np.zeros(len(diff), bool)
            near2 = np.abs(c - tau2) <= tol * abs(tau2) if np.isfinite(tau2) else np.zeros(len(diff), bool)
            bad = diff[~(near1 | near2)]
            assert bad.size == 0, (f"head ({bi},{g}): {bad.size} differing indices outside the tolerance band, "
                                   f"e.g. {bad[:5].tolist()}")
            swaps += int(diff.size)
    return swaps
