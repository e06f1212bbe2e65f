"""Second, independently written float64 statement of the pass in NumPy (test infrastructure).

Written from the paper's algorithms, without looking at the C oracle's loops, so
that the two can be compared on the tiny configuration.  Single batch item.
  Algorithm 2 lines 2-4: window softmax, mean over the window, max-pool
  Algorithm 1 lines 2-9: projected-value L1 norm, (A + eps) * norm, budget split, two Top-k stages
"""
import numpy as np


def pass_numpy(q_win, k, v, w_o, B, alpha, pool_kernel, eps=1e-4, scale=None):
    q_win, k, v, w_o = (np.asarray(x, dtype=np.float64) for x in (q_win, k, v, w_o))
    H, W, dh = q_win.shape
    Hkv, n, _ = k.shape
    G = H // Hkv
    scale = 1.0 / np.sqrt(dh) if scale is None else scale
    r = pool_kernel // 2
    abar = np.empty((H, n))
    norm = np.empty((H, n))
    for h in range(H):
        g = h // G
        logits = scale * (q_win[h] @ k[g].T)                      # [W, n]
        logits -= logits.max(axis=1, keepdims=True)
        p = np.exp(logits)
        p /= p.sum(axis=1, keepdims=True)
        a = p.mean(axis=0)
        padded = np.concatenate([np.full(r, -np.inf), a, np.full(r, -np.inf)])
        abar[h] = np.lib.stride_tricks.sliding_window_view(padded, pool_kernel).max(axis=1)
        norm[h] = np.abs(v[g] @ w_o[h * dh:(h + 1) * dh]).sum(axis=1)
    attn = abar.reshape(Hkv, G, n).mean(axis=1)
    crit = ((abar + eps) * norm).reshape(Hkv, G, n).mean(axis=1)
    b1 = int(np.floor(alpha * B))
    b2 = B - b1
    sets = []
    for g in range(Hkv):
        order1 = np.lexsort((np.arange(n), -attn[g]))             # descending value, then ascending index
        s1 = order1[:b1]
        rest = np.setdiff1d(np.arange(n), s1)
        order2 = rest[np.lexsort((rest, -crit[g][rest]))]
        s2 = order2[:b2]
        sets.append(np.sort(np.concatenate([s1, s2])).astype(np.int64))
    return attn, crit, sets
