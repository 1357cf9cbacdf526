"""Shared test helpers: the oracle's end-to-end decode step and the parity rules."""
import numpy as np


def oracle_step(oracle, wl, append=True, n_threads=4):
    """Run Alg. 1 with the CPU oracle on a synth.Workload.  Returns a dict of every intermediate.

    With ``append`` the step first appends (k_new, v_new) at row L and works on L+1 tokens.
    """
    g = 32
    K = wl.K.copy()
    V = wl.V.copy()
    L = wl.unit_lens.copy()
    bits, s, z = oracle.quantize(K, L, g, wl.dtype, n_threads)
    if append:
        oracle.append(K, V, L, wl.k_new, wl.v_new, bits, s, z, g, wl.dtype)
        L = (L + 1).astype(np.int32)
    scores = oracle.score(bits, s, z, wl.q, L, g, wl.dtype, n_threads)
    budgets = wl.unit_budgets
    max_budget = int(budgets.max())
    idx, count = oracle.topk(scores, L, budgets, max_budget)
    sm_scale = 1.0 / np.sqrt(wl.head_dim)
    out = oracle.attention(K, V, wl.q, L, sm_scale, wl.dtype, idx, count, n_threads)
    return dict(K=K, V=V, L=L, bits=bits, s=s, z=z, scores=scores, idx=idx, count=count, out=out,
                max_budget=max_budget, sm_scale=sm_scale)


def score_tolerance_ok(s_gpu, s_or, absterm):
    """Approximate scores: within 1e-3 relative, or within 1e-5 * sum_c |q_c K~_c| where the sum cancels."""
    err = np.abs(s_gpu.astype(np.float64) - s_or)
    return (err <= 1e-3 * np.abs(s_or)) | (err <= 1e-5 * absterm)


def check_index_sets(idx_gpu, cnt_gpu, idx_or, cnt_or, scores_or, L):
    """Selected sets equal, except members of the symmetric difference whose oracle score is within
    1e-3 relative of the oracle's B-th largest score (near-ties at the threshold)."""
    n_swapped = 0
    for u in range(len(L)):
        assert cnt_gpu[u] == cnt_or[u], (u, cnt_gpu[u], cnt_or[u])
        n = int(cnt_or[u])
        a = idx_gpu[u, :n]
        b = idx_or[u, :n]
        assert np.all(np.diff(a) > 0), f"unit {u}: indices not strictly ascending"
        assert n == 0 or (a[0] >= 0 and a[-1] < L[u])
        diff = np.setxor1d(a, b)
        if diff.size == 0:
            continue
        sc = scores_or[u]
        T = np.min(sc[b])
        gap = np.abs(sc[diff] - T)
        lim = 1e-3 * np.maximum(np.abs(T), np.abs(sc[diff]))
        assert np.all(gap <= lim), (u, diff, sc[diff], T)
        n_swapped += diff.size // 2
    return n_swapped
