"""Pins for the oracle's score (Alg. 1 step 2), top-k (step 3) and attention (step 4 / Sec. 3.1)."""
import numpy as np
import pytest
import scipy.special

from paper_2508_08256_amd import synth

F16, BF16 = 0, 1
G = 32


def _words(rng, shape, dtype, scale=1.0):
    return synth.f32_to_words(rng.standard_normal(shape).astype(np.float32) * scale, dtype)


def _val(w, dtype):
    return synth.words_to_f32(w, dtype).astype(np.float64)


# ------------------------------------------------------------------ score
@pytest.mark.parametrize("dtype,n_rep", [(F16, 1), (BF16, 4)])
def test_score_is_q_dot_dequantized_key(oracle, dtype, n_rep):
    rng = np.random.default_rng(20 + n_rep)
    U, L, D = 3, 5 * G, 128
    K = _words(rng, (U, L, D), dtype, 2.0)
    q = _words(rng, (U, n_rep, D), dtype)
    Lu = np.array([L, L - 7, 1], np.int32)
    bits, s, z = oracle.quantize(K, Lu, G, dtype)
    got = oracle.score(bits, s, z, q, Lu, G, dtype)
    # materialise K~ = code * s + z with numpy only, then a library matrix product
    Kt = bits.astype(np.float64) * np.repeat(_val(s, dtype), G, axis=1) + np.repeat(_val(z, dtype), G, axis=1)
    for u in range(U):
        n = int(Lu[u])
        want = Kt[u, :n] @ _val(q[u], dtype).T            # [n][n_rep]
        assert np.allclose(got[u, :n], want.sum(axis=1), rtol=1e-12, atol=1e-9)
        # summed-query form (linearity) and factorised form are algebraic identities of the same number
        qsum = _val(q[u], dtype).sum(axis=0)
        assert np.allclose(got[u, :n], Kt[u, :n] @ qsum, rtol=1e-11, atol=1e-9)
        zz = np.repeat(_val(z[u], dtype), G, axis=0)[:n]
        ss = np.repeat(_val(s[u], dtype), G, axis=0)[:n]
        fact = zz @ qsum + (bits[u, :n] * ss) @ qsum
        assert np.allclose(got[u, :n], fact, rtol=1e-11, atol=1e-9)
        assert np.all(got[u, n:] == 0)


def test_score_tracks_exact_logits_direction(oracle):
    """With a two-level key matrix the 1-bit key is exact, so the approximate score IS q.K."""
    rng = np.random.default_rng(22)
    U, L, D = 1, 2 * G, 128
    lvl = rng.integers(0, 2, (U, L, D)).astype(np.float32)
    lvl[:, 0::G] = 0
    lvl[:, 1::G] = 1
    K = synth.f32_to_words(lvl * 3.0 - 1.0, F16)
    q = _words(rng, (U, 1, D), F16)
    Lu = np.array([L], np.int32)
    bits, s, z = oracle.quantize(K, Lu, G, F16)
    got = oracle.score(bits, s, z, q, Lu, G, F16)
    want = _val(K[0], F16) @ _val(q[0, 0], F16)
    assert np.allclose(got[0], want, rtol=1e-12, atol=1e-10)


# ------------------------------------------------------------------ top-k
def test_topk_brute_force_tiny(oracle):
    rng = np.random.default_rng(23)
    for L in (1, 2, 7, 33, 64):
        sc = np.zeros((1, 64), np.float64)
        sc[0, :L] = rng.standard_normal(L)
        for B in list(range(1, L + 1)) + [L + 5]:
            idx, cnt = oracle.topk(sc, np.array([L], np.int32), np.array([B], np.int32), 80)
            n = min(B, L)
            assert cnt[0] == n
            order = np.argsort(-sc[0, :L], kind="stable")      # library sort; stable => lower index first
            want = np.sort(order[:n])
            assert np.array_equal(idx[0, :n], want)
            sel = np.zeros(L, bool)
            sel[idx[0, :n]] = True
            if n < L:
                assert sc[0, :L][sel].min() >= sc[0, :L][~sel].max()


def test_topk_ties_go_to_lower_index_and_budget_clamps(oracle):
    sc = np.array([[1.0, 5.0, 5.0, 5.0, 0.0, 5.0, 7.0, -1.0]])
    L = np.array([8], np.int32)
    idx, cnt = oracle.topk(sc, L, np.array([3], np.int32), 8)
    assert cnt[0] == 3 and list(idx[0, :3]) == [1, 2, 6]
    idx, cnt = oracle.topk(sc, L, np.array([4], np.int32), 8)
    assert list(idx[0, :4]) == [1, 2, 3, 6]
    idx, cnt = oracle.topk(sc, L, np.array([100], np.int32), 8)
    assert cnt[0] == 8 and list(idx[0]) == list(range(8))
    idx, cnt = oracle.topk(np.zeros((1, 8)), np.array([0], np.int32), np.array([3], np.int32), 8)
    assert cnt[0] == 0
    # only the first L entries compete
    idx, cnt = oracle.topk(sc, np.array([5], np.int32), np.array([2], np.int32), 8)
    assert list(idx[0, :2]) == [1, 2]


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("dtype,n_rep", [(F16, 1), (BF16, 4)])
def test_full_budget_equals_dense_softmax_attention(oracle, dtype, n_rep):
    rng = np.random.default_rng(24)
    U, L, D = 2, 100, 128
    K = _words(rng, (U, L, D), dtype)
    V = _words(rng, (U, L, D), dtype)
    q = _words(rng, (U, n_rep, D), dtype)
    Lu = np.array([L, 37], np.int32)
    sm = 1 / np.sqrt(D)
    dense = oracle.attention(K, V, q, Lu, sm, dtype)
    idx = np.tile(np.arange(L, dtype=np.int32), (U, 1))
    full = oracle.attention(K, V, q, Lu, sm, dtype, idx, Lu.copy())
    assert np.allclose(dense, full, rtol=0, atol=1e-14)
    for u in range(U):
        n = int(Lu[u])
        logits = sm * _val(q[u], dtype) @ _val(K[u, :n], dtype).T     # [n_rep][n]
        p = scipy.special.softmax(logits, axis=1)
        want = p @ _val(V[u, :n], dtype)
        assert np.allclose(dense[u], want, rtol=1e-12, atol=1e-13)


def test_attention_special_cases(oracle):
    rng = np.random.default_rng(25)
    U, L, D = 1, 64, 128
    K = _words(rng, (U, L, D), F16)
    V = _words(rng, (U, L, D), F16)
    q = _words(rng, (U, 2, D), F16)
    Lu = np.array([L], np.int32)
    sm = 1 / np.sqrt(D)
    # one selected row: the output is that value row
    idx = np.full((1, 8), -1, np.int32)
    idx[0, 0] = 17
    out = oracle.attention(K, V, q, Lu, sm, F16, idx, np.array([1], np.int32))
    assert np.array_equal(out[0, 0], _val(V[0, 17], F16)) and np.array_equal(out[0, 1], _val(V[0, 17], F16))
    # nothing selected: zeros
    out = oracle.attention(K, V, q, Lu, sm, F16, idx, np.array([0], np.int32))
    assert np.all(out == 0)
    # identical keys: uniform weights, the output is the mean of the selected value rows
    K2 = np.tile(K[:, :1], (1, L, 1))
    sel = np.array([[3, 9, 20, 41, 63, 0, 0, 0]], np.int32)
    out = oracle.attention(K2, V, q, Lu, sm, F16, sel, np.array([5], np.int32))
    assert np.allclose(out[0, 0], _val(V[0, sel[0, :5]], F16).mean(axis=0), rtol=1e-13, atol=1e-14)
    # the order of the selected set does not matter
    a = oracle.attention(K, V, q, Lu, sm, F16, sel, np.array([5], np.int32))
    b = oracle.attention(K, V, q, Lu, sm, F16, sel[:, [4, 2, 0, 1, 3, 5, 6, 7]].copy(), np.array([5], np.int32))
    assert np.allclose(a, b, rtol=1e-13, atol=1e-15)
    # a dominant logit wins: scale one key up along q so softmax is one-hot
    K3 = K.copy()
    K3[0, 30] = synth.f32_to_words(synth.words_to_f32(q[0, 0], F16) * 40.0, F16)
    out = oracle.attention(K3, V, q[:, :1].copy(), Lu, sm, F16)
    assert np.allclose(out[0, 0], _val(V[0, 30], F16), atol=1e-6)


# ------------------------------------------------------------------ the method's claim
def test_planted_tokens_are_recalled(oracle):
    """Observation 2: the top-k under 1-bit keys keeps the high-relevance tokens.  Every planted token of
    the synthetic workloads must be selected, for MHA (fp16) and for grouped queries (bf16)."""
    from helpers import oracle_step

    wl = synth.config1()
    r = oracle_step(oracle, wl, append=False)
    for u in range(wl.units):
        sel = set(r["idx"][u, :r["count"][u]].tolist())
        assert set(wl.planted[u].tolist()) <= sel
        assert r["count"][u] == 512
    wl = synth.make_workload("gqa", 3001, 2, 8, 2, [4096, 3000], [512, 330], BF16, chan="lognormal",
                             n_planted=16)
    r = oracle_step(oracle, wl, append=True)
    for u in range(wl.units):
        sel = set(r["idx"][u, :r["count"][u]].tolist())
        assert set(wl.planted[u].tolist()) <= sel


def test_end_to_end_full_budget_is_dense(oracle):
    """With budget >= L the whole of Alg. 1 collapses to the dense decode attention of Sec. 3.1."""
    from helpers import oracle_step

    wl = synth.make_workload("full", 77, 1, 2, 2, [200], [100000], F16, n_planted=4)
    r = oracle_step(oracle, wl, append=True)
    dense = oracle.attention(r["K"], r["V"], wl.q, r["L"], r["sm_scale"], wl.dtype)
    assert np.all(r["count"] == 201)
    assert np.allclose(r["out"], dense, atol=1e-14)
