"""Pins of the page-level oracle functions (the page-retrieval baseline of Sec. 3.2, Eq. 1-3, and the averaged
quantized score of the Sec. 4.4 ablation) against what the mathematics fixes: single-token pages reduce to library
routines, the channel-sum form bounds every key's dot product from above, a sign flip of q swaps the roles of the
maximum and minimum vectors, page means equal numpy means, page expansion equals a brute-force enumeration."""
import numpy as np
import pytest

from paper_2508_08256_amd import synth

F16, BF16 = 0, 1


def _rand_words(rng, shape, dtype, scale=1.0):
    return synth.f32_to_words((rng.standard_normal(shape) * scale).astype(np.float32), dtype)


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_single_token_pages_reduce_to_elementwise_max_and_dot(oracle, dtype):
    rng = np.random.default_rng(1)
    U, L, D = 3, 24, 128
    K = _rand_words(rng, (U, L, D), dtype)
    q = _rand_words(rng, (U, 1, D), dtype)
    lens = np.array([24, 7, 1], np.int32)
    kmin, kmax = oracle.page_minmax(K, lens, 1, dtype)
    assert np.array_equal(kmin[0], K[0]) and np.array_equal(kmax[0], K[0])      # one token: min = max = the key
    Kf = synth.words_to_f32(K, dtype).astype(np.float64)
    qf = synth.words_to_f32(q, dtype).astype(np.float64)[:, 0]
    s_max = oracle.page_score(kmin, kmax, q, lens, 1, dtype, 0)
    s_sum = oracle.page_score(kmin, kmax, q, lens, 1, dtype, 1)
    for u in range(U):
        n = lens[u]
        assert np.array_equal(s_max[u, :n], (Kf[u, :n] * qf[u]).max(axis=1))       # max_i q_i k_i
        np.testing.assert_allclose(s_sum[u, :n], Kf[u, :n] @ qf[u], rtol=1e-12, atol=1e-12)   # q . k
        assert np.all(np.isneginf(s_max[u, n:])) and np.all(np.isneginf(s_sum[u, n:]))


def test_channel_sum_form_bounds_every_key_of_the_page(oracle):
    rng = np.random.default_rng(2)
    U, L, D, page = 2, 160, 128, 16
    K = _rand_words(rng, (U, L, D), F16, 2.0)
    q = _rand_words(rng, (U, 2, D), F16)
    lens = np.array([160, 70], np.int32)
    kmin, kmax = oracle.page_minmax(K, lens, page, F16)
    s_sum = oracle.page_score(kmin, kmax, q, lens, page, F16, 1)
    s_max = oracle.page_score(kmin, kmax, q, lens, page, F16, 0)
    Kf = synth.words_to_f32(K, F16).astype(np.float64)
    qf = synth.words_to_f32(q, F16).astype(np.float64)
    for u in range(U):
        for p in range(-(-int(lens[u]) // page)):
            rows = Kf[u, p * page:min((p + 1) * page, lens[u])]
            per_head = rows @ qf[u].T                                    # [tokens][heads]
            assert s_sum[u, p] >= per_head.max(axis=0).sum() - 1e-9      # bound, head by head, then added
            # Eq. 3 as printed: the largest single product q_i k_i over the page's extreme vectors
            brute = sum(max((qf[u, h] * rows.max(axis=0)).max(), (qf[u, h] * rows.min(axis=0)).max()) for h in range(2))
            assert s_max[u, p] == brute
    # the extreme vectors are taken over the tokens present only
    assert np.array_equal(synth.words_to_f32(kmax[1, 4], F16), Kf[1, 64:70].max(axis=0).astype(np.float32))
    assert not kmin[1, 5:].any() and not kmax[1, 5:].any()


def test_negating_the_query_swaps_maximum_and_minimum_vectors(oracle):
    rng = np.random.default_rng(3)
    U, L, D, page = 1, 64, 128, 16
    K = _rand_words(rng, (U, L, D), BF16)
    q = _rand_words(rng, (U, 1, D), BF16)
    lens = np.array([64], np.int32)
    kmin, kmax = oracle.page_minmax(K, lens, page, BF16)
    Kn = synth.f32_to_words(-synth.words_to_f32(K, BF16), BF16)          # negation is exact
    qn = synth.f32_to_words(-synth.words_to_f32(q, BF16), BF16)
    kmin_n, kmax_n = oracle.page_minmax(Kn, lens, page, BF16)
    assert np.array_equal(synth.words_to_f32(kmin_n, BF16), -synth.words_to_f32(kmax, BF16))
    for mode in (0, 1):                                                   # (-q) . (-k) = q . k
        a = oracle.page_score(kmin, kmax, q, lens, page, BF16, mode)
        b = oracle.page_score(kmin_n, kmax_n, qn, lens, page, BF16, mode)
        assert np.array_equal(a, b)


def test_page_mean_equals_numpy_mean(oracle):
    rng = np.random.default_rng(4)
    sc = rng.standard_normal((2, 96))
    lens = np.array([96, 41], np.int32)
    pm = oracle.page_mean(sc, lens, 16)
    np.testing.assert_allclose(pm[0], sc[0].reshape(6, 16).mean(axis=1), rtol=1e-13)
    np.testing.assert_allclose(pm[1, :2], sc[1, :32].reshape(2, 16).mean(axis=1), rtol=1e-13)
    np.testing.assert_allclose(pm[1, 2], sc[1, 32:41].mean(), rtol=1e-13)            # partial page: 9 tokens
    assert np.all(np.isneginf(pm[1, 3:]))


def test_expand_pages_brute_force(oracle):
    page_idx = np.array([[0, 2, 5, -1], [1, 3, -1, -1]], np.int32)
    page_cnt = np.array([3, 2], np.int32)
    lens = np.array([85, 64], np.int32)                                   # page 5 of unit 0 holds tokens 80..84 only
    idx, cnt = oracle.expand_pages(page_idx, page_cnt, lens, 16, 48)
    want0 = list(range(0, 16)) + list(range(32, 48)) + list(range(80, 85))
    assert cnt[0] == len(want0) and idx[0, :cnt[0]].tolist() == want0
    assert cnt[1] == 32 and idx[1, :32].tolist() == list(range(16, 32)) + list(range(48, 64))
    idx, cnt = oracle.expand_pages(page_idx, page_cnt, lens, 16, 20)     # capacity cuts the list
    assert cnt[0] == 20 and idx[0, :20].tolist() == want0[:20]
