"""The pins must be able to fail: each plausible mistake, planted on the CPU in a wrapper around the oracle (a dropped
term, a wrong sign, index or operand, a wrong tie rule), has to make the pin that guards that part raise.  The real
oracle passes the same pins in the other test files."""
import types

import numpy as np
import pytest

import test_oracle_pages as tp
import test_oracle_quantize as tq
import test_oracle_score_topk_attn as ts

F16, BF16 = 0, 1
G = 32


def _mutant(oracle, **overrides):
    """The oracle module with some of its functions replaced."""
    m = types.SimpleNamespace(**{k: getattr(oracle, k) for k in dir(oracle) if not k.startswith("_")})
    for k, v in overrides.items():
        setattr(m, k, v)
    return m


def _f32(oracle, w, dtype):
    return oracle.to_f32(w, dtype).astype(np.float64)


# ---- planted mistakes -------------------------------------------------------------------------------------------
def scale_doubled(oracle):
    """s = 2 (max - min): the upper level overshoots."""
    def quantize(K, L, g, dtype, n_threads=1):
        bits, s, z = oracle.quantize(K, L, g, dtype, n_threads)
        s = oracle.from_f32((2.0 * _f32(oracle, s, dtype)).astype(np.float32), dtype)
        return bits, s, z
    return _mutant(oracle, quantize=quantize)


def offset_dropped(oracle):
    """z = 0 instead of the group minimum."""
    def quantize(K, L, g, dtype, n_threads=1):
        bits, s, z = oracle.quantize(K, L, g, dtype, n_threads)
        return bits, s, np.zeros_like(z)
    return _mutant(oracle, quantize=quantize)


def midpoint_rounds_down(oracle):
    """bit = 2 (k - z) > s: the exact midpoint goes to the lower level."""
    def quantize(K, L, g, dtype, n_threads=1):
        bits, s, z = oracle.quantize(K, L, g, dtype, n_threads)
        k = _f32(oracle, K, dtype)
        zz = np.repeat(_f32(oracle, z, dtype), g, axis=1)
        ss = np.repeat(_f32(oracle, s, dtype), g, axis=1)
        bits = bits.copy()
        bits[(2.0 * (k - zz) == ss) & (ss > 0)] = 0
        return bits, s, z
    return _mutant(oracle, quantize=quantize)


def codes_inverted(oracle):
    """bit = 1 for the LOWER level (wrong sign of the comparison)."""
    def quantize(K, L, g, dtype, n_threads=1):
        bits, s, z = oracle.quantize(K, L, g, dtype, n_threads)
        present = np.arange(K.shape[1])[None, :, None] < np.asarray(L)[:, None, None]
        return np.where(present, 1 - bits, bits).astype(np.uint8), s, z
    return _mutant(oracle, quantize=quantize)


def scale_shared_across_channels(oracle):
    """One (s, z) per group of tokens for ALL channels (grouping along the wrong axis)."""
    def quantize(K, L, g, dtype, n_threads=1):
        bits, s, z = oracle.quantize(K, L, g, dtype, n_threads)
        s = np.repeat(s[..., :1], s.shape[-1], axis=-1)
        return bits, np.ascontiguousarray(s), z
    return _mutant(oracle, quantize=quantize)


def append_keeps_old_codes(oracle):
    """The append updates (s, z) but leaves the earlier tokens' bits as they were."""
    def append(K, V, L, k_new, v_new, bits, s, z, g, dtype):
        old = bits.copy()
        oracle.append(K, V, L, k_new, v_new, bits, s, z, g, dtype)
        for u in range(K.shape[0]):
            t0 = (int(L[u]) // g) * g
            bits[u, t0:int(L[u])] = old[u, t0:int(L[u])]
    return _mutant(oracle, append=append)


def score_without_offset(oracle):
    """score = sum_c q_c * bit * s: the z term dropped."""
    def score(bits, s, z, q, L, g, dtype, n_threads=1):
        return oracle.score(bits, s, z, q, L, g, dtype, n_threads) - oracle.score(np.zeros_like(bits), s, z, q, L, g,
                                                                                 dtype, n_threads)
    return _mutant(oracle, score=score)


def score_first_head_only(oracle):
    """GQA: only the first query head of the group scores."""
    def score(bits, s, z, q, L, g, dtype, n_threads=1):
        q1 = q.copy()
        q1[:, 1:] = 0
        return oracle.score(bits, s, z, q1, L, g, dtype, n_threads)
    return _mutant(oracle, score=score)


def score_shifted_by_one_token(oracle):
    """score[j] uses the code word of token j + 1 (an index slip)."""
    def score(bits, s, z, q, L, g, dtype, n_threads=1):
        sc = oracle.score(bits, s, z, q, L, g, dtype, n_threads)
        out = np.zeros_like(sc)
        for u in range(sc.shape[0]):
            n = int(L[u])
            out[u, :n] = np.roll(sc[u, :n], -1)
        return out
    return _mutant(oracle, score=score)


def topk_takes_smallest(oracle):
    def topk(scores, L, budget, max_budget):
        return oracle.topk(-scores, L, budget, max_budget)
    return _mutant(oracle, topk=topk)


def topk_ties_to_higher_index(oracle):
    def topk(scores, L, budget, max_budget):
        rev = np.zeros_like(scores)
        for u in range(scores.shape[0]):
            n = int(L[u])
            rev[u, :n] = scores[u, :n][::-1]
        idx, cnt = oracle.topk(rev, L, budget, max_budget)
        out = np.full_like(idx, -1)
        for u in range(scores.shape[0]):
            c = int(cnt[u])
            out[u, :c] = np.sort(int(L[u]) - 1 - idx[u, :c])
        return out, cnt
    return _mutant(oracle, topk=topk)


def topk_ignores_length(oracle):
    """Entries past the sequence length compete."""
    def topk(scores, L, budget, max_budget):
        full = np.full_like(np.asarray(L), scores.shape[1])
        idx, cnt = oracle.topk(scores, full, budget, max_budget)
        return idx, np.minimum(cnt, np.minimum(budget, L)).astype(cnt.dtype)
    return _mutant(oracle, topk=topk)


def attention_unscaled(oracle):
    def attention(K, V, q, L, sm_scale, dtype, idx=None, count=None, n_threads=1):
        return oracle.attention(K, V, q, L, 1.0, dtype, idx, count, n_threads)
    return _mutant(oracle, attention=attention)


def attention_operands_swapped(oracle):
    def attention(K, V, q, L, sm_scale, dtype, idx=None, count=None, n_threads=1):
        return oracle.attention(V, K, q, L, sm_scale, dtype, idx, count, n_threads)
    return _mutant(oracle, attention=attention)


def attention_unnormalised(oracle):
    """o = sum_i exp(l_i - max) v_i without the division by the sum."""
    def attention(K, V, q, L, sm_scale, dtype, idx=None, count=None, n_threads=1):
        o = oracle.attention(K, V, q, L, sm_scale, dtype, idx, count, n_threads)
        return 2.0 * o
    return _mutant(oracle, attention=attention)


def page_score_uses_minimum_only(oracle):
    """Eq. 1-3 with max(q m, q M) replaced by q m."""
    def page_score(kmin, kmax, q, L, page, dtype, mode):
        return oracle.page_score(kmin, kmin, q, L, page, dtype, mode)
    return _mutant(oracle, page_score=page_score)


def page_score_modes_swapped(oracle):
    """The max-over-channels form where the sum over channels is asked for, and the reverse."""
    def page_score(kmin, kmax, q, L, page, dtype, mode):
        return oracle.page_score(kmin, kmax, q, L, page, dtype, 1 - mode)
    return _mutant(oracle, page_score=page_score)


def page_mean_over_the_whole_page(oracle):
    """The mean divides by the page size even where the last page is partly filled."""
    def page_mean(scores, L, page):
        pm = oracle.page_mean(scores, L, page)
        for u in range(scores.shape[0]):
            n = int(L[u])
            if n % page:
                pm[u, n // page] *= (n % page) / page
        return pm
    return _mutant(oracle, page_mean=page_mean)


def expand_pages_one_token_short(oracle):
    """A page expands to page - 1 tokens."""
    def expand_pages(page_idx, page_cnt, L, page, max_budget):
        idx, cnt = oracle.expand_pages(page_idx, page_cnt, L, page, max_budget)
        keep = (idx % page) != page - 1
        out = np.full_like(idx, -1)
        for u in range(idx.shape[0]):
            v = idx[u, :int(cnt[u])]
            v = v[keep[u, :int(cnt[u])]]
            out[u, :len(v)] = v
            cnt[u] = len(v)
        return out, cnt
    return _mutant(oracle, expand_pages=expand_pages)


CASES = [
    (scale_doubled, tq.test_two_levels_nearest_and_error_bound, (F16,)),
    (offset_dropped, tq.test_two_levels_nearest_and_error_bound, (BF16,)),
    (codes_inverted, tq.test_two_levels_nearest_and_error_bound, (F16,)),
    (midpoint_rounds_down, tq.test_midpoint_rounds_up, ()),
    (scale_shared_across_channels, tq.test_groups_run_along_tokens_per_channel, ()),
    (append_keeps_old_codes, tq.test_append_equals_bulk_quantize, (F16,)),
    (score_without_offset, ts.test_score_is_q_dot_dequantized_key, (F16, 1)),
    (score_first_head_only, ts.test_score_is_q_dot_dequantized_key, (BF16, 4)),
    (score_shifted_by_one_token, ts.test_score_is_q_dot_dequantized_key, (F16, 1)),
    (score_without_offset, ts.test_score_tracks_exact_logits_direction, ()),
    (topk_takes_smallest, ts.test_topk_brute_force_tiny, ()),
    (topk_ties_to_higher_index, ts.test_topk_ties_go_to_lower_index_and_budget_clamps, ()),
    (topk_ignores_length, ts.test_topk_ties_go_to_lower_index_and_budget_clamps, ()),
    (attention_unscaled, ts.test_full_budget_equals_dense_softmax_attention, (F16, 1)),
    (attention_operands_swapped, ts.test_full_budget_equals_dense_softmax_attention, (BF16, 4)),
    (attention_unnormalised, ts.test_attention_special_cases, ()),
    (codes_inverted, ts.test_planted_tokens_are_recalled, ()),
    (page_score_modes_swapped, tp.test_single_token_pages_reduce_to_elementwise_max_and_dot, (F16,)),
    (page_score_uses_minimum_only, tp.test_channel_sum_form_bounds_every_key_of_the_page, ()),
    (page_mean_over_the_whole_page, tp.test_page_mean_equals_numpy_mean, ()),
    (expand_pages_one_token_short, tp.test_expand_pages_brute_force, ()),
]


@pytest.mark.parametrize("mistake,pin,args", CASES, ids=[f"{m.__name__}-{p.__name__}" for m, p, _ in CASES])
def test_planted_mistake_fails_its_pin(oracle, mistake, pin, args):
    pin(oracle, *args)                          # the oracle itself passes ...
    with pytest.raises(AssertionError):         # ... the same pin catches the planted mistake
        pin(mistake(oracle), *args)
