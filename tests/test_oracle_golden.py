"""Pins for the oracle of the Golden Eviction label builder (Section 3.2 Eq. 3-5): the pooling as a linear
map on unit matrices, closed forms for uniform causal attention (harmonic numbers), the suffix-max
recurrence, planted needles the trace must keep, and exhaustive subset search on tiny traces."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import synth_inputs as si
from oracle import golden


def uniform_causal(Hq, T):
    A = np.zeros((Hq, T, T))
    for q in range(T):
        A[:, q, :q + 1] = 1.0 / (q + 1)
    return A


@pytest.mark.parametrize("T,B,L,M", [(100, 20, 10, 7), (101, 20, 10, 8), (30, 20, 10, 0), (31, 20, 10, 1), (20, 20, 10, 0),
                                     (32768, 2048, 128, 239), (8192, 1024, 256, 27)])
def test_number_of_steps(T, B, L, M):
    """M = ceil((T - B)/L) - 1 (Section 3.2); the last block holds between 1 and L queries."""
    assert golden.n_steps(T, B, L) == M
    if M > 0:
        assert B + M * L < T <= B + (M + 1) * L


def test_pooling_is_the_stated_linear_map_on_every_unit_matrix():
    """A single unit entry A^h[q, i] = 1 lands in group h // g, block (q - B) // L, key i with weight
    1 / (g L), and nowhere else; queries before B + L belong to no block."""
    Hq, g, T, B, L = 4, 2, 11, 3, 2
    M = golden.n_steps(T, B, L)
    assert M == 3
    for h in range(Hq):
        for q in range(T):
            for i in range(T):
                A = np.zeros((Hq, T, T))
                A[h, q, i] = 1.0
                a = golden.block_scores(A, g, B, L)
                want = np.zeros((Hq // g, M, T))
                if q >= B + L:
                    want[h // g, (q - B) // L - 1, i] = 1.0 / (g * L)
                assert np.array_equal(a, want), (h, q, i)


def test_pooling_is_linear():
    A1 = si.gen_attention(3, 4, 40).astype(np.float64)
    A2 = si.gen_attention(4, 4, 40).astype(np.float64)
    a = golden.block_scores(2.0 * A1 + 0.5 * A2, 2, 8, 5)
    np.testing.assert_allclose(a, 2.0 * golden.block_scores(A1, 2, 8, 5) + 0.5 * golden.block_scores(A2, 2, 8, 5), rtol=1e-13, atol=0)


def test_uniform_attention_closed_form_with_padded_last_block():
    """A[q, i] = 1/(q+1): for a key visible to the whole block, a~_t = (1/L) sum_{q in block} 1/(q+1),
    exact in rationals; the last block (3 of 10 queries present) divides by L all the same."""
    Hq, g, T, B, L = 2, 2, 63, 20, 10
    M = golden.n_steps(T, B, L)
    assert M == 4 and B + (M + 1) * L - T == 7
    a = golden.block_scores(uniform_causal(Hq, T), g, B, L)
    for t in range(1, M + 1):
        rows = range(B + t * L, min(B + (t + 1) * L, T))
        full = float(sum(Fraction(1, q + 1) for q in rows) / L)
        assert abs(a[0, t - 1, 0] - full) < 1e-15 and abs(a[0, t - 1, B + t * L] - full) < 1e-15
        # a key inside the block is seen only by the queries at or after it
        i = B + t * L + 1
        part = float(sum(Fraction(1, q + 1) for q in rows if q >= i) / L)
        assert abs(a[0, t - 1, i] - part) < 1e-15
        if rows[-1] + 1 < T:
            assert a[0, t - 1, rows[-1] + 1] == 0.0
    alpha = golden.future_scores(a)
    # block averages of 1/(q+1) fall with t, so the future score of an old key is its current block score
    assert np.array_equal(alpha[0, :, 0], a[0, :, 0])
    # all candidates tie at every step: the lowest positions stay
    kept = golden.trace(alpha.astype(np.float32), B, L)
    for t in range(1, M + 1):
        want = np.concatenate([np.arange(B - L), np.arange(B + t * L - L, B + t * L)])
        assert np.array_equal(kept[0, t - 1], want)


def test_future_score_obeys_the_suffix_max_recurrence():
    A = si.gen_attention(11, 6, 90).astype(np.float64)
    a = golden.block_scores(A, 3, 16, 8)
    alpha = golden.future_scores(a)
    M = a.shape[1]
    assert M == golden.n_steps(90, 16, 8) == 9
    assert np.array_equal(alpha[:, M - 1], a[:, M - 1])
    for t in range(M - 1, 0, -1):
        assert np.array_equal(alpha[:, t - 1], np.maximum(a[:, t - 1], alpha[:, t]))
    assert (np.diff(alpha, axis=1) <= 0).all() and (alpha >= a).all()


def test_group_pooling_ignores_head_order_inside_a_group_only():
    A = si.gen_attention(12, 4, 50).astype(np.float64)
    a = golden.block_scores(A, 2, 10, 5)
    assert np.allclose(golden.block_scores(A[[1, 0, 3, 2]], 2, 10, 5), a, rtol=1e-14, atol=0)
    assert not np.allclose(golden.block_scores(A[[0, 2, 1, 3]], 2, 10, 5), a, rtol=1e-3, atol=0)
    # g = 1: no pooling over heads
    a1 = golden.block_scores(A, 1, 10, 5)
    np.testing.assert_allclose(a, a1.reshape(2, 2, *a1.shape[1:]).mean(axis=1), rtol=1e-14, atol=0)


def test_trace_keeps_planted_needles_until_their_last_use():
    """Every query puts 0.1 on the key 2L before it and the rest on itself, except that the queries of
    block j move half their mass to needle key n_j (an early position).  So at step t the L pairs generated
    two chunks ago carry a small future score, due needles a large one, everything else none: Golden
    Eviction keeps each needle through every step up to its block and drops it right after."""
    T, B, L, g = 96, 16, 8, 1
    M = golden.n_steps(T, B, L)
    assert M == 9
    needles = {j: j - 3 for j in range(3, M + 1)}              # block j uses position j - 3
    A = np.zeros((1, T, T))
    for q in range(T):
        A[0, q, q] = 1.0
        if q >= 2 * L:
            A[0, q, q] -= 0.1
            A[0, q, q - 2 * L] = 0.1
        if q >= B + L and (q - B) // L in needles:
            A[0, q, q] -= 0.5
            A[0, q, needles[(q - B) // L]] += 0.5
    a = golden.block_scores(A, g, B, L)
    alpha = golden.future_scores(a)
    kept = golden.trace(alpha.astype(np.float32), B, L)
    for t in range(1, M + 1):
        s = set(kept[0, t - 1].tolist())
        assert set(range(B + t * L - L, B + t * L)) <= s                 # the L newest
        for j, n in needles.items():
            assert (n in s) == (j >= t), (t, j)                         # due needles stay, spent ones go
    # the current block alone does not see needle 9 at step 3; the future score does
    assert a[0, 2, needles[9]] == 0.0 and abs(alpha[0, 2, needles[9]] - 0.5) < 1e-15


def test_trace_against_exhaustive_subset_search():
    """Tiny traces: at every step the kept old pairs are the size-(B-L) subset of the candidates with the
    largest total future score (unique: the scores are distinct), candidates being what the previous step
    left plus nothing new; the L newest are kept on top."""
    T, B, L, g = 26, 6, 2, 2
    A = si.gen_attention(21, 4, T).astype(np.float64)
    alpha = golden.future_scores(golden.block_scores(A, g, B, L))
    a32 = alpha.astype(np.float32)
    kept = golden.trace(a32, B, L)
    M = golden.n_steps(T, B, L)
    assert kept.shape == (2, M, B) and M == 9
    for hp in range(2):
        cache = list(range(B + L))
        for t in range(1, M + 1):
            old, new = cache[:B], cache[B:]
            assert new == list(range(B + t * L - L, B + t * L))
            sc = a32[hp, t - 1].astype(np.float64)
            assert len(set(sc[old].tolist())) == len(old)
            best = max(itertools.combinations(old, B - L), key=lambda s: sum(sc[list(s)]))
            assert kept[hp, t - 1].tolist() == sorted(best) + new
            assert (np.diff(kept[hp, t - 1]) > 0).all()
            cache = kept[hp, t - 1].tolist() + list(range(B + t * L, B + (t + 1) * L))


def test_evicted_pairs_never_return_and_independent_topk_would_differ():
    """The trace is sequential: kept_t minus the L newest is a subset of kept_{t-1} plus the pairs that
    were new at step t - 1.  (Taking Top_{B-L} over ALL earlier positions at each step independently is not
    nested on this input, which is why the trace form is the reading taken.)"""
    T, B, L, g = 200, 32, 8, 2
    A = si.gen_attention(31, 4, T).astype(np.float64)
    a32 = golden.future_scores(golden.block_scores(A, g, B, L)).astype(np.float32)
    kept = golden.trace(a32, B, L)
    M = kept.shape[1]
    nested_everywhere = True
    for hp in range(2):
        for t in range(2, M + 1):
            prev = set(kept[hp, t - 2].tolist()) | set(range(B + (t - 1) * L, B + t * L))
            assert set(kept[hp, t - 1].tolist()) <= prev
            ind_prev = set(np.argsort(-a32[hp, t - 2, :B + (t - 1) * L - L], kind="stable")[:B - L].tolist())
            ind_now = set(np.argsort(-a32[hp, t - 1, :B + t * L - L], kind="stable")[:B - L].tolist())
            if not ind_now <= ind_prev | set(range(B + (t - 1) * L - L, B + t * L - L)):
                nested_everywhere = False
    assert not nested_everywhere
