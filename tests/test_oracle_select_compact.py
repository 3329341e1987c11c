"""Pins for the oracle's keep-selection and compaction (Section 3.1 eviction protocol:
the most recent L pairs stay, the others are pruned to the B - L most important)."""
import itertools

import numpy as np
import pytest

import synth_inputs as si
from util import random_cache


def brute_force_keep(scores, pos, n, budget, recent):
    """Exhaustive definition on tiny rows: among all subsets of the non-recent candidates of size
    budget - recent, the one in which every member outranks every non-member under
    (score desc, position asc); -0 == +0, NaN below everything."""
    order_newest = sorted(range(n), key=lambda i: -pos[i])
    prot = set(order_newest[:recent])
    cand = [i for i in range(n) if i not in prot]

    def key(i):
        s = float(scores[i])
        if np.isnan(s):
            return (1, 0.0, pos[i])          # after all numbers
        return (0, -(s + 0.0), pos[i])

    k = budget - recent
    for sub in itertools.combinations(cand, k):
        rest = [i for i in cand if i not in sub]
        if all(key(a) < key(b) for a in sub for b in rest):
            return sorted(prot | set(sub))
    raise AssertionError("no dominant subset")


@pytest.mark.parametrize("seed", range(6))
def test_tiny_rows_against_exhaustive_search(ora, seed):
    n, budget, recent, cap = 9, 6, 2, 12
    sc = si.gen_scores(100 + seed, (1, 1, cap), ties=3 if seed % 2 else 0)
    rng = np.random.default_rng(seed)
    pos = np.full((1, 1, cap), -1, np.int32)
    pos[0, 0, :n] = rng.permutation(50)[:n] if seed >= 3 else np.sort(rng.permutation(50)[:n])
    ln = np.array([n], np.int32)
    want = brute_force_keep(sc[0, 0], pos[0, 0], n, budget, recent)
    for method in ("rank", "sort"):
        got = ora.select_keep(sc, pos, ln, budget, recent, method)
        assert got[0, 0].tolist() == want


@pytest.mark.parametrize("ties", [0, 2, 7])
def test_rank_counting_and_sorting_agree(ora, ties):
    Bt, Hkv, cap, budget, recent = 3, 4, 300, 200, 32
    sc = si.gen_scores(7 + ties, (Bt, Hkv, cap), ties=ties)
    ln = np.array([300, 257, 120], np.int32)
    pos = np.tile(np.arange(cap, dtype=np.int32) * 2 + 1, (Bt, Hkv, 1))
    a = ora.select_keep(sc, pos, ln, budget, recent, "rank")
    b = ora.select_keep(sc, pos, ln, budget, recent, "sort")
    assert np.array_equal(a, b)
    # rows over budget hold exactly `budget` distinct ascending slots; the under-budget row is the identity
    for bi in range(2):
        for h in range(Hkv):
            row = a[bi, h]
            assert (np.diff(row) > 0).all() and row[0] >= 0 and row[-1] == ln[bi] - 1
            assert np.array_equal(row[-recent:], np.arange(ln[bi] - recent, ln[bi]))
    assert np.array_equal(a[2, :, :120], np.tile(np.arange(120), (Hkv, 1)))
    assert (a[2, :, 120:] == -1).all()


def test_all_scores_equal_keeps_lowest_positions_and_recent(ora):
    n, budget, recent = 40, 25, 5
    sc = np.full((1, 1, n), 0.75, np.float32)
    pos = (np.arange(n, dtype=np.int32) * 4 + 9)[None, None]
    got = ora.select_keep(sc, pos, np.array([n], np.int32), budget, recent)[0, 0]
    assert got.tolist() == list(range(20)) + list(range(35, 40))


def test_increasing_scores_keep_the_last_budget_slots(ora):
    n, budget, recent = 40, 25, 5
    sc = np.linspace(-3, 3, n).astype(np.float32)[None, None]
    pos = np.arange(n, dtype=np.int32)[None, None]
    got = ora.select_keep(sc, pos, np.array([n], np.int32), budget, recent)[0, 0]
    assert got.tolist() == list(range(15, 40))


def test_decreasing_scores_keep_head_and_recent(ora):
    n, budget, recent = 40, 25, 5
    sc = np.linspace(3, -3, n).astype(np.float32)[None, None]
    pos = np.arange(n, dtype=np.int32)[None, None]
    got = ora.select_keep(sc, pos, np.array([n], np.int32), budget, recent)[0, 0]
    assert got.tolist() == list(range(20)) + list(range(35, 40))


def test_special_values_order(ora):
    # ranking: +inf > 1 > +0 == -0 > -1 > -inf > NaN ; ties toward the lower position
    sc = np.array([np.nan, -np.inf, -0.0, 0.0, 1.0, np.inf, -1.0, np.nan, 5.0, 5.0], np.float32)[None, None]
    pos = np.arange(10, dtype=np.int32)[None, None]
    ln = np.array([10], np.int32)
    # recent = 2 protects slots 8, 9; candidates 0..7
    expect_order = [5, 4, 2, 3, 6, 1, 0, 7]
    for k in range(1, 8):
        got = ora.select_keep(sc, pos, ln, k + 2, 2)[0, 0].tolist()
        assert got == sorted(expect_order[:k]) + [8, 9], k


def test_recent_is_by_position_and_result_is_permutation_invariant(ora):
    n, budget, recent, cap = 64, 40, 8, 64
    sc = si.gen_scores(55, (1, 1, cap), ties=5)
    pos = (np.arange(n, dtype=np.int32) * 3)[None, None]
    ln = np.array([n], np.int32)
    base = ora.select_keep(sc, pos, ln, budget, recent)[0, 0]
    kept_positions = set(pos[0, 0, base].tolist())
    assert set(range(3 * (n - recent), 3 * n, 3)) <= kept_positions
    rng = np.random.default_rng(3)
    for _ in range(4):
        p = rng.permutation(n)
        got = ora.select_keep(np.ascontiguousarray(sc[:, :, p]), np.ascontiguousarray(pos[:, :, p]), ln, budget, recent)[0, 0]
        assert (np.diff(got) > 0).all()
        assert set(pos[0, 0, p][got].tolist()) == kept_positions


def test_bad_budget_is_rejected(ora):
    sc = np.zeros((1, 1, 8), np.float32)
    pos = np.arange(8, dtype=np.int32)[None, None]
    with pytest.raises(RuntimeError):
        ora.select_keep(sc, pos, np.array([8], np.int32), 4, 5)


# ----------------------------------------------------------------------------- compaction

@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compaction_equals_library_gather(ora, dtype):
    Bt, Hkv, cap, D, budget = 3, 2, 48, 16, 30
    c = random_cache(ora, 61, dtype, Bt, Hkv, cap, D, lens=[48, 31, 20])
    before = c.copy()
    rng = np.random.default_rng(5)
    keep = np.full((Bt, Hkv, budget), -1, np.int32)
    for b in range(Bt):
        for h in range(Hkv):
            n = int(c.len[b])
            keep[b, h, :min(n, budget)] = np.sort(rng.choice(n, size=budget, replace=False)) if n > budget else np.arange(n)
    ora.compact(c, keep, budget)
    assert c.len.tolist() == [30, 30, 20]
    for b in range(2):
        for h in range(Hkv):
            idx = keep[b, h]
            assert np.array_equal(c.K[b, h, :budget], before.K[b, h][idx])
            assert np.array_equal(c.V[b, h, :budget], before.V[b, h][idx])
            assert np.array_equal(c.pos[b, h, :budget], before.pos[b, h][idx])
            assert (np.diff(c.pos[b, h, :budget]) > 0).all()
    # the row at or under budget is untouched, bit for bit
    assert np.array_equal(c.K[2], before.K[2]) and np.array_equal(c.V[2], before.V[2]) and np.array_equal(c.pos[2], before.pos[2])


def test_compaction_identity_and_idempotence(ora):
    c = random_cache(ora, 62, "f32", 1, 1, 20, 8, lens=[20])
    before = c.copy()
    keep = np.arange(16, dtype=np.int32)[None, None]
    ora.compact(c, keep, 16)                       # keep the first 16: nothing moves
    assert c.len[0] == 16 and np.array_equal(c.K[0, 0, :16], before.K[0, 0, :16])
    again = c.copy()
    ora.compact(c, keep, 16)                       # len == budget now: no-op
    assert np.array_equal(c.K, again.K) and np.array_equal(c.pos, again.pos) and c.len[0] == 16


@pytest.mark.parametrize("pattern", ["first", "every_other", "block", "last_protected"])
def test_compaction_adversarial_overlaps(ora, pattern):
    """Patterns where a destination slot of one moved pair is the source slot of another."""
    n, budget, D = 64, 32, 4
    c = random_cache(ora, 63, "f32", 1, 1, n, D, lens=[n])
    before = c.copy()
    idx = {"first": np.arange(32, 64), "every_other": np.arange(0, 64, 2) + 1,
           "block": np.r_[np.arange(10), np.arange(42, 64)], "last_protected": np.r_[np.arange(0, 62, 2)[:31], 63]}[pattern]
    idx = np.sort(idx).astype(np.int32)
    ora.compact(c, idx[None, None], budget)
    assert np.array_equal(c.K[0, 0, :budget], before.K[0, 0][idx])
    assert np.array_equal(c.V[0, 0, :budget], before.V[0, 0][idx])
    assert np.array_equal(c.pos[0, 0, :budget], before.pos[0, 0][idx])
