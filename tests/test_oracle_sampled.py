"""Pins for the oracle's Top-K multinomial eviction (Section 3.1 Eq. 2, Appendix B.2): candidates are
the lowest-scored pairs, the evicted ones are drawn from them without replacement with probabilities
softmax(-score); the oracle takes the draw in Gumbel-top-k form on noise passed in."""
import itertools

import numpy as np
import pytest

import synth_inputs as si


def test_zero_noise_or_no_slack_reduces_to_deterministic_topk(ora):
    Bt, Hkv, cap, budget, recent = 2, 3, 260, 200, 32
    sc = si.gen_scores(901, (Bt, Hkv, cap), ties=5)
    pos = np.tile(np.arange(cap, dtype=np.int32) * 2, (Bt, Hkv, 1))
    ln = np.array([260, 231], np.int32)
    det = ora.select_keep(sc, pos, ln, budget, recent, "sort")
    zero = np.zeros_like(sc)
    wild = (si.normal(902, si.T_SCORE, 1, np.arange(sc.size)).reshape(sc.shape) * 50).astype(np.float32)
    for n_cand in (0, 1, 60, 120, 10000):
        assert np.array_equal(ora.select_keep_sampled(sc, zero, pos, ln, budget, recent, n_cand), det)
    # n_cand <= number to evict (60 and 31): every candidate goes, whatever the noise
    assert np.array_equal(ora.select_keep_sampled(sc, wild, pos, ln, budget, recent, 31), det)


def test_safe_pairs_and_recent_pairs_survive_any_noise(ora):
    cap, budget, recent, n_cand = 300, 200, 20, 150          # evict 100 of the 150 lowest
    sc = si.gen_scores(903, (1, 1, cap))
    pos = np.arange(cap, dtype=np.int32)[None, None]
    ln = np.array([cap], np.int32)
    order = np.argsort(-sc[0, 0, :cap - recent], kind="stable")          # distinct scores: plain ranking
    safe = set(order[:cap - recent - n_cand].tolist())
    for seed in range(5):
        noise = (si.normal(910 + seed, si.T_SCORE, 2, np.arange(cap)) * 100).astype(np.float32)[None, None]
        keep = ora.select_keep_sampled(sc, noise, pos, ln, budget, recent, n_cand)[0, 0]
        ks = set(keep.tolist())
        assert len(ks) == budget and (np.diff(keep) > 0).all()
        assert safe <= ks and set(range(cap - recent, cap)) <= ks
    # with strong noise the draw differs from the deterministic rule
    det = ora.select_keep(sc, pos, ln, budget, recent)[0, 0]
    assert not np.array_equal(keep, det)


def brute_force(scores, noise, pos, n, budget, recent, n_cand):
    newest = sorted(range(n), key=lambda i: -pos[i])[:recent]
    others = [i for i in range(n) if i not in newest]
    imp = sorted(others, key=lambda i: (-float(scores[i]), pos[i]))       # most important first
    E = n - budget
    K = min(max(n_cand, E), len(others))
    safe, cand = imp[:len(imp) - K], imp[len(imp) - K:]
    t = {i: np.float32(scores[i]) - np.float32(noise[i]) for i in cand}
    kept_c = sorted(cand, key=lambda i: (-float(t[i]), pos[i]))[:K - E]
    return sorted(newest + safe + kept_c)


@pytest.mark.parametrize("seed", range(8))
def test_small_rows_against_plain_python(ora, seed):
    rng = np.random.default_rng(seed)
    n, cap = 40, 48
    budget, recent, n_cand = int(rng.integers(10, 36)), int(rng.integers(0, 8)), int(rng.integers(0, 30))
    recent = min(recent, budget)
    sc = (np.round(rng.normal(size=(1, 1, cap)) * 2) / 2).astype(np.float32)      # many ties
    noise = (np.round(rng.gumbel(size=(1, 1, cap)) * 2) / 2).astype(np.float32)
    pos = np.full((1, 1, cap), -1, np.int32)
    pos[0, 0, :n] = np.sort(rng.permutation(200)[:n]) if seed % 2 else rng.permutation(200)[:n]
    got = ora.select_keep_sampled(sc, noise, pos, np.array([n], np.int32), budget, recent, n_cand)[0, 0]
    assert got.tolist() == brute_force(sc[0, 0], noise[0, 0], pos[0, 0], n, budget, recent, n_cand)


def test_draw_has_the_law_of_sampling_without_replacement(ora):
    """4 candidates, 2 evicted: the frequency of every evicted pair under Gumbel noise matches
    P({a,b}) = p_a p_b / (1 - p_a) + p_b p_a / (1 - p_b), p = softmax(-score): the law of two
    successive multinomial draws without replacement (Eq. 2)."""
    trials = 60000
    phi = np.array([0.3, -0.5, 1.2, 0.1], np.float64)                    # candidate scores
    high = np.array([5.0, 6.0, 7.0])                                      # safe pairs
    recent = 2
    row = np.concatenate([high, phi, [0.0, 0.0]]).astype(np.float32)      # 9 entries, last 2 protected
    n = len(row)
    sc = np.tile(row, (trials, 1, 1))
    pos = np.tile(np.arange(n, dtype=np.int32), (trials, 1, 1))
    rng = np.random.default_rng(7)
    noise = rng.gumbel(size=(trials, 1, n)).astype(np.float32)
    keep = ora.select_keep_sampled(sc, noise, pos, np.full(trials, n, np.int32), n - 2, recent, 4)
    p = np.exp(-phi) / np.exp(-phi).sum()
    counts = {}
    for r in range(trials):
        ev = tuple(sorted(set(range(n)) - set(keep[r, 0].tolist())))
        counts[ev] = counts.get(ev, 0) + 1
    assert all(3 <= a <= 6 and 3 <= b <= 6 for a, b in counts)           # only candidates are evicted
    for a, b in itertools.combinations(range(4), 2):
        want = p[a] * p[b] / (1 - p[a]) + p[b] * p[a] / (1 - p[b])
        got = counts.get((a + 3, b + 3), 0) / trials
        sigma = np.sqrt(want * (1 - want) / trials)
        assert abs(got - want) < 5 * sigma, (a, b, got, want)
