"""Pins for the oracle's retained-set attention (Appendix A, Problem Setup and Proposition A.1).

None of these re-types the oracle's loop: they are a library softmax + einsum on the same
stored values, closed forms, and the paper's renormalisation identities and error bound.
"""
import numpy as np
import pytest
from scipy.special import softmax

from util import random_cache, random_q, widen


def lib_attention(c, q, scale, g):
    """softmax(scale q K^T) V with scipy/numpy on the retained slots, GQA head h -> KV head h // g."""
    Bt, Hkv, cap, D = c.shape
    K, V, Q = widen(c.K, c.dtype), widen(c.V, c.dtype), widen(q, c.dtype)
    out = np.zeros((Bt, Q.shape[1], D))
    for b in range(Bt):
        n = int(c.len[b])
        for h in range(Q.shape[1]):
            logits = scale * (K[b, h // g, :n] @ Q[b, h])
            out[b, h] = softmax(logits) @ V[b, h // g, :n]
    return out


@pytest.mark.parametrize("dtype,D,Hq,Hkv", [("f32", 64, 8, 2), ("bf16", 128, 8, 2), ("bf16", 128, 7, 1), ("f32", 32, 3, 3)])
def test_matches_library_softmax_attention(ora, dtype, D, Hq, Hkv):
    Bt, cap = 3, 50
    c = random_cache(ora, 11, dtype, Bt, Hkv, cap, D, lens=[50, 17, 1])
    q = random_q(12, dtype, Bt, Hq, D)
    for scale in (D ** -0.5, 1.0):
        got = ora.decode_attn(c, q, scale)
        ref = lib_attention(c, q, scale, Hq // Hkv)
        np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-13)


def test_slots_beyond_len_are_ignored(ora):
    c = random_cache(ora, 3, "f32", 2, 2, 40, 16, lens=[10, 25])
    q = random_q(4, "f32", 2, 4, 16)
    a = ora.decode_attn(c, q, 0.25)
    c.K[0, :, 10:] = 1e6
    c.V[0, :, 10:] = -1e6
    c.K[1, :, 25:] = np.nan
    b = ora.decode_attn(c, q, 0.25)
    assert np.array_equal(a, b)


def test_identical_keys_give_mean_of_values(ora):
    c = random_cache(ora, 5, "f32", 1, 2, 33, 16, lens=[33])
    c.K[...] = c.K[:, :, :1]            # every key of a row equals the first one
    q = random_q(6, "f32", 1, 6, 16)
    out = ora.decode_attn(c, q, 0.7)
    mean_v = c.V.astype(np.float64).mean(axis=2)      # [1, Hkv, D]
    for h in range(6):
        np.testing.assert_allclose(out[0, h], mean_v[0, h // 3], rtol=1e-13, atol=1e-15)


def test_single_key_returns_its_value(ora):
    c = random_cache(ora, 7, "bf16", 2, 2, 8, 32, lens=[1, 1])
    q = random_q(8, "bf16", 2, 4, 32)
    out = ora.decode_attn(c, q, 1.0)
    V = widen(c.V, "bf16")
    for h in range(4):
        assert np.array_equal(out[:, h], V[:, h // 2, 0])


def test_dominant_logit_selects_that_value(ora):
    D = 16
    c = random_cache(ora, 9, "f32", 1, 1, 20, D, lens=[20], scale=0.01)
    q = random_q(10, "f32", 1, 2, D)
    j = 13
    c.K[0, 0, j] = 500.0 * q[0, 0]      # logit of key j for head 0 is 500 |q|^2 >> all others
    out = ora.decode_attn(c, q, 1.0)
    np.testing.assert_allclose(out[0, 0], c.V[0, 0, j].astype(np.float64), rtol=0, atol=1e-12)


def test_two_keys_closed_form(ora):
    # logits l0, l1 -> weights sigmoid(l0 - l1), sigmoid(l1 - l0)
    D = 4
    c = ora.new_cache("f32", 1, 1, 4, D)
    c.K[0, 0, 0] = [1, 0, 0, 0]
    c.K[0, 0, 1] = [0, 2, 0, 0]
    c.V[0, 0, 0] = [1, 2, 3, 4]
    c.V[0, 0, 1] = [-1, 0, 5, 8]
    c.len[0] = 2
    q = np.array([[[0.5, 0.75, 9, 9]]], np.float32)
    scale = 2.0
    l0, l1 = scale * 0.5, scale * 1.5
    w0 = 1.0 / (1.0 + np.exp(l1 - l0))
    want = w0 * np.array([1, 2, 3, 4.0]) + (1 - w0) * np.array([-1, 0, 5, 8.0])
    np.testing.assert_allclose(ora.decode_attn(c, q, scale)[0, 0], want, rtol=1e-14)


def test_invariant_under_slot_permutation(ora):
    c = random_cache(ora, 21, "f32", 2, 2, 64, 32, lens=[64, 40])
    q = random_q(22, "f32", 2, 8, 32)
    a = ora.decode_attn(c, q, 32 ** -0.5)
    rng = np.random.default_rng(0)
    for b in range(2):
        n = int(c.len[b])
        for h in range(2):
            p = rng.permutation(n)
            c.K[b, h, :n] = c.K[b, h, :n][p]
            c.V[b, h, :n] = c.V[b, h, :n][p]
            c.pos[b, h, :n] = c.pos[b, h, :n][p]
    b_ = ora.decode_attn(c, q, 32 ** -0.5)
    np.testing.assert_allclose(a, b_, rtol=1e-12, atol=1e-14)


def test_renormalisation_identities_and_error_bound(ora):
    """Appendix A: with eps = evicted mass of the full softmax, a_hat = a / (1 - eps),
    o_hat = h_S / (1 - eps), and Proposition A.1: |o - o_hat|_2 <= 2 C eps, C = max |v|_2."""
    D, n = 32, 96
    full = random_cache(ora, 31, "f32", 1, 1, n, D, lens=[n])
    q = random_q(32, "f32", 1, 4, D)
    scale = 0.5
    o = ora.decode_attn(full, q, scale)                       # [1, 4, D]
    K, V, Q = full.K.astype(np.float64), full.V.astype(np.float64), q.astype(np.float64)
    rng = np.random.default_rng(1)
    for trial in range(5):
        kept = np.sort(rng.choice(n, size=n - 20 - 5 * trial, replace=False))
        ev = np.setdiff1d(np.arange(n), kept)
        sub = ora.new_cache("f32", 1, 1, n, D)
        sub.K[0, 0, :len(kept)] = full.K[0, 0, kept]
        sub.V[0, 0, :len(kept)] = full.V[0, 0, kept]
        sub.len[0] = len(kept)
        o_hat = ora.decode_attn(sub, q, scale)
        C = np.linalg.norm(V[0, 0], axis=1).max()
        for h in range(4):
            a = softmax(scale * (K[0, 0] @ Q[0, h]))              # full attention weights
            eps = a[ev].sum()
            h_S = a[kept] @ V[0, 0, kept]
            np.testing.assert_allclose(o_hat[0, h], h_S / (1.0 - eps), rtol=1e-10, atol=1e-13)
            err = np.linalg.norm(o[0, h] - o_hat[0, h])
            assert err <= 2.0 * C * eps * (1 + 1e-9)
            # the bound is not vacuous on this data
            assert eps > 1e-3
