"""Pins for the oracle's MLP scorer (Appendix B.1: phi = sigma(x W1 + b1) W2 + b2, x = [k, v])."""
import numpy as np
import pytest
import torch

from util import random_cache, store, widen
import synth_inputs as si

# Phi(1), Phi(2), Phi(3): standard normal CDF values (textbook table), GELU(x) = x Phi(x)
PHI = {1.0: 0.8413447460685429, 2.0: 0.9772498680518208, 3.0: 0.9986501019683699}


def rand_weights(seed, dtype, nset, F, H):
    w1 = (si.normal(seed, si.T_W1, 0, np.arange(nset * F * H)).reshape(nset, F, H) / np.sqrt(F)).astype(np.float32)
    b1 = (si.normal(seed, si.T_B1, 0, np.arange(nset * H)).reshape(nset, H) * 0.3).astype(np.float32)
    w2 = (si.normal(seed, si.T_W2, 0, np.arange(nset * H)).reshape(nset, H) / np.sqrt(H)).astype(np.float32)
    b2 = (si.normal(seed, si.T_B2, 0, np.arange(nset)) * 0.5).astype(np.float32)
    return store(w1, dtype), b1, w2, b2


@pytest.mark.parametrize("dtype,D,H,shared", [("f32", 64, 64, False), ("bf16", 128, 256, False), ("bf16", 32, 16, True),
                                               ("f32", 16, 5, False)])
def test_matches_library_mlp(ora, dtype, D, H, shared):
    Bt, Hkv, cap = 2, 3, 21
    c = random_cache(ora, 41, dtype, Bt, Hkv, cap, D, lens=[21, 9])
    W1, b1, W2, b2 = rand_weights(42, dtype, 1 if shared else Hkv, 2 * D, H)
    got = ora.score_kv(c, W1, b1, W2, b2)
    K, V = torch.from_numpy(widen(c.K, dtype)), torch.from_numpy(widen(c.V, dtype))
    x = torch.cat([K, V], dim=-1)                                     # [Bt,Hkv,cap,2D]
    for h in range(Hkv):
        hw = 0 if shared else h
        w1 = torch.from_numpy(widen(W1[hw], dtype))                   # [F,H]
        hid = torch.nn.functional.gelu(
            torch.nn.functional.linear(x[:, h], w1.T.contiguous(), torch.from_numpy(b1[hw].astype(np.float64))),
            approximate="none")
        phi = torch.nn.functional.linear(hid, torch.from_numpy(W2[hw].astype(np.float64))[None, :],
                                         torch.from_numpy(b2[hw:hw + 1].astype(np.float64)))[..., 0]
        for b in range(Bt):
            n = int(c.len[b])
            np.testing.assert_allclose(got[b, h, :n], phi[b, :n].numpy(), rtol=1e-11, atol=1e-13)
            assert np.isnan(got[b, h, n:]).all()


def test_zero_first_layer_gives_constant_score(ora):
    D, H = 8, 4
    c = random_cache(ora, 43, "f32", 1, 1, 10, D, lens=[10])
    W1 = np.zeros((1, 2 * D, H), np.float32)
    b1 = np.array([[1.0, 2.0, 3.0, 0.0]], np.float32)
    W2 = np.array([[2.0, -1.0, 0.5, 7.0]], np.float32)
    b2 = np.array([0.25], np.float32)
    want = 2.0 * 1 * PHI[1.0] - 1.0 * 2 * PHI[2.0] + 0.5 * 3 * PHI[3.0] + 7.0 * 0.0 + 0.25
    got = ora.score_kv(c, W1, b1, W2, b2)[0, 0, :10]
    np.testing.assert_allclose(got, want, rtol=1e-14)


def test_zero_second_layer_gives_bias(ora):
    D, H = 8, 6
    c = random_cache(ora, 44, "f32", 2, 2, 10, D, lens=[10, 3])
    W1, b1, W2, b2 = rand_weights(45, "f32", 2, 2 * D, H)
    W2[...] = 0
    got = ora.score_kv(c, W1, b1, W2, b2)
    for h in range(2):
        assert np.array_equal(got[0, h, :10], np.full(10, np.float64(b2[h])))
        assert np.array_equal(got[1, h, :3], np.full(3, np.float64(b2[h])))


@pytest.mark.parametrize("f", [0, 5, 8, 15])
def test_one_hot_first_layer_picks_feature_and_order_of_concat(ora, f):
    """H = 1, W1 = e_f: phi = w2 gelu(x_f + b1) + b2 with x = [k (D entries), v (D entries)]."""
    D = 8
    c = ora.new_cache("f32", 1, 1, 8, D)
    vals = np.array([1.0, 2.0, 3.0, -1.0, -2.0, 0.0, 40.0, -40.0])
    c.len[0] = 8
    # put distinct garbage everywhere, the probed feature gets vals
    c.K[0, 0] = 0.123
    c.V[0, 0] = -0.456
    (c.K if f < D else c.V)[0, 0, :, f % D] = vals
    W1 = np.zeros((1, 2 * D, 1), np.float32)
    W1[0, f, 0] = 1.0
    b1 = np.zeros((1, 1), np.float32)
    W2 = np.array([[3.0]], np.float32)
    b2 = np.array([-0.5], np.float32)
    got = ora.score_kv(c, W1, b1, W2, b2)[0, 0, :8]
    gelu = np.array([PHI[1.0], 2 * PHI[2.0], 3 * PHI[3.0], -(1 - PHI[1.0]), -2 * (1 - PHI[2.0]), 0.0, 40.0, 0.0])
    np.testing.assert_allclose(got, 3.0 * gelu - 0.5, rtol=1e-13, atol=1e-13)


def test_first_layer_bias_enters_before_activation(ora):
    D = 4
    c = ora.new_cache("f32", 1, 1, 2, D)
    c.len[0] = 2
    c.K[0, 0, :, 0] = [0.5, -1.5]
    W1 = np.zeros((1, 2 * D, 1), np.float32)
    W1[0, 0, 0] = 2.0                      # z = 2 k_0 + b1 = 1 + 1, -3 + 1
    got = ora.score_kv(c, W1, np.array([[1.0]], np.float32), np.array([[1.0]], np.float32), np.array([0.0], np.float32))
    np.testing.assert_allclose(got[0, 0, :2], [2 * PHI[2.0], -2 * (1 - PHI[2.0])], rtol=1e-13)


def test_per_head_weights_are_indexed_by_kv_head(ora):
    D, H = 8, 3
    c = random_cache(ora, 46, "f32", 2, 2, 6, D, lens=[6, 6])
    W1, b1, W2, b2 = rand_weights(47, "f32", 2, 2 * D, H)
    both = ora.score_kv(c, W1, b1, W2, b2)
    for h in range(2):
        one = ora.new_cache("f32", 2, 1, 6, D)
        one.K[:, 0], one.V[:, 0], one.len[...] = c.K[:, h], c.V[:, h], c.len
        alone = ora.score_kv(one, W1[h:h + 1], b1[h:h + 1], W2[h:h + 1], b2[h:h + 1])
        assert np.array_equal(both[:, h], alone[:, 0])
