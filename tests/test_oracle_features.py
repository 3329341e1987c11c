"""Pins for the oracle's attention features (Appendix B.1, "Attention Features": recent-window sums
over 8 / 16 / 32 / L queries, cumulative sum over chunks, sum decayed by 0.9 per chunk) and for the
scorer on x = concat(k, v, a) (Section 3.1 Eq. 1)."""
import numpy as np
import torch
from scipy.special import softmax

import synth_inputs as si
from util import random_cache, random_q, store, widen

PHI1 = 0.8413447460685429


def test_probs_are_the_softmax_weights_and_out_is_unchanged(ora):
    c = random_cache(ora, 71, "bf16", 2, 2, 40, 32, lens=[40, 13])
    q = random_q(72, "bf16", 2, 6, 32)
    out, probs = ora.decode_attn_probs(c, q, 0.4)
    assert np.array_equal(out, ora.decode_attn(c, q, 0.4))
    K, Q = widen(c.K, "bf16"), widen(q, "bf16")
    for b, n in ((0, 40), (1, 13)):
        for h in range(6):
            np.testing.assert_allclose(probs[b, h, :n], softmax(0.4 * (K[b, h // 3, :n] @ Q[b, h])), rtol=1e-12, atol=1e-15)
            assert (probs[b, h, n:] == 0).all() and abs(probs[b, h].sum() - 1) < 1e-12


def test_feature_bookkeeping_against_the_definition_on_the_full_history(ora):
    """A small run with real evictions.  The test keeps, per absolute position, the weight the pair got
    from every query (recomputed with scipy from the cache contents), and at every event rebuilds the
    six features of every retained pair from that history by their definition."""
    Bt, Hkv, g, D, P, B, L, steps = 1, 2, 2, 8, 50, 90, 40, 205
    cap = B + L
    rngK = (si.normal(81, si.T_K, 0, np.arange(Hkv * (P + steps) * D)).reshape(Hkv, P + steps, D)).astype(np.float32)
    rngV = (si.normal(81, si.T_V, 0, np.arange(Hkv * (P + steps) * D)).reshape(Hkv, P + steps, D)).astype(np.float32)
    rngQ = (si.normal(81, si.T_Q, 0, np.arange(Hkv * g * steps * D)).reshape(Hkv * g, steps, D)).astype(np.float32)
    c = ora.new_cache("f32", Bt, Hkv, cap, D)
    c.K[0, :, :P], c.V[0, :, :P], c.pos[0, :, :P], c.len[0] = rngK[:, :P], rngV[:, :P], np.arange(P), P
    feat = ora.new_feat(Bt, Hkv, cap, g)
    F = 2 * D + 6 * g
    W1 = (si.normal(82, si.T_W1, 0, np.arange(Hkv * F * 12)).reshape(Hkv, F, 12) / 3).astype(np.float32)
    b1 = np.zeros((Hkv, 12), np.float32)
    W2 = (si.normal(82, si.T_W2, 0, np.arange(Hkv * 12)).reshape(Hkv, 12)).astype(np.float32)
    b2 = np.zeros(Hkv, np.float32)
    hist = {}            # (hkv, head, position) -> list of (step, weight)
    events = 0
    for t in range(steps):
        n0 = c.len.copy()
        ora.append(c, rngK[None, :, P + t], rngV[None, :, P + t], np.array([P + t], np.int32))
        q = np.ascontiguousarray(rngQ[None, :, t])
        out, probs = ora.decode_attn_probs(c, q, 0.5)
        ora.feat_step(feat, probs, n0, t % L, L)
        n = int(c.len[0])
        for hk in range(Hkv):
            for j in range(g):
                w = softmax(0.5 * (c.K[0, hk, :n].astype(np.float64) @ q[0, hk * g + j].astype(np.float64)))
                for i in range(n):
                    hist.setdefault((hk, j, int(c.pos[0, hk, i])), []).append((t, w[i]))
        if (t + 1) % L == 0:
            events += 1
            fv = ora.feat_vectors(feat)                                    # [1,Hkv,cap,6g]
            for hk in range(Hkv):
                for i in range(n):
                    for j in range(g):
                        hs = hist[(hk, j, int(c.pos[0, hk, i]))]
                        want = []
                        for wnd in (8, 16, 32, L):
                            want.append(sum(w for (s, w) in hs if t - min(wnd, L) < s <= t))
                        want.append(sum(w for (s, w) in hs))
                        chunk_of = lambda s: s // L
                        want.append(sum(w * 0.9 ** (chunk_of(t) - chunk_of(s)) for (s, w) in hs))
                        np.testing.assert_allclose(fv[0, hk, i, 6 * j:6 * j + 6], want, rtol=1e-10, atol=1e-14)
            sc = ora.score_kv_feat(c, fv, W1, b1, W2, b2)
            keep = ora.select_keep(sc.astype(np.float32), c.pos, c.len, B, L)
            before = c.len.copy()
            ora.compact(c, keep, B)
            ora.feat_roll_and_compact(feat, keep, before, B)
            assert (feat[0, :, :, :, :4] == 0).all()
    assert events == 5 and c.len[0] == B + steps % L


def test_identical_keys_closed_form(ora):
    """All keys equal: every weight is 1/n, so after a chunk of L queries over a cache growing from
    n0+1 to n0+L an old pair has wL = sum_{k=1..L} 1/(n0+k) and w8 the last 8 terms."""
    Bt, Hkv, g, D, n0, L = 1, 1, 3, 4, 20, 12
    c = ora.new_cache("f32", Bt, Hkv, 64, D)
    c.K[...] = 0.25
    c.len[0] = n0
    feat = ora.new_feat(Bt, Hkv, 64, g)
    q = np.ones((1, g, D), np.float32)
    for t in range(L):
        before = c.len.copy()
        ora.append(c, np.full((1, 1, D), 0.25, np.float32), np.zeros((1, 1, D), np.float32), np.array([100 + t], np.int32))
        _, probs = ora.decode_attn_probs(c, q, 1.0)
        ora.feat_step(feat, probs, before, t, L)
    fv = ora.feat_vectors(feat)[0, 0]
    terms = np.array([1.0 / (n0 + k) for k in range(1, L + 1)])
    for j in range(g):
        np.testing.assert_allclose(fv[5, 6 * j:6 * j + 6], [terms[-8:].sum(), terms.sum(), terms.sum(), terms.sum(), terms.sum(), terms.sum()], rtol=1e-13)
    # the pair appended at chunk step 9 has only seen queries 9, 10, 11
    np.testing.assert_allclose(fv[n0 + 9, :6], [terms[9:].sum()] * 6, rtol=1e-13)


def test_scorer_with_features_matches_library_mlp_and_feature_order(ora):
    Bt, Hkv, cap, D, g, H = 2, 2, 15, 16, 2, 10
    A = 6 * g
    c = random_cache(ora, 91, "bf16", Bt, Hkv, cap, D, lens=[15, 7])
    fvec = np.abs(si.normal(92, si.T_SCORE, 0, np.arange(Bt * Hkv * cap * A)).reshape(Bt, Hkv, cap, A)) * 3
    F = 2 * D + A
    W1 = store((si.normal(93, si.T_W1, 0, np.arange(Hkv * F * H)).reshape(Hkv, F, H) / np.sqrt(F)).astype(np.float32), "bf16")
    b1 = (si.normal(93, si.T_B1, 0, np.arange(Hkv * H)).reshape(Hkv, H) * 0.1).astype(np.float32)
    W2 = (si.normal(93, si.T_W2, 0, np.arange(Hkv * H)).reshape(Hkv, H)).astype(np.float32)
    b2 = np.array([0.5, -0.25], np.float32)
    got = ora.score_kv_feat(c, fvec, W1, b1, W2, b2)
    x = torch.cat([torch.from_numpy(widen(c.K, "bf16")), torch.from_numpy(widen(c.V, "bf16")), torch.from_numpy(fvec)], dim=-1)
    for h in range(Hkv):
        hid = torch.nn.functional.gelu(torch.nn.functional.linear(x[:, h], torch.from_numpy(widen(W1[h], "bf16")).T.contiguous(),
                                                                  torch.from_numpy(b1[h].astype(np.float64))), approximate="none")
        phi = hid @ torch.from_numpy(W2[h].astype(np.float64)) + float(b2[h])
        for b, n in ((0, 15), (1, 7)):
            np.testing.assert_allclose(got[b, h, :n], phi[b, :n].numpy(), rtol=1e-11, atol=1e-13)
    # zero feature rows: the plain scorer
    W1z = si.from_bf16_bits(W1).copy()
    W1z[:, 2 * D:] = 0
    plain = ora.score_kv(c, store(W1z[:, :2 * D], "bf16"), b1, W2, b2)
    np.testing.assert_allclose(ora.score_kv_feat(c, fvec, store(W1z, "bf16"), b1, W2, b2)[0, :, :15], plain[0, :, :15], rtol=1e-13)
    # one-hot on feature a (head 1, plane 4): phi = gelu(a_value) for that entry
    W1o = np.zeros((1, F, 1), np.float32)
    W1o[0, 2 * D + 6 * 1 + 4, 0] = 1.0
    fv1 = np.zeros((1, 1, 4, A))
    fv1[0, 0, :, 6 * 1 + 4] = [1.0, 0.0, 1.0, 0.0]
    c1 = ora.new_cache("f32", 1, 1, 4, D)
    c1.len[0] = 4
    s1 = ora.score_kv_feat(c1, fv1, W1o, np.zeros((1, 1), np.float32), np.ones((1, 1), np.float32), np.zeros(1, np.float32))
    np.testing.assert_allclose(s1[0, 0], [PHI1, 0.0, PHI1, 0.0], rtol=1e-14, atol=1e-15)
