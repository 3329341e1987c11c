"""Parity of the attention-feature path (Appendix B.1) against the oracle: fk_decode_step_feat keeps the
six attention sums per (pair, query head), fk_score_kv_feat scores x = concat(k, v, a), fk_compact_feat
closes the chunk and compacts the features with the cache.

Tolerances.  The device forms the weights in fp32 from fp32 logits (bf16 products, fp32 accumulation
over 128 channels): a logit carries an absolute error of a few 1e-6 at |s| of order 10, so a weight is
off by a few 1e-6 relative, and a sum of up to L such weights by no more than that relative to the sum.
The bar is 2e-4 relative plus 1e-7 absolute.  Scores: the usual 1e-3 bar (features enter the MFMA as
bf16 head + remainder, 2^-17 relative).  Keep-sets, K, V, pos, len: bit exact (both sides select on the
oracle's fp32 scores)."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from util import bulk_step_inputs, workload_cache

pytestmark = pytest.mark.gpu

FEAT_RTOL, FEAT_ATOL = 2e-4, 1e-7


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    import paper_2602_03203_amd as fk
    fk.lib()
    return gpu_util


def dev_feat_rows(feat_dev, b, h, n, g):
    """device state [Bt,Hkv,6,cap,GP] -> [n, g, 6] float64 of one row (and the padded heads)."""
    f = feat_dev[b, h].cpu().numpy().astype(np.float64)          # [6, cap, GP]
    return f[:, :n, :g].transpose(1, 2, 0), f[:, :n, g:]


def assert_feat_close(got, ref, what):
    err = np.abs(got - ref) - (FEAT_ATOL + FEAT_RTOL * np.abs(ref))
    assert (err <= 0).all(), f"{what}: worst excess {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"


def lockstep_feat(gpu, ora, w, n_steps, sample_rows=None, scale=None, check_every=1, cold=False):
    import paper_2602_03203_amd as fk
    scale = w.softmax_scale if scale is None else scale
    lens0 = si.initial_lengths(w)
    B, L, g = w.budget, w.interval, w.group
    print(f"lockstep_feat {w.name}: g={g} B={B} L={L}", flush=True)
    full = workload_cache(ora, w)
    dev = gpu.DevCache(full, w.n_q_heads)
    dev.desc.cold = cold
    feat = fk.new_feat(dev.desc)
    fws = fk.new_feat_workspace(dev.desc)
    W1, b1, W2, b2 = si.gen_scorer_feat(w, 0)
    W1 = si.storage_array(W1, w.dtype)
    dW = [gpu.to_dev(x) for x in (W1, b1, W2, b2)]
    rows = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)] if sample_rows is None else sample_rows
    subs, ofeat = {}, {}
    for (b, h) in rows:
        subs[(b, h)] = ora.Cache(w.dtype, full.K[b:b + 1, h:h + 1].copy(), full.V[b:b + 1, h:h + 1].copy(),
                                 full.pos[b:b + 1, h:h + 1].copy(), full.len[b:b + 1].copy())
        ofeat[(b, h)] = ora.new_feat(1, 1, w.capacity, g)
    del full
    q_all, k_all, v_all, p_all = bulk_step_inputs(w, 0, 0, n_steps, lens0)
    dq, dk, dv, dp = (gpu.to_dev(x) for x in (q_all, k_all, v_all, p_all))
    keep_dev = torch.full((w.batch, w.n_kv_heads, B), -1, dtype=torch.int32, device="cuda")
    events = 0
    max_len = int(lens0.max())
    for t in range(n_steps):
        max_len += 1
        cp = t % L
        fk.fk_decode_step_feat(dev.desc, dq[t], dev.K, dev.V, dev.pos, dev.len, dk[t], dv[t], dp[t], min(max_len, w.capacity),
                               scale, feat, cp, L, dev.out, fws)
        check = t % check_every == 0 or (t + 1) % L == 0
        got = gpu.out_to_f64(dev.out) if check else None
        for (b, h), c in subs.items():
            n0 = c.len.copy()
            ora.append(c, k_all[t, b:b + 1, h:h + 1], v_all[t, b:b + 1, h:h + 1], p_all[t, b:b + 1])
            ref, probs = ora.decode_attn_probs(c, q_all[t, b:b + 1, h * g:(h + 1) * g], scale)
            ora.feat_step(ofeat[(b, h)], probs, n0, cp, L)
            if check:
                gpu.assert_attn_close(got[b, h * g:(h + 1) * g], ref[0], w.dtype, f"step {t} row ({b},{h})")
                n = int(c.len[0])
                f, pad = dev_feat_rows(feat, b, h, n, g)
                assert_feat_close(f, ofeat[(b, h)][0, 0, :n], f"features at step {t} row ({b},{h})")
                assert (pad == 0).all(), "padded heads must hold zeros"
        if (t + 1) % L == 0:
            print(f"  event after step {t}, max_len {max_len}", flush=True)
            ml = min(max_len, w.capacity)
            fk.fk_score_kv_feat(dev.desc, dev.K, dev.V, feat, dev.len, ml, *dW, dev.scores)
            own_h = dev.scores.cpu().numpy()
            inject = own_h.copy()
            refs = {}
            for (b, h), c in subs.items():
                n = int(c.len[0])
                fv = ora.feat_vectors(ofeat[(b, h)])
                sc = ora.score_kv_feat(c, fv, W1[h:h + 1], b1[h:h + 1], W2[h:h + 1], b2[h:h + 1])
                gpu.assert_scores_close(own_h[b:b + 1, h:h + 1], sc, [n], f"event at step {t}")
                # the features must matter: without them the scores differ by far more than the bar
                sc0 = ora.score_kv(c, np.ascontiguousarray(W1[h:h + 1, :2 * w.head_dim]), b1[h:h + 1], W2[h:h + 1], b2[h:h + 1])
                assert np.abs(sc0[0, 0, :n] - sc[0, 0, :n]).max() > 20e-3 * np.sqrt(np.mean(sc[0, 0, :n] ** 2))
                sc32 = sc.astype(np.float32)
                refs[(b, h)] = (sc32, n)
                inject[b, h, :n] = sc32[0, 0, :n]
            dev.scores.copy_(torch.from_numpy(inject).cuda())
            fk.fk_select_keep(dev.desc, dev.scores, dev.pos, dev.len, ml, B, L, keep_dev)
            keep_h = keep_dev.cpu().numpy()
            fk.fk_compact_feat(dev.desc, dev.K, dev.V, dev.pos, feat, dev.len, keep_dev, B)
            host = dev.host(ora)
            for (b, h), c in subs.items():
                sc32, n = refs[(b, h)]
                keep_ref = ora.select_keep(sc32, c.pos, c.len, B, L, "sort")
                if n > B:
                    assert np.array_equal(keep_h[b, h], keep_ref[0, 0]), f"keep-set differs at step {t}, row ({b},{h})"
                before = c.len.copy()
                ora.compact(c, keep_ref, B)
                ora.feat_roll_and_compact(ofeat[(b, h)], keep_ref, before, B)
                m = int(c.len[0])
                assert host.len[b] == m
                assert np.array_equal(host.pos[b, h, :m], c.pos[0, 0, :m])
                assert np.array_equal(host.K[b, h, :m], c.K[0, 0, :m]) and np.array_equal(host.V[b, h, :m], c.V[0, 0, :m])
                f, pad = dev_feat_rows(feat, b, h, m, g)
                assert_feat_close(f, ofeat[(b, h)][0, 0, :m], f"features after the event at step {t} row ({b},{h})")
                assert (f[:, :, :4] == 0).all() and (pad == 0).all()
            max_len = min(max_len, B) if max_len > B else max_len
            events += 1
    return events


def small(g, n_kv=2, batch=2, **kw):
    base = dict(name=f"feat-g{g}", batch=batch, n_q_heads=n_kv * g, n_kv_heads=n_kv, prompt=150, budget=192, interval=64,
                hidden=64, steps=300)
    base.update(kw)
    return si.config(1).scaled(**base)


@pytest.mark.parametrize("g", [4, 1, 7, 8, 3])
def test_small_runs_every_row_every_step(gpu, ora, g):
    """Several events, rows below and above budget, every group size class (padding 4 and 8)."""
    w = small(g)
    assert lockstep_feat(gpu, ora, w, 300) == 4


def test_events_on_rows_still_under_budget(gpu, ora):
    """Short prompt: the first two events find every row under budget (the chunk is closed, nothing moves)."""
    w = small(4, prompt=60)
    assert lockstep_feat(gpu, ora, w, 260) == 4


def test_cold_cache_hint(gpu, ora):
    """The cold-cache flag (non-temporal K / V loads) on the feature path: same parity."""
    assert lockstep_feat(gpu, ora, small(4), 150, cold=True) == 2
    assert lockstep_feat(gpu, ora, small(7), 70, cold=True) == 1


def test_interval_shorter_than_the_windows(gpu, ora):
    """L = 16: the 16- and 32-query windows cover the whole chunk, the 8-query window half of it."""
    w = small(4, interval=16, budget=96, prompt=90)
    assert lockstep_feat(gpu, ora, w, 100) == 6


def test_peaked_softmax(gpu, ora):
    w = small(4)
    lockstep_feat(gpu, ora, w, 140, scale=1.0)


def test_ragged_tail_lengths(gpu, ora):
    """Budget and interval that are no multiples of the 32-key tile."""
    w = small(2, interval=37, budget=131, prompt=100, batch=3)
    assert lockstep_feat(gpu, ora, w, 160) == 4


def test_qwen3_4b_layer_shape_sampled_rows(gpu, ora):
    """configs[1] shapes (batch 16, 32/8 heads, D 128, bf16, B 2048, L 128, H 256) with a long prompt so that
    two events fall inside 300 steps; the oracle follows 3 sampled rows."""
    w = si.config(1).scaled(prompt=1920)
    assert lockstep_feat(gpu, ora, w, 300, sample_rows=[(0, 0), (7, 3), (15, 7)], check_every=16) >= 2


@pytest.mark.parametrize("g,dtype,D", [(4, "f32", 64), (2, "bf16", 64), (3, "f32", 128), (7, "bf16", 64), (5, "f32", 64)])
def test_other_storage_types_and_head_sizes(gpu, ora, g, dtype, D):
    """fp32 (vector-ALU attention, one-thread-per-pair scorer) and head_dim 64 (MFMA q.K^T only)."""
    w = small(g, dtype=dtype, head_dim=D)
    assert lockstep_feat(gpu, ora, w, 200) == 3


def test_tiny_workload_full_run_with_features(gpu, ora):
    """configs[0] end to end (fp32, head_dim 64, 512 steps, 16 event clocks) with the feature path."""
    w = si.config(0)
    assert lockstep_feat(gpu, ora, w, w.steps) == 16


def test_window_call_equals_the_single_steps(gpu):
    """fk_decode_window_feat enqueues the same launches as the per-step calls: every buffer ends bit-identical (the
    per-step path is the one the other tests of this file hold against the oracle)."""
    import paper_2602_03203_amd as fk
    Bt, Hq, Hkv, D, cap, L, n0, steps, c0 = 3, 8, 2, 128, 300, 32, 200, 20, 7
    d = fk.CacheDesc(Bt, Hq, Hkv, D, cap, "bf16")
    g = torch.Generator(device="cuda").manual_seed(5)
    mk = lambda *shape: (torch.randn(shape, generator=g, device="cuda") / 8).to(torch.bfloat16)
    K0, V0 = mk(Bt, Hkv, cap, D), mk(Bt, Hkv, cap, D)
    q, k, v = mk(steps, Bt, Hq, D), mk(steps, Bt, Hkv, D), mk(steps, Bt, Hkv, D)
    ps = (torch.arange(steps, dtype=torch.int32, device="cuda")[:, None] + n0).expand(steps, Bt).contiguous()
    pos0 = torch.arange(cap, dtype=torch.int32, device="cuda").expand(Bt, Hkv, cap).contiguous()
    feat0 = torch.rand((Bt, Hkv, 6, cap, fk.feat_heads(d)), generator=g, device="cuda")
    results = []
    for window in (False, True):
        K, V, pos, feat = K0.clone(), V0.clone(), pos0.clone(), feat0.clone()
        ln = torch.full((Bt, Hkv), n0, dtype=torch.int32, device="cuda")
        out = torch.zeros((steps, Bt, Hq, D), dtype=torch.bfloat16, device="cuda")
        ws = fk.new_feat_workspace(d)
        if window:
            fk.fk_decode_window_feat(d, q, K, V, pos, ln, k, v, ps, steps, n0 + 1, 0.7, feat, c0, L, out, ws)
        else:
            for t in range(steps):
                fk.fk_decode_step_feat(d, q[t], K, V, pos, ln, k[t], v[t], ps[t], n0 + 1 + t, 0.7, feat, c0 + t, L, out[t], ws)
        torch.cuda.synchronize()
        results.append((K, V, pos, feat, ln, out))
    for a, b in zip(*results):
        assert torch.equal(a.view(torch.uint8) if a.dtype == torch.bfloat16 else a, b.view(torch.uint8) if b.dtype == torch.bfloat16 else b)
    assert (results[0][4] == n0 + steps).all()
    with pytest.raises(fk.FkError):   # the window must end inside the chunk
        fk.fk_decode_window_feat(d, q, K, V, pos, ln, k, v, ps, steps, n0 + 1, 0.7, feat, L - steps + 1, L, out, ws)


def test_bad_arguments_are_refused(gpu):
    import paper_2602_03203_amd as fk
    z = torch.zeros(64 * 128 * 4, dtype=torch.bfloat16, device="cuda")
    f = torch.zeros(6 * 64 * 4, dtype=torch.float32, device="cuda")
    i = torch.zeros(64, dtype=torch.int32, device="cuda")
    ws = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    d = fk.CacheDesc(1, 4, 1, 128, 64, "bf16")
    with pytest.raises(fk.FkError) as e:
        fk.fk_decode_step_feat(d, z, z, z, i, i, z, z, i, 8, 1.0, f, 4, 4, z, ws)   # chunk_pos out of range
    assert e.value.code == 1
    with pytest.raises(fk.FkError) as e:
        fk.fk_decode_step_feat(d, z, z, z, i, i, z, z, i, 8, 1.0, f, 0, 4, z, ws[:64])   # workspace too small
    assert e.value.code == 3
    W1 = torch.zeros((1, 2 * 128 + 24, 44), dtype=torch.bfloat16, device="cuda")         # hidden not a multiple of 8
    b = torch.zeros((1, 44), dtype=torch.float32, device="cuda")
    sc = torch.zeros((1, 1, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(fk.FkError) as e:
        fk.fk_score_kv_feat(d, z, z, f, i, 8, W1, b, b, b[:, 0].contiguous(), sc)
    assert e.value.code == 2
