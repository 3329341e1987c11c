"""Lock-step parity of the whole path (append, attention, score, select, compact) against the
oracle over real step / event sequences.

At every step the attention outputs are compared; at every event the device scores are compared
with the oracle's, then BOTH sides select on the oracle's fp32 scores (keep-sets bit exact), and
after compaction K, V, pos and len are compared bit for bit.  The device's own scores also go
through device selection and must equal the oracle's selection on those same fp32 values.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from util import bulk_step_inputs, scorer_storage, workload_cache, workload_cache_replicated

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    import paper_2602_03203_amd as fk
    fk.lib()
    return gpu_util


def lockstep(gpu, ora, w, n_steps, sample_rows=None, scale=None, check_every=1, fused=True, sampled=False, replicate=False):
    """Run the device on the whole workload and the oracle on `sample_rows` [(b, h), ...]
    (None = every row).  Returns the number of events checked."""
    import paper_2602_03203_amd as fk
    scale = w.softmax_scale if scale is None else scale
    lens0 = si.initial_lengths(w)
    B, L, g = w.budget, w.interval, w.group
    print(f"lockstep {w.name}: building prompt cache", flush=True)
    full = workload_cache_replicated(ora, w, sample_rows) if replicate else workload_cache(ora, w)
    dev = gpu.DevCache(full, w.n_q_heads)
    W1, b1, W2, b2 = scorer_storage(w)
    dW = [gpu.to_dev(x) for x in (W1, b1, W2, b2)]
    rows = [(b, h) for b in range(w.batch) for h in range(w.n_kv_heads)] if sample_rows is None else sample_rows
    # one single-row oracle cache per sampled row (rows are independent)
    subs = {}
    for (b, h) in rows:
        subs[(b, h)] = ora.Cache(w.dtype, full.K[b:b + 1, h:h + 1].copy(), full.V[b:b + 1, h:h + 1].copy(),
                                 full.pos[b:b + 1, h:h + 1].copy(), full.len[b:b + 1].copy())
    del full
    q_all, k_all, v_all, p_all = bulk_step_inputs(w, 0, 0, n_steps, lens0)
    dq, dk, dv, dp = (gpu.to_dev(x) for x in (q_all, k_all, v_all, p_all))
    keep_dev = torch.full((w.batch, w.n_kv_heads, B), -1, dtype=torch.int32, device="cuda")
    keep_own = torch.full_like(keep_dev, -1)
    events = 0
    max_len = int(lens0.max())
    for t in range(n_steps):
        max_len += 1
        if fused:      # one launch: append + attention (what bench.py times)
            fk.fk_decode_step(dev.desc, dq[t], dev.K, dev.V, dev.pos, dev.len, dk[t], dv[t], dp[t], min(max_len, w.capacity),
                              scale, dev.out, dev.ws)
        else:
            fk.fk_append(dev.desc, dev.K, dev.V, dev.pos, dev.len, dk[t], dv[t], dp[t])
            fk.fk_decode_attn(dev.desc, dq[t], dev.K, dev.V, dev.len, min(max_len, w.capacity), scale, dev.out, dev.ws)
        for (b, h), c in subs.items():
            ora.append(c, k_all[t, b:b + 1, h:h + 1], v_all[t, b:b + 1, h:h + 1], p_all[t, b:b + 1])
        if t % check_every == 0 or (t + 1) % L == 0:
            got = gpu.out_to_f64(dev.out)
            for (b, h), c in subs.items():
                ref = ora.decode_attn(c, q_all[t, b:b + 1, h * g:(h + 1) * g], scale)
                gpu.assert_attn_close(got[b, h * g:(h + 1) * g], ref[0], w.dtype, f"step {t} row ({b},{h})")
        if (t + 1) % L == 0:
            print(f"  event after step {t}, max_len {max_len}", flush=True)
            fk.fk_score_kv(dev.desc, dev.K, dev.V, dev.len, min(max_len, w.capacity), *dW, dev.scores)
            own = dev.scores.clone()
            fk.fk_select_keep(dev.desc, own, dev.pos, dev.len, min(max_len, w.capacity), B, L, keep_own)
            own_h, keep_own_h = own.cpu().numpy(), keep_own.cpu().numpy()
            inject = own_h.copy()
            refs = {}
            for (b, h), c in subs.items():
                n = int(c.len[0])
                sc = ora.score_kv(c, W1[h:h + 1], b1[h:h + 1], W2[h:h + 1], b2[h:h + 1])
                gpu.assert_scores_close(own_h[b:b + 1, h:h + 1], sc, [n], f"event at step {t}")
                sc32 = sc.astype(np.float32)
                refs[(b, h)] = (sc32, n)
                inject[b, h, :n] = sc32[0, 0, :n]
                # the device's own fp32 scores, selected by the oracle, equal the device's selection
                k_own = ora.select_keep(np.ascontiguousarray(own_h[b:b + 1, h:h + 1]), c.pos, c.len, B, L, "sort")
                if n > B:
                    assert np.array_equal(keep_own_h[b, h], k_own[0, 0]), f"own-score keep-set differs, row ({b},{h})"
            # both sides select on the oracle's scores
            dev.scores.copy_(torch.from_numpy(inject).cuda())
            if sampled:   # Top-K multinomial policy: 2L candidates, Gumbel noise per slot and event
                noise = si.gen_gumbel(w.seed, (w.batch, w.n_kv_heads, w.capacity), event=events)
                fk.fk_select_keep_sampled(dev.desc, dev.scores, gpu.to_dev(noise), dev.pos, dev.len, min(max_len, w.capacity),
                                          B, L, 2 * L, keep_dev)
            else:
                fk.fk_select_keep(dev.desc, dev.scores, dev.pos, dev.len, min(max_len, w.capacity), B, L, keep_dev)
            keep_h = keep_dev.cpu().numpy()
            fk.fk_compact(dev.desc, dev.K, dev.V, dev.pos, dev.len, keep_dev, B)
            host = dev.host(ora)
            for (b, h), c in subs.items():
                sc32, n = refs[(b, h)]
                if sampled:
                    keep_ref = ora.select_keep_sampled(sc32, np.ascontiguousarray(noise[b:b + 1, h:h + 1]), c.pos, c.len, B, L, 2 * L)
                else:
                    keep_ref = ora.select_keep(sc32, c.pos, c.len, B, L, "sort")
                if n > B:
                    assert np.array_equal(keep_h[b, h], keep_ref[0, 0]), f"keep-set differs at step {t}, row ({b},{h})"
                ora.compact(c, keep_ref, B)
                m = int(c.len[0])
                assert host.len[b] == m
                assert np.array_equal(host.pos[b, h, :m], c.pos[0, 0, :m])
                assert np.array_equal(host.K[b, h, :m], c.K[0, 0, :m]) and np.array_equal(host.V[b, h, :m], c.V[0, 0, :m])
            max_len = min(max_len, B) if max_len > B else max_len
            events += 1
    return events


@pytest.mark.parametrize("fused", [True, False])
def test_tiny_workload_full_run(gpu, ora, fused):
    """configs[0] end to end: 512 steps, 16 event clocks (14 with rows over budget), every row."""
    w = si.config(0)
    assert lockstep(gpu, ora, w, w.steps, fused=fused) == 16


def test_tiny_workload_peaked_softmax(gpu, ora):
    w = si.config(0)
    lockstep(gpu, ora, w, 200, scale=1.0)


def test_qwen3_4b_layer_shape_sampled_rows(gpu, ora):
    """configs[1] shapes and launch configuration (batch 16, 32/8 heads, D 128, bf16, B 2048, L 128,
    capacity 2176); the prompt is lengthened so that two events fall inside 400 steps.  The device
    runs all 128 rows; the oracle follows 4 sampled rows."""
    w = si.config(1).scaled(prompt=1920)
    rows = [(0, 0), (5, 3), (11, 6), (15, 7)]
    for scale in (w.softmax_scale, 128.0 ** 0.5):       # near-uniform and unit-variance logits
        assert lockstep(gpu, ora, w, 400 if scale == w.softmax_scale else 260, sample_rows=rows, scale=scale, check_every=16,
                        fused=scale == w.softmax_scale) >= 2


def test_qwen3_4b_layer_all_rows_around_an_event(gpu, ora):
    """configs[1] at the steady state bench.py times (batch 16, 32/8 heads, D 128, bf16, B 2048, L 128, rows at
    B + L - 2 pairs): EVERY one of the 128 rows is compared with the oracle for the two decode steps before an
    eviction event (enqueued by one fk_decode_window call, as bench.py does), the event itself (scores; keep-sets on
    the oracle's scores and on the device's own; K, V, positions and lengths after the compaction, bit for bit)
    and the two steps after it."""
    import paper_2602_03203_amd as fk
    w = si.config(1)
    B, L, g, Bt, Hkv = w.budget, w.interval, w.group, w.batch, w.n_kv_heads
    start = B + L - 2
    lens0 = np.full(Bt, start, np.int32)
    print("all rows: building the cache", flush=True)
    c = workload_cache(ora, w, lens=lens0)
    dev = gpu.DevCache(c, w.n_q_heads)
    W = scorer_storage(w)
    dW = [gpu.to_dev(x) for x in W]
    q, k, v, p = bulk_step_inputs(w, 0, 0, 4, lens0)
    dq, dk, dv, dp = (gpu.to_dev(x) for x in (q, k, v, p))
    outs = torch.empty((4, Bt, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device="cuda")
    for scale in (w.softmax_scale, 128.0 ** 0.5):   # near-uniform and unit-variance logits, each on a fresh copy
        cc = c.copy()
        d2 = gpu.DevCache(cc, w.n_q_heads)
        fk.fk_decode_window(d2.desc, dq[:2], d2.K, d2.V, d2.pos, d2.len, dk[:2], dv[:2], dp[:2], 2, start + 1, scale, outs[:2], d2.ws)
        for t in range(2):
            ora.append(cc, k[t], v[t], p[t])
            gpu.assert_attn_close(gpu.out_to_f64(outs[t]), ora.decode_attn(cc, q[t], scale), "bf16", f"scale {scale:.3f} step {t}")
        assert int(d2.len.min()) == B + L == int(d2.len.max())
        print("all rows: event", flush=True)
        fk.fk_score_kv(d2.desc, d2.K, d2.V, d2.len, B + L, *dW, d2.scores, skip_len=B)
        sc = ora.score_kv(cc, *W)
        own = d2.scores.cpu().numpy()
        gpu.assert_scores_close(own, sc, cc.len, "all rows scores")
        keep = torch.full((Bt, Hkv, B), -1, dtype=torch.int32, device="cuda")
        fk.fk_select_keep(d2.desc, d2.scores, d2.pos, d2.len, B + L, B, L, keep)          # on the device's own scores
        gpu.assert_keep_equal(keep.cpu().numpy(), ora.select_keep(own, cc.pos, cc.len, B, L, "sort"), cc.len, B, "own scores")
        sc32 = sc.astype(np.float32)
        keep_ref = ora.select_keep(sc32, cc.pos, cc.len, B, L, "sort")
        d2.scores.copy_(torch.from_numpy(sc32).cuda())
        fk.fk_select_keep(d2.desc, d2.scores, d2.pos, d2.len, B + L, B, L, keep)          # on the oracle's scores
        gpu.assert_keep_equal(keep.cpu().numpy(), keep_ref, cc.len, B, "oracle scores")
        fk.fk_compact(d2.desc, d2.K, d2.V, d2.pos, d2.len, keep, B)
        ora.compact(cc, keep_ref, B)
        h = d2.host(ora)
        assert np.array_equal(h.len, cc.len) and (h.len == B).all()
        assert np.array_equal(h.pos[:, :, :B], cc.pos[:, :, :B])
        assert np.array_equal(h.K[:, :, :B], cc.K[:, :, :B]) and np.array_equal(h.V[:, :, :B], cc.V[:, :, :B])
        fk.fk_decode_window(d2.desc, dq[2:], d2.K, d2.V, d2.pos, d2.len, dk[2:], dv[2:], dp[2:], 2, B + 1, scale, outs[2:], d2.ws)
        for t in range(2, 4):
            ora.append(cc, k[t], v[t], p[t])
            gpu.assert_attn_close(gpu.out_to_f64(outs[t]), ora.decode_attn(cc, q[t], scale), "bf16", f"scale {scale:.3f} step {t}")
        assert int(d2.len.min()) == B + 2 == int(d2.len.max())
    del dev


def test_gqa7_mixture_sampled_rows(gpu, ora):
    """configs[3] shapes (28/4 heads, D 128, B 4096, L 64) with duplicate-heavy keys: exact score ties."""
    w = si.config(3).scaled(layers=1, batch=4, prompt=4096 - 64)
    rows = [(0, 0), (3, 2)]
    assert lockstep(gpu, ora, w, 200, sample_rows=rows, scale=128.0 ** 0.5, check_every=16) >= 2


def test_long_budget_shape_sampled_rows(gpu, ora):
    """configs[2] row shape (32/8 heads, D 128, B 16384, L 128, capacity 16512), two sequences of one
    layer: rows are split across workgroups (few rows) and compaction / selection run several tiles."""
    w = si.config(2).scaled(layers=1, batch=2, prompt=16384 - 128)
    rows = [(0, 1), (1, 6)]
    assert lockstep(gpu, ora, w, 300, sample_rows=rows, scale=128.0 ** 0.5, check_every=32) >= 2


def test_ragged_batch_shape_sampled_rows(gpu, ora):
    """configs[4] shape (ragged lengths up to 32768, B 8192, L 128, capacity 32896), four sequences: the
    first event prunes rows far over budget in one go, rows under budget are left alone."""
    w = si.config(4).scaled(batch=4)
    lens0 = si.initial_lengths(w)
    assert lens0.max() > w.budget + w.interval and len(set(lens0.tolist())) == 4
    b_long = int(np.argmax(lens0))
    b_short = int(np.argmin(lens0))
    rows = [(b_long, 0), (b_short, 5)]
    assert lockstep(gpu, ora, w, 260, sample_rows=rows, scale=128.0 ** 0.5, check_every=32) >= 2


def test_stack_layer_shapes_at_full_batch_sampled_rows(gpu, ora):
    """One layer of configs[2] (batch 8, B 16384: 64 rows, two splits per row) and of configs[3] (batch 16,
    GQA 7, B 4096: 64 rows) in the launch configuration bench.py uses, caches just under the first event;
    the oracle follows two rows of each, the other rows hold copies of their data."""
    w = si.config(2).scaled(layers=1, prompt=16384 - 64)
    assert lockstep(gpu, ora, w, 200, sample_rows=[(0, 0), (7, 5)], check_every=40, replicate=True) >= 1
    w = si.config(3).scaled(layers=1, prompt=4096 - 32)
    assert lockstep(gpu, ora, w, 140, sample_rows=[(2, 1), (15, 3)], check_every=20, replicate=True) >= 2


def test_ragged_batch_at_full_size_sampled_rows(gpu, ora):
    """configs[4] as bench.py runs it: 64 sequences (512 rows, 8.6 GB of cache), lengths 1024 .. 32768, B 8192;
    the oracle follows one row far over budget, one under it and the longest one."""
    w = si.config(4)
    lens = si.initial_lengths(w)
    over = int(np.argmax(lens > 20000))
    under = int(np.argmax(lens < 8000))
    longest = int(np.argmax(lens))
    rows = sorted({(over, 0), (under, 3), (longest, 7)})
    assert lockstep(gpu, ora, w, 130, sample_rows=rows, check_every=32, replicate=True) == 1


def test_one_shot_prefill_compression(gpu, ora):
    """Long-input use of the same calls (Section 4.3, long-context tasks: the cache is compressed once
    after the prefill, no repeated eviction): a 65536-token prompt is scored, pruned to B = 2048
    (128 newest protected) and compacted in one event, then decoding continues over the pruned cache."""
    import paper_2602_03203_amd as fk
    n, B, R = 65536, 2048, 128
    w = si.config(1).scaled(batch=1, n_q_heads=8, n_kv_heads=2, prompt=n, budget=B, interval=R, ragged_max=n)
    print(f"one-shot: building {n}-token prompt cache, capacity {w.capacity}", flush=True)
    c = workload_cache(ora, w, lens=[n])
    dev = gpu.DevCache(c, w.n_q_heads)
    W1, b1, W2, b2 = scorer_storage(w)
    fk.fk_score_kv(dev.desc, dev.K, dev.V, dev.len, n, *[gpu.to_dev(x) for x in (W1, b1, W2, b2)], dev.scores)
    sc = ora.score_kv(c, W1, b1, W2, b2)
    gpu.assert_scores_close(dev.scores.cpu().numpy(), sc, [n], "one-shot scores")
    sc32 = sc.astype(np.float32)
    keep_ref = ora.select_keep(sc32, c.pos, c.len, B, R, "sort")
    dev.scores.copy_(torch.from_numpy(sc32).cuda())
    keep = torch.full((1, 2, B), -1, dtype=torch.int32, device="cuda")
    fk.fk_select_keep(dev.desc, dev.scores, dev.pos, dev.len, n, B, R, keep)
    gpu.assert_keep_equal(keep.cpu().numpy(), keep_ref, c.len, B)
    fk.fk_compact(dev.desc, dev.K, dev.V, dev.pos, dev.len, keep, B)
    ora.compact(c, keep_ref, B)
    h = dev.host(ora)
    assert h.len[0] == B and np.array_equal(h.pos[:, :, :B], c.pos[:, :, :B])
    assert np.array_equal(h.K[:, :, :B], c.K[:, :, :B]) and np.array_equal(h.V[:, :, :B], c.V[:, :, :B])
    q, k_new, v_new, p_new = bulk_step_inputs(w, 0, 0, 3, [n])
    for t in range(3):
        fk.fk_decode_step(dev.desc, gpu.to_dev(q[t]), dev.K, dev.V, dev.pos, dev.len, gpu.to_dev(k_new[t]), gpu.to_dev(v_new[t]),
                          gpu.to_dev(p_new[t]), B + 3, 128.0 ** 0.5, dev.out, dev.ws)
        ora.append(c, k_new[t], v_new[t], p_new[t])
        gpu.assert_attn_close(gpu.out_to_f64(dev.out), ora.decode_attn(c, q[t], 128.0 ** 0.5), "bf16", f"after one-shot, step {t}")


def test_sampled_policy_tiny_workload_full_run(gpu, ora):
    """configs[0] end to end under the Top-K multinomial eviction policy (Section 3.1 Eq. 2): every event
    draws the evicted pairs among the 2L lowest-scored ones; keep-sets and caches stay bit exact."""
    w = si.config(0)
    assert lockstep(gpu, ora, w, w.steps, sampled=True) == 16


def test_sampled_policy_qwen3_shape_sampled_rows(gpu, ora):
    w = si.config(1).scaled(prompt=1920)
    assert lockstep(gpu, ora, w, 400, sample_rows=[(1, 2), (14, 5)], scale=128.0 ** 0.5, check_every=32, sampled=True) >= 2
