"""Pins for the budgeted-cache protocol (Section 3.1) on the tiny fp32 workload, and for the
workload shapes against the figures the paper prints."""
import os

import numpy as np
from scipy.special import softmax

import synth_inputs as si
from util import step_inputs, widen, workload_cache

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def read_golden():
    vals = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            k, v = line.split("=")
            vals[k.strip()] = float(v)
    return vals


def test_qwen3_4b_shape_reproduces_printed_kv_footprint():
    """Section 1: the KV cache of one 32K-token sequence of Qwen3-4B in bf16 is 4.5 GB."""
    g = read_golden()
    w = si.config(2)
    bytes_per_seq = w.layers * w.n_kv_heads * w.head_dim * 2 * w.elem_bytes * int(g["kv_tokens"])
    assert abs(bytes_per_seq / 2 ** 30 - g["kv_cache_gb_at_32k"]) < 0.01
    assert w.steps + w.prompt == int(g["kv_tokens"])


def test_event_count_matches_eviction_step_formula():
    """Section 3.2: with T tokens, budget B and eviction length L there are M = ceil((T-B)/L) - 1
    eviction steps before the end; the step-clock rule fires one more after the last token when
    (T - B) is a multiple of L."""
    for i in (0, 1):
        w = si.config(i)
        T = w.prompt + w.steps
        M = int(np.ceil((T - w.budget) / w.interval)) - 1
        lens, events = w.prompt, 0
        for t in range(w.steps):
            lens += 1
            if (t + 1) % w.interval == 0 and lens > w.budget:
                assert lens == w.budget + w.interval      # first and every eviction at B + L
                lens = w.budget
                events += 1
        assert events == M + 1


def test_tiny_workload_protocol_invariants(ora):
    w = si.config(0)
    lens0 = si.initial_lengths(w)
    c = workload_cache(ora, w)
    scorer = si.gen_scorer(w, 0)
    scorer = (si.storage_array(scorer[0], w.dtype),) + scorer[1:]
    seen = {"events": 0, "max_len": 0}
    full_K, full_V = si.gen_kv(w, 0, 0, w.prompt + w.steps)

    def on_step(t, out):
        n = int(c.len[0])
        seen["max_len"] = max(seen["max_len"], n)
        assert n <= w.budget + w.interval
        # positions strictly increasing, newest is the token just generated
        for h in range(w.n_kv_heads):
            p = c.pos[0, h, :n]
            assert (np.diff(p) > 0).all() and p[-1] == w.prompt + t
            # the cache rows are the generator's rows for those positions, bit for bit
            assert np.array_equal(c.K[0, h, :n], full_K[0, h, p]) and np.array_equal(c.V[0, h, :n], full_V[0, h, p])
        if n == w.prompt + t + 1:      # nothing evicted yet: equals full causal attention
            q = si.gen_q(w, 0, w.prompt + t, w.prompt + t + 1)[0, :, 0].astype(np.float64)
            for hq in range(w.n_q_heads):
                hk = hq // w.group
                a = softmax(w.softmax_scale * (full_K[0, hk, :n].astype(np.float64) @ q[hq]))
                np.testing.assert_allclose(out[0, hq], a @ full_V[0, hk, :n].astype(np.float64), rtol=1e-11, atol=1e-13)

    def on_event(t, sc, keep, before):
        n_before = int(before.len[0])
        if n_before <= w.budget:
            assert c.len[0] == n_before
            return
        seen["events"] += 1
        assert n_before == w.budget + w.interval and c.len[0] == w.budget
        for h in range(w.n_kv_heads):
            kept = keep[0, h]
            assert len(set(kept.tolist())) == w.budget
            # the L newest always survive
            assert np.array_equal(kept[-w.interval:], np.arange(n_before - w.interval, n_before))
            # every kept older pair outranks every evicted one on (score desc, position asc)
            old = np.arange(n_before - w.interval)
            s32 = sc[0, h, :n_before].astype(np.float32)
            ev = np.setdiff1d(old, kept)
            ko = np.intersect1d(old, kept)
            assert len(ko) == w.budget - w.interval
            worst_kept = min((s32[i], -before.pos[0, h, i]) for i in ko)
            best_ev = max((s32[i], -before.pos[0, h, i]) for i in ev)
            assert worst_kept > best_ev

    ora.run_protocol(c, lambda t: step_inputs(w, 0, t, lens0), w.steps, scorer, w.budget, w.interval,
                     w.softmax_scale, on_step=on_step, on_event=on_event)
    assert seen["max_len"] == w.budget + w.interval
    assert seen["events"] == 14 and c.len[0] == w.budget


def test_budget_at_least_sequence_length_is_full_attention(ora):
    w = si.config(0).scaled(budget=1024, steps=96)
    lens0 = si.initial_lengths(w)
    c = workload_cache(ora, w)
    scorer = si.gen_scorer(w, 0)
    outs = {}
    ora.run_protocol(c, lambda t: step_inputs(w, 0, t, lens0), w.steps, scorer, w.budget, w.interval,
                     w.softmax_scale, on_step=lambda t, o: outs.__setitem__(t, o.copy()))
    assert c.len[0] == w.prompt + w.steps
    K, V = si.gen_kv(w, 0, 0, w.prompt + w.steps)
    for t in (0, 31, 32, 95):
        n = w.prompt + t + 1
        q = si.gen_q(w, 0, n - 1, n)[0, :, 0].astype(np.float64)
        for hq in range(w.n_q_heads):
            hk = hq // w.group
            a = softmax(w.softmax_scale * (K[0, hk, :n].astype(np.float64) @ q[hq]))
            np.testing.assert_allclose(outs[t][0, hq], a @ V[0, hk, :n].astype(np.float64), rtol=1e-11, atol=1e-13)


def test_eviction_error_bound_on_every_event(ora):
    """Proposition A.1 on the tiny workload: for the query that follows each eviction, the output
    over the pruned cache differs from the output over the cache before pruning (plus the same new
    token) by at most 2 C eps, eps = softmax mass of the pruned pairs."""
    w = si.config(0)
    lens0 = si.initial_lengths(w)
    c = workload_cache(ora, w)
    scorer = si.gen_scorer(w, 0)
    checked = []

    def on_event(t, sc, keep, before):
        if int(before.len[0]) <= w.budget or t + 1 >= w.steps:
            return
        q, k_new, v_new, pos_new = step_inputs(w, 0, t + 1, lens0)
        unpruned = before.copy()
        # before has capacity B + L and is full: evaluate in a cache one slot larger
        big = ora.new_cache(w.dtype, 1, w.n_kv_heads, w.capacity + 1, w.head_dim)
        n = int(unpruned.len[0])
        big.K[:, :, :n], big.V[:, :, :n], big.pos[:, :, :n] = unpruned.K[:, :, :n], unpruned.V[:, :, :n], unpruned.pos[:, :, :n]
        big.len[0] = n
        ora.append(big, k_new, v_new, pos_new)
        pruned = c.copy()
        ora.append(pruned, k_new, v_new, pos_new)
        o = ora.decode_attn(big, q, w.softmax_scale)
        o_hat = ora.decode_attn(pruned, q, w.softmax_scale)
        for hq in range(w.n_q_heads):
            hk = hq // w.group
            Kf = widen(big.K[0, hk, :n + 1], w.dtype)
            Vf = widen(big.V[0, hk, :n + 1], w.dtype)
            a = softmax(w.softmax_scale * (Kf @ widen(q[0, hq], w.dtype)))
            evicted = np.setdiff1d(np.arange(n), keep[0, hk])
            eps = a[evicted].sum()
            C = np.linalg.norm(Vf, axis=1).max()
            assert np.linalg.norm(o[0, hq] - o_hat[0, hq]) <= 2 * C * eps * (1 + 1e-9)
            checked.append(eps)

    ora.run_protocol(c, lambda t: step_inputs(w, 0, t, lens0), 200, scorer, w.budget, w.interval,
                     w.softmax_scale, on_event=on_event)
    assert len(checked) == 4 * w.n_q_heads and max(checked) > 1e-4
