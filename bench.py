#!/usr/bin/env python3
"""Benchmark of the budgeted-KV decode + evict path on one MI355X.

A "step" is one pass of the whole hot path over one batch: append the new pair, attend over the
retained cache, and after every L-th step run the eviction event (score, select, compact).
Default workload: the Qwen3-4B single-layer shape (batch 16, 32 query / 8 KV heads, head_dim 128,
bf16 K/V, prompt 512, budget 2048, eviction every 128 steps, 8192 decode steps).  All inputs are
seeded synthetic data, resident in HBM before the timed region starts.

Prints ONE JSON line: decode tokens/s for the whole run, the roofline record of the dominant kernel
(decode attention; algorithmic bytes / HIP-event time of its launches) and the CPU oracle timed on a
bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gen_step_inputs(w: si.Workload, lens0: np.ndarray, n_steps: int, threads: int):
    """q [T,Bt,Hq,D], k_new, v_new [T,Bt,Hkv,D] storage arrays and pos_new [T,Bt] for steps 0..T-1."""
    D, Bt = w.head_dim, w.batch
    st = np.float32 if w.dtype == "f32" else np.uint16
    q = np.empty((n_steps, Bt, w.n_q_heads, D), st)
    k = np.empty((n_steps, Bt, w.n_kv_heads, D), st)
    v = np.empty((n_steps, Bt, w.n_kv_heads, D), st)
    pos = np.empty((n_steps, Bt), np.int32)
    chunk = 256
    jobs = [(b, t0, min(t0 + chunk, n_steps)) for b in range(Bt) for t0 in range(0, n_steps, chunk)]

    def work(job):
        b, t0, t1 = job
        p0 = int(lens0[b]) + t0
        pos[t0:t1, b] = np.arange(p0, p0 + (t1 - t0))
        qq = si.gen_q(w, 0, p0, p0 + (t1 - t0), batch_sel=[b])[0]
        kk, vv = si.gen_kv(w, 0, p0, p0 + (t1 - t0), batch_sel=[b])
        q[t0:t1, b] = si.storage_array(qq.transpose(1, 0, 2), w.dtype)
        k[t0:t1, b] = si.storage_array(kk[0].transpose(1, 0, 2), w.dtype)
        v[t0:t1, b] = si.storage_array(vv[0].transpose(1, 0, 2), w.dtype)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, jobs))
    return q, k, v, pos


def gen_prompt(w: si.Workload, lens0: np.ndarray, threads: int):
    """Prompt cache as storage arrays K, V [Bt,Hkv,cap,D], pos [Bt,Hkv,cap]."""
    st = np.float32 if w.dtype == "f32" else np.uint16
    K = np.zeros((w.batch, w.n_kv_heads, w.capacity, w.head_dim), st)
    V = np.zeros_like(K)
    pos = np.full((w.batch, w.n_kv_heads, w.capacity), -1, np.int32)

    def work(b):
        n = int(lens0[b])
        kk, vv = si.gen_kv(w, 0, 0, n, batch_sel=[b])
        K[b, :, :n] = si.storage_array(kk[0], w.dtype)
        V[b, :, :n] = si.storage_array(vv[0], w.dtype)
        pos[b, :, :n] = np.arange(n, dtype=np.int32)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(work, range(w.batch)))
    return K, V, pos


def len_schedule(w: si.Workload, lens0: np.ndarray, n_steps: int):
    """Host replay of the protocol's cache sizes: lens_at_attn [T, Bt] (after the append of step t)."""
    lens = lens0.astype(np.int64).copy()
    out = np.empty((n_steps, w.batch), np.int64)
    ev = []
    for t in range(n_steps):
        lens += 1
        out[t] = lens
        if (t + 1) % w.interval == 0:
            ev.append(lens.copy())
            lens = np.minimum(lens, w.budget)
    return out, ev


def measured_traffic(w: si.Workload, steps: int, features: bool = False):
    """HBM bytes per attention launch from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE runs of this same command, each scaled on a plain copy of known size); None when the
    summary does not cover this workload / step count."""
    if w.name != "cfg1-qwen3-4b-layer" or steps != w.steps or features:
        return None
    path = os.path.join(ROOT, "profiles", "attn_kernel_cfg1_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def profile_value(fname: str, key: str):
    """A `key = number` line of a committed profile summary, or None."""
    try:
        for line in open(os.path.join(ROOT, "profiles", fname)):
            if line.startswith(key):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def attn_bytes(w: si.Workload, lens_row: np.ndarray) -> float:
    """Algorithmic bytes of one attention launch: K and V once per KV head, plus q and out."""
    e = w.elem_bytes
    return float(w.n_kv_heads * lens_row.sum() * w.head_dim * 2 * e + w.batch * w.n_q_heads * w.head_dim * 2 * e)


def feat_bytes(w: si.Workload, lens_row: np.ndarray, chunk_pos: int) -> float:
    """Algorithmic bytes the attention features add to a launch: the chunk plane, and each window plane
    that is open at this step, is read and written once per (live pair, query head), fp32."""
    planes = 1 + sum(1 for wnd in (8, 16, 32) if chunk_pos >= w.interval - wnd)
    return float(w.n_kv_heads * lens_row.sum() * w.group * 4 * 2 * planes)


def cpu_baseline(w: si.Workload, threads: int, windows: int = 5):
    """Time the CPU oracle, as it stands, on a bounded sample of the same workload: the full batch at
    steady state (cache at budget) for `windows` eviction windows, each L decode steps (append +
    attention) and one eviction event (score + select + compact)."""
    import oracle
    oracle.set_threads(threads)
    B, L, Bt = w.budget, w.interval, w.batch
    wl = w.scaled(prompt=B)  # steady state: rows already hold B pairs
    c = oracle.new_cache(w.dtype, Bt, w.n_kv_heads, w.capacity, w.head_dim)
    K, V = si.gen_kv(wl, 0, 0, B)
    c.K[:, :, :B], c.V[:, :, :B] = si.storage_array(K, w.dtype), si.storage_array(V, w.dtype)
    c.pos[:, :, :B] = np.arange(B, dtype=np.int32)
    c.len[:] = B
    W1, b1, W2, b2 = si.gen_scorer(w, 0)
    scorer = (si.storage_array(W1, w.dtype), b1, W2, b2)
    n_steps = windows * L
    qs = si.storage_array(si.gen_q(wl, 0, B, B + n_steps), w.dtype)
    ks, vs = (si.storage_array(x, w.dtype) for x in si.gen_kv(wl, 0, B, B + n_steps))
    step_in = [(np.ascontiguousarray(qs[:, :, t]), np.ascontiguousarray(ks[:, :, t]), np.ascontiguousarray(vs[:, :, t]),
                np.full(Bt, B + t, np.int32)) for t in range(n_steps)]
    t0 = time.perf_counter()
    oracle.run_protocol(c, lambda t: step_in[t], n_steps, scorer, B, L, w.softmax_scale, method="sort")
    dt = time.perf_counter() - t0
    assert int(c.len[0]) == B
    # the same loop on ONE core, one window (the cache is back at B after the run above)
    oracle.set_threads(1)
    t0 = time.perf_counter()
    oracle.run_protocol(c, lambda t: step_in[t], L, scorer, B, L, w.softmax_scale, method="sort")
    dt1 = time.perf_counter() - t0
    oracle.set_threads(threads)
    return {"value": Bt * n_steps / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": f"full batch ({Bt} sequences x {w.n_kv_heads} KV heads) at steady state (cache {B}..{B + L}): "
                      f"{windows} windows of {L} decode steps + 1 eviction event each = {n_steps} steps, {dt:.1f}s CPU",
            "value_1core": Bt * L / dt1, "sample_1core": f"one such window on one core, {dt1:.1f}s CPU"}


def bench_golden(args):
    """Golden Eviction label builder (Section 3.2 Eq. 3-5) at the Qwen3-4B layer shape: 32 query / 8 KV
    heads, one 8192-token trace, B 2048, L 128, bf16 attention (4.3 GB, HBM resident).  A step = block
    pooling + future scores + the 47-step eviction trace."""
    import torch
    import paper_2602_03203_amd as fk
    fk.lib()
    torch.cuda.set_device(0)
    Hq, Hkv, T, B, L = 32, 8, 8192, 2048, 128
    g = Hq // Hkv
    M = fk.fk_golden_steps(T, B, L)
    K_steps = args.steps if args.steps is not None else 20
    W_steps = min(args.warmup, 5)
    gen = torch.Generator(device="cuda").manual_seed(2602)
    A = torch.empty((Hq, T, T), dtype=torch.bfloat16, device="cuda")
    causal = torch.ones((T, T), dtype=torch.bool, device="cuda").tril_()
    for h in range(Hq):
        z = 1.5 * torch.randn((T, T), generator=gen, device="cuda")
        z.masked_fill_(~causal, float("-inf"))
        A[h] = torch.softmax(z, dim=1).to(torch.bfloat16)
    del z, causal
    a_t = torch.empty((Hkv, M, T), dtype=torch.float32, device="cuda")
    alpha = torch.empty_like(a_t)
    kept = torch.empty((Hkv, M, B), dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()

    def step():
        fk.fk_golden_scores(A, Hkv, T, B, L, a_t, alpha, stream)
        fk.fk_golden_trace(alpha, T, B, L, kept, stream)

    for _ in range(W_steps):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(K_steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    entries = Hq * sum(q + 1 for q in range(B + L, T))          # causal entries of the pooled queries
    e0 = [torch.cuda.Event(enable_timing=True) for _ in range(K_steps)]
    e1 = [torch.cuda.Event(enable_timing=True) for _ in range(K_steps)]
    for i in range(K_steps):
        e0[i].record(stream)
        fk.fk_golden_scores(A, Hkv, T, B, L, a_t, alpha, stream)
        e1[i].record(stream)
        fk.fk_golden_trace(alpha, T, B, L, kept, stream)
    torch.cuda.synchronize()
    ms = float(np.mean([a.elapsed_time(b) for a, b in zip(e0, e1)]))
    bytes_alg = entries * 2 + 2 * Hkv * M * T * 4 * 2           # A once; block scores written, read, future scores written
    achieved = bytes_alg / (ms * 1e-3) / 1e9
    result = {
        "metric": "Golden Eviction label builder: causal attention entries pooled per second (pooling + future scores + trace), one layer",
        "value": entries * K_steps / wall, "unit": "entries/s", "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": 1e3 * wall / K_steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "golden-qwen3-4b-layer-8k", "n_q_heads": Hq, "n_kv_heads": Hkv, "trace_tokens": T, "budget": B,
                   "eviction_interval": L, "steps_M": M},
        "roofline": {"kernel": "golden_pool_kernel + golden_future_kernel (fk_golden_scores)", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": profile_value("golden_pool_kernel_qwen3_4b_8k_trace.txt", "traffic_bytes_per_launch"),
                     "avg_launch_us": ms * 1e3, "algorithmic_bytes_per_launch": bytes_alg},
    }
    if not args.no_cpu:
        from oracle import golden
        ncol = 2048
        cols = torch.arange(0, T, T // ncol, device="cuda")
        sub = A[:, :, cols].float().cpu().numpy().astype(np.float64)
        t0 = time.perf_counter()
        a_ref = golden.block_scores(sub, g, B, L)
        golden.future_scores(a_ref)
        dt = time.perf_counter() - t0
        frac = sum(int((cols.cpu().numpy() <= q).sum()) for q in range(B + L, T)) * Hq
        result["cpu_baseline"] = {"value": frac / dt, "unit": "entries/s", "cores": 1, "kind": "oracle",
                                  "sample": f"{ncol} of {T} key columns, all heads and blocks, pooling + future scores, {dt:.1f}s CPU"}
    print(json.dumps(result), flush=True)


def bench_stack(args, w: si.Workload):
    """Whole layer stack of a multi-layer configuration (--stack): every decode step runs the fused append +
    attention of EVERY layer, every L-th step the eviction event of every layer; every layer has its own cache,
    lengths and scorer weights.  The run starts near the steady state (prompt = budget - L/2 unless --prompt) and
    its inputs are drawn on the device with seeded torch ops in the distributions of the configuration
    (N(0,1)/sqrt(D), 1 % of the positions with 3x key norm); step inputs cycle through a pool of 64."""
    import torch
    import paper_2602_03203_amd as fk
    fk.lib()
    torch.cuda.set_device(0)
    NL, Bt, Hq, Hkv, D, B, L, cap = w.layers, w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.budget, w.interval, w.capacity
    P0 = args.prompt if args.prompt is not None else B - L // 2
    K_steps = args.steps if args.steps is not None else 2 * L
    W_steps = min(args.warmup, L)
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    gen = torch.Generator(device="cuda").manual_seed(w.seed % (2 ** 31))
    sd = 1.0 / np.sqrt(D)
    K0 = torch.empty((NL, Bt, Hkv, cap, D), dtype=dt, device="cuda")
    V0 = torch.empty_like(K0)
    for l in range(NL):
        heavy = 1.0 + 2.0 * (torch.rand((Bt, 1, cap, 1), generator=gen, device="cuda") < 0.01).float()
        K0[l] = (torch.randn((Bt, Hkv, cap, D), generator=gen, device="cuda") * sd * heavy).to(dt)
        V0[l] = (torch.randn((Bt, Hkv, cap, D), generator=gen, device="cuda") * sd).to(dt)
    pos0 = torch.arange(cap, dtype=torch.int32, device="cuda").expand(NL, Bt, Hkv, cap).contiguous()
    len0 = torch.full((NL, Bt, Hkv), P0, dtype=torch.int32, device="cuda")
    NP = 64
    dq = (torch.randn((NP, Bt, Hq, D), generator=gen, device="cuda") * sd).to(dt)
    dk = (torch.randn((NP, Bt, Hkv, D), generator=gen, device="cuda") * sd).to(dt)
    dv = (torch.randn((NP, Bt, Hkv, D), generator=gen, device="cuda") * sd).to(dt)
    F, H = 2 * D, w.hidden
    W1 = (torch.randn((NL, Hkv, F, H), generator=gen, device="cuda") / np.sqrt(F)).to(dt)
    b1 = torch.randn((NL, Hkv, H), generator=gen, device="cuda") / np.sqrt(F)
    W2 = torch.randn((NL, Hkv, H), generator=gen, device="cuda") / np.sqrt(H)
    b2 = torch.randn((NL, Hkv), generator=gen, device="cuda") / np.sqrt(H)
    desc = fk.CacheDesc(Bt, Hq, Hkv, D, cap, w.dtype, cold=NL * Bt * Hkv * cap * D * 2 * w.elem_bytes > (256 << 20))
    Kc, Vc, posc, lenc = (torch.empty_like(x) for x in (K0, V0, pos0, len0))
    ws = fk.new_attn_workspace(desc)
    out = torch.empty((Bt, Hq, D), dtype=dt, device="cuda")
    scores = torch.zeros((Bt, Hkv, cap), dtype=torch.float32, device="cuda")
    keep = torch.zeros((Bt, Hkv, B), dtype=torch.int32, device="cuda")
    dp = torch.zeros((Bt,), dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream()
    scale = w.softmax_scale
    n_tot = max(K_steps, W_steps)
    lens = np.empty(n_tot, np.int64)     # cache length at the attention of step t (all rows alike)
    cur = P0
    for t in range(n_tot):
        cur += 1
        lens[t] = cur
        if (t + 1) % L == 0:
            cur = min(cur, B)

    def reset():
        Kc.copy_(K0); Vc.copy_(V0); posc.copy_(pos0); lenc.copy_(len0)

    def run(n_steps, brackets=None):
        for t in range(n_steps):
            ml = int(min(lens[t], cap))
            dp.fill_(P0 + t)
            if brackets is not None:
                brackets[t][0].record(stream)
            for l in range(NL):
                fk.fk_decode_step(desc, dq[(t + l) % NP], Kc[l], Vc[l], posc[l], lenc[l], dk[(t + 3 * l) % NP], dv[(t + 5 * l) % NP],
                                  dp, ml, scale, out, ws, stream)
            if brackets is not None:
                brackets[t][1].record(stream)
            if (t + 1) % L == 0:
                for l in range(NL):
                    fk.fk_score_kv(desc, Kc[l], Vc[l], lenc[l], ml, W1[l], b1[l], W2[l], b2[l], scores, stream, skip_len=B)
                    fk.fk_select_keep(desc, scores, posc[l], lenc[l], ml, B, L, keep, stream)
                    fk.fk_compact(desc, Kc[l], Vc[l], posc[l], lenc[l], keep, B, stream)

    reset()
    run(W_steps)
    torch.cuda.synchronize()
    reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(K_steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    fl = lenc.cpu().numpy()
    assert (fl == fl.flat[0]).all() and fl.flat[0] == (min(lens[K_steps - 1], B) if K_steps % L == 0 else lens[K_steps - 1])
    e = w.elem_bytes
    step_bytes = [NL * (Bt * Hkv * int(lens[t]) * D * 2 * e + Bt * Hq * D * 2 * e) for t in range(K_steps)]
    result = {
        "metric": "decode tokens/s, budgeted KV decode+evict (attention + scorer + top-k + compaction), whole layer stack",
        "value": Bt * K_steps / wall, "unit": "tokens/s", "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": 1e3 * wall / K_steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic (drawn on the device)",
        "config": {"workload": f"{w.name} (all {NL} layers, prompt {P0})", "layers": NL, "batch": Bt, "n_q_heads": Hq,
                   "n_kv_heads": Hkv, "head_dim": D, "budget": B, "eviction_interval": L, "capacity": cap, "scorer_hidden": H},
        "path_gbs_algorithmic": sum(step_bytes) / wall / 1e9,
    }
    reset()
    br = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K_steps)]
    run(K_steps, br)
    torch.cuda.synchronize()
    ms = sum(a.elapsed_time(b) for a, b in br)
    achieved = sum(step_bytes) / (ms * 1e-3) / 1e9
    result["roofline"] = {"kernel": "attn_kernel (fk_decode_step), all layers of a step between one pair of HIP events", "bound": "hbm",
                          "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                          "avg_launch_us": ms * 1e3 / (K_steps * NL), "algorithmic_bytes_per_launch": sum(step_bytes) / (K_steps * NL)}
    print(json.dumps(result), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed decode steps (default: the workload's)")
    ap.add_argument("--warmup", type=int, default=256)
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--prompt", type=int, default=None, help="override the prompt length (to start near the steady state)")
    ap.add_argument("--policy", choices=["topk", "sampled"], default="topk",
                    help="eviction action: deterministic top-k (default) or Top-K multinomial over 2L candidates")
    ap.add_argument("--features", action="store_true",
                    help="scorer inputs concat(k, v, attention features): the decode step also keeps the attention sums "
                         "(bf16, head_dim 128 only; the default run scores on k and v alone)")
    ap.add_argument("--stack", action="store_true", help="multi-layer configurations: run every layer at every step")
    ap.add_argument("--hidden", type=int, default=None, help="override the scorer's hidden width (the paper trains with 16)")
    ap.add_argument("--workload", choices=["decode", "golden"], default="decode",
                    help="decode: the budgeted decode + evict path (the headline); golden: the Golden Eviction label builder")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-kernel-timing", action="store_true", help="skip the HIP-event pass over the attention launches")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (rows are independent: batch or KV-head sharding needs no exchange inside this path); use --gpus 1")

    if args.workload == "golden":
        return bench_golden(args)
    import torch
    import paper_2602_03203_amd as fk
    fk.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    host_threads = min(16, os.cpu_count() or 1)

    w = si.config(args.config)
    if w.layers != 1 and args.stack:
        if args.hidden is not None:
            w = w.scaled(hidden=args.hidden)
        return bench_stack(args, w)
    if w.layers != 1:   # stacks: every layer runs the same kernels on its own cache; without --stack one layer is timed
        w = w.scaled(name=f"{w.name} (one layer of {w.layers})", layers=1)
    if args.prompt is not None:
        w = w.scaled(name=f"{w.name} (prompt {args.prompt})", prompt=args.prompt)
    if args.hidden is not None:
        w = w.scaled(name=f"{w.name} (scorer hidden {args.hidden})", hidden=args.hidden)
    K_steps = args.steps if args.steps is not None else w.steps
    W_steps = args.warmup
    n_gen = max(K_steps, W_steps)
    lens0 = si.initial_lengths(w)
    B, L = w.budget, w.interval

    t0 = time.time()
    Kh, Vh, posh = gen_prompt(w, lens0, host_threads)
    qh, kh, vh, ph = gen_step_inputs(w, lens0, n_gen, host_threads)
    log(f"[bench] generated {w.name}: prompt + {n_gen} steps in {time.time() - t0:.1f}s")

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    K0, V0, pos0 = dev(Kh), dev(Vh), dev(posh)
    len0 = dev(np.repeat(lens0.astype(np.int32)[:, None], w.n_kv_heads, axis=1))      # one count per row
    dq, dk, dv, dp = dev(qh), dev(kh), dev(vh), dev(ph)
    del Kh, Vh, qh, kh, vh
    W1, b1, W2, b2 = si.gen_scorer_feat(w, 0) if args.features else si.gen_scorer(w, 0)
    dW = [dev(si.storage_array(W1, w.dtype)), dev(b1), dev(W2), dev(b2)]
    desc = fk.CacheDesc(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.capacity, w.dtype)
    Kc, Vc, posc, lenc = (torch.empty_like(x) for x in (K0, V0, pos0, len0))
    ws = fk.new_attn_workspace(desc)
    feat = fk.new_feat(desc) if args.features else None
    fws = fk.new_feat_workspace(desc) if args.features else None
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=desc.torch_dtype, device="cuda")
    scores = torch.zeros((w.batch, w.n_kv_heads, w.capacity), dtype=torch.float32, device="cuda")
    keep = torch.zeros((w.batch, w.n_kv_heads, B), dtype=torch.int32, device="cuda")
    noise_pool = None
    if args.policy == "sampled":   # Gumbel noise per slot, a pool of 8 independent draws cycled over the events
        noise_pool = [dev(si.gen_gumbel(w.seed, (w.batch, w.n_kv_heads, w.capacity), event=e)) for e in range(8)]
    lens_at, _ = len_schedule(w, lens0, n_gen)
    max_at = lens_at.max(axis=1)
    scale = w.softmax_scale
    stream = torch.cuda.current_stream()

    def reset():
        Kc.copy_(K0); Vc.copy_(V0); posc.copy_(pos0); lenc.copy_(len0)
        if feat is not None:
            feat.zero_()

    ev_kernels = []

    def run(n_steps, ev_pairs=None):
        for t in range(n_steps):
            ml = int(min(max_at[t], w.capacity))
            if ev_pairs is not None and t % L == 0:
                ev_pairs[t // L][0].record(stream)
            if feat is None:
                fk.fk_decode_step(desc, dq[t], Kc, Vc, posc, lenc, dk[t], dv[t], dp[t], ml, scale, out, ws, stream)
            else:
                fk.fk_decode_step_feat(desc, dq[t], Kc, Vc, posc, lenc, dk[t], dv[t], dp[t], ml, scale, feat, t % L, L, out,
                                       fws, stream)
            if ev_pairs is not None and ((t + 1) % L == 0 or t + 1 == n_steps):
                ev_pairs[t // L][1].record(stream)
            if (t + 1) % L == 0:
                kev = None
                if ev_pairs is not None:   # per-kernel brackets of the event: [start, after score, after select, after compact]
                    kev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                    ev_kernels.append((t, kev))
                    kev[0].record(stream)
                if feat is None:
                    fk.fk_score_kv(desc, Kc, Vc, lenc, ml, *dW, scores, stream, skip_len=B)
                else:
                    fk.fk_score_kv_feat(desc, Kc, Vc, feat, lenc, ml, *dW, scores, stream, skip_len=B)
                if kev:
                    kev[1].record(stream)
                if noise_pool is None:
                    fk.fk_select_keep(desc, scores, posc, lenc, ml, B, L, keep, stream)
                else:
                    fk.fk_select_keep_sampled(desc, scores, noise_pool[(t // L) % 8], posc, lenc, ml, B, L, 2 * L, keep, stream)
                if kev:
                    kev[2].record(stream)
                if feat is None:
                    fk.fk_compact(desc, Kc, Vc, posc, lenc, keep, B, stream)
                else:
                    fk.fk_compact_feat(desc, Kc, Vc, posc, feat, lenc, keep, B, stream)
                if kev:
                    kev[3].record(stream)

    # warm-up (untimed), then restart from the prompt
    reset()
    run(W_steps)
    torch.cuda.synchronize()
    reset()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(K_steps)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    final_len = lenc.cpu().numpy()
    assert (final_len == final_len[:, :1]).all()
    final_len = final_len[:, 0]
    expect_len = len_schedule(w, lens0, K_steps)[0][-1]
    expect_len = np.where((K_steps % L == 0) & (expect_len > B), B, expect_len)
    assert np.array_equal(final_len, expect_len), (final_len, expect_len)

    tokens_per_s = w.batch * K_steps / wall
    total_attn_bytes = sum(attn_bytes(w, lens_at[t]) for t in range(K_steps))
    if args.features:
        total_attn_bytes += sum(feat_bytes(w, lens_at[t], t % L) for t in range(K_steps))
    result = {
        "metric": "decode tokens/s, budgeted KV decode+evict (attention + scorer + top-k + compaction), one layer",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": 1e3 * wall / K_steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "prompt": w.prompt, "budget": B, "eviction_interval": L,
                   "capacity": w.capacity, "scorer_hidden": w.hidden, "eviction_policy": args.policy,
                   "scorer_inputs": "k, v, attention features" if args.features else "k, v"},
        "path_gbs_algorithmic": total_attn_bytes / wall / 1e9,
    }
    # the same with the eviction events' algorithmic bytes added (rows over budget at the event: every retained
    # pair scored, its score read by the selection, the kept slots written, every kept pair that is not already in
    # place moved; "every kept pair" is taken, an upper bound)
    ev_bytes = 0.0
    for t in range(L - 1, K_steps, L):
        over = lens_at[t] > B
        pairs = float(lens_at[t][over].sum()) * w.n_kv_heads
        rows_over = float(over.sum()) * w.n_kv_heads
        ev_bytes += pairs * (2 * w.head_dim * w.elem_bytes + 4) + 4 * pairs + rows_over * 4 * B \
            + rows_over * B * (4 * w.head_dim * w.elem_bytes + 8)
    result["path_with_events"] = {"gbs_algorithmic": (total_attn_bytes + ev_bytes) / wall / 1e9,
                                  "frac_of_hbm_peak": (total_attn_bytes + ev_bytes) / wall / 1e9 / HBM_PEAK_GBS,
                                  "event_bytes_share": ev_bytes / (total_attn_bytes + ev_bytes)}

    if not args.no_kernel_timing:
        # second pass over the same steps with HIP events (on the launch stream) bracketing the attention
        # launches of every eviction window: first launch of the window .. last launch before the event
        # kernels.  elapsed / launches is the average launch duration, inter-launch gaps included.
        reset()
        n_win = (K_steps + L - 1) // L
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_win)]
        run(K_steps, pairs)
        torch.cuda.synchronize()
        total_ms = sum(a.elapsed_time(b) for a, b in pairs)
        ms = np.array([total_ms / K_steps])
        avg_bytes = total_attn_bytes / K_steps
        achieved = avg_bytes / (ms.mean() * 1e-3) / 1e9
        result["roofline"] = {"kernel": "attn_kernel (fk_decode_step_feat: append + attention + attention-feature update, one launch)" if args.features
                              else "attn_kernel (fk_decode_step: append + split-K attention + merge, one launch)", "bound": "hbm", "achieved": achieved,
                              "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                              "traffic": measured_traffic(w, K_steps, args.features),
                              "avg_launch_us": float(ms.mean() * 1e3), "algorithmic_bytes_per_launch": avg_bytes}
        # the event kernels, over the events in which every row is over budget (HIP events between the calls)
        full = [(t, kev) for (t, kev) in ev_kernels if lens_at[t].min() > B]
        if full:
            us = [float(np.mean([k[i].elapsed_time(k[i + 1]) for _, k in full])) * 1e3 for i in range(3)]
            pairs = float(np.mean([lens_at[t].sum() for t, _ in full])) * w.n_kv_heads   # retained pairs scored per event
            rows_ = w.batch * w.n_kv_heads
            e = w.elem_bytes
            sc_bytes = pairs * (2 * w.head_dim * e + 4)
            sc_flops = pairs * (2.0 * (2 * w.head_dim + (6 * w.group if args.features else 0)) * w.hidden + 4 * w.hidden)
            sel_bytes = 4 * pairs + rows_ * 4 * B
            cp_bytes = rows_ * B * (2 * 2 * w.head_dim * e + 8)
            result["event_kernels"] = {
                "events_timed": len(full), "pairs_per_event": pairs,
                "score": {"us": us[0], "algorithmic_gbs": sc_bytes / us[0] / 1e3, "tflops": sc_flops / us[0] / 1e6},
                "select": {"us": us[1], "algorithmic_gbs": sel_bytes / us[1] / 1e3},
                "compact": {"us": us[2], "algorithmic_gbs_upper": cp_bytes / us[2] / 1e3,
                            "note": "bytes if every kept pair moved; includes the length clamp launch"}}
    if "roofline" in result:
        # achievable streaming-read bandwidth on this machine, beside the nominal peak: the K cache of this
        # workload (fits the Infinity Cache at the default shape) and a 4 GiB buffer (HBM resident)
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        big = torch.empty(1 << 30, dtype=torch.int32, device="cuda")
        big.fill_(1)
        def stream_gbs(t, iters):
            for _ in range(3):
                fk.fk_stream_read(t, sink, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(iters):
                fk.fk_stream_read(t, sink, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            return t.numel() * t.element_size() * iters / (e0.elapsed_time(e1) * 1e-3) / 1e9
        result["roofline"]["stream_read_gbs"] = {"k_cache": stream_gbs(Kc, 50), "buffer_4gib": stream_gbs(big, 10)}
        del big
    if not args.no_cpu and not args.features:   # the oracle's protocol loop covers the default path
        result["cpu_baseline"] = cpu_baseline(w, host_threads)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
