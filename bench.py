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


def cpu_baseline(w: si.Workload, threads: int, start_len: int, clock0: int, n_steps: int, budget_s: float = 25.0):
    """Time the CPU oracle, as it stands, on the window the GPU timed: the full batch with every row holding
    `start_len` pairs, step clock at `clock0` (an eviction event after every step t with (clock0 + t + 1) % L
    == 0), `n_steps` decode steps.  If that is more than about `budget_s` seconds of CPU work, the sample is
    the first whole eviction windows of it (same cache lengths) and the rate is an extrapolation to the whole
    region.  Seconds are kept per part: append + attention, score, select, compact."""
    import oracle
    B, L, Bt = w.budget, w.interval, w.batch
    # about 22 ms per step of the Qwen3-4B layer shape on 16 cores: bound the sample by whole windows
    per_step = 2.2e-2 * (Bt * w.n_kv_heads * (B + L) * w.head_dim) / (128 * 2176 * 128) * (16.0 / max(threads, 1))
    max_steps = max(L, int(budget_s / max(per_step, 1e-9)) // L * L)
    sample = n_steps if n_steps <= max_steps else max_steps
    wl = w
    W1, b1, W2, b2 = si.gen_scorer(w, 0)
    scorer = (si.storage_array(W1, w.dtype), b1, W2, b2)
    K, V = si.gen_kv(wl, 0, 0, start_len)
    K, V = si.storage_array(K, w.dtype), si.storage_array(V, w.dtype)
    qs = si.storage_array(si.gen_q(wl, 0, start_len, start_len + sample), w.dtype)
    ks, vs = (si.storage_array(x, w.dtype) for x in si.gen_kv(wl, 0, start_len, start_len + sample))
    step_in = [(np.ascontiguousarray(qs[:, :, t]), np.ascontiguousarray(ks[:, :, t]), np.ascontiguousarray(vs[:, :, t]),
                np.full(Bt, start_len + t, np.int32)) for t in range(sample)]

    def run(nthreads):
        oracle.set_threads(nthreads)
        c = oracle.new_cache(w.dtype, Bt, w.n_kv_heads, w.capacity, w.head_dim)
        c.K[:, :, :start_len], c.V[:, :, :start_len] = K, V
        c.pos[:, :, :start_len] = np.arange(start_len, dtype=np.int32)
        c.len[:] = start_len
        part = {"append_attention": 0.0, "score": 0.0, "select": 0.0, "compact": 0.0}
        events = 0
        t_all = time.perf_counter()
        for t in range(sample):
            q, kn, vn, pn = step_in[t]
            t0 = time.perf_counter()
            oracle.append(c, kn, vn, pn)
            oracle.decode_attn(c, q, w.softmax_scale)
            t1 = time.perf_counter()
            part["append_attention"] += t1 - t0
            if (clock0 + t + 1) % L == 0:
                sc = oracle.score_kv(c, *scorer)
                t2 = time.perf_counter()
                keep = oracle.select_keep(sc.astype(np.float32), c.pos, c.len, B, L, "sort")
                t3 = time.perf_counter()
                oracle.compact(c, keep, B)
                t4 = time.perf_counter()
                part["score"] += t2 - t1
                part["select"] += t3 - t2
                part["compact"] += t4 - t3
                events += 1
        return time.perf_counter() - t_all, part, events

    dt, part, events = run(threads)
    what = (f"full batch ({Bt} sequences x {w.n_kv_heads} KV heads), rows at {start_len} pairs, {sample} decode steps "
            f"with {events} eviction event(s)")
    out = {"value": Bt * sample / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
           "sample": f"{what}, {dt:.1f}s CPU on {threads} cores"
                     + ("" if sample == n_steps else f"; EXTRAPOLATED: the first {sample} of the {n_steps} timed steps, same cache lengths in every window"),
           "extrapolated": sample != n_steps, "seconds_by_part": {k: round(v, 3) for k, v in part.items()},
           "events_in_sample": events}
    if dt * threads * 0.7 <= 40.0:   # the same sample on ONE core, when that stays within the time bound
        dt1, part1, _ = run(1)
        out["value_1core"] = Bt * sample / dt1
        out["sample_1core"] = f"the same sample on one core, {dt1:.1f}s CPU"
        out["seconds_by_part_1core"] = {k: round(v, 3) for k, v in part1.items()}
    oracle.set_threads(threads)
    return out


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
    e2 = [torch.cuda.Event(enable_timing=True) for _ in range(K_steps)]
    for i in range(K_steps):
        e0[i].record(stream)
        fk.fk_golden_scores(A, Hkv, T, B, L, a_t, alpha, stream)
        e1[i].record(stream)
        fk.fk_golden_trace(alpha, T, B, L, kept, stream)
        e2[i].record(stream)
    torch.cuda.synchronize()
    ms = float(np.mean([a.elapsed_time(b) for a, b in zip(e0, e1)]))
    ms_trace = float(np.mean([a.elapsed_time(b) for a, b in zip(e1, e2)]))
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
        "trace": {"kernel": "golden_trace_kernel (fk_golden_trace): M sequential selections, one workgroup per KV group",
                  "us": ms_trace * 1e3, "us_per_step": ms_trace * 1e3 / M},
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


def bench_oneshot(args):
    """One-shot compression after the prefill (Section 4.3, long-input tasks: the cache is compressed once, no repeated
    eviction): rows of n = 65536 and of 131072 pairs are scored, pruned to B = 2048 (128 newest protected) and compacted
    in one event.  Qwen3-4B layer heads (32 query / 8 KV heads, head_dim 128, bf16), 2 GiB of K + V per case, inputs
    drawn on the device in the distribution of the single-layer workload.  A step = one event; the cache prefix that
    the compaction overwrites is restored between steps, outside the timed brackets."""
    import torch
    import paper_2602_03203_amd as fk
    fk.lib()
    torch.cuda.set_device(0)
    Hq, Hkv, D, B, R, H = 32, 8, 128, 2048, 128, 256
    K_steps = args.steps if args.steps is not None else 10
    W_steps = min(args.warmup, 3)
    gen = torch.Generator(device="cuda").manual_seed(2602)
    sd = 1.0 / np.sqrt(D)
    W1 = (torch.randn((Hkv, 2 * D, H), generator=gen, device="cuda") / np.sqrt(2 * D)).to(torch.bfloat16)
    b1 = torch.randn((Hkv, H), generator=gen, device="cuda") / np.sqrt(2 * D)
    W2 = torch.randn((Hkv, H), generator=gen, device="cuda") / np.sqrt(H)
    b2 = torch.randn((Hkv,), generator=gen, device="cuda") / np.sqrt(H)
    stream = torch.cuda.current_stream()
    cases = []
    for n, Bt in ((65536, 8), (131072, 4)):
        rows = Bt * Hkv
        desc = fk.CacheDesc(Bt, Hq, Hkv, D, n, "bf16")
        heavy = 1.0 + 2.0 * (torch.rand((Bt, 1, n, 1), generator=gen, device="cuda") < 0.01).float()
        K = (torch.randn((Bt, Hkv, n, D), generator=gen, device="cuda") * sd * heavy).to(torch.bfloat16)
        V = (torch.randn((Bt, Hkv, n, D), generator=gen, device="cuda") * sd).to(torch.bfloat16)
        del heavy
        pos = torch.arange(n, dtype=torch.int32, device="cuda").expand(Bt, Hkv, n).contiguous()
        ln = torch.full((Bt, Hkv), n, dtype=torch.int32, device="cuda")
        K0, V0, pos0 = K[:, :, :B].clone(), V[:, :, :B].clone(), pos[:, :, :B].clone()
        scores = torch.zeros((Bt, Hkv, n), dtype=torch.float32, device="cuda")
        keep = torch.zeros((Bt, Hkv, B), dtype=torch.int32, device="cuda")
        sel_ws = torch.empty(max(fk.fk_select_keep_workspace(desc, n, B, R), 16), dtype=torch.uint8, device="cuda")
        us = np.zeros(3)
        wall = 0.0
        for it in range(W_steps + K_steps):
            K[:, :, :B].copy_(K0); V[:, :, :B].copy_(V0); pos[:, :, :B].copy_(pos0); ln.fill_(n)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev[0].record(stream)
            fk.fk_score_kv(desc, K, V, ln, n, W1, b1, W2, b2, scores, stream, skip_len=B)
            ev[1].record(stream)
            fk.fk_select_keep_ws(desc, scores, pos, ln, n, B, R, keep, sel_ws, stream)
            ev[2].record(stream)
            fk.fk_compact(desc, K, V, pos, ln, keep, B, stream)
            ev[3].record(stream)
            torch.cuda.synchronize()
            if it >= W_steps:
                wall += time.perf_counter() - t0
                us += np.array([ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(3)])
        assert int(ln.min()) == B and int(ln.max()) == B
        us /= K_steps
        pairs = float(rows) * n
        moved = float((keep != torch.arange(B, dtype=torch.int32, device="cuda")).sum().item())
        sc_bytes, sc_flops = pairs * (2 * D * 2 + 4), pairs * (2.0 * 2 * D * H + 4 * H)
        sel_bytes = 4 * pairs + rows * 4 * B
        cp_bytes = moved * (2 * 2 * D * 2 + 8)
        cases.append({"pairs_per_row": n, "rows": rows, "ms_per_event": 1e3 * wall / K_steps, "pairs_per_s": pairs * K_steps / wall,
                      "score": {"us": us[0], "algorithmic_gbs": sc_bytes / us[0] / 1e3, "tflops": sc_flops / us[0] / 1e6},
                      "select": {"us": us[1], "algorithmic_gbs": sel_bytes / us[1] / 1e3},
                      "compact": {"us": us[2], "algorithmic_gbs": cp_bytes / us[2] / 1e3, "moved_pairs": moved}})
        del K, V, pos, scores
    big = cases[-1]
    result = {
        "metric": "one-shot post-prefill compression: retained pairs scored + selected + compacted per second (n = 131072 per row -> budget 2048), one layer",
        "value": big["pairs_per_s"], "unit": "pairs/s", "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": big["ms_per_event"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic (drawn on the device)",
        "config": {"workload": "oneshot-qwen3-4b-layer", "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "budget": B,
                   "protect_recent": R, "scorer_hidden": H, "cases": [(c["pairs_per_row"], c["rows"]) for c in cases]},
        "cases": cases,
        "roofline": {"kernel": "score_mfma_kernel (fk_score_kv) at n = 131072", "bound": "mfma", "achieved": big["score"]["tflops"],
                     "peak": 2500.0, "unit": "TFLOP/s", "frac": big["score"]["tflops"] / 2500.0, "traffic": None,
                     "avg_launch_us": big["score"]["us"], "algorithmic_flops_per_launch": big["score"]["tflops"] * big["score"]["us"] * 1e6,
                     "hbm_gbs": big["score"]["algorithmic_gbs"], "frac_of_hbm_peak": big["score"]["algorithmic_gbs"] / HBM_PEAK_GBS},
    }
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
    cfg_no = {"cfg2": 2, "cfg3": 3}.get(w.name[:4])
    ratio = profile_value(f"attn_kernel_cfg{cfg_no}_stack.txt", "traffic_over_algorithmic") if cfg_no and args.prompt is None and args.hidden is None else None
    avg_bytes = sum(step_bytes) / (K_steps * NL)
    result["roofline"] = {"kernel": "attn_kernel (fk_decode_step), all layers of a step between one pair of HIP events", "bound": "hbm",
                          "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                          "traffic": None if ratio is None else ratio * avg_bytes,
                          "traffic_source": None if ratio is None else f"profiles/attn_kernel_cfg{cfg_no}_stack.txt: counter bytes / algorithmic bytes of this command, times this run's algorithmic bytes",
                          "avg_launch_us": ms * 1e3 / (K_steps * NL), "algorithmic_bytes_per_launch": avg_bytes,
                          "working_set_mb": NL * Bt * Hkv * float(np.mean(lens[:K_steps])) * D * 2 * e / 1e6, "resident_in": "hbm"}
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
    ap.add_argument("--workload", choices=["decode", "golden", "oneshot"], default="decode",
                    help="decode: the budgeted decode + evict path (the headline); golden: the Golden Eviction label builder; "
                         "oneshot: one compression event on rows of 65536 / 131072 pairs (long-input use)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-cold", action="store_true", help="skip the HBM-resident (rotating cache copies) attention measurement")
    ap.add_argument("--no-kernel-timing", action="store_true", help="skip the HIP-event pass over the attention launches")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (rows are independent: batch or KV-head sharding needs no exchange inside this path); use --gpus 1")

    if args.workload == "golden":
        return bench_golden(args)
    if args.workload == "oneshot":
        return bench_oneshot(args)
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
    if args.hidden is not None:
        w = w.scaled(name=f"{w.name} (scorer hidden {args.hidden})", hidden=args.hidden)
    B, L = w.budget, w.interval
    K_steps = args.steps if args.steps is not None else w.steps
    W_steps = args.warmup
    # Where the run starts.  Default: the steady state of the protocol (Section 3.1: the cache swings between B and
    # B + L).  Rows start at B + c0 pairs with the step clock at c0, c0 chosen so that the LAST timed step is followed
    # by an eviction event: any number of steps, also fewer than L, times real events at the cache sizes of a long
    # generation.  --prompt P: start from a prompt of P tokens at clock 0 instead (the cache first grows to B + L).
    # Workloads with ragged initial lengths start from those lengths.
    ragged = len(set(int(x) for x in si.initial_lengths(w))) > 1
    steady = args.prompt is None and not ragged
    if steady:
        clock0 = (L - K_steps % L) % L
        start_len = B + clock0
        clock0_w = (L - W_steps % L) % L
        start_len_w = B + clock0_w
    else:
        if args.prompt is not None:
            w = w.scaled(name=f"{w.name} (prompt {args.prompt})", prompt=args.prompt)
        clock0 = clock0_w = 0
        start_len = start_len_w = None
    lens0 = si.initial_lengths(w) if not steady else np.full(w.batch, start_len, np.int32)
    lens0_w = lens0 if not steady else np.full_like(lens0, start_len_w)
    n_gen = max(K_steps, W_steps)

    t0 = time.time()
    # the cache is generated up to the longest start in use, so that the warm-up can start from its own length
    fill = lens0 if not steady else np.full_like(lens0, max(start_len, start_len_w))
    Kh, Vh, posh = gen_prompt(w, fill, host_threads)
    qh, kh, vh, ph = gen_step_inputs(w, lens0, n_gen, host_threads)
    log(f"[bench] generated {w.name}: cache + {n_gen} steps in {time.time() - t0:.1f}s")

    def dev(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    K0, V0, pos0 = dev(Kh), dev(Vh), dev(posh)
    rep = lambda l: np.repeat(l.astype(np.int32)[:, None], w.n_kv_heads, axis=1)      # one count per row
    len0, len0_w = dev(rep(lens0)), dev(rep(lens0_w))
    dq, dk, dv, dp = dev(qh), dev(kh), dev(vh), dev(ph)
    dp_w = dev((ph - lens0[None, :] + lens0_w[None, :]).astype(np.int32))   # the warm-up counts positions from its own start
    del Kh, Vh, qh, kh, vh
    W1, b1, W2, b2 = si.gen_scorer_feat(w, 0) if args.features else si.gen_scorer(w, 0)
    dW = [dev(si.storage_array(W1, w.dtype)), dev(b1), dev(W2), dev(b2)]
    desc = fk.CacheDesc(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.capacity, w.dtype)
    Kc, Vc, posc, lenc = (torch.empty_like(x) for x in (K0, V0, pos0, len0))
    ws = fk.new_attn_workspace(desc)
    feat = fk.new_feat(desc) if args.features else None
    fws = fk.new_feat_workspace(desc) if args.features else None
    dout = torch.empty((L, w.batch, w.n_q_heads, w.head_dim), dtype=desc.torch_dtype, device="cuda")  # outputs of one window
    scores = torch.zeros((w.batch, w.n_kv_heads, w.capacity), dtype=torch.float32, device="cuda")
    keep = torch.zeros((w.batch, w.n_kv_heads, B), dtype=torch.int32, device="cuda")
    slot_idx = torch.arange(B, dtype=torch.int32, device="cuda")
    noise_pool = None
    if args.policy == "sampled":   # Gumbel noise per slot, a pool of 8 independent draws cycled over the events
        noise_pool = [dev(si.gen_gumbel(w.seed, (w.batch, w.n_kv_heads, w.capacity), event=e)) for e in range(8)]
    scale = w.softmax_scale
    stream = torch.cuda.current_stream()

    def schedule(l0, c0, n_steps):
        """Host replay of the protocol's cache sizes: lens [n_steps, Bt] at the attention of step t, and the steps
        after which an event runs."""
        lens = l0.astype(np.int64).copy()
        out = np.empty((n_steps, w.batch), np.int64)
        ev = []
        for t in range(n_steps):
            lens += 1
            out[t] = lens
            if (c0 + t + 1) % L == 0:
                ev.append(t)
                lens = np.minimum(lens, B)
        return out, ev

    def reset(l0_dev):
        Kc.copy_(K0); Vc.copy_(V0); posc.copy_(pos0); lenc.copy_(l0_dev)
        if feat is not None:
            feat.zero_()

    def plan(n_steps, c0, lens_at, pos_dev, rec=None):
        """The library calls of n_steps decode steps from the step clock c0, marshalled NOW (fk.prepare) so that the
        timed loop only makes the calls: a list of zero-argument callables.  Steps between two events go to the
        library as ONE fk_decode_window call (the host comes back once per window, not once per step).  rec: dict
        of lists that receives HIP-event pairs around every window's attention launches and around each of the
        three event kernels, and the number of moved pairs per event (the callables then also record the events)."""
        calls = []
        t = 0
        while t < n_steps:
            seg = min(L - (c0 + t) % L, n_steps - t)
            ml = int(min(lens_at[t].max(), w.capacity))
            if rec is not None:
                e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
                calls.append(lambda ev=e[0]: ev.record(stream))
            if feat is None:
                calls.append(fk.prepare(fk.fk_decode_window, desc, dq[t:t + seg], Kc, Vc, posc, lenc, dk[t:t + seg], dv[t:t + seg],
                                        pos_dev[t:t + seg], seg, ml, scale, dout[:seg], ws, stream))
            else:
                calls.append(fk.prepare(fk.fk_decode_window_feat, desc, dq[t:t + seg], Kc, Vc, posc, lenc, dk[t:t + seg], dv[t:t + seg],
                                        pos_dev[t:t + seg], seg, ml, scale, feat, (c0 + t) % L, L, dout[:seg], fws, stream))
            if rec is not None:
                calls.append(lambda ev=e[1]: ev.record(stream))
                rec["attn"].append((t, seg, e))
            t += seg
            if (c0 + t) % L == 0:
                ml = int(min(lens_at[t - 1].max(), w.capacity))
                kev = None
                if rec is not None:   # [start, after score, after select, after compact]
                    kev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
                    calls.append(lambda ev=kev[0]: ev.record(stream))
                if feat is None:
                    calls.append(fk.prepare(fk.fk_score_kv, desc, Kc, Vc, lenc, ml, *dW, scores, stream, skip_len=B))
                else:
                    calls.append(fk.prepare(fk.fk_score_kv_feat, desc, Kc, Vc, feat, lenc, ml, *dW, scores, stream, skip_len=B))
                if kev:
                    calls.append(lambda ev=kev[1]: ev.record(stream))
                if noise_pool is None:
                    calls.append(fk.prepare(fk.fk_select_keep, desc, scores, posc, lenc, ml, B, L, keep, stream))
                else:
                    calls.append(fk.prepare(fk.fk_select_keep_sampled, desc, scores, noise_pool[((c0 + t) // L) % 8], posc, lenc, ml, B, L,
                                            2 * L, keep, stream))
                if kev:
                    calls.append(lambda ev=kev[2]: ev.record(stream))
                if feat is None:
                    calls.append(fk.prepare(fk.fk_compact, desc, Kc, Vc, posc, lenc, keep, B, stream))
                else:
                    calls.append(fk.prepare(fk.fk_compact_feat, desc, Kc, Vc, posc, feat, lenc, keep, B, stream))
                if kev:
                    calls.append(lambda ev=kev[3]: ev.record(stream))
                    rec["events"].append((t - 1, kev))
                    # pairs whose slot changes (the kept ones already in place cost the compaction nothing)
                    full = bool((lens_at[t - 1] > B).all())
                    calls.append(lambda full=full: rec["moved"].append((keep != slot_idx).sum() if full else None))
        return calls

    def run(n_steps, c0, lens_at, pos_dev, rec=None):
        for call in plan(n_steps, c0, lens_at, pos_dev, rec):
            call()

    lens_at_w, _ = schedule(lens0_w, clock0_w, W_steps) if W_steps else (None, [])
    lens_at, ev_steps = schedule(lens0, clock0, K_steps)
    # warm-up (untimed; with the default start it ends with a full eviction event), then set the timed start state
    if W_steps:
        reset(len0_w)
        run(W_steps, clock0_w, lens_at_w, dp_w)
    torch.cuda.synchronize()
    reset(len0)
    # The reset rewrote the caches; three untimed attention passes WITHOUT append (they change nothing) bring them to
    # where a running generation has them (this layer's K and V last touched by an attention launch) and the clocks up.
    ml0 = int(min(lens0.max(), w.capacity))
    for _ in range(3):
        fk.fk_decode_attn(desc, dq[0], Kc, Vc, lenc, ml0, scale, dout[0], ws, stream)
    torch.cuda.synchronize()
    done = torch.cuda.Event()
    timed_calls = plan(K_steps, clock0, lens_at, dp)   # marshalled before the clock starts
    t0 = time.perf_counter()
    for call in timed_calls:
        call()
    done.record(stream)
    while not done.query():   # poll instead of sleeping in the driver: the wake-up of a blocking wait costs tens of microseconds
        pass
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    final_len = lenc.cpu().numpy()
    assert (final_len == final_len[:, :1]).all()
    final_len = final_len[:, 0]
    expect_len = lens_at[-1].copy()
    if ev_steps and ev_steps[-1] == K_steps - 1:
        expect_len = np.minimum(expect_len, B)
    assert np.array_equal(final_len, expect_len), (final_len, expect_len)

    tokens_per_s = w.batch * K_steps / wall
    total_attn_bytes = sum(attn_bytes(w, lens_at[t]) for t in range(K_steps))
    if args.features:
        total_attn_bytes += sum(feat_bytes(w, lens_at[t], (clock0 + t) % L) for t in range(K_steps))
    ws_mb = 2 * w.batch * w.n_kv_heads * float(lens_at.mean()) * w.head_dim * w.elem_bytes / 1e6
    n_events = len(ev_steps)
    parts = "attention + scorer + top-k + compaction" if n_events else "attention only: no eviction event falls into the timed steps"
    result = {
        "metric": f"decode tokens/s, budgeted KV decode+evict ({parts}), one layer",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": 1e3 * wall / K_steps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": w.batch, "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads,
                   "head_dim": w.head_dim, "budget": B, "eviction_interval": L,
                   "capacity": w.capacity, "scorer_hidden": w.hidden, "eviction_policy": args.policy,
                   "scorer_inputs": "k, v, attention features" if args.features else "k, v",
                   "start": ("steady state of the protocol: rows pre-filled to start_len, step clock offset so that the last timed step is followed by an eviction event"
                             if steady else "prompt, step clock 0"),
                   "start_len": int(lens0.max()) if steady else [int(lens0.min()), int(lens0.max())],
                   "cache_len_range_timed": [int(lens_at.min()), int(lens_at.max())],
                   "events_in_timed_region": n_events, "events_in_warmup": len(schedule(lens0_w, clock0_w, W_steps)[1]) if W_steps else 0},
        "path_gbs_algorithmic": total_attn_bytes / wall / 1e9,
    }

    if not args.no_kernel_timing:
        # second pass over the same steps with HIP events (on the launch stream) around every window's attention
        # launches and around each kernel of every event
        reset(len0)
        rec = {"attn": [], "events": [], "moved": []}
        run(K_steps, clock0, lens_at, dp, rec)
        torch.cuda.synchronize()
        attn_ms = sum(e[0].elapsed_time(e[1]) for _, _, e in rec["attn"])
        attn_us = attn_ms * 1e3 / K_steps
        avg_bytes = total_attn_bytes / K_steps
        achieved = avg_bytes / (attn_us * 1e-6) / 1e9
        ratio, ratio_file = None, None
        if not args.features and args.hidden is None and args.policy == "topk":
            if w.name == "cfg1-qwen3-4b-layer" and steady:
                ratio_file = "attn_kernel_cfg1_hbm_traffic.txt"
            elif w.name == "cfg4-ragged-batch64" and K_steps == w.steps:
                ratio_file = "attn_kernel_cfg4_ragged.txt"
            if ratio_file:
                ratio = profile_value(ratio_file, "traffic_over_algorithmic")
        result["roofline"] = {
            "kernel": "attn_kernel (fk_decode_step_feat: append + attention + attention-feature update, one launch)" if args.features
            else "attn_kernel (fk_decode_step via fk_decode_window: append + attention, one launch per step)",
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": None if ratio is None else ratio * avg_bytes,
            "traffic_source": None if ratio is None else f"profiles/{ratio_file}: counter bytes / algorithmic bytes of the same workload, times this run's algorithmic bytes",
            "avg_launch_us": attn_us, "algorithmic_bytes_per_launch": avg_bytes,
            "working_set_mb": ws_mb,
            "resident_in": "infinity cache (the K + V of this one layer are re-read every step and fit its 256 MB)" if ws_mb < 256 else "hbm"}
        # the event kernels over the events in which every row is over budget
        full = [(t, kev) for (t, kev) in rec["events"] if lens_at[t].min() > B]
        if full:
            us = [float(np.mean([k[i].elapsed_time(k[i + 1]) for _, k in full])) * 1e3 for i in range(3)]
            pairs = float(np.mean([lens_at[t].sum() for t, _ in full])) * w.n_kv_heads   # retained pairs scored per event
            moved = [float(m.item()) for m in rec["moved"] if m is not None]
            moved = float(np.mean(moved)) if moved else 0.0
            rows_ = w.batch * w.n_kv_heads
            e = w.elem_bytes
            sc_bytes = pairs * (2 * w.head_dim * e + 4)
            sc_flops = pairs * (2.0 * (2 * w.head_dim + (6 * w.group if args.features else 0)) * w.hidden + 4 * w.hidden)
            sel_bytes = 4 * pairs + rows_ * 4 * B
            cp_bytes = moved * (2 * 2 * w.head_dim * e + 8)      # read + write of K, V rows and the position of every moved pair
            ev_us = sum(us)
            result["event_kernels"] = {
                "events_timed": len(full), "pairs_per_event": pairs, "moved_pairs_per_event": moved, "event_us": ev_us,
                "score": {"us": us[0], "algorithmic_gbs": sc_bytes / us[0] / 1e3, "tflops": sc_flops / us[0] / 1e6,
                          "frac_of_hbm_peak": sc_bytes / us[0] / 1e3 / HBM_PEAK_GBS, "frac_of_bf16_mfma_peak": sc_flops / us[0] / 1e6 / 2500.0},
                "select": {"us": us[1], "algorithmic_gbs": sel_bytes / us[1] / 1e3},
                "compact": {"us": us[2], "algorithmic_gbs": cp_bytes / us[2] / 1e3}}
            ev_bytes = len(full) * (sc_bytes + sel_bytes + cp_bytes)
            result["path_with_events"] = {"gbs_algorithmic": (total_attn_bytes + ev_bytes) / wall / 1e9,
                                          "frac_of_hbm_peak": (total_attn_bytes + ev_bytes) / wall / 1e9 / HBM_PEAK_GBS,
                                          "event_bytes_share": ev_bytes / (total_attn_bytes + ev_bytes)}
            # what a long generation pays per step: one attention launch plus 1/L of an event
            result["amortised"] = {"tokens_per_s": w.batch / ((attn_us + ev_us / L) * 1e-6), "us_per_step": attn_us + ev_us / L,
                                   "note": "AMORTISED over a whole eviction window from the HIP-event component times: attention launch + event / L; "
                                           "`value` is the wall clock of the timed steps as they ran"}
        # wall clock per step of the plain pass minus the HIP-event kernel time per step of the instrumented pass
        result["host_gap_us_per_step"] = 1e6 * wall / K_steps - (attn_us + (sum(k[0].elapsed_time(k[3]) for _, k in rec["events"]) * 1e3 / K_steps))

        if w.dtype == "bf16" and w.head_dim == 128 and not args.features and not args.no_cold:
            # The same launches with the cache coming from HBM: the attention of a deep stack visits another layer's
            # cache at every launch.  Here: copies of this layer's cache, enough of them to exceed the Infinity Cache
            # several times, visited in turn with the cold-cache flag set; len is restored between rounds.
            n_copies = max(4, int(np.ceil(1536.0 / ws_mb)))
            cdesc = fk.CacheDesc(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.capacity, w.dtype, cold=True)
            cws = fk.new_attn_workspace(cdesc)
            reset(len0)
            copies = [(Kc.clone(), Vc.clone(), posc.clone(), lenc.clone()) for _ in range(n_copies)]
            n_round = min(16, w.capacity - int(lens0.max()) - 1)
            ml = int(min(lens0.max() + n_round + 1, w.capacity))
            def cold_pass():
                for r in range(n_round):
                    for (Kx, Vx, px, lx) in copies:
                        fk.fk_decode_step(cdesc, dq[r], Kx, Vx, px, lx, dk[r], dv[r], dp[r], ml, scale, dout[0], cws, stream)
            cold_pass()
            for c_ in copies:
                c_[3].copy_(len0)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            cold_pass()
            e1.record(stream)
            torch.cuda.synchronize()
            c_us = e0.elapsed_time(e1) * 1e3 / (n_round * n_copies)
            c_bytes = float(np.mean([attn_bytes(w, lens0 + r + 1) for r in range(n_round)]))
            result["roofline_hbm_resident"] = {
                "kernel": "attn_kernel (fk_decode_step with FK_CACHE_COLD), one launch per cache copy in turn", "bound": "hbm",
                "achieved": c_bytes / c_us / 1e3, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": c_bytes / c_us / 1e3 / HBM_PEAK_GBS,
                "avg_launch_us": c_us, "algorithmic_bytes_per_launch": c_bytes, "cache_copies": n_copies,
                "working_set_mb": ws_mb * n_copies, "resident_in": "hbm"}
            del copies
    if "roofline" in result:
        # achievable streaming-read bandwidth on this machine, beside the nominal peak: the K cache of this
        # workload (fits the Infinity Cache at the default shape) and a 4 GiB buffer (HBM resident)
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        big = torch.empty(1 << 30, dtype=torch.int32, device="cuda")
        big.random_(0, 1 << 30)
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
    if not args.no_cpu and not args.features and steady:   # the oracle's protocol loop covers the default path
        result["cpu_baseline"] = cpu_baseline(w, host_threads, int(lens0.max()), clock0, K_steps)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
