"""Helpers shared by the test files: build oracle-side caches from the seeded generator."""
from __future__ import annotations

import numpy as np

import synth_inputs as si


def store(x32: np.ndarray, dtype: str) -> np.ndarray:
    return si.storage_array(si.round_to_storage(x32, dtype), dtype)


def widen(a: np.ndarray, dtype: str) -> np.ndarray:
    """storage array -> float64 values"""
    if dtype == "f32":
        return a.astype(np.float64)
    return si.from_bf16_bits(a).astype(np.float64)


def random_cache(oracle, seed, dtype, Bt, Hkv, cap, D, lens, scale=1.0, shuffle_pos=False):
    """Cache filled from the counter generator; positions ascending (or shuffled) per row."""
    rng_idx = np.arange(Bt * Hkv * cap * D)
    K = (si.normal(seed, si.T_K, 0, rng_idx).reshape(Bt, Hkv, cap, D) * scale).astype(np.float32)
    V = (si.normal(seed, si.T_V, 0, rng_idx).reshape(Bt, Hkv, cap, D) * scale).astype(np.float32)
    c = oracle.new_cache(dtype, Bt, Hkv, cap, D)
    c.K[...] = store(K, dtype)
    c.V[...] = store(V, dtype)
    c.len[...] = np.asarray(lens, np.int32)
    for b in range(Bt):
        for h in range(Hkv):
            n = int(c.len[b])
            p = np.arange(n, dtype=np.int32) * 3 + 5
            if shuffle_pos:
                perm = np.argsort(si.uniform01(seed, si.T_FLAG, 0, np.arange(n) + 1000 * (b * Hkv + h)))
                p = p[perm]
            c.pos[b, h, :n] = p
    return c


def random_q(seed, dtype, Bt, Hq, D, scale=1.0):
    q = (si.normal(seed, si.T_Q, 0, np.arange(Bt * Hq * D)).reshape(Bt, Hq, D) * scale).astype(np.float32)
    return store(q, dtype)


def workload_cache(oracle, w: si.Workload, layer=0, batch_sel=None, head_sel=None, lens=None):
    """Prompt-filled oracle cache for (a slice of) a workload."""
    bs = np.arange(w.batch) if batch_sel is None else np.asarray(batch_sel)
    hs = np.arange(w.n_kv_heads) if head_sel is None else np.asarray(head_sel)
    lens_all = si.initial_lengths(w) if lens is None else np.asarray(lens, np.int32)
    lens_sel = lens_all[bs]
    c = oracle.new_cache(w.dtype, len(bs), len(hs), w.capacity, w.head_dim)
    pmax = int(lens_sel.max())
    K, V = si.gen_kv(w, layer, 0, pmax, batch_sel=bs, head_sel=hs)
    c.K[:, :, :pmax] = si.storage_array(K, w.dtype)
    c.V[:, :, :pmax] = si.storage_array(V, w.dtype)
    for i in range(len(bs)):
        n = int(lens_sel[i])
        c.pos[i, :, :n] = np.arange(n, dtype=np.int32)
        c.pos[i, :, n:] = -1
    c.len[...] = lens_sel
    return c


def step_inputs(w: si.Workload, layer, t, lens0, batch_sel=None, kv_head_sel=None):
    """(q, k_new, v_new, pos_new) in storage form for decode step t (absolute position = len0 + t)."""
    bs = np.arange(w.batch) if batch_sel is None else np.asarray(batch_sel)
    hk = np.arange(w.n_kv_heads) if kv_head_sel is None else np.asarray(kv_head_sel)
    g = w.group
    hq = (hk[:, None] * g + np.arange(g)[None, :]).reshape(-1)
    D = w.head_dim
    q = np.empty((len(bs), len(hq), D), np.float32)
    k = np.empty((len(bs), len(hk), D), np.float32)
    v = np.empty((len(bs), len(hk), D), np.float32)
    pos_new = np.empty(len(bs), np.int32)
    for i, b in enumerate(bs):
        p = int(lens0[b]) + t
        pos_new[i] = p
        q[i] = si.gen_q(w, layer, p, p + 1, batch_sel=[b], head_sel=hq)[0, :, 0]
        kk, vv = si.gen_kv(w, layer, p, p + 1, batch_sel=[b], head_sel=hk)
        k[i], v[i] = kk[0, :, 0], vv[0, :, 0]
    return (si.storage_array(q, w.dtype), si.storage_array(k, w.dtype), si.storage_array(v, w.dtype), pos_new)


def scorer_storage(w: si.Workload, layer=0, head_sel=None):
    """(W1, b1, W2, b2) with W1 in storage form, optionally restricted to some KV heads."""
    W1, b1, W2, b2 = si.gen_scorer(w, layer)
    if head_sel is not None:
        hs = np.asarray(head_sel)
        W1, b1, W2, b2 = W1[hs], b1[hs], W2[hs], b2[hs]
    return si.storage_array(W1, w.dtype), b1, W2, b2


def bulk_step_inputs(w: si.Workload, layer, t0, t1, lens0, batch_sel=None, kv_head_sel=None):
    """Inputs of decode steps t0 .. t1-1 at once, storage form:
    q [steps, nb, nhq, D], k_new, v_new [steps, nb, nhk, D], pos_new [steps, nb]."""
    bs = np.arange(w.batch) if batch_sel is None else np.asarray(batch_sel)
    hk = np.arange(w.n_kv_heads) if kv_head_sel is None else np.asarray(kv_head_sel)
    g = w.group
    hq = (hk[:, None] * g + np.arange(g)[None, :]).reshape(-1)
    steps, D = t1 - t0, w.head_dim
    st = np.float32 if w.dtype == "f32" else np.uint16
    q = np.empty((steps, len(bs), len(hq), D), st)
    k = np.empty((steps, len(bs), len(hk), D), st)
    v = np.empty((steps, len(bs), len(hk), D), st)
    pos = np.empty((steps, len(bs)), np.int32)
    for i, b in enumerate(bs):
        p0 = int(lens0[b]) + t0
        pos[:, i] = np.arange(p0, p0 + steps)
        qq = si.gen_q(w, layer, p0, p0 + steps, batch_sel=[b], head_sel=hq)[0]          # [nhq, steps, D]
        kk, vv = si.gen_kv(w, layer, p0, p0 + steps, batch_sel=[b], head_sel=hk)
        q[:, i] = si.storage_array(qq.transpose(1, 0, 2), w.dtype)
        k[:, i] = si.storage_array(kk[0].transpose(1, 0, 2), w.dtype)
        v[:, i] = si.storage_array(vv[0].transpose(1, 0, 2), w.dtype)
    return q, k, v, pos


def workload_cache_replicated(oracle, w: si.Workload, rows, layer=0):
    """Prompt-filled cache of the whole workload in which only the (b, h) rows listed in ``rows`` hold the
    generator's data; every other row is a copy of one of them, cut to its own sequence's length.  For full-size
    parity runs: the device works on every row, the oracle follows ``rows`` only, and drawing tens of
    gigabytes from the counter generator on the host would take minutes."""
    lens = si.initial_lengths(w)
    c = oracle.new_cache(w.dtype, w.batch, w.n_kv_heads, w.capacity, w.head_dim)
    c.len[...] = lens
    src = []
    for (b, h) in rows:
        n = int(lens[b])
        K, V = si.gen_kv(w, layer, 0, n, batch_sel=[b], head_sel=[h])
        c.K[b, h, :n] = si.storage_array(K, w.dtype)[0, 0]
        c.V[b, h, :n] = si.storage_array(V, w.dtype)[0, 0]
        src.append((b, h, n))
    longest = max(src, key=lambda t: t[2])
    i = 0
    for b in range(w.batch):
        n = int(lens[b])
        c.pos[b, :, :n] = np.arange(n, dtype=np.int32)
        for h in range(w.n_kv_heads):
            if (b, h) in rows:
                continue
            sb, sh, sn = src[i % len(src)] if src[i % len(src)][2] >= n else longest
            i += 1
            m = min(n, sn)
            c.K[b, h, :m], c.V[b, h, :m] = c.K[sb, sh, :m], c.V[sb, sh, :m]
            if m < n:   # longer than any sampled row: repeat the source
                for o in range(m, n, sn):
                    e = min(o + sn, n)
                    c.K[b, h, o:e], c.V[b, h, o:e] = c.K[sb, sh, :e - o], c.V[sb, sh, :e - o]
    return c
