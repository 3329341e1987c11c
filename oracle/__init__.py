"""CPU oracle of the budgeted-KV decode + evict path (TEST INFRASTRUCTURE ONLY).

Thin ctypes access to ``fk_oracle.c`` plus the step/event protocol of Section 3.1
written as a plain Python loop.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; it imports nothing from the HIP package
and the HIP package imports nothing from here.

Arrays are numpy, host memory.  K, V, q, W1 are passed in the storage type of the
workload: float32 arrays for 'f32', uint16 bit patterns for 'bf16'.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fk_oracle.c")
# FK_ORACLE_SANITIZE=1: the same source built with AddressSanitizer + UndefinedBehaviorSanitizer into a library of its
# own (the process must have the ASan runtime preloaded); the tests run the pins under it in a child process.
_SANITIZE = os.environ.get("FK_ORACLE_SANITIZE", "") == "1"
_SO = os.path.join(_HERE, "libfk_oracle_san.so" if _SANITIZE else "libfk_oracle.so")
_lib = None

F32, BF16 = 0, 1
_DT = {"f32": F32, "bf16": BF16}


def build(force: bool = True) -> str:
    """Compile the oracle with gcc (-O2, OpenMP for the trivially parallel row loops)."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-fopenmp", "-shared", "-fPIC", "-Wall", "-o", _SO, _SRC, "-lm"])
    return _SO


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        _lib = ctypes.CDLL(_SO)
        _lib.ora_select_keep.restype = ctypes.c_int
        _lib.ora_select_keep_sampled.restype = ctypes.c_int
        _lib.ora_append.restype = ctypes.c_int
        _lib.ora_max_threads.restype = ctypes.c_int
        _lib.ora_get_threads.restype = ctypes.c_int
    return _lib


def set_threads(n: int) -> None:
    lib().ora_set_threads(ctypes.c_int(int(n)))


def max_threads() -> int:
    return int(lib().ora_max_threads())


def _p(a: np.ndarray):
    assert a.flags["C_CONTIGUOUS"], "oracle arrays must be C contiguous"
    return a.ctypes.data_as(ctypes.c_void_p)


def _check_store(a: np.ndarray, dtype: str):
    want = np.float32 if dtype == "f32" else np.uint16
    assert a.dtype == want, f"storage array for {dtype} must be {want}, got {a.dtype}"


@dataclass
class Cache:
    """Host copy of one layer's cache: K, V [Bt,Hkv,cap,D] storage, pos [Bt,Hkv,cap], len [Bt]."""
    dtype: str
    K: np.ndarray
    V: np.ndarray
    pos: np.ndarray
    len: np.ndarray

    @property
    def shape(self):
        return self.K.shape

    def copy(self) -> "Cache":
        return Cache(self.dtype, self.K.copy(), self.V.copy(), self.pos.copy(), self.len.copy())


def new_cache(dtype: str, batch: int, n_kv: int, cap: int, D: int) -> Cache:
    st = np.float32 if dtype == "f32" else np.uint16
    return Cache(dtype, np.zeros((batch, n_kv, cap, D), st), np.zeros((batch, n_kv, cap, D), st),
                 np.full((batch, n_kv, cap), -1, np.int32), np.zeros(batch, np.int32))


def append(c: Cache, k_new: np.ndarray, v_new: np.ndarray, pos_new: np.ndarray) -> None:
    """One new (k, v, position) per sequence joins every KV-head row (Section 3.1)."""
    Bt, Hkv, cap, D = c.shape
    _check_store(k_new, c.dtype)
    _check_store(v_new, c.dtype)
    assert k_new.shape == (Bt, Hkv, D) and v_new.shape == (Bt, Hkv, D)
    pn = np.ascontiguousarray(pos_new, dtype=np.int32)
    rc = lib().ora_append(_DT[c.dtype], Bt, Hkv, D, cap, _p(c.K), _p(c.V), _p(c.pos), _p(c.len),
                          _p(np.ascontiguousarray(k_new)), _p(np.ascontiguousarray(v_new)), _p(pn))
    if rc != 0:
        raise RuntimeError("append beyond capacity")


def decode_attn(c: Cache, q: np.ndarray, scale: float) -> np.ndarray:
    """Retained-set attention (Appendix A, Problem Setup).  q [Bt,Hq,D] storage -> float64 [Bt,Hq,D]."""
    Bt, Hkv, cap, D = c.shape
    _check_store(q, c.dtype)
    Hq = q.shape[1]
    assert q.shape == (Bt, Hq, D) and Hq % Hkv == 0
    out = np.empty((Bt, Hq, D), np.float64)
    lib().ora_decode_attn(_DT[c.dtype], Bt, Hq, Hkv, D, cap, _p(np.ascontiguousarray(q)), _p(c.K), _p(c.V),
                          _p(c.len), ctypes.c_double(scale), _p(out))
    return out


def score_kv(c: Cache, W1: np.ndarray, b1: np.ndarray, W2: np.ndarray, b2: np.ndarray) -> np.ndarray:
    """MLP scorer on concat(k, v) (Appendix B.1).  W1 [Hkv or 1, 2D, H] storage; b1, W2 [., H], b2 [.]
    float32.  Returns float64 [Bt,Hkv,cap]; slots >= len hold NaN."""
    Bt, Hkv, cap, D = c.shape
    _check_store(W1, c.dtype)
    nset, F, H = W1.shape
    assert F == 2 * D and nset in (1, Hkv)
    assert b1.shape == (nset, H) and W2.shape == (nset, H) and b2.shape == (nset,)
    sc = np.full((Bt, Hkv, cap), np.nan, np.float64)
    lib().ora_score_kv(_DT[c.dtype], Bt, Hkv, D, cap, _p(c.K), _p(c.V), _p(c.len), _p(np.ascontiguousarray(W1)),
                       _p(np.ascontiguousarray(b1, np.float32)), _p(np.ascontiguousarray(W2, np.float32)),
                       _p(np.ascontiguousarray(b2, np.float32)), H, int(nset == 1 and Hkv != 1), _p(sc))
    return sc


def select_keep(scores: np.ndarray, pos: np.ndarray, length: np.ndarray, budget: int, recent: int,
                method: str = "rank") -> np.ndarray:
    """Keep the ``recent`` newest pairs plus the top ``budget - recent`` of the others, order
    (score desc, position asc) (Section 3.1).  scores float32 [Bt,Hkv,cap].  Returns int32
    [Bt,Hkv,budget], kept slots ascending; -1 where a row under budget has fewer entries."""
    Bt, Hkv, cap = scores.shape
    assert scores.dtype == np.float32, "selection decides on the fp32 scores both sides see"
    keep = np.full((Bt, Hkv, budget), -1, np.int32)
    rc = lib().ora_select_keep(Bt, Hkv, cap, _p(np.ascontiguousarray(scores)), _p(np.ascontiguousarray(pos, np.int32)),
                               _p(np.ascontiguousarray(length, np.int32)), budget, recent,
                               {"rank": 0, "sort": 1}[method], _p(keep))
    if rc != 0:
        raise RuntimeError(f"ora_select_keep failed ({rc})")
    return keep


def select_keep_sampled(scores: np.ndarray, noise: np.ndarray, pos: np.ndarray, length: np.ndarray, budget: int,
                        recent: int, n_cand: int) -> np.ndarray:
    """Top-K multinomial eviction (Section 3.1 Eq. 2, Appendix B.2) in Gumbel-top-k form: the ``n_cand``
    lowest-scored non-recent pairs are candidates; of them the ``len - budget`` with the smallest fp32
    ``score - noise`` are evicted.  scores, noise float32 [Bt,Hkv,cap].  Returns int32 [Bt,Hkv,budget]."""
    Bt, Hkv, cap = scores.shape
    assert scores.dtype == np.float32 and noise.dtype == np.float32 and noise.shape == scores.shape
    keep = np.full((Bt, Hkv, budget), -1, np.int32)
    rc = lib().ora_select_keep_sampled(Bt, Hkv, cap, _p(np.ascontiguousarray(scores)), _p(np.ascontiguousarray(noise)),
                                       _p(np.ascontiguousarray(pos, np.int32)), _p(np.ascontiguousarray(length, np.int32)),
                                       budget, recent, n_cand, _p(keep))
    if rc != 0:
        raise RuntimeError(f"ora_select_keep_sampled failed ({rc})")
    return keep


def compact(c: Cache, keep_idx: np.ndarray, budget: int) -> None:
    """Stable in-place compaction of K, V, pos to ``budget`` entries for rows over budget."""
    Bt, Hkv, cap, D = c.shape
    assert keep_idx.shape == (Bt, Hkv, budget) and keep_idx.dtype == np.int32
    lib().ora_compact(_DT[c.dtype], Bt, Hkv, D, cap, _p(c.K), _p(c.V), _p(c.pos), _p(c.len),
                      _p(np.ascontiguousarray(keep_idx)), budget)


def evict(c: Cache, scorer, budget: int, recent: int, method: str = "rank"):
    """One eviction event: score every retained pair, select, compact.  Returns (scores64, keep_idx)."""
    sc = score_kv(c, *scorer)
    keep = select_keep(sc.astype(np.float32), c.pos, c.len, budget, recent, method)
    compact(c, keep, budget)
    return sc, keep


def run_protocol(c: Cache, step_inputs, n_steps: int, scorer, budget: int, interval: int, scale: float,
                 t0: int = 0, on_step=None, on_event=None, method: str = "rank") -> None:
    """Generation with a budgeted cache (Section 3.1): each step appends the new pair and attends
    over the retained set; after every ``interval`` steps the rows over ``budget`` are scored,
    pruned to the ``interval`` newest plus the top ``budget - interval`` others, and compacted.

    step_inputs(t) -> (q, k_new, v_new, pos_new) in storage form.  on_step(t, out64) and
    on_event(t, scores64, keep_idx, cache_before) are optional observers.
    """
    for t in range(t0, t0 + n_steps):
        q, k_new, v_new, pos_new = step_inputs(t)
        append(c, k_new, v_new, pos_new)
        out = decode_attn(c, q, scale)
        if on_step is not None:
            on_step(t, out)
        if (t + 1) % interval == 0:
            before = c.copy() if on_event is not None else None
            sc, keep = evict(c, scorer, budget, interval, method)
            if on_event is not None:
                on_event(t, sc, keep, before)


# ---------------------------------------------------------------------------------------------
# Attention features of the scoring model (Appendix B.1, "Attention Features")
#
# For every retained pair n and every query head h of its group, six numbers built from the
# attention weights a_hat the pair has received:
#   w8, w16, w32, wL : sums over the last 8 / 16 / 32 / L queries before the eviction event
#                      (L = the update length; a window longer than the chunk is the whole chunk),
#   cum              : sum over all chunks since the pair entered the cache (direct sum),
#   dec              : the same with a decay of 0.9 per chunk, dec <- 0.9 dec + wL at every event.
# a_n concatenates the six numbers of head 0, then head 1, ... (6 g values).
# Readings (the paper gives one sentence): "attention scores" are the softmax weights; a chunk is
# the L queries between two events; a pair appended mid-chunk starts from zero and counts the
# weight of its own query.
# ---------------------------------------------------------------------------------------------
FEAT_WINDOWS = (8, 16, 32)
FEAT_DECAY = 0.9
W8, W16, W32, WL, CUM, DEC = range(6)


def decode_attn_probs(c: Cache, q: np.ndarray, scale: float):
    """decode_attn plus the attention weights: (out [Bt,Hq,D], probs [Bt,Hq,cap], 0 past len)."""
    Bt, Hkv, cap, D = c.shape
    _check_store(q, c.dtype)
    Hq = q.shape[1]
    out = np.empty((Bt, Hq, D), np.float64)
    probs = np.zeros((Bt, Hq, cap), np.float64)
    lib().ora_decode_attn_probs(_DT[c.dtype], Bt, Hq, Hkv, D, cap, _p(np.ascontiguousarray(q)), _p(c.K), _p(c.V),
                                _p(c.len), ctypes.c_double(scale), _p(out), _p(probs))
    return out, probs


def new_feat(batch: int, n_kv: int, cap: int, g: int) -> np.ndarray:
    """Feature state [Bt, Hkv, cap, g, 6] float64, all zero."""
    return np.zeros((batch, n_kv, cap, g, 6), np.float64)


def feat_step(feat: np.ndarray, probs: np.ndarray, lens_before: np.ndarray, chunk_pos: int, L: int) -> None:
    """Account one query (chunk step ``chunk_pos`` in 0..L-1): every live slot gains its weight in wL
    and in the windows that reach back to this step; the slot appended at this step starts from zero."""
    Bt, Hkv, cap, g, _ = feat.shape
    p = probs.reshape(Bt, Hkv, g, cap).transpose(0, 1, 3, 2)          # [Bt,Hkv,cap,g]
    for b in range(Bt):
        feat[b, :, int(lens_before[b])] = 0.0                        # the new pair's slot
    feat[..., WL] += p
    for plane, wnd in ((W8, 8), (W16, 16), (W32, 32)):
        if chunk_pos >= L - wnd:
            feat[..., plane] += p


def feat_vectors(feat: np.ndarray) -> np.ndarray:
    """The scorer's view at an event: [Bt,Hkv,cap,6g] with cum and dec already including this chunk."""
    f = feat.copy()
    f[..., CUM] = feat[..., CUM] + feat[..., WL]
    f[..., DEC] = FEAT_DECAY * feat[..., DEC] + feat[..., WL]
    Bt, Hkv, cap, g, _ = f.shape
    return np.ascontiguousarray(f.reshape(Bt, Hkv, cap, 6 * g))


def feat_roll_and_compact(feat: np.ndarray, keep_idx: np.ndarray, lens_before: np.ndarray, budget: int) -> None:
    """Close the chunk: cum += wL, dec = 0.9 dec + wL, windows cleared; rows over budget are gathered
    to the kept slots in order, like K and V."""
    Bt, Hkv, cap, g, _ = feat.shape
    feat[..., CUM] += feat[..., WL]
    feat[..., DEC] = FEAT_DECAY * feat[..., DEC] + feat[..., WL]
    feat[..., :4] = 0.0
    for b in range(Bt):
        if lens_before[b] > budget:
            for h in range(Hkv):
                feat[b, h, :budget] = feat[b, h, keep_idx[b, h]]
                feat[b, h, budget:] = 0.0


def score_kv_feat(c: Cache, fvec: np.ndarray, W1: np.ndarray, b1: np.ndarray, W2: np.ndarray, b2: np.ndarray) -> np.ndarray:
    """Scorer on x = concat(k, v, a) (Section 3.1 Eq. 1).  fvec [Bt,Hkv,cap,A] float64; W1 [., 2D + A, H]."""
    Bt, Hkv, cap, D = c.shape
    _check_store(W1, c.dtype)
    A = fvec.shape[-1]
    nset, F, H = W1.shape
    assert F == 2 * D + A and nset in (1, Hkv) and fvec.shape == (Bt, Hkv, cap, A) and fvec.dtype == np.float64
    sc = np.full((Bt, Hkv, cap), np.nan, np.float64)
    lib().ora_score_kv_feat(_DT[c.dtype], Bt, Hkv, D, cap, _p(c.K), _p(c.V), _p(np.ascontiguousarray(fvec)), A, _p(c.len),
                            _p(np.ascontiguousarray(W1)), _p(np.ascontiguousarray(b1, np.float32)),
                            _p(np.ascontiguousarray(W2, np.float32)), _p(np.ascontiguousarray(b2, np.float32)), H,
                            int(nset == 1 and Hkv != 1), _p(sc))
    return sc
