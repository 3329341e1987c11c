"""CPU oracle of the Golden Eviction label builder (TEST INFRASTRUCTURE ONLY), Section 3.2 Eq. 3-5.

Given the causal attention matrices A^h [T, T] (row = query, column = key, 0-based positions) of the
query heads of one layer on a full trace of T tokens, a budget B and an eviction length L:

  * the queries from position B + L on are cut into blocks of L; block t = 1 .. M holds the queries
    B + tL .. B + (t+1)L - 1 (the L queries that run on the cache left by eviction step t), with
    M = ceil((T - B) / L) - 1; the last block is zero padded to L queries;
  * Eq. 3: a_t^h = average over the block's L query rows of A^h                  (a vector over keys);
  * Eq. 4: a~_t^{h'} = average of a_t^h over the g query heads of KV group h';
  * Eq. 5: alpha_{i,t} = max over t <= j <= M of a~_{i,j};  eviction step t keeps Top_{B-L} by alpha_{.,t}.

The trace applies Eq. 5 step after step under the cache protocol of Section 3.1: at step t the cache
holds the B pairs kept by step t - 1 (all of 0 .. B + L - 1 before step 1) plus the L pairs generated
since; the L newest stay, the other B are pruned to the B - L with the largest alpha_{.,t} (ties: the
lower position first), and an evicted pair never comes back.

Plain numpy in float64, loops in the order of the definition; nothing here is shared with the HIP path.
"""
from __future__ import annotations

import numpy as np

from . import select_keep


def n_steps(T: int, B: int, L: int) -> int:
    """M = ceil((T - B) / L) - 1 eviction steps (Section 3.2), 0 when the trace never exceeds B + L."""
    return max(-(-(T - B) // L) - 1, 0)


def block_scores(A: np.ndarray, g: int, B: int, L: int) -> np.ndarray:
    """Eq. 3 and 4.  A float64 [Hq, T, C] with C = T, or any subset of the key columns (columns do not
    interact); returns a~ [Hq / g, M, C] (index t - 1 along the block axis)."""
    Hq, T, C = A.shape
    assert Hq % g == 0 and A.dtype == np.float64
    M = n_steps(T, B, L)
    out = np.zeros((Hq // g, M, C), np.float64)
    for t in range(1, M + 1):
        q0, q1 = B + t * L, min(B + (t + 1) * L, T)
        for hp in range(Hq // g):
            acc = np.zeros(C, np.float64)
            for h in range(hp * g, (hp + 1) * g):
                a_h = np.zeros(C, np.float64)
                for q in range(q0, q1):
                    a_h += A[h, q]
                acc += a_h / L              # Eq. 3: average over the L (zero padded) query rows
            out[hp, t - 1] = acc / g        # Eq. 4: average over the group's heads
    return out


def future_scores(a_tilde: np.ndarray) -> np.ndarray:
    """Eq. 5, first half: alpha[h', t - 1, i] = max_{t <= j <= M} a~[h', j - 1, i]."""
    Hkv, M, T = a_tilde.shape
    alpha = np.empty_like(a_tilde)
    for t in range(1, M + 1):
        alpha[:, t - 1] = a_tilde[:, t - 1:M].max(axis=1)
    return alpha


def trace(alpha32: np.ndarray, B: int, L: int) -> np.ndarray:
    """Eq. 5, second half, as an eviction trace.  alpha32 float32 [Hkv, M, T] (the fp32 values both
    sides select on).  Returns int32 [Hkv, M, B]: the positions retained after step t, ascending."""
    Hkv, M, T = alpha32.shape
    assert alpha32.dtype == np.float32
    kept = np.empty((Hkv, M, B), np.int32)
    for hp in range(Hkv):
        cache = np.arange(B + L, dtype=np.int32)            # positions held before step 1
        for t in range(1, M + 1):
            assert cache.size == B + L and cache[-1] == B + t * L - 1
            sc = np.ascontiguousarray(alpha32[hp, t - 1, cache]).reshape(1, 1, B + L)
            idx = select_keep(sc, cache.reshape(1, 1, -1), np.array([B + L], np.int32), B, L, "sort")[0, 0]
            kept[hp, t - 1] = cache[idx]
            cache = np.concatenate([kept[hp, t - 1], np.arange(B + t * L, B + (t + 1) * L, dtype=np.int32)])
    return kept
