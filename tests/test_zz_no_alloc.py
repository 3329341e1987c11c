"""fk_decode_step_static (the entry point that allocates nothing, for callers that cannot call hipMalloc) against
fk_decode_step on a caller workspace: same kernels, same plan, so outputs and cache contents must agree bit for
bit.  Two calls in a row on the library's one scratch array, the second on a smaller input."""
import numpy as np
import pytest
import torch

import synth_inputs as si
import paper_2602_03203_amd as fk
from gpu_util import to_dev, to_host
from util import store

pytestmark = pytest.mark.gpu


def _case(seed, dtype, Bt, Hq, Hkv, D, cap, n):
    """Random cache with n live slots per row plus one step's inputs, as device tensors."""
    rng = np.arange(Bt * Hkv * cap * D)
    K = store((si.normal(seed, si.T_K, 0, rng).reshape(Bt, Hkv, cap, D) * 0.5).astype(np.float32), dtype)
    V = store((si.normal(seed, si.T_V, 0, rng).reshape(Bt, Hkv, cap, D)).astype(np.float32), dtype)
    q = store((si.normal(seed, si.T_Q, 0, np.arange(Bt * Hq * D)).reshape(Bt, Hq, D)).astype(np.float32), dtype)
    kn = store((si.normal(seed + 1, si.T_K, 1, np.arange(Bt * Hkv * D)).reshape(Bt, Hkv, D) * 0.5).astype(np.float32), dtype)
    vn = store((si.normal(seed + 1, si.T_V, 1, np.arange(Bt * Hkv * D)).reshape(Bt, Hkv, D)).astype(np.float32), dtype)
    pos = np.tile(np.arange(cap, dtype=np.int32), (Bt, Hkv, 1))
    ln = np.full((Bt, Hkv), n, np.int32)
    ln[0, 0] = max(n - 37, 0)      # ragged: one shorter row
    pn = np.full(Bt, cap + 5, np.int32)
    return [to_dev(x) for x in (K, V, pos, ln, q, kn, vn, pn)]


def _step_both(desc, case, n_steps, scale):
    """Run n_steps decode steps twice from the same state: on a caller workspace and on the static scratch."""
    K, V, pos, ln, q, kn, vn, pn = case
    outs = []
    for static in (False, True):
        Kc, Vc, pc, lc = K.clone(), V.clone(), pos.clone(), ln.clone()
        out = torch.zeros_like(q)
        ws = None if static else fk.new_attn_workspace(desc)
        res = []
        for t in range(n_steps):
            ml = min(int(ln.max()) + t + 1, desc.capacity)
            if static:
                fk.fk_decode_step_static(desc, q, Kc, Vc, pc, lc, kn, vn, pn, ml, scale, out)
            else:
                fk.fk_decode_step(desc, q, Kc, Vc, pc, lc, kn, vn, pn, ml, scale, out, ws)
            res.append(to_host(out).copy())
        torch.cuda.synchronize()
        outs.append((res, to_host(Kc), to_host(Vc), to_host(pc), to_host(lc)))
    return outs


def _assert_same(a, b, what):
    for t, (x, y) in enumerate(zip(a[0], b[0])):
        assert np.array_equal(x, y), f"{what}: attention output of step {t} differs"
    for i, name in enumerate(("K", "V", "pos", "len"), start=1):
        assert np.array_equal(a[i], b[i]), f"{what}: {name} differs"


def test_static_scratch_matches_workspace_two_calls_in_a_row():
    # first: 2 sequences x 2 KV heads, long rows -> every row is cut into many splits, the scratch holds their records
    d1 = fk.CacheDesc(2, 8, 2, 128, 3000, "bf16")
    c1 = _case(11, "bf16", 2, 8, 2, 128, 3000, 2900)
    ref1, got1 = _step_both(d1, c1, 3, 0.11)
    _assert_same(ref1, got1, "first call")
    assert ref1[4].max() == 2903
    # second, smaller: fewer rows, shorter, other group size and dtype; the scratch still holds the first call's records
    d2 = fk.CacheDesc(1, 6, 2, 64, 700, "f32")
    c2 = _case(12, "f32", 1, 6, 2, 64, 700, 650)
    ref2, got2 = _step_both(d2, c2, 2, 0.2)
    _assert_same(ref2, got2, "second call")
    # and the first shape once more: the counters were left at zero
    ref3, got3 = _step_both(d1, c1, 1, 0.11)
    _assert_same(ref3, got3, "third call")


def test_static_scratch_rejects_what_does_not_fit():
    import ctypes
    L = fk.lib()
    big = fk.CacheDesc(4096, 64, 8, 128, 4096, "f32")    # 32768 rows x 16 splits ... far beyond 8 MiB of records
    assert fk.fk_decode_attn_workspace(big, 4096) > (8 << 20)
    p = 4096
    rc = L.fk_decode_step_static(ctypes.byref(big.c()), p, p, p, p, p, p, p, p, 4096, ctypes.c_float(1.0), p, 0)
    assert rc == fk.binding.FK_ERR_WORKSPACE
