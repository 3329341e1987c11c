"""Parity of every C-ABI entry point against the CPU oracle, element by element, on seeded inputs
that span several tiles and a ragged tail, plus the edge cases each kernel has."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from util import random_cache, random_q, store

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    import paper_2602_03203_amd as fk
    fk.lib()                       # the HIP library must be there: no fallback
    return gpu_util


ATTN_SHAPES = [
    # dtype, D, Hq, Hkv, cap, lens
    ("f32", 64, 8, 2, 160, [160]),
    ("bf16", 128, 32, 8, 2176, [2176, 2049]),
    ("bf16", 128, 8, 2, 700, [700, 513, 1, 0, 64, 65]),
    ("bf16", 128, 28, 4, 1100, [1100, 777]),          # group of 7
    ("bf16", 64, 6, 3, 300, [300, 37]),
    ("f32", 128, 2, 2, 200, [200, 129]),
    ("f32", 64, 5, 1, 90, [90, 3]),                    # group of 5
    ("bf16", 128, 8, 1, 260, [260]),                   # group of 8
]


@pytest.mark.parametrize("dtype,D,Hq,Hkv,cap,lens", ATTN_SHAPES)
def test_decode_attn_matches_oracle(gpu, ora, dtype, D, Hq, Hkv, cap, lens):
    import paper_2602_03203_amd as fk
    Bt = len(lens)
    print(f"attn case {dtype} D={D} Hq={Hq} Hkv={Hkv} cap={cap} lens={lens}", flush=True)
    c = random_cache(ora, 1000 + D + Hq, dtype, Bt, Hkv, cap, D, lens=lens)
    q = random_q(2000 + D, dtype, Bt, Hq, D)
    dev = gpu.DevCache(c, Hq)
    qd = gpu.to_dev(q)
    for scale in (D ** -0.5, 0.02, 3.0 * D ** -0.5):      # usual, near-uniform, peaked softmax
        ref = ora.decode_attn(c, q, scale)
        got = dev.attn(qd, scale)
        gpu.assert_attn_close(got, ref, dtype, f"scale {scale}")
    # a tighter max_len hint that still covers every row gives the same answer
    got = dev.attn(qd, D ** -0.5, max_len=max(max(lens), 1))
    gpu.assert_attn_close(got, ora.decode_attn(c, q, D ** -0.5), dtype, "max_len hint")
    # the "cold cache" hint changes how K and V are fetched, not a bit of the result
    plain = dev.attn(qd, D ** -0.5)
    dev.desc.cold = True
    ws_small, dev.ws = dev.ws, fk.new_attn_workspace(dev.desc)     # a cold cache may be cut into more splits
    cold = dev.attn(qd, D ** -0.5)
    gpu.assert_attn_close(cold, ora.decode_attn(c, q, D ** -0.5), dtype, "cold-cache hint")
    if Bt * Hkv >= 128 or dtype != "bf16" or D != 128:
        assert np.array_equal(cold, plain)                          # same splits: the same bits
    dev.desc.cold, dev.ws = False, ws_small
    # a hint that is too small only costs time: the last split runs on to the end of the row
    for hint in (1, 33, max(max(lens) // 3, 1)):
        got = dev.attn(qd, D ** -0.5, max_len=hint)
        gpu.assert_attn_close(got, ora.decode_attn(c, q, D ** -0.5), dtype, f"max_len hint {hint} below the lengths")


def test_decode_attn_closed_forms_on_device(gpu, ora):
    """identical keys -> mean of V; one dominant key -> its value."""
    D, cap = 128, 1000
    c = random_cache(ora, 77, "bf16", 1, 2, cap, D, lens=[cap])
    c.K[...] = c.K[:, :, :1]
    q = random_q(78, "bf16", 1, 8, D)
    dev = gpu.DevCache(c, 8)
    got = dev.attn(gpu.to_dev(q), 0.3)
    mean_v = si.from_bf16_bits(c.V).astype(np.float64).mean(axis=2)
    for h in range(8):
        gpu.assert_attn_close(got[0, h], mean_v[0, h // 4], "bf16", "mean of V")
    c2 = random_cache(ora, 79, "f32", 1, 1, 300, 64, lens=[300], scale=0.01)
    q2 = random_q(80, "f32", 1, 4, 64)
    c2.K[0, 0, 217] = 300.0 * q2[0, 2]
    got2 = gpu.DevCache(c2, 4).attn(gpu.to_dev(q2), 1.0)
    np.testing.assert_allclose(got2[0, 2], c2.V[0, 0, 217].astype(np.float64), atol=1e-5)


def test_split_merge_many_splits_back_to_back(gpu, ora):
    """One row cut into as many splits as the plan ever uses (128 workgroups whose records are merged by the last one to
    arrive), 64 launches in a row on one workspace with no host synchronisation in between: every launch must find the
    arrival counter at zero and every merge must see all records of its own launch.  Cold-cache variant too."""
    import paper_2602_03203_amd as fk
    D, cap, n, g, nq = 128, 20000, 19777, 4, 64
    c = random_cache(ora, 4711, "bf16", 1, 1, cap, D, lens=[n], scale=0.5)
    for cold in (False, True):
        desc = fk.CacheDesc(1, g, 1, D, cap, "bf16", cold=cold)
        dev = gpu.DevCache(c, g)
        ws = fk.new_attn_workspace(desc)
        qs = [random_q(9000 + i, "bf16", 1, g, D, scale=1.0 + 0.05 * i) for i in range(nq)]
        dq = gpu.to_dev(np.stack(qs))
        outs = torch.empty((nq, 1, g, D), dtype=torch.bfloat16, device="cuda")
        for i in range(nq):
            fk.fk_decode_attn(desc, dq[i], dev.K, dev.V, dev.len, n, 0.2, outs[i], ws)
        torch.cuda.synchronize()
        assert int(ws[:4].view(torch.int32)[0]) == 0          # the row's arrival counter is back at zero
        for i in range(nq):
            gpu.assert_attn_close(gpu.out_to_f64(outs[i]), ora.decode_attn(c, qs[i], 0.2), "bf16", f"launch {i} (cold={cold})")


def test_rows_of_a_sequence_may_hold_different_counts(gpu, ora):
    """Every row carries its own length: heads of one sequence with different counts (the oracle sees
    each row as a one-head sequence)."""
    import paper_2602_03203_amd as fk
    Bt, Hkv, G, D, cap = 3, 4, 4, 128, 900
    lens = np.array([[900, 31, 0, 512], [1, 899, 450, 33], [64, 65, 700, 2]], np.int32)
    c = random_cache(ora, 8100, "bf16", Bt * Hkv, 1, cap, D, lens=lens.reshape(-1))        # oracle: rows as sequences
    q = random_q(8101, "bf16", Bt * Hkv, G, D)
    desc = fk.CacheDesc(Bt, Hkv * G, Hkv, D, cap, "bf16")
    K, V = gpu.to_dev(c.K.reshape(Bt, Hkv, cap, D)), gpu.to_dev(c.V.reshape(Bt, Hkv, cap, D))
    pos, ln = gpu.to_dev(c.pos.reshape(Bt, Hkv, cap)), gpu.to_dev(lens)
    ws, out = fk.new_attn_workspace(desc), torch.empty((Bt, Hkv * G, D), dtype=torch.bfloat16, device="cuda")
    k_new, v_new = random_q(8102, "bf16", Bt * Hkv, 1, D), random_q(8103, "bf16", Bt * Hkv, 1, D)
    pos_new = np.array([5000, 5001, 5002], np.int32)
    fk.fk_decode_step(desc, gpu.to_dev(q.reshape(Bt, Hkv * G, D)), K, V, pos, ln, gpu.to_dev(k_new.reshape(Bt, Hkv, D)),
                      gpu.to_dev(v_new.reshape(Bt, Hkv, D)), gpu.to_dev(pos_new), cap, 0.1, out, ws)
    for r in range(Bt * Hkv):
        if c.len[r] < cap:
            sub = ora.Cache("bf16", c.K[r:r + 1], c.V[r:r + 1], c.pos[r:r + 1], c.len[r:r + 1])
            ora.append(sub, k_new[r:r + 1], v_new[r:r + 1], pos_new[r // Hkv:r // Hkv + 1])
    ref = ora.decode_attn(c, q, 0.1)
    gpu.assert_attn_close(gpu.out_to_f64(out).reshape(Bt * Hkv, G, D), ref, "bf16", "per-row lengths")
    assert np.array_equal(gpu.to_host(ln).reshape(-1), c.len)
    assert np.array_equal(gpu.to_host(K).reshape(c.K.shape), c.K) and np.array_equal(gpu.to_host(pos).reshape(c.pos.shape), c.pos)
    # eviction on rows with different counts: scores -> select -> compact, row by row against the oracle
    sc = si.gen_scores(8104, (Bt * Hkv, 1, cap), ties=4)
    budget, recent = 400, 50
    keep_ref = ora.select_keep(sc, c.pos, c.len, budget, recent, "sort")
    keep = torch.full((Bt, Hkv, budget), -1, dtype=torch.int32, device="cuda")
    fk.fk_select_keep(desc, gpu.to_dev(sc.reshape(Bt, Hkv, cap)), pos, ln, cap, budget, recent, keep)
    gpu.assert_keep_equal(keep.cpu().numpy().reshape(keep_ref.shape), keep_ref, c.len, budget, "per-row lengths")
    fk.fk_compact(desc, K, V, pos, ln, keep, budget)
    ora.compact(c, keep_ref, budget)
    assert np.array_equal(gpu.to_host(ln).reshape(-1), c.len)
    assert np.array_equal(gpu.to_host(K).reshape(c.K.shape), c.K) and np.array_equal(gpu.to_host(V).reshape(c.V.shape), c.V)
    assert np.array_equal(gpu.to_host(pos).reshape(c.pos.shape), c.pos)


SCORE_SHAPES = [
    ("f32", 64, 64, 2, 160, [160, 33], True),
    ("bf16", 128, 256, 8, 2176, [2176], True),
    ("bf16", 128, 256, 2, 600, [600, 257, 1, 0], True),
    ("bf16", 128, 32, 2, 100, [100, 64], False),       # shared weights, narrow hidden
    ("bf16", 64, 96, 3, 130, [130, 65], True),
    ("f32", 128, 20, 1, 70, [70], True),
    ("bf16", 128, 16, 8, 2176, [2176, 1500], True),    # the paper's hidden width (Section 4.1): padded to one MFMA tile
    ("bf16", 128, 48, 2, 300, [300, 31], True),        # a width that is no multiple of 32
    # more widths: hidden tiles partly empty, shared weights, rows that end inside a tile / a workgroup's share
    ("bf16", 128, 72, 2, 700, [700, 33], True),
    ("bf16", 128, 128, 2, 1100, [1100, 1087, 32], False),
    ("bf16", 128, 200, 3, 520, [520, 97], True),
    ("bf16", 64, 256, 2, 1300, [1300, 64], True),
    ("bf16", 64, 136, 2, 300, [300, 299], False),
    ("bf16", 64, 512, 1, 200, [200], True),
]


@pytest.mark.parametrize("dtype,D,H,Hkv,cap,lens,per_head", SCORE_SHAPES)
def test_score_kv_matches_oracle(gpu, ora, dtype, D, H, Hkv, cap, lens, per_head):
    import paper_2602_03203_amd as fk
    Bt = len(lens)
    print(f"score case {dtype} D={D} H={H} Hkv={Hkv} cap={cap} lens={lens}", flush=True)
    c = random_cache(ora, 3000 + H, dtype, Bt, Hkv, cap, D, lens=lens, scale=0.5)
    nset = Hkv if per_head else 1
    F = 2 * D
    W1 = store((si.normal(5, si.T_W1, 0, np.arange(nset * F * H)).reshape(nset, F, H) / np.sqrt(F)).astype(np.float32), dtype)
    b1 = (si.normal(5, si.T_B1, 0, np.arange(nset * H)).reshape(nset, H) * 0.2).astype(np.float32)
    W2 = (si.normal(5, si.T_W2, 0, np.arange(nset * H)).reshape(nset, H) / np.sqrt(H)).astype(np.float32)
    b2 = (si.normal(5, si.T_B2, 0, np.arange(nset)) * 0.3).astype(np.float32)
    ref = ora.score_kv(c, W1, b1, W2, b2)
    dev = gpu.DevCache(c, Hkv)
    fk.fk_score_kv(dev.desc, dev.K, dev.V, dev.len, cap, gpu.to_dev(W1), gpu.to_dev(b1), gpu.to_dev(W2), gpu.to_dev(b2), dev.scores)
    got = dev.scores.cpu().numpy()
    gpu.assert_scores_close(got, ref, lens, "scores")
    for b in range(Bt):                                   # slots past len are not written
        assert np.isnan(got[b, :, lens[b]:]).all()
    if dtype == "f32":
        # fp32 path (plain FMA, library erf): besides the bar above, every score within 1e-5 of the sum of the
        # magnitudes of its terms, so that an fp32 regression cannot hide under the row-scale floor of that bar
        from scipy.special import erf
        for b in range(Bt):
            n = lens[b]
            for h in range(Hkv):
                x = np.concatenate([c.K[b, h, :n], c.V[b, h, :n]], axis=1).astype(np.float64)
                hw = h if per_head else 0
                z = x @ W1[hw].astype(np.float64) + b1[hw]
                terms = np.abs(0.5 * z * (1.0 + erf(z / np.sqrt(2.0))) * W2[hw]).sum(axis=1) + abs(float(b2[hw]))
                assert (np.abs(got[b, h, :n] - ref[b, h, :n]) <= 1e-5 * terms).all(), f"fp32 scores row ({b},{h})"
    # rows at or under skip_len (the budget, in the protocol) are left alone, the others get the same scores
    skip = sorted(lens)[len(lens) // 2]
    dev.scores.fill_(float("nan"))
    fk.fk_score_kv(dev.desc, dev.K, dev.V, dev.len, cap, gpu.to_dev(W1), gpu.to_dev(b1), gpu.to_dev(W2), gpu.to_dev(b2), dev.scores,
                   skip_len=skip)
    got2 = dev.scores.cpu().numpy()
    for b in range(Bt):
        if lens[b] <= skip:
            assert np.isnan(got2[b]).all()
        else:
            assert np.array_equal(got2[b, :, :lens[b]], got[b, :, :lens[b]])


SELECT_CASES = [
    # Bt, Hkv, cap, lens, budget, recent, ties
    (1, 2, 160, [160], 128, 32, 0),
    (16, 8, 2176, [2176] * 16, 2048, 128, 0),
    (2, 4, 2176, [2176, 2100], 2048, 128, 6),          # heavy ties
    (3, 2, 5000, [5000, 3001, 2999], 3000, 64, 3),     # far over budget, exactly at budget + 1, under budget
    (2, 1, 300, [300, 300], 200, 0, 2),                # nothing protected
    (2, 1, 300, [300, 300], 200, 200, 0),              # everything kept is protected
    (1, 3, 1500, [1500], 1, 0, 2),                     # budget 1
    (2, 2, 40000, [40000, 33000], 8192, 128, 0),       # long rows (ragged-batch first event)
]


@pytest.mark.parametrize("Bt,Hkv,cap,lens,budget,recent,ties", SELECT_CASES)
def test_select_keep_bit_exact(gpu, ora, Bt, Hkv, cap, lens, budget, recent, ties):
    import paper_2602_03203_amd as fk
    print(f"select case Bt={Bt} Hkv={Hkv} cap={cap} lens={lens} B={budget} R={recent} ties={ties}", flush=True)
    sc = si.gen_scores(4000 + cap + ties, (Bt, Hkv, cap), ties=ties)
    pos = np.tile(np.arange(cap, dtype=np.int32) * 2 + 3, (Bt, Hkv, 1))
    ln = np.asarray(lens, np.int32)
    ref = ora.select_keep(sc, pos, ln, budget, recent, "sort")
    desc = fk.CacheDesc(Bt, Hkv, Hkv, 128, cap, "bf16")
    keep = torch.full((Bt, Hkv, budget), -1, dtype=torch.int32, device="cuda")
    fk.fk_select_keep(desc, gpu.to_dev(sc), gpu.to_dev(pos), gpu.to_dev(np.repeat(ln[:, None], Hkv, 1)), cap, budget, recent, keep)
    gpu.assert_keep_equal(keep.cpu().numpy(), ref, ln, budget)


@pytest.mark.parametrize("cluster,dup", [(1, 0), (2, 1), (33, 0), (63, 1), (64, 0), (64, 1), (65, 0), (65, 1), (200, 1)])
@pytest.mark.parametrize("gap_bits", [0, 9, 15])
def test_select_keep_threshold_inside_a_small_cluster(gpu, ora, cluster, dup, gap_bits):
    """The cut falls inside a cluster of scores that share their leading bits (1 + j * 2^(gap_bits - 23), all in
    [1, 2)); 500 scores lie above it in [2, 4), the rest below in [0.25, 0.5).  Clusters of at most 64 are resolved by
    ranking a list, larger ones by further histograms.  With dup the cluster holds every value twice (ties at the cut go
    to the lower position)."""
    import paper_2602_03203_amd as fk
    cap, recent, others = 900, 50, 500
    rng = np.random.default_rng(cluster * 100 + dup * 10 + gap_bits)
    sc = np.empty((1, 2, cap), np.float32)
    for h in range(2):
        row = (0.25 + 0.25 * rng.random(cap)).astype(np.float32)
        slots = rng.permutation(cap - recent)
        row[slots[:others]] = (2.0 + 2.0 * rng.random(others)).astype(np.float32)
        j = np.arange(cluster) // 2 if dup else np.arange(cluster)
        row[slots[others:others + cluster]] = (1.0 + (j << gap_bits) * 2.0 ** -23).astype(np.float32)
        sc[0, h] = row
        mid = sc[0, h, : cap - recent]
        assert ((mid >= 1.0) & (mid < 2.0)).sum() == cluster and (mid >= 2.0).sum() == others
    budget = others + (cluster + 1) // 2 + recent                           # the cut lies in the middle of the cluster
    pos = np.tile(np.arange(cap, dtype=np.int32), (1, 2, 1))
    ln = np.array([cap], np.int32)
    ref = ora.select_keep(sc, pos, ln, budget, recent, "sort")
    desc = fk.CacheDesc(1, 2, 2, 128, cap, "bf16")
    keep = torch.full((1, 2, budget), -1, dtype=torch.int32, device="cuda")
    fk.fk_select_keep(desc, gpu.to_dev(sc), None, gpu.to_dev(np.repeat(ln[:, None], 2, 1)), cap, budget, recent, keep)
    gpu.assert_keep_equal(keep.cpu().numpy(), ref, ln, budget)


SPLIT_SELECT_CASES = [
    # Bt, Hkv, cap, lens, max_len hint, budget, recent, ties -- few long rows: fk_select_keep_ws cuts them into chunks
    (1, 4, 131072, [131072], 131072, 2048, 128, 0),            # the one-shot benchmark's row: 9 chunks
    (2, 2, 40000, [40000, 33000], 40000, 8192, 128, 0),         # large budget: two chunks is all that fits the merge
    (2, 2, 70000, [70000, 20011], 70000, 2048, 0, 5),           # ragged, heavy ties, nothing protected
    (3, 1, 50000, [50000, 1500, 17000], 50000, 1600, 64, 3),    # a row under budget, a row inside the first chunks
    (1, 2, 65536, [65536], 65536, 1, 0, 2),                     # budget 1: sixteen chunks
    (2, 1, 90000, [90000, 88000], 20000, 4096, 4096, 0),        # everything kept is protected; hint far below the lengths
    (1, 2, 90000, [90000], 30000, 3000, 100, 4),                # hint below the length: the last chunk runs on
]


@pytest.mark.parametrize("Bt,Hkv,cap,lens,hint,budget,recent,ties", SPLIT_SELECT_CASES)
def test_select_keep_split_rows_bit_exact(gpu, ora, Bt, Hkv, cap, lens, hint, budget, recent, ties):
    import paper_2602_03203_amd as fk
    print(f"split select case Bt={Bt} Hkv={Hkv} cap={cap} lens={lens} hint={hint} B={budget} R={recent} ties={ties}", flush=True)
    sc = si.gen_scores(9000 + cap + ties, (Bt, Hkv, cap), ties=ties)
    pos = np.tile(np.arange(cap, dtype=np.int32), (Bt, Hkv, 1))
    ln = np.asarray(lens, np.int32)
    ref = ora.select_keep(sc, pos, ln, budget, recent, "sort")
    desc = fk.CacheDesc(Bt, Hkv, Hkv, 128, cap, "bf16")
    nbytes = fk.fk_select_keep_workspace(desc, hint, budget, recent)
    assert (nbytes > 0) == (budget > recent)       # these shapes are split unless nothing is selected
    ws = torch.full((max(nbytes, 16),), 0xA5, dtype=torch.uint8, device="cuda")   # contents undefined: no zeroing needed
    d_sc, d_ln = gpu.to_dev(sc), gpu.to_dev(np.repeat(ln[:, None], Hkv, 1))
    for _ in range(2):                             # twice on the same workspace
        keep = torch.full((Bt, Hkv, budget), -1, dtype=torch.int32, device="cuda")
        fk.fk_select_keep_ws(desc, d_sc, None, d_ln, hint, budget, recent, keep, ws)
        gpu.assert_keep_equal(keep.cpu().numpy(), ref, ln, budget)
    keep1 = torch.full((Bt, Hkv, budget), -1, dtype=torch.int32, device="cuda")
    fk.fk_select_keep(desc, d_sc, None, d_ln, hint, budget, recent, keep1)
    assert torch.equal(keep1, keep)                # and the one-launch call agrees
    if nbytes:
        with pytest.raises(fk.FkError):
            fk.fk_select_keep_ws(desc, d_sc, None, d_ln, hint, budget, recent, keep, ws[:nbytes - 1])


def test_select_keep_ws_on_short_rows_is_the_plain_call(gpu, ora):
    import paper_2602_03203_amd as fk
    Bt, Hkv, cap, budget, recent = 16, 8, 2176, 2048, 128
    desc = fk.CacheDesc(Bt, Hkv, Hkv, 128, cap, "bf16")
    assert fk.fk_select_keep_workspace(desc, cap, budget, recent) == 0
    sc = si.gen_scores(31, (Bt, Hkv, cap), ties=2)
    ln = np.full(Bt, cap, np.int32)
    ref = ora.select_keep(sc, np.tile(np.arange(cap, dtype=np.int32), (Bt, Hkv, 1)), ln, budget, recent, "sort")
    keep = torch.full((Bt, Hkv, budget), -1, dtype=torch.int32, device="cuda")
    fk.fk_select_keep_ws(desc, gpu.to_dev(sc), None, gpu.to_dev(np.repeat(ln[:, None], Hkv, 1)), cap, budget, recent, keep, None)
    gpu.assert_keep_equal(keep.cpu().numpy(), ref, ln, budget)


def test_prepared_call_replays_the_direct_call(gpu, ora):
    """fk.prepare marshals once; the callable it returns makes the same library call each time it is used."""
    import paper_2602_03203_amd as fk
    Bt, Hkv, cap, budget, recent = 2, 4, 2176, 2048, 128
    sc = si.gen_scores(777, (Bt, Hkv, cap), ties=3)
    ln = np.array([cap, 2100], np.int32)
    ref = ora.select_keep(sc, np.tile(np.arange(cap, dtype=np.int32), (Bt, Hkv, 1)), ln, budget, recent, "sort")
    desc = fk.CacheDesc(Bt, Hkv, Hkv, 128, cap, "bf16")
    d_sc, d_ln = gpu.to_dev(sc), gpu.to_dev(np.repeat(ln[:, None], Hkv, 1))
    keep = torch.full((Bt, Hkv, budget), -1, dtype=torch.int32, device="cuda")
    call = fk.prepare(fk.fk_select_keep, desc, d_sc, None, d_ln, cap, budget, recent, keep)
    torch.cuda.synchronize()
    assert (keep == -1).all()                      # preparing calls nothing
    for _ in range(2):
        keep.fill_(-1)
        call()
        gpu.assert_keep_equal(keep.cpu().numpy(), ref, ln, budget)
    with pytest.raises(fk.FkError):                # an error status still raises, when prepared and when replayed
        fk.prepare(fk.fk_select_keep, desc, d_sc, None, d_ln, cap, cap + 1, recent, keep)()


def test_select_keep_special_values(gpu, ora):
    import paper_2602_03203_amd as fk
    cap, budget, recent = 1200, 700, 100
    sc = si.gen_scores(4242, (1, 4, cap), ties=4)
    flat = sc.reshape(-1)
    special = np.array([np.nan, -np.nan, np.inf, -np.inf, 0.0, -0.0, 1e-45, -1e-45, 3.4e38, -3.4e38], np.float32)
    idx = (si.hash_u64(1, si.T_FLAG, 0, np.arange(1500)) % np.uint64(flat.size)).astype(np.int64)
    flat[idx] = special[np.arange(1500) % len(special)]
    sc[0, 3] = 0.0
    sc[0, 3, ::2] = -0.0                                   # a row of +0 / -0 only: pure position tie-break
    pos = np.arange(cap, dtype=np.int32)[None, None].repeat(4, 1)
    ln = np.array([cap], np.int32)
    ref = ora.select_keep(sc, pos, ln, budget, recent, "rank")
    desc = fk.CacheDesc(1, 4, 4, 128, cap, "bf16")
    keep = torch.full((1, 4, budget), -1, dtype=torch.int32, device="cuda")
    fk.fk_select_keep(desc, gpu.to_dev(sc), None, gpu.to_dev(np.repeat(ln[:, None], 4, 1)), cap, budget, recent, keep)
    gpu.assert_keep_equal(keep.cpu().numpy(), ref, ln, budget)
    assert keep[0, 3].cpu().tolist() == list(range(600)) + list(range(1100, 1200))


SAMPLED_CASES = [
    # Bt, Hkv, cap, lens, budget, recent, n_cand, ties (score levels), noise levels
    (16, 8, 2176, [2176] * 16, 2048, 128, 256, 0, 0),        # the paper's policy at the benchmark shape: 2L candidates, L evicted
    (2, 4, 2176, [2176, 2100], 2048, 128, 256, 6, 6),        # heavy ties in scores and in score - noise
    (3, 2, 5000, [5000, 3001, 2999], 3000, 64, 3000, 3, 4),  # far over budget; one row just over; one under
    (2, 2, 700, [700, 650], 500, 0, 100000, 0, 0),           # every non-recent pair is a candidate
    (2, 2, 700, [700, 650], 500, 100, 0, 2, 2),              # n_cand below the number to evict: deterministic rule
    (1, 3, 1500, [1500], 1, 0, 7, 2, 3),                     # budget 1
    (2, 2, 40000, [40000, 33000], 8192, 128, 50000, 0, 0),   # long rows
]


@pytest.mark.parametrize("Bt,Hkv,cap,lens,budget,recent,n_cand,ties,nlev", SAMPLED_CASES)
def test_select_keep_sampled_bit_exact(gpu, ora, Bt, Hkv, cap, lens, budget, recent, n_cand, ties, nlev):
    import paper_2602_03203_amd as fk
    print(f"sampled case Bt={Bt} Hkv={Hkv} cap={cap} lens={lens} B={budget} R={recent} K'={n_cand} ties={ties}/{nlev}", flush=True)
    sc = si.gen_scores(4500 + cap + ties, (Bt, Hkv, cap), ties=ties)
    noise = si.gen_gumbel(4600 + cap, (Bt, Hkv, cap), event=3, levels=nlev)
    if ties:   # a few special values among the scores
        flat = sc.reshape(-1)
        idx = (si.hash_u64(2, si.T_FLAG, 0, np.arange(200)) % np.uint64(flat.size)).astype(np.int64)
        flat[idx] = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0], np.float32)[np.arange(200) % 5]
    pos = np.tile(np.arange(cap, dtype=np.int32) * 2 + 3, (Bt, Hkv, 1))
    ln = np.asarray(lens, np.int32)
    ref = ora.select_keep_sampled(sc, noise, pos, ln, budget, recent, n_cand)
    desc = fk.CacheDesc(Bt, Hkv, Hkv, 128, cap, "bf16")
    keep = torch.full((Bt, Hkv, budget), -1, dtype=torch.int32, device="cuda")
    dln = gpu.to_dev(np.repeat(ln[:, None], Hkv, 1))
    fk.fk_select_keep_sampled(desc, gpu.to_dev(sc), gpu.to_dev(noise), gpu.to_dev(pos), dln, cap, budget, recent, n_cand, keep)
    gpu.assert_keep_equal(keep.cpu().numpy(), ref, ln, budget)
    # zero noise: the deterministic entry point's answer
    det = torch.full_like(keep, -1)
    fk.fk_select_keep(desc, gpu.to_dev(sc), None, dln, cap, budget, recent, det)
    fk.fk_select_keep_sampled(desc, gpu.to_dev(sc), gpu.to_dev(np.zeros_like(noise)), None, dln, cap, budget, recent, n_cand, keep)
    assert torch.equal(keep, det)


COMPACT_CASES = [("f32", 64, 1, 2, 160, [160], 128), ("bf16", 128, 3, 2, 2176, [2176, 2050, 2048], 2048),
                 ("bf16", 64, 2, 3, 333, [333, 100], 150), ("f32", 128, 1, 1, 700, [700], 300)]


@pytest.mark.parametrize("dtype,D,Bt,Hkv,cap,lens,budget", COMPACT_CASES)
def test_compact_bit_exact(gpu, ora, dtype, D, Bt, Hkv, cap, lens, budget):
    import paper_2602_03203_amd as fk
    print(f"compact case {dtype} D={D} Bt={Bt} Hkv={Hkv} cap={cap} lens={lens} B={budget}", flush=True)
    c = random_cache(ora, 5000 + cap, dtype, Bt, Hkv, cap, D, lens=lens)
    recent = min(32, budget)
    sc = si.gen_scores(5001 + cap, (Bt, Hkv, cap), ties=5)
    keep = ora.select_keep(sc, c.pos, c.len, budget, recent)
    patterns = [keep]
    # adversarial overlaps on the first row: evict the head block / every other / a middle block
    n0 = lens[0]
    if n0 > budget:
        for pat in (np.arange(n0 - budget, n0), np.sort(np.r_[np.arange(0, 2 * (n0 - budget), 2), np.arange(2 * (n0 - budget), n0)])[:budget],
                    np.r_[np.arange(7), np.arange(7 + n0 - budget, n0)]):
            k2 = keep.copy()
            k2[0, :] = pat.astype(np.int32)
            patterns.append(k2)
    for kp in patterns:
        host = c.copy()
        dev = gpu.DevCache(c, Hkv)
        ora.compact(host, kp, budget)
        fk.fk_compact(dev.desc, dev.K, dev.V, dev.pos, dev.len, gpu.to_dev(kp), budget)
        got = dev.host(ora)
        assert np.array_equal(got.len, host.len)
        assert np.array_equal(got.pos, host.pos)
        assert np.array_equal(got.K, host.K) and np.array_equal(got.V, host.V)


@pytest.mark.parametrize("dtype,D,Hq,Hkv,cap,lens", [
    ("bf16", 128, 32, 8, 2176, [2175, 2048, 0, 1087, 1088]),      # split boundaries, empty row, last free slot
    ("bf16", 128, 28, 4, 600, [600, 599, 31, 32]),                # one sequence is full: no append, attention still runs
    ("f32", 64, 8, 2, 160, [159, 0, 77]),
    ("bf16", 64, 4, 2, 100, [5, 99]),
])
def test_decode_step_equals_append_then_attention(gpu, ora, dtype, D, Hq, Hkv, cap, lens):
    """The fused launch against the oracle's append followed by the oracle's attention; cache bits exact."""
    import paper_2602_03203_amd as fk
    Bt = len(lens)
    print(f"decode_step case {dtype} D={D} Hq={Hq} Hkv={Hkv} cap={cap} lens={lens}", flush=True)
    c = random_cache(ora, 7000 + cap, dtype, Bt, Hkv, cap, D, lens=lens)
    dev = gpu.DevCache(c, Hq)
    scale = D ** -0.5
    for rep in range(3):                                      # consecutive steps reuse the workspace counters
        q = random_q(7001 + rep, dtype, Bt, Hq, D)
        k_new = random_q(7101 + rep, dtype, Bt, Hkv, D)
        v_new = random_q(7201 + rep, dtype, Bt, Hkv, D)
        pos_new = (np.arange(Bt) + 10000 + rep).astype(np.int32)
        fk.fk_decode_step(dev.desc, gpu.to_dev(q), dev.K, dev.V, dev.pos, dev.len, gpu.to_dev(k_new), gpu.to_dev(v_new),
                          gpu.to_dev(pos_new), cap, scale, dev.out, dev.ws)
        for b in range(Bt):
            if c.len[b] < cap:
                sub = ora.Cache(dtype, c.K[b:b + 1], c.V[b:b + 1], c.pos[b:b + 1], c.len[b:b + 1])   # views: appended in place
                ora.append(sub, k_new[b:b + 1], v_new[b:b + 1], pos_new[b:b + 1])
        ref = ora.decode_attn(c, q, scale)
        gpu.assert_attn_close(gpu.out_to_f64(dev.out), ref, dtype, f"fused step {rep}")
        got = dev.host(ora)
        assert np.array_equal(got.len, c.len) and np.array_equal(got.pos, c.pos)
        assert np.array_equal(got.K, c.K) and np.array_equal(got.V, c.V)
    assert int(torch.count_nonzero(dev.ws[:4 * Bt * Hkv])) == 0        # counters are back to zero


@pytest.mark.parametrize("dtype,D", [("f32", 64), ("bf16", 128), ("bf16", 64), ("f32", 128)])
def test_append_bit_exact(gpu, ora, dtype, D):
    import paper_2602_03203_amd as fk
    Bt, Hkv, cap = 5, 3, 40
    lens = [0, 39, 40, 17, 5]                           # one sequence is full: must be left alone
    c = random_cache(ora, 6000 + D, dtype, Bt, Hkv, cap, D, lens=lens)
    dev = gpu.DevCache(c, Hkv)
    k_new = random_q(6001, dtype, Bt, Hkv, D)
    v_new = random_q(6002, dtype, Bt, Hkv, D)
    pos_new = np.array([0, 500, 501, 502, 503], np.int32)
    fk.fk_append(dev.desc, dev.K, dev.V, dev.pos, dev.len, gpu.to_dev(k_new), gpu.to_dev(v_new), gpu.to_dev(pos_new))
    got = dev.host(ora)
    host = c.copy()
    for b in range(Bt):                                   # oracle append refuses the full row as a whole; do rows one by one
        if lens[b] < cap:
            sub = ora.Cache(dtype, host.K[b:b + 1].copy(), host.V[b:b + 1].copy(), host.pos[b:b + 1].copy(), host.len[b:b + 1].copy())
            ora.append(sub, k_new[b:b + 1], v_new[b:b + 1], pos_new[b:b + 1])
            host.K[b], host.V[b], host.pos[b], host.len[b] = sub.K[0], sub.V[0], sub.pos[0], sub.len[0]
    assert np.array_equal(got.len, host.len) and np.array_equal(got.pos, host.pos)
    assert np.array_equal(got.K, host.K) and np.array_equal(got.V, host.V)


def test_select_and_compact_random_shapes(gpu, ora):
    """Forty seeded random shapes (capacity, lengths, budget, protected tail, tie density, candidate count):
    both selection policies and the compaction they feed, bit for bit against the oracle.  The draws favour the
    boundaries: len = budget + 1, recent = 0 or = budget, budget = capacity, n_cand around the number evicted."""
    import paper_2602_03203_amd as fk
    rng = np.random.default_rng(20260203)
    for case in range(40):
        Bt, Hkv = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        cap = int(rng.choice([33, 64, 257, 1000, 1025, 2049, 3000]))
        budget = int(rng.choice([1, cap // 3 + 1, cap // 2, cap - 1, cap]))
        recent = int(rng.choice([0, 1, budget // 2, budget]))
        lens = [int(rng.choice([0, 1, budget, min(budget + 1, cap), cap, int(rng.integers(0, cap + 1))])) for _ in range(Bt)]
        ties = int(rng.choice([0, 2, 5]))
        n_cand = int(rng.choice([0, 1, max(cap - budget, 1), 2 * max(cap - budget, 1), cap]))
        D, dtype = (64, "f32") if case % 2 else (128, "bf16")
        print(f"random case {case}: Bt={Bt} Hkv={Hkv} cap={cap} lens={lens} B={budget} R={recent} ties={ties} K'={n_cand} {dtype}", flush=True)
        c = random_cache(ora, 7000 + case, dtype, Bt, Hkv, cap, D, lens=lens)
        sc = si.gen_scores(7100 + case, (Bt, Hkv, cap), ties=ties)
        noise = si.gen_gumbel(7200 + case, (Bt, Hkv, cap), event=case, levels=ties)
        dev = gpu.DevCache(c, Hkv)
        dsc, dnz = gpu.to_dev(sc), gpu.to_dev(noise)
        keep = torch.full((Bt, Hkv, budget), -1, dtype=torch.int32, device="cuda")
        fk.fk_select_keep_sampled(dev.desc, dsc, dnz, dev.pos, dev.len, cap, budget, recent, n_cand, keep)
        ref_s = ora.select_keep_sampled(sc, noise, c.pos, c.len, budget, recent, n_cand)
        fk.fk_select_keep(dev.desc, dsc, dev.pos, dev.len, cap, budget, recent, keep)
        ref = ora.select_keep(sc, c.pos, c.len, budget, recent, "sort")
        gpu.assert_keep_equal(keep.cpu().numpy(), ref, lens, budget, f"case {case}")
        fk.fk_select_keep_sampled(dev.desc, dsc, dnz, dev.pos, dev.len, cap, budget, recent, n_cand, keep)
        gpu.assert_keep_equal(keep.cpu().numpy(), ref_s, lens, budget, f"case {case} (sampled)")
        fk.fk_compact(dev.desc, dev.K, dev.V, dev.pos, dev.len, keep, budget)
        ora.compact(c, ref_s, budget)
        host = dev.host(ora)
        assert np.array_equal(host.len, c.len)
        for b in range(Bt):
            m = int(c.len[b])
            assert np.array_equal(host.pos[b, :, :m], c.pos[b, :, :m])
            assert np.array_equal(host.K[b, :, :m], c.K[b, :, :m]) and np.array_equal(host.V[b, :, :m], c.V[b, :, :m])


def test_attention_and_fused_step_random_shapes(gpu, ora):
    """Thirty seeded random shapes: every group size 1 .. 8, both head sizes and storage types, lengths around
    the 32-key tile and the split boundaries (0, 1, 31 .. 33, capacity - 1, capacity), random max_len hints;
    attention and the fused append + attention step against the oracle."""
    import paper_2602_03203_amd as fk
    rng = np.random.default_rng(26020302)
    for case in range(30):
        g = int(rng.integers(1, 9))
        Hkv, Bt = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        D, dtype = (64, 128)[case % 2], ("bf16", "f32")[(case // 2) % 2]
        cap = int(rng.choice([34, 65, 130, 513, 1500]))
        choices = [0, 1, 31, 32, 33, cap - 1, cap, int(rng.integers(0, cap + 1))]
        lens = [int(rng.choice(choices)) for _ in range(Bt)]
        scale = float(rng.choice([D ** -0.5, 0.02, 2.0 * D ** -0.5]))
        print(f"random attn case {case}: {dtype} D={D} g={g} Hkv={Hkv} cap={cap} lens={lens} scale={scale:.3f}", flush=True)
        c = random_cache(ora, 8000 + case, dtype, Bt, Hkv, cap, D, lens=lens)
        q = random_q(8100 + case, dtype, Bt, Hkv * g, D)
        dev = gpu.DevCache(c, Hkv * g)
        qd = gpu.to_dev(q)
        hint = int(rng.choice([cap, max(max(lens), 1), max(max(lens) // 2, 1)]))
        gpu.assert_attn_close(dev.attn(qd, scale, max_len=hint), ora.decode_attn(c, q, scale), dtype, f"case {case}")
        # fused step: rows at capacity are left alone, the others grow by one
        kn, vn = random_q(8200 + case, dtype, Bt, Hkv, D), random_q(8300 + case, dtype, Bt, Hkv, D)
        pn = np.array([3 * cap + 7 + b for b in range(Bt)], np.int32)
        fk.fk_decode_step(dev.desc, qd, dev.K, dev.V, dev.pos, dev.len, gpu.to_dev(kn), gpu.to_dev(vn), gpu.to_dev(pn),
                          min(max(lens) + 1, cap), scale, dev.out, dev.ws)
        for b in range(Bt):      # the oracle refuses a full row; the device leaves it alone
            if c.len[b] < cap:
                ora.append(ora.Cache(dtype, c.K[b:b + 1], c.V[b:b + 1], c.pos[b:b + 1], c.len[b:b + 1]), kn[b:b + 1], vn[b:b + 1], pn[b:b + 1])
        gpu.assert_attn_close(gpu.out_to_f64(dev.out), ora.decode_attn(c, q, scale), dtype, f"case {case} fused")
        host = dev.host(ora)
        assert np.array_equal(host.len, c.len)
        for b in range(Bt):
            m = int(c.len[b])
            assert np.array_equal(host.pos[b, :, :m], c.pos[b, :, :m]) and np.array_equal(host.K[b, :, :m], c.K[b, :, :m])
            assert np.array_equal(host.V[b, :, :m], c.V[b, :, :m])


def test_scorer_random_shapes(gpu, ora):
    """Twenty seeded random scorer shapes: hidden widths that are and are not multiples of 32, shared and
    per-head weights, both head sizes and storage types, lengths around the 32-pair tile."""
    import paper_2602_03203_amd as fk
    rng = np.random.default_rng(26020303)
    for case in range(20):
        D, dtype = (64, 128)[case % 2], ("bf16", "f32")[(case // 2) % 2]
        H = int(rng.choice([8, 16, 24, 40, 64, 72, 128, 200, 256])) if dtype == "bf16" else int(rng.choice([1, 5, 16, 63, 64, 65, 130]))
        Hkv, Bt = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        per_head = bool(rng.integers(0, 2)) or Hkv == 1
        cap = int(rng.choice([33, 100, 520, 1100]))
        lens = [int(rng.choice([0, 1, 31, 32, 33, cap, int(rng.integers(0, cap + 1))])) for _ in range(Bt)]
        print(f"random score case {case}: {dtype} D={D} H={H} Hkv={Hkv} per_head={per_head} cap={cap} lens={lens}", flush=True)
        c = random_cache(ora, 9000 + case, dtype, Bt, Hkv, cap, D, lens=lens, scale=0.5)
        nset, F = (Hkv if per_head else 1), 2 * D
        W1 = store((si.normal(9100 + case, si.T_W1, 0, np.arange(nset * F * H)).reshape(nset, F, H) / np.sqrt(F)).astype(np.float32), dtype)
        b1 = (si.normal(9100 + case, si.T_B1, 0, np.arange(nset * H)).reshape(nset, H) * 0.2).astype(np.float32)
        W2 = (si.normal(9100 + case, si.T_W2, 0, np.arange(nset * H)).reshape(nset, H) / np.sqrt(H)).astype(np.float32)
        b2 = (si.normal(9100 + case, si.T_B2, 0, np.arange(nset)) * 0.3).astype(np.float32)
        ref = ora.score_kv(c, W1, b1, W2, b2)
        dev = gpu.DevCache(c, Hkv)
        fk.fk_score_kv(dev.desc, dev.K, dev.V, dev.len, cap, gpu.to_dev(W1), gpu.to_dev(b1), gpu.to_dev(W2), gpu.to_dev(b2), dev.scores)
        got = dev.scores.cpu().numpy()
        gpu.assert_scores_close(got, ref, lens, f"case {case}")
        for b in range(Bt):
            assert np.isnan(got[b, :, lens[b]:]).all()
