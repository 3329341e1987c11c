"""Parity of the Golden Eviction label builder (Section 3.2 Eq. 3-5) against the oracle.

Block scores and future scores: fp32 sums of up to g*L non-negative terms against fp64, bar
|x - ref| <= 1e-9 + 1e-5 |ref| (2^-24 * sqrt(terms) relative, a decade of margin).  The trace is
index work: bit exact, both sides selecting on the same fp32 future scores (the oracle's, and
separately the device's own)."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    import paper_2602_03203_amd as fk
    fk.lib()
    return gpu_util


def to_dev_padded(gpu, A32, dtype, ld):
    """[Hq,T,T] float32 values (already rounded to the storage type) -> device [Hq,T,ld] with junk-free padding."""
    Hq, T, _ = A32.shape
    pad = np.zeros((Hq, T, ld), np.float32)
    pad[:, :, :T] = A32
    return gpu.to_dev(si.storage_array(pad, dtype))


def run_case(gpu, dtype, Hq, g, T, B, L, seed=5, ld=None):
    import paper_2602_03203_amd as fk
    from oracle import golden
    ld = (T + 7) // 8 * 8 if ld is None else ld
    print(f"golden {dtype} Hq={Hq} g={g} T={T} B={B} L={L} ld={ld}", flush=True)
    A32 = si.gen_attention(seed, Hq, T, dtype)
    M = golden.n_steps(T, B, L)
    assert fk.fk_golden_steps(T, B, L) == M
    Hkv = Hq // g
    dA = to_dev_padded(gpu, A32, dtype, ld)
    d_a = torch.full((Hkv, max(M, 1), T), float("nan"), dtype=torch.float32, device="cuda")
    d_alpha = torch.full_like(d_a, float("nan"))
    fk.fk_golden_scores(dA, Hkv, T, B, L, d_a, d_alpha)
    if M == 0:
        assert torch.isnan(d_a).all() and torch.isnan(d_alpha).all()
        return 0
    a_ref = golden.block_scores(A32.astype(np.float64), g, B, L)
    alpha_ref = golden.future_scores(a_ref)
    for got, ref, what in ((d_a, a_ref, "block scores"), (d_alpha, alpha_ref, "future scores")):
        gh = got.cpu().numpy().astype(np.float64)
        err = np.abs(gh - ref) - (1e-9 + 1e-5 * np.abs(ref))
        assert (err <= 0).all(), f"{what}: worst excess {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"
    assert a_ref.max() > 0
    # the device's future scores are exactly the running maximum of ITS block scores
    ah = d_a.cpu().numpy()
    assert np.array_equal(d_alpha.cpu().numpy(), np.maximum.accumulate(ah[:, ::-1], axis=1)[:, ::-1])
    # trace on the oracle's fp32 future scores: bit exact
    a32 = alpha_ref.astype(np.float32)
    d_kept = torch.full((Hkv, M, B), -1, dtype=torch.int32, device="cuda")
    fk.fk_golden_trace(torch.from_numpy(a32).cuda(), T, B, L, d_kept)
    assert np.array_equal(d_kept.cpu().numpy(), golden.trace(a32, B, L))
    # and on the device's own
    d_kept.fill_(-1)
    fk.fk_golden_trace(d_alpha, T, B, L, d_kept)
    assert np.array_equal(d_kept.cpu().numpy(), golden.trace(d_alpha.cpu().numpy(), B, L))
    return M


@pytest.mark.parametrize("dtype,Hq,g,T,B,L", [
    ("f32", 4, 2, 300, 64, 16),       # last block partial (12 of 16 queries)
    ("bf16", 8, 4, 517, 96, 32),      # T not a multiple of the tile nor of 8 (padded leading dimension)
    ("f32", 3, 1, 200, 40, 8),        # no head pooling
    ("bf16", 7, 7, 260, 48, 24),      # one group of 7 heads
    ("f32", 2, 2, 129, 32, 32),       # B == L: no old pair survives a step
    ("bf16", 2, 1, 2700, 2500, 50),   # cache far larger than the workgroup: several passes of the ordered scan
])
def test_small_traces(gpu, dtype, Hq, g, T, B, L):
    assert run_case(gpu, dtype, Hq, g, T, B, L) > 0


@pytest.mark.parametrize("T", [48, 49])
def test_traces_that_never_evict_or_evict_once(gpu, T):
    """T <= B + L: M = 0 and nothing is written; T = B + L + 1: one step whose block holds one query."""
    assert run_case(gpu, "f32", 2, 2, T, 32, 16) == (0 if T == 48 else 1)


def test_exact_ties_keep_the_lower_position(gpu):
    """Uniform causal attention: all candidates tie at every step (closed form of the oracle pins)."""
    import paper_2602_03203_amd as fk
    from oracle import golden
    Hq, g, T, B, L = 2, 2, 63, 20, 10
    A = np.zeros((Hq, T, T), np.float32)
    for q in range(T):
        A[:, q, :q + 1] = np.float32(1.0 / (q + 1))
    M = golden.n_steps(T, B, L)
    dA = to_dev_padded(gpu, A, "f32", 64)
    d_a = torch.zeros((1, M, T), dtype=torch.float32, device="cuda")
    d_alpha = torch.zeros_like(d_a)
    fk.fk_golden_scores(dA, 1, T, B, L, d_a, d_alpha)
    # fp32 sums of equal terms in a different order may differ in the last bit, so select on the oracle's values
    a32 = golden.future_scores(golden.block_scores(A.astype(np.float64), g, B, L)).astype(np.float32)
    np.testing.assert_allclose(d_alpha.cpu().numpy(), a32, rtol=1e-6)
    d_kept = torch.full((1, M, B), -1, dtype=torch.int32, device="cuda")
    fk.fk_golden_trace(torch.from_numpy(a32).cuda(), T, B, L, d_kept)
    kept = d_kept.cpu().numpy()
    for t in range(1, M + 1):
        assert np.array_equal(kept[0, t - 1], np.concatenate([np.arange(B - L), np.arange(B + t * L - L, B + t * L)]))


@pytest.mark.parametrize("Hkv,T,B,L", [
    (2, 16000, 9000, 1100),   # a wavefront's stretch of candidates is 9 x 64 wide, more than 1024 newest pairs per step
    (1, 9000, 4096, 512),     # stretches of exactly 4 x 64
    (3, 5000, 2049, 7),       # one candidate beyond two full stretches per lane
])
def test_trace_on_large_budgets(gpu, Hkv, T, B, L):
    """The trace alone on synthetic future scores (random, with repeated values so that ties at the cut occur):
    budgets whose candidates span many slots per lane.  Bit exact against the oracle's trace."""
    import paper_2602_03203_amd as fk
    from oracle import golden
    M = golden.n_steps(T, B, L)
    rng = np.random.default_rng(T + B + L)
    alpha = (rng.integers(0, 4096, size=(Hkv, M, T)) / 4096.0).astype(np.float32)
    print(f"trace Hkv={Hkv} T={T} B={B} L={L} M={M}", flush=True)
    d_kept = torch.full((Hkv, M, B), -1, dtype=torch.int32, device="cuda")
    fk.fk_golden_trace(torch.from_numpy(alpha).cuda(), T, B, L, d_kept)
    assert np.array_equal(d_kept.cpu().numpy(), golden.trace(alpha, B, L))


def test_layer_slice_at_paper_budget(gpu):
    """Budget 256, L 64 on a 2048-token trace, 8 query heads in 2 groups, bf16: 27 steps, tiles on and
    off the diagonal, every output compared."""
    assert run_case(gpu, "bf16", 8, 4, 2048, 256, 64, seed=9) == 27


def test_qwen3_4b_layer_full_size_sampled_columns(gpu):
    """The shape bench.py --workload golden times: 32 query / 8 KV heads, 8192-token trace, B 2048, L 128,
    bf16 (4.3 GB of attention, 47 steps).  The attention is drawn on the device (seeded torch ops, an input
    like any other); the oracle recomputes 96 sampled key columns of every group and block, and the whole
    trace from the device's own future scores."""
    import paper_2602_03203_amd as fk
    from oracle import golden
    Hq, Hkv, T, B, L = 32, 8, 8192, 2048, 128
    g = Hq // Hkv
    M = golden.n_steps(T, B, L)
    assert M == 47
    print("drawing the attention", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(2602)
    A = torch.empty((Hq, T, T), dtype=torch.bfloat16, device="cuda")
    causal = torch.ones((T, T), dtype=torch.bool, device="cuda").tril_()
    keyb = (torch.rand((Hq, 1, T), generator=gen, device="cuda") < 0.02).float() * 3.0
    for h in range(Hq):
        z = 1.5 * torch.randn((T, T), generator=gen, device="cuda") + keyb[h]
        z.masked_fill_(~causal, float("-inf"))
        A[h] = torch.softmax(z, dim=1).to(torch.bfloat16)
    del z, causal
    d_a = torch.empty((Hkv, M, T), dtype=torch.float32, device="cuda")
    d_alpha = torch.empty_like(d_a)
    print("fk_golden_scores", flush=True)
    fk.fk_golden_scores(A, Hkv, T, B, L, d_a, d_alpha)
    torch.cuda.synchronize()
    cols = np.unique(np.concatenate([np.array([0, 1, 63, 64, 127, 128, 2047, 2048, 2175, 2176, 2177, 2303, 2304, 8191, 8064, 8063]),
                                     (si.uniform01(77, si.T_FLAG, 0, np.arange(80)) * T).astype(np.int64)]))
    sub = A[:, :, torch.from_numpy(cols).cuda()].float().cpu().numpy().astype(np.float64)
    a_ref = golden.block_scores(sub, g, B, L)
    alpha_ref = golden.future_scores(a_ref)
    for got, ref, what in ((d_a, a_ref, "block scores"), (d_alpha, alpha_ref, "future scores")):
        gh = got[:, :, torch.from_numpy(cols).cuda()].cpu().numpy().astype(np.float64)
        err = np.abs(gh - ref) - (1e-9 + 1e-5 * np.abs(ref))
        assert (err <= 0).all(), f"{what}: worst excess {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"
    ah = d_a.cpu().numpy()
    assert np.array_equal(d_alpha.cpu().numpy(), np.maximum.accumulate(ah[:, ::-1], axis=1)[:, ::-1])
    print("fk_golden_trace", flush=True)
    d_kept = torch.full((Hkv, M, B), -1, dtype=torch.int32, device="cuda")
    fk.fk_golden_trace(d_alpha, T, B, L, d_kept)
    assert np.array_equal(d_kept.cpu().numpy(), golden.trace(d_alpha.cpu().numpy(), B, L))


def test_bad_arguments(gpu):
    import paper_2602_03203_amd as fk
    A = torch.zeros((2, 64, 60), dtype=torch.float32, device="cuda")     # ld not a multiple of 8
    o = torch.zeros((1, 4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(fk.FkError) as e:
        fk.fk_golden_scores(A, 1, 60, 16, 8, o, o)
    assert e.value.code == 1
    k = torch.zeros((1, 4, 16), dtype=torch.int32, device="cuda")
    with pytest.raises(fk.FkError) as e:
        fk.fk_golden_trace(o, 64, 20000, 8, k)                          # cache larger than the kernel's LDS plan
    assert e.value.code == 2
    assert fk.fk_golden_steps(100, 8, 16) == -1                         # L > B
