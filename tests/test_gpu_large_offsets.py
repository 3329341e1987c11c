"""One pass of every call on a cache whose rows lie beyond 2^31 elements and 2^32 bytes from the start of
the tensors (1 sequence x 3 KV heads x 2^23 slots x 128 channels, bf16: 6.4 GB per tensor), to catch
32-bit index arithmetic.  The data are aperiodic on purpose (every slot carries its own index in two
channels, dominant keys sit near the end of each row): a wrapped address would read different values."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    if torch.cuda.get_device_properties(0).total_memory < 60 * 2 ** 30:
        pytest.skip("needs 60 GB of device memory")
    import gpu_util
    import paper_2602_03203_amd as fk
    fk.lib()
    return gpu_util


def test_rows_beyond_four_gigabytes(gpu, ora):
    import paper_2602_03203_amd as fk
    Hkv, g, D, cap = 3, 2, 128, 1 << 23
    n = cap - 3
    B, R, H = cap - 5000, 128, 32
    print("building the cache", flush=True)
    blk = si.round_to_storage(si.normal(91, si.T_K, 0, np.arange(2 * 8192 * D)).reshape(2, 8192, D).astype(np.float32) * 0.1, "bf16")
    c = ora.new_cache("bf16", 1, Hkv, cap, D)
    idx = np.arange(cap)
    for h in range(Hkv):
        for name, src in (("K", blk[0]), ("V", blk[1])):
            t = np.tile(src, (cap // 8192, 1))
            t[:, 2 * h] = (idx % 251) / 251.0                     # the slot's own index, aperiodic against 8192
            t[:, 2 * h + 1] = ((idx // 251) % 241) / 241.0
            getattr(c, name)[0, h] = si.storage_array(si.round_to_storage(t, "bf16"), "bf16")
            del t
    c.pos[0, :, :n] = np.arange(n, dtype=np.int32)
    c.len[0] = n
    q = si.storage_array(si.round_to_storage(si.normal(92, si.T_Q, 0, np.arange(Hkv * g * D)).reshape(1, Hkv * g, D).astype(np.float32), "bf16"), "bf16")
    qf = si.from_bf16_bits(q).astype(np.float32)
    for h in range(Hkv):                                          # a dominant key near the end of every row
        c.K[0, h, n - 7 - h] = si.storage_array(si.round_to_storage(2.0 * qf[0, h * g], "bf16"), "bf16")
    dev = gpu.DevCache(c, Hkv * g)

    print("attention", flush=True)
    got = dev.attn(gpu.to_dev(q), 1.0)
    ref = ora.decode_attn(c, q, 1.0)
    gpu.assert_attn_close(got, ref, "bf16", "attention over 2^23 keys")
    vdom = si.from_bf16_bits(c.V[0, 2, n - 9]).astype(np.float64)
    assert np.abs(got[0, 2 * g] - vdom).max() < 0.05              # head 4 sees (almost only) its dominant key in row 2

    print("scores on sampled windows", flush=True)
    w = si.config(1).scaled(n_q_heads=Hkv * g, n_kv_heads=Hkv, hidden=H)
    W1, b1, W2, b2 = si.gen_scorer(w, 0)
    W1 = si.storage_array(W1, "bf16")
    fk.fk_score_kv(dev.desc, dev.K, dev.V, dev.len, n, gpu.to_dev(W1), gpu.to_dev(b1), gpu.to_dev(W2), gpu.to_dev(b2), dev.scores)
    sc_dev = dev.scores.cpu().numpy()
    for lo in (0, cap // 2 - 100, n - 300):
        sub = ora.Cache("bf16", c.K[:, :, lo:lo + 300].copy(), c.V[:, :, lo:lo + 300].copy(), c.pos[:, :, lo:lo + 300].copy(),
                        np.array([300], np.int32))
        ref_sc = ora.score_kv(sub, W1, b1, W2, b2)
        gpu.assert_scores_close(sc_dev[:, :, lo:lo + 300], ref_sc, [300], f"scores at slots {lo}..")

    print("selection", flush=True)
    scores = si.gen_scores(93, (1, Hkv, cap))
    dev.scores.copy_(torch.from_numpy(scores).cuda())
    keep = torch.full((1, Hkv, B), -1, dtype=torch.int32, device="cuda")
    fk.fk_select_keep(dev.desc, dev.scores, dev.pos, dev.len, n, B, R, keep)
    keep_ref = ora.select_keep(scores, c.pos, c.len, B, R, "sort")
    gpu.assert_keep_equal(keep.cpu().numpy(), keep_ref, c.len, B)

    print("compaction", flush=True)
    fk.fk_compact(dev.desc, dev.K, dev.V, dev.pos, dev.len, keep, B)
    ora.compact(c, keep_ref, B)
    host = dev.host(ora)
    assert host.len[0] == B == c.len[0]
    for h in range(Hkv):
        assert np.array_equal(host.pos[0, h, :B], c.pos[0, h, :B])
        assert np.array_equal(host.K[0, h, :B], c.K[0, h, :B]) and np.array_equal(host.V[0, h, :B], c.V[0, h, :B])

    print("append + fused step at the end of the rows", flush=True)
    kn = gpu.to_dev(np.ascontiguousarray(c.K[:, :, 5]))
    vn = gpu.to_dev(np.ascontiguousarray(c.V[:, :, 6]))
    pn = torch.tensor([n + 10], dtype=torch.int32, device="cuda")
    fk.fk_decode_step(dev.desc, gpu.to_dev(q), dev.K, dev.V, dev.pos, dev.len, kn, vn, pn, B + 1, 1.0, dev.out, dev.ws)
    ora.append(c, np.ascontiguousarray(c.K[:, :, 5]), np.ascontiguousarray(c.V[:, :, 6]), np.array([n + 10], np.int32))
    gpu.assert_attn_close(gpu.out_to_f64(dev.out), ora.decode_attn(c, q, 1.0), "bf16", "fused step")
    host = dev.host(ora)
    assert host.len[0] == B + 1 and np.array_equal(host.K[0, :, B], c.K[0, :, B]) and np.array_equal(host.pos[0, :, B], c.pos[0, :, B])
