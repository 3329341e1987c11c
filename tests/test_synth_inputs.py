"""The seeded generator: reproducible in isolation, right storage rounding, stated distributions."""
import numpy as np
import torch

import synth_inputs as si


def test_slices_regenerate_identically():
    w = si.config(1)
    K, V = si.gen_kv(w, 0, 100, 108, batch_sel=[3, 9], head_sel=[1, 6])
    K2, V2 = si.gen_kv(w, 0, 104, 105, batch_sel=[9], head_sel=[6])
    assert np.array_equal(K[1, 1, 4], K2[0, 0, 0]) and np.array_equal(V[1, 1, 4], V2[0, 0, 0])
    q = si.gen_q(w, 0, 7, 9, batch_sel=[2], head_sel=[31])
    q2 = si.gen_q(w, 0, 0, 9)
    assert np.array_equal(q[0, 0], q2[2, 31, 7:9])
    assert not np.array_equal(si.gen_kv(w, 1, 100, 101)[0], si.gen_kv(w, 0, 100, 101)[0])


def test_bf16_rounding_matches_library_cast():
    x = (si.normal(1, 0, 0, np.arange(20000)) * 3).astype(np.float32)
    x[:5] = [0.0, -0.0, np.inf, -np.inf, 1e-40]
    bits = si.to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)
    assert np.array_equal(si.from_bf16_bits(bits), torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_distributions():
    z = si.normal(9, 3, 0, np.arange(400000))
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01 and abs((z ** 4).mean() - 3) < 0.1
    w0 = si.config(0)
    K, _ = si.gen_kv(w0, 0, 0, 64)
    assert K[0, :, :4].std() > 3.0 and abs(K[0, :, 4:].std() - 1.0) < 0.05       # sink-like keys
    w1 = si.config(1)
    m = si.heavy_positions(w1, np.arange(16)[:, None], np.arange(4096)[None, :])
    assert 0.005 < (m == 3.0).mean() < 0.015
    w3 = si.config(3)
    K, V = si.gen_kv(w3, 0, 0, 256, batch_sel=[0], head_sel=[0])
    x = np.concatenate([K, V], -1)[0, 0]
    uniq = np.unique(x, axis=0)
    assert len(uniq) < 256 - 20          # exact duplicate rows exist (score ties)
    lens = si.initial_lengths(si.config(4))
    assert lens.min() >= 1024 and lens.max() <= 32768 and len(set(lens.tolist())) > 32


def test_config_shapes():
    c = [si.config(i) for i in range(5)]
    assert [w.capacity for w in c] == [160, 2176, 16512, 4160, 32896]
    assert [w.group for w in c] == [4, 4, 4, 7, 4]
    assert c[1].prompt + 13 * c[1].interval == c[1].capacity
