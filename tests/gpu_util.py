"""Device-side helpers for the GPU parity tests: move oracle-format host arrays to device
buffers and back.  No arithmetic of the method here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2602_03203_amd as fk


def to_dev(a: np.ndarray, dtype: str | None = None) -> torch.Tensor:
    """numpy -> device tensor; uint16 bf16 bit patterns become torch.bfloat16."""
    if a.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def out_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.float().cpu().numpy().astype(np.float64)


class DevCache:
    """Device copy of an oracle cache plus the descriptor and an attention workspace."""

    def __init__(self, c, n_q_heads: int):
        Bt, Hkv, cap, D = c.shape
        self.desc = fk.CacheDesc(Bt, n_q_heads, Hkv, D, cap, c.dtype)
        self.K, self.V = to_dev(c.K), to_dev(c.V)
        # the device keeps one length per row; the oracle one per sequence (all heads equal)
        self.pos, self.len = to_dev(c.pos), to_dev(np.repeat(c.len[:, None], Hkv, axis=1).astype(np.int32))
        self.ws = fk.new_attn_workspace(self.desc)
        self.out = torch.empty((Bt, n_q_heads, D), dtype=self.desc.torch_dtype, device="cuda")
        self.scores = torch.full((Bt, Hkv, cap), float("nan"), dtype=torch.float32, device="cuda")

    def host(self, oracle):
        ln = to_host(self.len)
        assert (ln == ln[:, :1]).all(), "rows of a sequence must hold equal counts"
        return oracle.Cache(self.desc.dtype, to_host(self.K), to_host(self.V), to_host(self.pos), np.ascontiguousarray(ln[:, 0]))

    def attn(self, q_dev, scale, max_len=None):
        fk.fk_decode_attn(self.desc, q_dev, self.K, self.V, self.len, max_len or self.desc.capacity, scale, self.out, self.ws)
        return out_to_f64(self.out)


def attn_tolerance(dtype: str):
    """(atol, rtol) of the attention parity bar: bf16 from the benchmark statement, fp32 derived
    from fp32 accumulation over a few thousand terms."""
    return (1e-2, 2e-2) if dtype == "bf16" else (1e-5, 1e-4)


def assert_attn_close(got, ref, dtype, what=""):
    atol, rtol = attn_tolerance(dtype)
    err = np.abs(got - ref) - (atol + rtol * np.abs(ref))
    assert (err <= 0).all(), f"{what}: worst excess {err.max():.3e} at {np.unravel_index(err.argmax(), err.shape)}"


def assert_scores_close(got, ref, lens, what=""):
    """|phi_gpu - phi_ref| <= 1e-3 * max(|phi_ref|, rms of the row's reference scores)."""
    Bt, Hkv, _ = ref.shape
    for b in range(Bt):
        n = int(lens[b])
        if n == 0:
            continue
        for h in range(Hkv):
            r, g = ref[b, h, :n], got[b, h, :n].astype(np.float64)
            bound = 1e-3 * np.maximum(np.abs(r), np.sqrt(np.mean(r * r)))
            bad = np.abs(g - r) > bound
            assert not bad.any(), f"{what} row ({b},{h}): {bad.sum()} scores off, worst {np.abs(g - r).max():.3e} vs bound {bound.min():.3e}"


def assert_keep_equal(got, ref, lens, budget, what=""):
    """Keep-sets bit for bit.  Rows over budget: the device's kept slots equal the oracle's.  Rows at or under budget
    (nothing to prune): the device writes the identity over all `budget` entries, the oracle j for j < len and -1
    beyond; both say "every live slot stays where it is"."""
    got, ref = np.asarray(got), np.asarray(ref)
    assert got.shape == ref.shape and got.shape[-1] == budget
    Bt, Hkv, _ = ref.shape
    ident = np.arange(budget, dtype=ref.dtype)
    for b in range(Bt):
        n = int(lens[b])
        for h in range(Hkv):
            if n > budget:
                assert np.array_equal(got[b, h], ref[b, h]), f"{what} row ({b},{h}): keep-set differs"
            else:
                assert np.array_equal(ref[b, h, :n], ident[:n]) and (ref[b, h, n:] == -1).all(), f"{what} row ({b},{h}): oracle convention"
                assert np.array_equal(got[b, h], ident), f"{what} row ({b},{h}): identity expected at or under budget"
