"""Seeded synthetic inputs for the budgeted-KV decode + evict path.

This module is the only code shared by the CPU oracle's tests and the HIP path's
tests / benchmark.  It holds no arithmetic of the method itself (no attention, no
scorer, no selection, no compaction): it only turns (seed, tensor, coordinates)
into numbers, rounds them to the storage type, and describes the workload shapes.

Generator.  Counter based: every element of every tensor is a pure function of
(seed, tensor id, layer, batch, head, position, channel), so any slice can be
regenerated in isolation (a sampled row of a large workload, one decode step).
A 64-bit mixing hash of the counter gives two 24-bit uniforms; Box-Muller turns
them into a pair of standard normals shared by the two channels 2j, 2j+1.

Workloads.  ``config(i)`` returns the i-th workload of the benchmark description
(tiny fp32 case; Qwen3-4B single layer; 36-layer stack; GQA-7 mixture stack; ragged
large batch).  The value recipes stand in for the KV statistics of reasoning traces
(attention sinks, sparse heavy keys, clustered keys with exact duplicates); no item
of any public benchmark is used.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLD = np.uint64(0x9E3779B97F4A7C15)
_C1 = np.uint64(0xBF58476D1CE4E5B9)
_C2 = np.uint64(0x94D049BB133111EB)

# tensor ids of the counter streams
T_Q, T_K, T_V, T_W1, T_B1, T_W2, T_B2, T_FLAG, T_MIXMEAN, T_MIXSEL, T_LEN, T_SCORE, T_GUMBEL, T_W1A, T_ATT, T_ATTKEY = range(16)

BASE_SEED = 2602032030


def _mix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on uint64 arrays (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        x = (x ^ (x >> np.uint64(30))) * _C1
        x = (x ^ (x >> np.uint64(27))) * _C2
        x = x ^ (x >> np.uint64(31))
    return x


def _stream_base(seed: int, tensor: int, layer: int) -> np.uint64:
    s = np.array([(seed & 0xFFFFFFFFFFFFFFFF)], dtype=np.uint64)
    t = np.array([(tensor + (layer << 8) + 1)], dtype=np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(s ^ _mix64(t * _GOLD))[0]


def hash_u64(seed: int, tensor: int, layer: int, counter: np.ndarray) -> np.ndarray:
    """64 hashed bits for every entry of the integer array ``counter``."""
    c = np.asarray(counter).astype(np.uint64)
    with np.errstate(over="ignore"):
        return _mix64(_stream_base(seed, tensor, layer) + c * _GOLD)


def uniform01(seed: int, tensor: int, layer: int, counter: np.ndarray) -> np.ndarray:
    """Uniform in [0, 1) with 53 bits, one per counter."""
    return (hash_u64(seed, tensor, layer, counter) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def normal(seed: int, tensor: int, layer: int, counter: np.ndarray) -> np.ndarray:
    """Standard normal for every flat element index in ``counter`` (float64).

    Elements 2j and 2j+1 are the cosine / sine branch of one Box-Muller pair.
    """
    c = np.asarray(counter).astype(np.uint64)
    h = hash_u64(seed, tensor, layer, c >> np.uint64(1))
    u1 = ((h >> np.uint64(40)).astype(np.float64) + 1.0) * (1.0 / (1 << 24))  # (0, 1]
    u2 = ((h >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) * (1.0 / (1 << 24))
    r = np.sqrt(-2.0 * np.log(u1))
    ang = 2.0 * np.pi * u2
    odd = (c & np.uint64(1)).astype(bool)
    return np.where(odd, r * np.sin(ang), r * np.cos(ang))


def normal_rows(seed: int, tensor: int, layer: int, row_base: np.ndarray, D: int) -> np.ndarray:
    """Same values as ``normal`` for the flat indices row_base[...] + (0 .. D-1), D even and
    row_base even: one hash per Box-Muller pair.  Returns float64 [..., D]."""
    rb = np.asarray(row_base).astype(np.uint64)
    pair = (rb[..., None] >> np.uint64(1)) + np.arange(D // 2, dtype=np.uint64)
    h = hash_u64(seed, tensor, layer, pair)
    u1 = ((h >> np.uint64(40)).astype(np.float64) + 1.0) * (1.0 / (1 << 24))
    u2 = ((h >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) * (1.0 / (1 << 24))
    r = np.sqrt(-2.0 * np.log(u1))
    ang = 2.0 * np.pi * u2
    out = np.empty(pair.shape + (2,), np.float64)
    out[..., 0] = r * np.cos(ang)
    out[..., 1] = r * np.sin(ang)
    return out.reshape(rb.shape + (D,))


# ----------------------------------------------------------------------------
# storage formats
# ----------------------------------------------------------------------------

def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    r = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), r)
    return r.astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """Widen 16-bit bfloat16 patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Return ``x`` as float32 values that are exactly representable in ``dtype``."""
    x32 = np.asarray(x, dtype=np.float32)
    if dtype == "f32":
        return x32
    if dtype == "bf16":
        return from_bf16_bits(to_bf16_bits(x32))
    raise ValueError(dtype)


def storage_array(x32: np.ndarray, dtype: str) -> np.ndarray:
    """Pack float32 values (already representable) into the storage array:
    float32 for 'f32', uint16 bit patterns for 'bf16'."""
    if dtype == "f32":
        return np.ascontiguousarray(x32, dtype=np.float32)
    return to_bf16_bits(x32)


# ----------------------------------------------------------------------------
# workloads
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class Workload:
    name: str
    layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str            # 'f32' | 'bf16' : storage type of q, K, V, W1, out
    prompt: int           # prompt length P (ragged workloads: lower bound)
    steps: int            # decode steps
    budget: int           # B
    interval: int         # L : eviction every L steps; also the protected recent count R
    hidden: int           # scorer hidden width H
    value_scale: float    # multiplier on N(0,1) for q, k, v
    heavy: str            # 'sink4' | 'sparse1pct' | 'mixture16'
    seed: int
    ragged_max: int = 0   # >0: initial lengths uniform in [prompt, ragged_max]

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def capacity(self) -> int:
        return max(self.budget, self.ragged_max, self.prompt) + self.interval

    @property
    def rows(self) -> int:
        return self.batch * self.n_kv_heads

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def softmax_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


def config(i: int) -> Workload:
    s = BASE_SEED + i
    inv = 1.0 / float(np.sqrt(128.0))
    if i == 0:
        return Workload("cfg0-tiny-f32", 1, 1, 8, 2, 64, "f32", 64, 512, 128, 32, 64, 1.0, "sink4", s)
    if i == 1:
        return Workload("cfg1-qwen3-4b-layer", 1, 16, 32, 8, 128, "bf16", 512, 8192, 2048, 128, 256, inv, "sparse1pct", s)
    if i == 2:
        return Workload("cfg2-qwen3-4b-stack", 36, 8, 32, 8, 128, "bf16", 512, 32768 - 512, 16384, 128, 256, inv, "sparse1pct", s)
    if i == 3:
        return Workload("cfg3-7b-distill-gqa7", 28, 16, 28, 4, 128, "bf16", 512, 16384 - 512, 4096, 64, 256, inv, "mixture16", s)
    if i == 4:
        return Workload("cfg4-ragged-batch64", 1, 64, 32, 8, 128, "bf16", 1024, 2048, 8192, 128, 256, inv, "sparse1pct", s,
                        ragged_max=32768)
    raise IndexError(i)


_POS_SPAN = 1 << 20   # positions per (batch, head) stream in the flat counter
_HEAD_SPAN = 64       # heads per batch entry in the flat counter


def _flat_index(b: np.ndarray, h: np.ndarray, pos: np.ndarray, d: np.ndarray, D: int) -> np.ndarray:
    b, h, pos, d = np.broadcast_arrays(b, h, pos, d)
    return ((b.astype(np.int64) * _HEAD_SPAN + h) * _POS_SPAN + pos) * D + d


def initial_lengths(w: Workload) -> np.ndarray:
    """Per-sequence prompt length (int32 [batch])."""
    if w.ragged_max <= 0:
        return np.full(w.batch, w.prompt, dtype=np.int32)
    u = uniform01(w.seed, T_LEN, 0, np.arange(w.batch))
    return (w.prompt + np.floor(u * (w.ragged_max - w.prompt + 1))).astype(np.int32)


def heavy_positions(w: Workload, b: np.ndarray, pos: np.ndarray) -> np.ndarray:
    """Multiplier applied to the key at (sequence b, position pos); shared by all heads."""
    b, pos = np.broadcast_arrays(np.asarray(b), np.asarray(pos))
    if w.heavy == "sink4":
        return np.where(pos < 4, 4.0, 1.0)
    if w.heavy == "sparse1pct":
        u = uniform01(w.seed, T_FLAG, 0, b.astype(np.int64) * _POS_SPAN + pos)
        return np.where(u < 0.01, 3.0, 1.0)
    return np.ones(b.shape)


def _mixture_kv(w: Workload, layer: int, bs, hs, ps) -> tuple[np.ndarray, np.ndarray]:
    """(k ‖ v) rows drawn jointly from a 16-component Gaussian mixture with a quarter
    of the rows being exact copies of their component mean (score ties)."""
    D = w.head_dim
    ncomp = 16
    means = normal(w.seed, T_MIXMEAN, layer, np.arange(ncomp * 2 * D)).reshape(ncomp, 2 * D) * w.value_scale
    B_, H_, P_ = np.meshgrid(bs, hs, ps, indexing="ij")
    cnt = (B_.astype(np.int64) * _HEAD_SPAN + H_) * _POS_SPAN + P_
    hsel = hash_u64(w.seed, T_MIXSEL, layer, cnt)
    comp = (hsel & np.uint64(15)).astype(np.int64)
    exact = ((hsel >> np.uint64(8)) & np.uint64(3)) == np.uint64(0)      # probability 1/4
    rb = _flat_index(B_, H_, P_, 0, D)
    kn = normal_rows(w.seed, T_K, layer, rb, D)
    vn = normal_rows(w.seed, T_V, layer, rb, D)
    sig = 0.02 * w.value_scale
    noise_k = np.where(exact[..., None], 0.0, sig * kn)
    noise_v = np.where(exact[..., None], 0.0, sig * vn)
    k = means[comp][..., :D] + noise_k
    v = means[comp][..., D:] + noise_v
    return k, v


def gen_kv(w: Workload, layer: int, pos_lo: int, pos_hi: int, batch_sel=None, head_sel=None):
    """Keys and values for absolute positions [pos_lo, pos_hi).

    Returns float32 arrays K, V of shape [nb, nh, npos, D] whose values are exactly
    representable in the workload's storage type.
    """
    bs = np.arange(w.batch) if batch_sel is None else np.asarray(batch_sel)
    hs = np.arange(w.n_kv_heads) if head_sel is None else np.asarray(head_sel)
    ps = np.arange(pos_lo, pos_hi)
    D = w.head_dim
    if w.heavy == "mixture16":
        k, v = _mixture_kv(w, layer, bs, hs, ps)
    else:
        rb = _flat_index(bs[:, None, None], hs[None, :, None], ps[None, None, :], 0, D)
        k = normal_rows(w.seed, T_K, layer, rb, D) * w.value_scale
        v = normal_rows(w.seed, T_V, layer, rb, D) * w.value_scale
        k = k * heavy_positions(w, bs[:, None, None, None], ps[None, None, :, None])
    return round_to_storage(k, w.dtype), round_to_storage(v, w.dtype)


def gen_q(w: Workload, layer: int, pos_lo: int, pos_hi: int, batch_sel=None, head_sel=None) -> np.ndarray:
    """Queries for absolute positions [pos_lo, pos_hi): float32 [nb, nh_q, npos, D]."""
    bs = np.arange(w.batch) if batch_sel is None else np.asarray(batch_sel)
    hs = np.arange(w.n_q_heads) if head_sel is None else np.asarray(head_sel)
    ps = np.arange(pos_lo, pos_hi)
    D = w.head_dim
    rb = _flat_index(bs[:, None, None], hs[None, :, None], ps[None, None, :], 0, D)
    q = normal_rows(w.seed, T_Q, layer, rb, D) * w.value_scale
    return round_to_storage(q, w.dtype)


def gen_scorer(w: Workload, layer: int):
    """Random-init scorer weights, one set per KV head of the layer.

    W1 [Hkv, 2D, H] ~ N(0, 1/(2D)) rounded to the storage type; b1 [Hkv, H] ~ N(0, 1/(2D));
    W2 [Hkv, H] ~ N(0, 1/H); b2 [Hkv] ~ N(0, 1/H).  b1, W2, b2 stay float32.
    """
    F, H, Hkv = 2 * w.head_dim, w.hidden, w.n_kv_heads
    w1 = normal(w.seed, T_W1, layer, np.arange(Hkv * F * H)).reshape(Hkv, F, H) / np.sqrt(F)
    b1 = normal(w.seed, T_B1, layer, np.arange(Hkv * H)).reshape(Hkv, H) / np.sqrt(F)
    w2 = normal(w.seed, T_W2, layer, np.arange(Hkv * H)).reshape(Hkv, H) / np.sqrt(H)
    b2 = normal(w.seed, T_B2, layer, np.arange(Hkv)) / np.sqrt(H)
    return (round_to_storage(w1, w.dtype), b1.astype(np.float32), w2.astype(np.float32), b2.astype(np.float32))


def gen_scorer_feat(w: Workload, layer: int, gain: float = 8.0):
    """Scorer weights for inputs with attention features: W1 [Hkv, 2D + 6g, H], whose first 2D rows are
    gen_scorer's and whose 6g feature rows are ~ N(0, gain^2 / (6g)) (attention sums are small numbers;
    the gain makes them move the scores); b1, W2, b2 as gen_scorer."""
    w1, b1, w2, b2 = gen_scorer(w, layer)
    A, H, Hkv = 6 * w.group, w.hidden, w.n_kv_heads
    wa = normal(w.seed, T_W1A, layer, np.arange(Hkv * A * H)).reshape(Hkv, A, H) * (gain / np.sqrt(A))
    return (np.concatenate([w1, round_to_storage(wa, w.dtype)], axis=1), b1, w2, b2)


def gen_scores(seed: int, shape, ties: int = 0) -> np.ndarray:
    """Standalone float32 scores for selection tests; ``ties`` > 0 quantises them to
    that many distinct levels so that exact ties are frequent."""
    n = int(np.prod(shape))
    s = normal(seed, T_SCORE, 0, np.arange(n)).reshape(shape)
    if ties > 0:
        s = np.round(s * ties / 4.0) * (4.0 / ties)
    return s.astype(np.float32)


def gen_gumbel(seed: int, shape, event: int = 0, levels: int = 0) -> np.ndarray:
    """Standard Gumbel noise g = -log(-log u), float32, one value per cache slot, for the sampled
    eviction policy; ``event`` selects an independent stream per eviction event.  ``levels`` > 0
    quantises the noise so that exact ties with quantised scores occur."""
    n = int(np.prod(shape))
    u = uniform01(seed, T_GUMBEL, event, np.arange(n))
    u = np.clip(u, 2.0 ** -53, 1.0 - 2.0 ** -53)
    g = -np.log(-np.log(u)).reshape(shape)
    if levels > 0:
        g = np.round(g * levels / 4.0) * (4.0 / levels)
    return g.astype(np.float32)


def gen_attention(seed: int, n_heads: int, T: int, dtype: str = "f32", spread: float = 1.5, sinks: int = 4,
                  heavy_frac: float = 0.02, recency: float = 96.0) -> np.ndarray:
    """Synthetic causal attention matrices [n_heads, T, T] of a full trace, float32 values rounded to the
    storage type: row-wise softmax of random logits with the structure reasoning traces show (a few sink
    positions, sparse heavy keys whose weight comes and goes per query, a recency ramp); zero above the
    diagonal.  Stands in for the attention of a real model on a real trace."""
    A = np.zeros((n_heads, T, T), np.float32)
    key_u = uniform01(seed, T_ATTKEY, 0, np.arange(n_heads * T)).reshape(n_heads, T)
    key_bias = np.where(key_u < heavy_frac, 3.0, 0.0)
    key_bias[:, :sinks] += 4.0
    dist = np.arange(T)[:, None] - np.arange(T)[None, :]              # q - i
    ramp = -np.minimum(np.maximum(dist, 0), 4 * recency) / recency
    for h in range(n_heads):
        z = spread * normal(seed, T_ATT, h, np.arange(T * T)).reshape(T, T) + key_bias[h][None, :] + ramp
        z = np.where(dist >= 0, z, -np.inf)
        z -= z.max(axis=1, keepdims=True)
        e = np.exp(z)
        A[h] = (e / e.sum(axis=1, keepdims=True)).astype(np.float32)
    return round_to_storage(A, dtype)
