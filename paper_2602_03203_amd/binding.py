"""ctypes binding of libfk.so: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used as plain device buffers; every step of the
path runs in the library's HIP kernels.  bf16 buffers may be torch.bfloat16 or raw
torch.uint16 / torch.int16 bit patterns.  There is no fallback: if the library is not
built, importing the functions raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfk.so")

FK_OK, FK_ERR_INVALID_ARG, FK_ERR_UNSUPPORTED, FK_ERR_WORKSPACE, FK_ERR_LAUNCH = range(5)
FK_F32, FK_BF16 = 0, 1

SYMBOLS = ["fk_status_string", "fk_version", "fk_append", "fk_decode_attn_workspace", "fk_decode_attn", "fk_decode_step", "fk_decode_window", "fk_decode_step_static",
           "fk_score_kv", "fk_select_keep", "fk_select_keep_workspace", "fk_select_keep_ws", "fk_select_keep_sampled", "fk_compact", "fk_decode_step_feat_workspace",
           "fk_decode_step_feat", "fk_decode_window_feat", "fk_score_kv_feat", "fk_compact_feat", "fk_golden_steps", "fk_golden_scores",
           "fk_golden_trace", "fk_stream_read"]


class fk_cache_desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("capacity", ctypes.c_int32), ("dtype", ctypes.c_int32), ("flags", ctypes.c_int32)]


class fk_scorer(ctypes.Structure):
    _fields_ = [("w1", ctypes.c_void_p), ("b1", ctypes.c_void_p), ("w2", ctypes.c_void_p), ("b2", ctypes.c_void_p),
                ("hidden", ctypes.c_int32), ("per_head", ctypes.c_int32), ("skip_len", ctypes.c_int32)]


class FkError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (fk_status {code})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libfk.so (built in-tree by paper_2602_03203_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built: run `python -m paper_2602_03203_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        dp, sp = ctypes.POINTER(fk_cache_desc), ctypes.POINTER(fk_scorer)
        L.fk_status_string.restype, L.fk_status_string.argtypes = ctypes.c_char_p, [ctypes.c_int]
        L.fk_version.restype, L.fk_version.argtypes = ctypes.c_char_p, []
        L.fk_append.restype, L.fk_append.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.fk_decode_attn_workspace.restype, L.fk_decode_attn_workspace.argtypes = sz, [dp, i32]
        L.fk_decode_attn.restype, L.fk_decode_attn.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, i32, f32, vp, vp, sz, vp]
        L.fk_decode_step.restype, L.fk_decode_step.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp, sz, vp]
        L.fk_decode_window.restype, L.fk_decode_window.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, f32, vp, vp, sz, vp]
        L.fk_decode_step_static.restype, L.fk_decode_step_static.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp]
        L.fk_score_kv.restype, L.fk_score_kv.argtypes = ctypes.c_int, [dp, vp, vp, vp, i32, sp, vp, vp]
        L.fk_select_keep.restype, L.fk_select_keep.argtypes = ctypes.c_int, [dp, vp, vp, vp, i32, i32, i32, vp, vp]
        L.fk_select_keep_workspace.restype, L.fk_select_keep_workspace.argtypes = sz, [dp, i32, i32, i32]
        L.fk_select_keep_ws.restype, L.fk_select_keep_ws.argtypes = ctypes.c_int, [dp, vp, vp, vp, i32, i32, i32, vp, vp, sz, vp]
        L.fk_select_keep_sampled.restype, L.fk_select_keep_sampled.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp]
        L.fk_compact.restype, L.fk_compact.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, vp, i32, vp]
        L.fk_decode_step_feat_workspace.restype, L.fk_decode_step_feat_workspace.argtypes = sz, [dp]
        L.fk_decode_step_feat.restype, L.fk_decode_step_feat.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, i32, i32, vp, vp, sz, vp]
        L.fk_decode_window_feat.restype, L.fk_decode_window_feat.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, f32, vp, i32, i32, vp, vp, sz, vp]
        L.fk_score_kv_feat.restype, L.fk_score_kv_feat.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, i32, sp, vp, vp]
        L.fk_compact_feat.restype, L.fk_compact_feat.argtypes = ctypes.c_int, [dp, vp, vp, vp, vp, vp, vp, i32, vp]
        L.fk_golden_steps.restype, L.fk_golden_steps.argtypes = i32, [i32, i32, i32]
        L.fk_golden_scores.restype, L.fk_golden_scores.argtypes = ctypes.c_int, [vp, i32, i32, i32, i32, ctypes.c_int64, i32, i32, vp, vp, vp]
        L.fk_golden_trace.restype, L.fk_golden_trace.argtypes = ctypes.c_int, [vp, i32, i32, i32, i32, vp, vp]
        L.fk_stream_read.restype, L.fk_stream_read.argtypes = ctypes.c_int, [vp, sz, vp, vp]
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().fk_status_string(int(code)).decode()


def version() -> str:
    return lib().fk_version().decode()


def _check(code: int, where: str) -> None:
    if code != FK_OK:
        raise FkError(code, where)


_recording = None  # while prepare() runs: the list that receives the library calls instead of the library


def _call(name: str, *cargs) -> None:
    f = getattr(lib(), name)
    if _recording is not None:
        _recording.append((f, cargs, name))
        return
    _check(f(*cargs), name)


def prepare(fn, *args, **kwargs):
    """Marshal once, call many times.  Runs the wrapper `fn(*args, **kwargs)` WITHOUT calling the library and returns a
    zero-argument callable that makes the same library call(s) with the arguments as converted now (device pointers,
    sizes, stream handle).  For loops in which Python's per-call marshalling would show in the timing.  The tensors
    must stay alive and in place for as long as the callable is used."""
    global _recording
    assert _recording is None, "prepare() does not nest"
    _recording = calls = []
    try:
        fn(*args, **kwargs)
    finally:
        _recording = None
    if len(calls) == 1:
        f, cargs, name = calls[0]

        def run_one():
            code = f(*cargs)
            if code:
                _check(code, name)
        return run_one

    def run_all():
        for f, cargs, name in calls:
            code = f(*cargs)
            if code:
                _check(code, name)
    return run_all


def _ptr(t) -> int:
    if t is None:
        return 0
    assert t.is_cuda and t.is_contiguous(), "fk buffers must be contiguous device tensors"
    return t.data_ptr()


def _stream(stream) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


@dataclass
class CacheDesc:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    capacity: int
    dtype: str  # 'f32' | 'bf16'
    cold: bool = False  # FK_CACHE_COLD: the cache is not cache resident between calls (a layer of a deep stack)

    def c(self) -> fk_cache_desc:
        return fk_cache_desc(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.capacity,
                             FK_F32 if self.dtype == "f32" else FK_BF16, 1 if self.cold else 0)

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


def fk_append(desc: CacheDesc, K, V, pos, length, k_new, v_new, pos_new, stream=None) -> None:
    _call("fk_append", ctypes.byref(desc.c()), _ptr(K), _ptr(V), _ptr(pos), _ptr(length), _ptr(k_new),
                           _ptr(v_new), _ptr(pos_new), _stream(stream))


def fk_decode_attn_workspace(desc: CacheDesc, max_len: int) -> int:
    return int(lib().fk_decode_attn_workspace(ctypes.byref(desc.c()), int(max_len)))


def new_attn_workspace(desc: CacheDesc) -> "torch.Tensor":
    """Zero-filled device workspace for fk_decode_attn / fk_decode_step (the counters must start at zero)."""
    return torch.zeros(max(fk_decode_attn_workspace(desc, desc.capacity), 16), dtype=torch.uint8, device="cuda")


def fk_decode_attn(desc: CacheDesc, q, K, V, length, max_len: int, softmax_scale: float, out, workspace,
                   stream=None) -> None:
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _call("fk_decode_attn", ctypes.byref(desc.c()), _ptr(q), _ptr(K), _ptr(V), _ptr(length), int(max_len),
                                float(softmax_scale), _ptr(out), _ptr(workspace), nbytes, _stream(stream))


def fk_decode_step(desc: CacheDesc, q, K, V, pos, length, k_new, v_new, pos_new, max_len: int, softmax_scale: float,
                   out, workspace, stream=None) -> None:
    """fk_append + fk_decode_attn in one launch; max_len bounds len[b] + 1."""
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _call("fk_decode_step", ctypes.byref(desc.c()), _ptr(q), _ptr(K), _ptr(V), _ptr(pos), _ptr(length), _ptr(k_new),
                                _ptr(v_new), _ptr(pos_new), int(max_len), float(softmax_scale), _ptr(out),
                                _ptr(workspace), nbytes, _stream(stream))


def fk_decode_step_static(desc: CacheDesc, q, K, V, pos, length, k_new, v_new, pos_new, max_len: int, softmax_scale: float,
                          out, stream=None) -> None:
    """fk_decode_step on the library's own fixed scratch: no workspace argument, nothing allocated."""
    _call("fk_decode_step_static", ctypes.byref(desc.c()), _ptr(q), _ptr(K), _ptr(V), _ptr(pos), _ptr(length), _ptr(k_new),
                                       _ptr(v_new), _ptr(pos_new), int(max_len), float(softmax_scale), _ptr(out),
                                       _stream(stream))


def fk_decode_window(desc: CacheDesc, q_seq, K, V, pos, length, k_seq, v_seq, pos_seq, n_steps: int, max_len_first: int,
                     softmax_scale: float, out_seq, workspace, stream=None) -> None:
    """n_steps consecutive decode steps enqueued by one call: step t uses q_seq[t], k_seq[t], v_seq[t], pos_seq[t]
    and writes out_seq[t]; max_len_first bounds len + 1 at the first step."""
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _call("fk_decode_window", ctypes.byref(desc.c()), _ptr(q_seq), _ptr(K), _ptr(V), _ptr(pos), _ptr(length), _ptr(k_seq),
                                  _ptr(v_seq), _ptr(pos_seq), int(n_steps), int(max_len_first), float(softmax_scale),
                                  _ptr(out_seq), _ptr(workspace), nbytes, _stream(stream))


def fk_score_kv(desc: CacheDesc, K, V, length, max_len: int, W1, b1, W2, b2, scores, stream=None, skip_len: int = 0) -> None:
    """W1 [n_sets, 2D, H] cache dtype; b1, W2 [n_sets, H] fp32; b2 [n_sets] fp32; n_sets in {1, n_kv_heads};
    rows with len <= skip_len are not scored."""
    n_sets, _, hidden = W1.shape
    sc = fk_scorer(_ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), int(hidden), 1 if n_sets == desc.n_kv_heads and n_sets > 1 else 0,
                   int(skip_len))
    _call("fk_score_kv", ctypes.byref(desc.c()), _ptr(K), _ptr(V), _ptr(length), int(max_len), ctypes.byref(sc),
                             _ptr(scores), _stream(stream))


def fk_select_keep(desc: CacheDesc, scores, pos, length, max_len: int, budget: int, protect_recent: int, keep_idx,
                   stream=None) -> None:
    _call("fk_select_keep", ctypes.byref(desc.c()), _ptr(scores), _ptr(pos), _ptr(length), int(max_len),
                                int(budget), int(protect_recent), _ptr(keep_idx), _stream(stream))


def fk_select_keep_workspace(desc: CacheDesc, max_len: int, budget: int, protect_recent: int) -> int:
    return int(lib().fk_select_keep_workspace(ctypes.byref(desc.c()), int(max_len), int(budget), int(protect_recent)))


def fk_select_keep_ws(desc: CacheDesc, scores, pos, length, max_len: int, budget: int, protect_recent: int, keep_idx,
                      workspace, stream=None) -> None:
    """fk_select_keep that may split few, long rows over several workgroups; workspace: a device byte tensor of at least
    fk_select_keep_workspace(...) bytes, or None when that is 0."""
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _call("fk_select_keep_ws", ctypes.byref(desc.c()), _ptr(scores), _ptr(pos), _ptr(length), int(max_len), int(budget),
          int(protect_recent), _ptr(keep_idx), _ptr(workspace), nbytes, _stream(stream))


def fk_select_keep_sampled(desc: CacheDesc, scores, noise, pos, length, max_len: int, budget: int, protect_recent: int,
                           n_candidates: int, keep_idx, stream=None) -> None:
    _call("fk_select_keep_sampled", ctypes.byref(desc.c()), _ptr(scores), _ptr(noise), _ptr(pos), _ptr(length),
                                        int(max_len), int(budget), int(protect_recent), int(n_candidates),
                                        _ptr(keep_idx), _stream(stream))


def fk_compact(desc: CacheDesc, K, V, pos, length, keep_idx, budget: int, stream=None) -> None:
    _call("fk_compact", ctypes.byref(desc.c()), _ptr(K), _ptr(V), _ptr(pos), _ptr(length), _ptr(keep_idx),
                            int(budget), _stream(stream))


def feat_heads(desc: CacheDesc) -> int:
    """Heads per slot in the attention-feature state (the group size padded to 4 or 8)."""
    return 4 if desc.n_q_heads // desc.n_kv_heads <= 4 else 8


def new_feat(desc: CacheDesc) -> "torch.Tensor":
    """Zero attention-feature state [batch, n_kv_heads, 6, capacity, GP] fp32."""
    return torch.zeros((desc.batch, desc.n_kv_heads, 6, desc.capacity, feat_heads(desc)), dtype=torch.float32, device="cuda")


def new_feat_workspace(desc: CacheDesc) -> "torch.Tensor":
    return torch.zeros(max(int(lib().fk_decode_step_feat_workspace(ctypes.byref(desc.c()))), 16), dtype=torch.uint8, device="cuda")


def fk_decode_step_feat(desc: CacheDesc, q, K, V, pos, length, k_new, v_new, pos_new, max_len: int, softmax_scale: float,
                        feat, chunk_pos: int, chunk_len: int, out, workspace, stream=None) -> None:
    """fk_decode_step that also accounts the step's attention weights in the feature state."""
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _call("fk_decode_step_feat", ctypes.byref(desc.c()), _ptr(q), _ptr(K), _ptr(V), _ptr(pos), _ptr(length),
                                     _ptr(k_new), _ptr(v_new), _ptr(pos_new), int(max_len), float(softmax_scale),
                                     _ptr(feat), int(chunk_pos), int(chunk_len), _ptr(out), _ptr(workspace), nbytes,
                                     _stream(stream))


def fk_decode_window_feat(desc: CacheDesc, q_seq, K, V, pos, length, k_seq, v_seq, pos_seq, n_steps: int, max_len_first: int,
                          softmax_scale: float, feat, chunk_pos_first: int, chunk_len: int, out_seq, workspace, stream=None) -> None:
    """n_steps consecutive fk_decode_step_feat calls (chunk positions chunk_pos_first ..) enqueued by one call."""
    nbytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _call("fk_decode_window_feat", ctypes.byref(desc.c()), _ptr(q_seq), _ptr(K), _ptr(V), _ptr(pos), _ptr(length), _ptr(k_seq),
          _ptr(v_seq), _ptr(pos_seq), int(n_steps), int(max_len_first), float(softmax_scale), _ptr(feat), int(chunk_pos_first),
          int(chunk_len), _ptr(out_seq), _ptr(workspace), nbytes, _stream(stream))


def fk_score_kv_feat(desc: CacheDesc, K, V, feat, length, max_len: int, W1, b1, W2, b2, scores, stream=None,
                     skip_len: int = 0) -> None:
    """fk_score_kv on concat(k, v, a); W1 [n_sets, 2D + 6g, H]."""
    n_sets, _, hidden = W1.shape
    sc = fk_scorer(_ptr(W1), _ptr(b1), _ptr(W2), _ptr(b2), int(hidden), 1 if n_sets == desc.n_kv_heads and n_sets > 1 else 0,
                   int(skip_len))
    _call("fk_score_kv_feat", ctypes.byref(desc.c()), _ptr(K), _ptr(V), _ptr(feat), _ptr(length), int(max_len),
                                  ctypes.byref(sc), _ptr(scores), _stream(stream))


def fk_compact_feat(desc: CacheDesc, K, V, pos, feat, length, keep_idx, budget: int, stream=None) -> None:
    _call("fk_compact_feat", ctypes.byref(desc.c()), _ptr(K), _ptr(V), _ptr(pos), _ptr(feat), _ptr(length),
                                 _ptr(keep_idx), int(budget), _stream(stream))


def fk_golden_steps(T: int, budget: int, interval: int) -> int:
    return int(lib().fk_golden_steps(int(T), int(budget), int(interval)))


def fk_golden_scores(A, n_kv_heads: int, T: int, budget: int, interval: int, block_scores, alpha, stream=None) -> None:
    """A [n_q_heads, T, ld] fp32 or bf16 (ld = A.shape[2] >= T); block_scores, alpha [n_kv_heads, M, T] fp32."""
    _call("fk_golden_scores", _ptr(A), FK_F32 if A.dtype == torch.float32 else FK_BF16, int(A.shape[0]), int(n_kv_heads),
                                  int(T), int(A.shape[2]), int(budget), int(interval), _ptr(block_scores), _ptr(alpha),
                                  _stream(stream))


def fk_golden_trace(alpha, T: int, budget: int, interval: int, kept, stream=None) -> None:
    """alpha [n_kv_heads, M, T] fp32; kept [n_kv_heads, M, budget] int32."""
    _call("fk_golden_trace", _ptr(alpha), int(alpha.shape[0]), int(T), int(budget), int(interval), _ptr(kept),
                                 _stream(stream))


def fk_stream_read(src, sink, stream=None) -> None:
    """Measurement helper: stream-read the whole tensor `src` once (sink: >= 4 bytes of device memory)."""
    _call("fk_stream_read", _ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream(stream))
