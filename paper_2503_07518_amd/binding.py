"""ctypes binding of libtokenbutler.so: argument marshalling only.

Every function has the name of the C entry point it calls (``include/tokenbutler.h``) and
passes device pointers of torch tensors plus the current HIP stream.  No step of the path is
computed here; if the HIP library is missing or does not load, importing the ops fails loudly
(there is no fallback).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtokenbutler.so")

TB_OK, TB_ERR_INVALID_ARG, TB_ERR_UNSUPPORTED, TB_ERR_WORKSPACE, TB_ERR_HIP = 0, 1, 2, 3, 4
TB_F32, TB_BF16 = 0, 1
TB_OP_SELECT, TB_OP_ATTN, TB_OP_DECODE_STEP = 1, 2, 3

EXPORTS = (
    "tb_project_keys", "tb_score", "tb_select_topk", "tb_expand_neighbors", "tb_sparse_decode_attn",
    "tb_sparse_decode_attn_shared", "tb_sparse_decode_attn_static",
    "tb_gather_kv", "tb_gather_important", "tb_buffered_decode_attn", "tb_predict_queries", "tb_decode_step", "tb_workspace_bytes", "tb_workspace_init", "tb_read_stream_probe", "tb_status_string", "tb_version",
)


class TbError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {status_string(code)} (tb_status {code})")


class tb_cache_desc(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("Dimp", ctypes.c_int32), ("dtype", ctypes.c_int32), ("N", ctypes.c_int64),
        ("k_stride_b", ctypes.c_int64), ("k_stride_h", ctypes.c_int64), ("k_stride_n", ctypes.c_int64),
        ("v_stride_b", ctypes.c_int64), ("v_stride_h", ctypes.c_int64), ("v_stride_n", ctypes.c_int64),
        ("ki_stride_b", ctypes.c_int64), ("ki_stride_h", ctypes.c_int64), ("ki_stride_n", ctypes.c_int64),
    ]


class tb_predictor_desc(ctypes.Structure):
    _fields_ = [
        ("E", ctypes.c_int32), ("hidden", ctypes.c_int32), ("G", ctypes.c_int32), ("Hq", ctypes.c_int32),
        ("Dimp", ctypes.c_int32), ("dtype", ctypes.c_int32), ("ln_eps", ctypes.c_float),
    ]


_lib: Optional[ctypes.CDLL] = None


def load_library() -> ctypes.CDLL:
    """Load libtokenbutler.so from the package directory.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2503_07518_amd.build` "
            "(hipcc, --offload-arch=gfx950).  There is no fallback implementation.")
    L = ctypes.CDLL(LIB_PATH)
    i32, i64, f32, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
    dp = ctypes.POINTER(tb_cache_desc)
    L.tb_project_keys.argtypes = [dp, vp, vp, i32, vp, i64, i64, vp]
    L.tb_score.argtypes = [dp, vp, vp, f32, vp, i64, vp]
    L.tb_select_topk.argtypes = [dp, vp, i64, i32, i32, i32, vp, vp, i64, vp, sz, vp]
    L.tb_expand_neighbors.argtypes = [i32, i32, i64, i32, i32, vp, vp, i64, vp, vp, i64, vp]
    L.tb_sparse_decode_attn.argtypes = [dp, vp, vp, vp, vp, vp, i64, i64, i64, i64, f32, vp, vp, vp, sz, vp]
    L.tb_sparse_decode_attn_shared.argtypes = L.tb_sparse_decode_attn.argtypes
    L.tb_sparse_decode_attn_static.argtypes = [dp, vp, vp, vp, vp, vp, i64, i64, i64, i64, f32, vp, vp, vp]
    L.tb_decode_step.argtypes = [dp, vp, vp, f32, vp, vp, vp, i32, i32, i32, f32, vp, i64, vp, vp, i64, vp, vp,
                                 vp, sz, vp]
    L.tb_gather_kv.argtypes = [dp, vp, vp, vp, vp, i64, i64, vp, vp, i64, vp]
    L.tb_gather_important.argtypes = [dp, vp, vp, vp, vp, i64, i64, i32, i32, vp, vp, i64, vp, vp]
    L.tb_buffered_decode_attn.argtypes = [dp, vp, vp, vp, i64, vp, i64, vp, vp, i64, i64, f32, vp, vp, vp, sz, vp]
    L.tb_predict_queries.argtypes = [ctypes.POINTER(tb_predictor_desc), i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.tb_workspace_bytes.argtypes = [i32, dp, i64]
    L.tb_workspace_bytes.restype = sz
    L.tb_workspace_init.argtypes = [vp, sz, vp]
    L.tb_read_stream_probe.argtypes = [vp, sz, vp, vp]
    L.tb_status_string.argtypes = [ctypes.c_int]
    L.tb_status_string.restype = ctypes.c_char_p
    L.tb_version.restype = i32
    for name in EXPORTS:
        if name not in ("tb_workspace_bytes", "tb_status_string", "tb_version"):
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def status_string(code: int) -> str:
    return load_library().tb_status_string(int(code)).decode()


def _check(code: int, what: str) -> None:
    if code != TB_OK:
        raise TbError(code, what)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return TB_F32
    if t.dtype == torch.bfloat16:
        return TB_BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def _strides3(t: Optional[torch.Tensor], inner: int) -> Tuple[int, int, int]:
    if t is None:
        return (0, 0, inner)
    assert t.dim() == 4 and t.stride(3) == 1, "cache tensors are [B, Hkv, N, D] with D contiguous"
    return (t.stride(0), t.stride(1), t.stride(2))


def make_desc(N: int, Hq: int, K: Optional[torch.Tensor] = None, V: Optional[torch.Tensor] = None,
              Kimp: Optional[torch.Tensor] = None, D: Optional[int] = None, Dimp: Optional[int] = None) -> tb_cache_desc:
    """Describe one layer's cache from the tensors at hand.  Missing tensors get neutral
    strides; D / Dimp may be given explicitly when the tensor that carries them is absent."""
    ref = K if K is not None else (Kimp if Kimp is not None else V)
    assert ref is not None
    B, Hkv = ref.shape[0], ref.shape[1]
    D = D if D is not None else (K.shape[3] if K is not None else (V.shape[3] if V is not None else 128))
    Dimp = Dimp if Dimp is not None else (Kimp.shape[3] if Kimp is not None else 32)
    d = tb_cache_desc()
    d.B, d.Hq, d.Hkv, d.D, d.Dimp, d.dtype, d.N = B, Hq, Hkv, D, Dimp, _dtype_code(ref), N
    d.k_stride_b, d.k_stride_h, d.k_stride_n = _strides3(K, D)
    d.v_stride_b, d.v_stride_h, d.v_stride_n = _strides3(V if V is not None else K, D)
    d.ki_stride_b, d.ki_stride_h, d.ki_stride_n = _strides3(Kimp, Dimp)
    return d


def tb_version() -> int:
    return int(load_library().tb_version())


def tb_workspace_bytes(op: int, desc: tb_cache_desc, max_count: int = 0) -> int:
    return int(load_library().tb_workspace_bytes(op, ctypes.byref(desc), int(max_count)))


def tb_workspace_init(ws: torch.Tensor, stream=None) -> None:
    _check(load_library().tb_workspace_init(_ptr(ws), ws.numel() * ws.element_size(), _stream(stream)),
           "tb_workspace_init")


def tb_read_stream_probe(src: torch.Tensor, sink: torch.Tensor, stream=None) -> None:
    """Read `src` once with a plain streaming kernel (a bandwidth calibration, see the header)."""
    _check(load_library().tb_read_stream_probe(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                               _stream(stream)), "tb_read_stream_probe")


def new_workspace(op: int, desc: tb_cache_desc, max_count: int = 0, device="cuda") -> torch.Tensor:
    """Allocate (torch, device memory) and zero a workspace for `op`."""
    nbytes = tb_workspace_bytes(op, desc, max_count)
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    tb_workspace_init(ws)
    return ws


def tb_project_keys(desc, K, W, Kimp, n_begin: int, n_end: int, stream=None) -> None:
    Hw = W.shape[0]
    assert W.is_contiguous()
    _check(load_library().tb_project_keys(ctypes.byref(desc), _ptr(K), _ptr(W), Hw, _ptr(Kimp), n_begin, n_end,
                                          _stream(stream)), "tb_project_keys")


def tb_score(desc, q_imp, Kimp, scale: float, scores, stream=None) -> None:
    assert q_imp.is_contiguous() and scores.stride(-1) == 1
    _check(load_library().tb_score(ctypes.byref(desc), _ptr(q_imp), _ptr(Kimp), scale, _ptr(scores),
                                   scores.stride(-2), _stream(stream)), "tb_score")


def tb_select_topk(desc, scores, k: int, sink: int, window: int, idx, count, ws, stream=None) -> None:
    _check(load_library().tb_select_topk(ctypes.byref(desc), _ptr(scores), scores.stride(-2), k, sink, window,
                                         _ptr(idx), _ptr(count), idx.stride(-2), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)), "tb_select_topk")


def tb_gather_kv(desc, K, V, idx, count, max_count: int, Kbuf, Vbuf, stream=None) -> None:
    assert Kbuf.is_contiguous() and Vbuf.is_contiguous() and Kbuf.shape == Vbuf.shape
    _check(load_library().tb_gather_kv(ctypes.byref(desc), _ptr(K), _ptr(V), _ptr(idx), _ptr(count), idx.stride(-2),
                                       max_count, _ptr(Kbuf), _ptr(Vbuf), Kbuf.shape[2], _stream(stream)),
           "tb_gather_kv")


def tb_gather_important(desc, K, V, idx, count, max_count: int, skip_front: int, skip_back: int, Kbuf, Vbuf,
                        count_out, stream=None) -> None:
    assert Kbuf.is_contiguous() and Vbuf.is_contiguous() and Kbuf.shape == Vbuf.shape
    _check(load_library().tb_gather_important(ctypes.byref(desc), _ptr(K), _ptr(V), _ptr(idx), _ptr(count),
                                              idx.stride(-2), max_count, skip_front, skip_back, _ptr(Kbuf), _ptr(Vbuf),
                                              Kbuf.shape[2], _ptr(count_out), _stream(stream)), "tb_gather_important")


def tb_buffered_decode_attn(desc, q, Kbuf, Vbuf, count, max_count: int, K, V, sm_scale: float, out, lse, ws,
                            tail_begin: int = 0, tail_end: int = 0, stream=None) -> None:
    assert Kbuf.is_contiguous() and Vbuf.is_contiguous() and Kbuf.shape == Vbuf.shape
    _check(load_library().tb_buffered_decode_attn(ctypes.byref(desc), _ptr(q), _ptr(Kbuf), _ptr(Vbuf), Kbuf.shape[2],
                                                  _ptr(count), max_count, _ptr(K), _ptr(V), tail_begin, tail_end,
                                                  sm_scale, _ptr(out), _ptr(lse), _ptr(ws),
                                                  ws.numel() * ws.element_size(), _stream(stream)),
           "tb_buffered_decode_attn")


def tb_predict_queries(h, gamma, beta, W1, b1, W2, b2, G: int, Hq: int, Dimp: int, hidden_act, ln_act, q_imp,
                       ln_eps: float = 1e-5, stream=None) -> None:
    """q_imp[G][B][Hq][Dimp] = MLP(LN(h)); W1 [hidden][E], W2 [G*Hq*Dimp][hidden] (torch Linear layout)."""
    B, E = h.shape
    hidden = W1.shape[0]
    for t in (h, gamma, beta, W1, b1, W2, b2, hidden_act, ln_act, q_imp):
        assert t.is_contiguous()
    assert W1.shape == (hidden, E) and W2.shape == (G * Hq * Dimp, hidden)
    assert hidden_act.dtype == torch.float32 and hidden_act.shape == (B, hidden)
    assert ln_act.dtype == torch.float32 and ln_act.shape == (B, E)
    assert q_imp.shape == (G, B, Hq, Dimp) and q_imp.dtype == h.dtype
    p = tb_predictor_desc(E, hidden, G, Hq, Dimp, _dtype_code(h), ln_eps)
    _check(load_library().tb_predict_queries(ctypes.byref(p), B, _ptr(h), _ptr(gamma), _ptr(beta), _ptr(W1), _ptr(b1),
                                             _ptr(W2), _ptr(b2), _ptr(hidden_act), _ptr(ln_act), _ptr(q_imp), _stream(stream)),
           "tb_predict_queries")


def tb_expand_neighbors(B: int, Hq: int, N: int, radius: int, mode: int, idx_in, count_in, idx_out, count_out,
                        stream=None) -> None:
    _check(load_library().tb_expand_neighbors(B, Hq, N, radius, mode, _ptr(idx_in), _ptr(count_in),
                                              idx_in.stride(-2), _ptr(idx_out), _ptr(count_out), idx_out.stride(-2),
                                              _stream(stream)), "tb_expand_neighbors")


def tb_sparse_decode_attn(desc, q, K, V, idx, count, max_count: int, sm_scale: float, out, lse, ws,
                          tail_begin: int = 0, tail_end: int = 0, stream=None) -> None:
    assert q.is_contiguous() and out.is_contiguous()
    _check(load_library().tb_sparse_decode_attn(ctypes.byref(desc), _ptr(q), _ptr(K), _ptr(V), _ptr(idx),
                                                _ptr(count), idx.stride(-2), max_count, tail_begin, tail_end,
                                                sm_scale, _ptr(out), _ptr(lse), _ptr(ws),
                                                ws.numel() * ws.element_size(), _stream(stream)),
           "tb_sparse_decode_attn")


def tb_sparse_decode_attn_static(desc, q, K, V, idx, count, max_count: int, sm_scale: float, out, lse,
                                 tail_begin: int = 0, tail_end: int = 0, stream=None) -> None:
    """tb_sparse_decode_attn with the library's own scratch (no workspace, no allocation)."""
    assert q.is_contiguous() and out.is_contiguous()
    _check(load_library().tb_sparse_decode_attn_static(ctypes.byref(desc), _ptr(q), _ptr(K), _ptr(V), _ptr(idx),
                                                       _ptr(count), idx.stride(-2), max_count, tail_begin,
                                                       tail_end, sm_scale, _ptr(out), _ptr(lse), _stream(stream)),
           "tb_sparse_decode_attn_static")


def tb_sparse_decode_attn_shared(desc, q, K, V, idx, count, max_count: int, sm_scale: float, out, lse, ws,
                                 tail_begin: int = 0, tail_end: int = 0, stream=None) -> None:
    """idx: int32 [B][idx_cap] (or [B][1][idx_cap]), count: int32 [B]; one list for all heads."""
    assert q.is_contiguous() and out.is_contiguous()
    _check(load_library().tb_sparse_decode_attn_shared(ctypes.byref(desc), _ptr(q), _ptr(K), _ptr(V), _ptr(idx),
                                                       _ptr(count), idx.stride(-2), max_count, tail_begin,
                                                       tail_end, sm_scale, _ptr(out), _ptr(lse), _ptr(ws),
                                                       ws.numel() * ws.element_size(), _stream(stream)),
           "tb_sparse_decode_attn_shared")


def tb_decode_step(desc, q_imp, Kimp, score_scale: float, q, K, V, k: int, sink: int, window: int, sm_scale: float,
                   scores, idx, count, out, lse, ws, stream=None) -> None:
    assert q.is_contiguous() and q_imp.is_contiguous() and out.is_contiguous()
    _check(load_library().tb_decode_step(ctypes.byref(desc), _ptr(q_imp), _ptr(Kimp), score_scale, _ptr(q), _ptr(K),
                                         _ptr(V), k, sink, window, sm_scale, _ptr(scores), scores.stride(-2),
                                         _ptr(idx), _ptr(count), idx.stride(-2), _ptr(out), _ptr(lse), _ptr(ws),
                                         ws.numel() * ws.element_size(), _stream(stream)), "tb_decode_step")


def policy_count(N: int, k: int, sink: int, window: int) -> int:
    """Length of the list the selection policy emits (host-side sizing helper)."""
    lo = min(sink, N)
    hi = max(lo, N - window)
    return lo + min(k, hi - lo) + (N - hi)
