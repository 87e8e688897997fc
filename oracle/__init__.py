"""Plain CPU oracle for the TokenButler decode hot path.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The product package never imports this module and this
module never imports the product package.

The arithmetic lives in ``tb_oracle.c`` (plain C, fp64 accumulation); this file only marshals
numpy arrays into it and holds the prediction-interval driver, which is orchestration of the
C steps in the order Sec. 3.4 gives them.

bf16 tensors are passed as ``uint16`` numpy arrays together with ``dtype="bf16"``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tb_oracle.c")
_LIB = os.path.join(_HERE, "libtb_oracle.so")

F32, BF16 = 0, 1
_DT = {"f32": F32, "fp32": F32, "float32": F32, "bf16": BF16, "bfloat16": BF16, 0: F32, 1: BF16}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i32, i64, dbl, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        L.tbo_num_threads.restype = ctypes.c_int
        L.tbo_set_num_threads.argtypes = [ctypes.c_int]
        L.tbo_round_bf16.restype = ctypes.c_uint16
        L.tbo_round_bf16.argtypes = [dbl]
        L.tbo_project_keys.argtypes = [i32, i32, i32, i64, i32, i32, i32, vp, vp, i64, i64, vp]
        L.tbo_score.argtypes = [i32, i32, i32, i32, i64, i32, vp, vp, dbl, vp]
        L.tbo_select_topk.argtypes = [i64, i64, vp, i64, i32, i32, i32, vp, vp, i64]
        L.tbo_select_topk_bruteforce.argtypes = [i64, vp, i32, i32, i32, vp, vp, i64]
        L.tbo_expand_neighbors.argtypes = [i64, i64, i32, vp, vp, i64, vp, vp, i64]
        L.tbo_expand_neighbors_cluster.argtypes = [i64, i64, vp, vp, i64, vp, vp, i64]
        L.tbo_sparse_decode_attn.argtypes = [i32, i32, i32, i32, i64, i32, vp, vp, vp, vp, vp, i64, dbl, vp, vp]
        L.tbo_dense_decode_attn.argtypes = [i32, i32, i32, i32, i64, i32, vp, vp, vp, dbl, vp]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().tbo_num_threads())


def set_num_threads(n: int) -> None:
    lib().tbo_set_num_threads(int(n))


def _elt(dtype) -> np.dtype:
    return np.dtype(np.float32) if _DT[dtype] == F32 else np.dtype(np.uint16)


def _arr(a, dtype, shape=None) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def to_numpy(t):
    """torch CPU/GPU tensor (fp32, bf16, int32) -> contiguous numpy array; bf16 as uint16."""
    import torch  # local: the oracle itself does not need torch

    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def round_bf16(x: float) -> int:
    return int(lib().tbo_round_bf16(float(x)))


def bf16_to_f64(a: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64 values (exact)."""
    return (np.asarray(a, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def project_keys(K, W, dtype, n_begin: int = 0, n_end: Optional[int] = None, out=None) -> np.ndarray:
    """Sec. 3.1 key-cache projection.  K [B,Hkv,N,D], W [Hw,D,Dimp] -> Kimp [B,Hkv,N,Dimp]."""
    et = _elt(dtype)
    K = _arr(K, et)
    W = _arr(W, et)
    B, Hkv, N, D = K.shape
    Hw, D2, Dimp = W.shape
    assert D2 == D
    n_end = N if n_end is None else n_end
    if out is None:
        out = np.zeros((B, Hkv, N, Dimp), dtype=et)
    assert out.flags.c_contiguous and out.shape == (B, Hkv, N, Dimp) and out.dtype == et
    _check(lib().tbo_project_keys(_DT[dtype], B, Hkv, N, D, Dimp, Hw, _p(K), _p(W), n_begin, n_end, _p(out)),
           "project_keys")
    return out


def score(q_imp, Kimp, dtype, scale: float = 1.0) -> np.ndarray:
    """Importance scores.  q_imp [B,Hq,Dimp], Kimp [B,Hkv,N,Dimp] -> fp32 [B,Hq,N]."""
    et = _elt(dtype)
    q_imp = _arr(q_imp, et)
    Kimp = _arr(Kimp, et)
    B, Hq, Dimp = q_imp.shape
    B2, Hkv, N, Dimp2 = Kimp.shape
    assert B2 == B and Dimp2 == Dimp
    out = np.empty((B, Hq, N), dtype=np.float32)
    _check(lib().tbo_score(_DT[dtype], B, Hq, Hkv, N, Dimp, _p(q_imp), _p(Kimp), float(scale), _p(out)), "score")
    return out


def select_topk(scores, k: int, sink: int = 0, window: int = 0, N: Optional[int] = None,
                cap: Optional[int] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Selection policy of Sec. 4.  scores fp32 [..., >=N] -> (idx int32 [..., cap], count int32 [...])."""
    scores = _arr(scores, np.float32)
    lead = scores.shape[:-1]
    stride = scores.shape[-1]
    N = stride if N is None else N
    assert N <= stride
    U = int(np.prod(lead)) if lead else 1
    lo = min(sink, N)
    hi = max(lo, N - window)
    need = lo + min(k, hi - lo) + (N - hi)
    cap = need if cap is None else cap
    idx = np.full(lead + (max(cap, 1),), -1, dtype=np.int32)
    count = np.zeros(lead, dtype=np.int32)
    _check(lib().tbo_select_topk(U, N, _p(scores), stride, k, sink, window, _p(idx), _p(count), idx.shape[-1]),
           "select_topk")
    return idx, count


def select_topk_bruteforce(scores_1d, k: int, sink: int = 0, window: int = 0) -> np.ndarray:
    s = _arr(scores_1d, np.float32)
    assert s.ndim == 1
    N = s.shape[0]
    idx = np.full((max(N, 1),), -1, dtype=np.int32)
    cnt = np.zeros((1,), dtype=np.int32)
    _check(lib().tbo_select_topk_bruteforce(N, _p(s), k, sink, window, _p(idx), _p(cnt), idx.shape[0]),
           "select_topk_bruteforce")
    return idx[: int(cnt[0])].copy()


def expand_neighbors(idx, count, N: int, radius: int, cap_out: Optional[int] = None,
                     mode: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Neighbour fetching (Sec. 3.4).  mode 0: union of [i-r, i+r]; mode 1: cluster-aware."""
    idx = _arr(idx, np.int32)
    count = _arr(count, np.int32, idx.shape[:-1])
    lead = idx.shape[:-1]
    U = int(np.prod(lead)) if lead else 1
    cap_in = idx.shape[-1]
    mult = (2 * radius + 1) if mode == 0 else 2
    if cap_out is None:
        cap_out = max(1, min(N, mult * int(count.max()) if count.size else 1))
    out = np.full(lead + (cap_out,), -1, dtype=np.int32)
    cnt = np.zeros(lead, dtype=np.int32)
    if mode == 0:
        rc = lib().tbo_expand_neighbors(U, N, radius, _p(idx), _p(count), cap_in, _p(out), _p(cnt), cap_out)
    else:
        rc = lib().tbo_expand_neighbors_cluster(U, N, _p(idx), _p(count), cap_in, _p(out), _p(cnt), cap_out)
    _check(rc, "expand_neighbors")
    return out, cnt


def sparse_decode_attn(q, K, V, idx, count, dtype, sm_scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Attention over the selected rows.  q [B,Hq,D]; K,V [B,Hkv,N,D]; idx [B,Hq,cap]; count [B,Hq]."""
    et = _elt(dtype)
    q = _arr(q, et)
    K = _arr(K, et)
    V = _arr(V, et, K.shape)
    B, Hq, D = q.shape
    _, Hkv, N, _ = K.shape
    idx = _arr(idx, np.int32)
    count = _arr(count, np.int32, (B, Hq))
    assert idx.shape[:2] == (B, Hq)
    out = np.empty((B, Hq, D), dtype=np.float32)
    lse = np.empty((B, Hq), dtype=np.float32)
    _check(lib().tbo_sparse_decode_attn(_DT[dtype], B, Hq, Hkv, N, D, _p(q), _p(K), _p(V), _p(idx), _p(count),
                                         idx.shape[-1], float(sm_scale), _p(out), _p(lse)), "sparse_decode_attn")
    return out, lse


def sparse_decode_attn_shared(q, K, V, idx, count, dtype, sm_scale: float) -> Tuple[np.ndarray, np.ndarray]:
    """Head-less selection (Appendix "Additional Efficiency Evaluation": one importance per token
    per layer): the single list idx [B,cap], count [B] is what every head of the batch element
    attends over.  By definition this is sparse_decode_attn with the list repeated for each head."""
    B, Hq, _ = np.asarray(q).shape
    idx = _arr(idx, np.int32).reshape(B, 1, -1)
    count = _arr(count, np.int32).reshape(B, 1)
    return sparse_decode_attn(q, K, V, np.repeat(idx, Hq, axis=1), np.repeat(count, Hq, axis=1), dtype, sm_scale)


def predict_queries(h, gamma, beta, W1, b1, W2, b2, G: int, Hq: int, Dimp: int, dtype, ln_eps: float = 1e-5):
    """Query prediction of a producer layer (Sec. 3.1 "Query prediction"): LayerNorm over the
    model dimension, then a two-layer MLP (exact-erf GELU; the paper does not name the
    nonlinearity), all in fp64, one rounding to the storage type at the end.
    h [B,E]; W1 [hidden,E]; W2 [G*Hq*Dimp,hidden].  Returns (q_imp [G,B,Hq,Dimp], z [B,hidden] fp64)."""
    import math

    def f64(a):
        a = np.asarray(a)
        return bf16_to_f64(a) if dtype == "bf16" else a.astype(np.float64)

    h, gamma, beta, W1, b1, W2, b2 = (f64(a) for a in (h, gamma, beta, W1, b1, W2, b2))
    B, E = h.shape
    mean = h.sum(axis=1, keepdims=True) / E
    var = ((h - mean) ** 2).sum(axis=1, keepdims=True) / E
    x = (h - mean) / np.sqrt(var + ln_eps) * gamma + beta
    pre = x @ W1.T + b1
    z = 0.5 * pre * (1.0 + np.vectorize(math.erf)(pre / math.sqrt(2.0)))
    y = z @ W2.T + b2  # [B, G*Hq*Dimp], output row (slot, head, j) with the slot outermost
    y = y.reshape(B, G, Hq, Dimp).transpose(1, 0, 2, 3)
    if dtype == "bf16":
        q = np.vectorize(round_bf16, otypes=[np.uint16])(y)
    else:
        q = y.astype(np.float32)
    return np.ascontiguousarray(q), z


def gather_kv(K, V, idx, count, buf_cap: int) -> Tuple[np.ndarray, np.ndarray]:
    """Migration of selected rows into per-query-head buffers (Sec. 3.3, the Important Buffer):
    buf[b,h,i,:] = cache[b, h // g, idx[b,h,i], :] for i < count[b,h]; the rest stays zero.
    Written out as the definition, one (b, h) at a time."""
    B, Hkv, N, D = K.shape
    idx = np.asarray(idx)
    count = np.asarray(count)
    Hq = idx.shape[1]
    g = Hq // Hkv
    Kbuf = np.zeros((B, Hq, buf_cap, D), dtype=K.dtype)
    Vbuf = np.zeros((B, Hq, buf_cap, D), dtype=V.dtype)
    for b in range(B):
        for h in range(Hq):
            c = int(count[b, h])
            rows = idx[b, h, :c].astype(np.int64)
            Kbuf[b, h, :c] = K[b, h // g, rows]
            Vbuf[b, h, :c] = V[b, h // g, rows]
    return Kbuf, Vbuf


def dense_decode_attn(q, K, V, dtype, sm_scale: float) -> np.ndarray:
    et = _elt(dtype)
    q = _arr(q, et)
    K = _arr(K, et)
    V = _arr(V, et, K.shape)
    B, Hq, D = q.shape
    _, Hkv, N, _ = K.shape
    out = np.empty((B, Hq, D), dtype=np.float32)
    _check(lib().tbo_dense_decode_attn(_DT[dtype], B, Hq, Hkv, N, D, _p(q), _p(K), _p(V), float(sm_scale), _p(out)),
           "dense_decode_attn")
    return out


def decode_step(q, q_imp, K, V, Kimp, dtype, k: int, sink: int, window: int, sm_scale: float,
                scale: float = 1.0):
    """One prediction step: score -> select -> attend (Sec. 3.4, "prediction steps")."""
    s = score(q_imp, Kimp, dtype, scale)
    idx, cnt = select_topk(s, k, sink, window)
    out, lse = sparse_decode_attn(q, K, V, idx, cnt, dtype, sm_scale)
    return s, idx, cnt, out, lse


class IntervalDriver:
    """Prediction interval with neighbour fetching (Sec. 3.4).

    Step t sees the first ``N0 + t`` tokens of the cache.  If ``t % P == 0`` the importance
    scores and the selection are recomputed and attention runs on the selected set; the
    selection widened by ``radius`` neighbours is stored.  On the other steps attention runs
    on the stored widened set plus every token appended since the last prediction (the local
    window is refreshed every step).
    """

    def __init__(self, dtype, k: int, P: int, radius: int, sink: int = 0, window: int = 0,
                 sm_scale: float = 1.0, scale: float = 1.0, expand_on_predict: bool = False, mode: int = 0,
                 headless: bool = False, ring: int = 0):
        self.dtype, self.k, self.P, self.radius = dtype, k, P, radius
        self.sink, self.window, self.sm_scale, self.scale = sink, window, sm_scale, scale
        self.expand_on_predict, self.mode = expand_on_predict, mode
        # head-less variant (Appendix "Additional Efficiency Evaluation"): q_imp [B,1,d'], Kimp
        # [B,1,N,d']; one list per batch element, attended by every head
        self.headless = headless
        # ring > 0: the three-buffer layout of Sec. 3.3 "Inference Setup" with a Local Window
        # Buffer of `ring` tokens (replaces `window`).  Starting from the post-prefill state the
        # window fills over the first `ring` steps, so at step t it holds the W_t = min(ring, t)
        # newest tokens; those are attended on EVERY step without a score and are no candidates.
        # A prediction step selects among [sink, N_t - W_t), widens the list and attends over the
        # widened list (the Important Buffer holds the widened selection); the other steps attend
        # over the stored widened list WITHOUT the window rows of the prediction step, followed by
        # the window as it is now -- rows that have left the window since the prediction and were
        # not selected are not attended until the next prediction.
        self.ring = ring
        assert ring == 0 or (ring >= P and window == 0), "the window must cover a prediction interval"
        self.N0 = None
        self.W_pred = 0
        self.N_pred = None
        self.exp_idx = None
        self.exp_cnt = None

    def lists(self, t: int, N_t: int, q_imp, Kimp):
        """The token lists that step t attends over: (idx, count).  On a prediction step the
        scores and the selection are made (and the widened selection is stored); on the other
        steps the stored widened list is followed by the tokens appended since the prediction."""
        if self.N0 is None:
            self.N0 = N_t - t
        W_t = min(self.ring, N_t - self.N0) if self.ring else self.window
        if t % self.P == 0:
            s = score(q_imp, np.ascontiguousarray(Kimp[:, :, :N_t]), self.dtype, self.scale)
            sel, cnt = select_topk(s, self.k, self.sink, W_t)
            self.N_pred, self.W_pred = N_t, W_t
            self.exp_idx, self.exp_cnt = expand_neighbors(sel, cnt, N_t, self.radius, mode=self.mode)
            return (self.exp_idx, self.exp_cnt) if (self.expand_on_predict or self.ring) else (sel, cnt)
        B, Hq = self.exp_cnt.shape
        if self.ring:
            # widened list minus its last W_pred entries (the window rows of the prediction step:
            # the largest positions of the list), then the window of this step
            drop, tail = self.W_pred, np.arange(N_t - W_t, N_t, dtype=np.int32)
        else:
            drop, tail = 0, np.arange(self.N_pred, N_t, dtype=np.int32)
        extra = len(tail)
        cap = self.exp_idx.shape[-1] + extra
        use_idx = np.full((B, Hq, cap), -1, dtype=np.int32)
        use_cnt = self.exp_cnt - drop + extra
        for b in range(B):
            for h in range(Hq):
                c = int(self.exp_cnt[b, h]) - drop
                use_idx[b, h, :c] = self.exp_idx[b, h, :c]
                use_idx[b, h, c:c + extra] = tail
        return use_idx, use_cnt

    def step(self, t: int, N_t: int, q, q_imp, K, V, Kimp):
        """K, V, Kimp hold at least N_t rows; only the first N_t are visible.  Returns
        (out, lse, idx_used, count_used)."""
        use_idx, use_cnt = self.lists(t, N_t, q_imp, Kimp)
        Kt = np.ascontiguousarray(K[:, :, :N_t])
        Vt = np.ascontiguousarray(V[:, :, :N_t])
        if self.headless:
            out, lse = sparse_decode_attn_shared(q, Kt, Vt, use_idx[:, 0], use_cnt[:, 0], self.dtype, self.sm_scale)
        else:
            out, lse = sparse_decode_attn(q, Kt, Vt, use_idx, use_cnt, self.dtype, self.sm_scale)
        return out, lse, use_idx, use_cnt
