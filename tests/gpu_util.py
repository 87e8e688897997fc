"""Helpers for the GPU parity tests: thin wrappers that allocate outputs with torch, call the
C ABI through the binding and hand results to the oracle as numpy arrays."""
from __future__ import annotations

import numpy as np
import torch

from paper_2503_07518_amd import binding as tb

DEV = "cuda"


def np_of(t: torch.Tensor) -> np.ndarray:
    """Device/host tensor -> contiguous numpy; bf16 as uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def dtype_name(t: torch.Tensor) -> str:
    return "f32" if t.dtype == torch.float32 else "bf16"


def gpu_project(K, W, N, n_begin=0, n_end=None, Kimp=None):
    B, Hkv, Ncap, D = K.shape
    Dimp = W.shape[2]
    if Kimp is None:
        Kimp = torch.zeros((B, Hkv, Ncap, Dimp), dtype=K.dtype, device=K.device)
    d = tb.make_desc(N, Hkv, K=K, Kimp=Kimp)
    tb.tb_project_keys(d, K, W, Kimp, n_begin, N if n_end is None else n_end)
    return Kimp


def gpu_score(q_imp, Kimp, N, scale=1.0, stride=None):
    B, Hq, _ = q_imp.shape
    stride = stride or (N + 3) // 4 * 4
    scores = torch.full((B, Hq, max(stride, 4)), float("nan"), dtype=torch.float32, device=q_imp.device)
    d = tb.make_desc(N, Hq, Kimp=Kimp)
    tb.tb_score(d, q_imp, Kimp, scale, scores)
    return scores


def gpu_select(scores, N, k, sink=0, window=0, cap=None, ws=None, Hkv=None):
    B, Hq, _ = scores.shape
    need = tb.policy_count(N, k, sink, window)
    cap = need if cap is None else cap
    idx = torch.full((B, Hq, max(cap, 1)), -7, dtype=torch.int32, device=scores.device)
    cnt = torch.full((B, Hq), -7, dtype=torch.int32, device=scores.device)
    d = tb.tb_cache_desc()
    d.B, d.Hq, d.Hkv, d.D, d.Dimp, d.dtype, d.N = B, Hq, Hkv or Hq, 128, 32, tb.TB_F32, N
    d.k_stride_n = d.v_stride_n = 128
    d.ki_stride_n = 32
    if ws is None:
        ws = tb.new_workspace(tb.TB_OP_SELECT, d, need)  # long rows on few heads: two-stage selection
    tb.tb_select_topk(d, scores, k, sink, window, idx, cnt, ws)
    return idx, cnt


def gpu_expand(idx, cnt, N, radius, mode=0, cap_out=None):
    B, Hq, cap_in = idx.shape
    mult = 2 * radius + 1 if mode == 0 else 2
    cap_out = cap_out or max(1, min(N, mult * cap_in))
    out = torch.full((B, Hq, cap_out), -7, dtype=torch.int32, device=idx.device)
    oc = torch.full((B, Hq), -7, dtype=torch.int32, device=idx.device)
    tb.tb_expand_neighbors(B, Hq, N, radius, mode, idx, cnt, out, oc)
    return out, oc


def gpu_attn(q, K, V, idx, cnt, N, sm_scale, max_count=None, tail=(0, 0), ws=None):
    B, Hq, D = q.shape
    d = tb.make_desc(N, Hq, K=K, V=V)
    max_count = idx.shape[2] if max_count is None else max_count
    if ws is None:
        ws = tb.new_workspace(tb.TB_OP_ATTN, d, max_count + tail[1] - tail[0])
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device=q.device)
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=q.device)
    tb.tb_sparse_decode_attn(d, q, K, V, idx, cnt, max_count, sm_scale, out, lse, ws, tail[0], tail[1])
    return out, lse


def gpu_decode_step(q, q_imp, K, V, Kimp, N, k, sink, window, sm_scale, scale=1.0, ws=None):
    B, Hq, D = q.shape
    d = tb.make_desc(N, Hq, K=K, V=V, Kimp=Kimp)
    need = tb.policy_count(N, k, sink, window)
    stride = (N + 3) // 4 * 4
    scores = torch.full((B, Hq, max(stride, 4)), float("nan"), dtype=torch.float32, device=q.device)
    idx = torch.full((B, Hq, max(need, 1)), -7, dtype=torch.int32, device=q.device)
    cnt = torch.full((B, Hq), -7, dtype=torch.int32, device=q.device)
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device=q.device)
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=q.device)
    if ws is None:
        ws = tb.new_workspace(tb.TB_OP_DECODE_STEP, d, need)
    tb.tb_decode_step(d, q_imp, Kimp, scale, q, K, V, k, sink, window, sm_scale, scores, idx, cnt, out, lse, ws)
    return scores, idx, cnt, out, lse


def score_tolerance(oracle, q_imp_np, Kimp_np, dtype, scale, g):
    """|gpu - ref| <= 1e-4 |ref| + 1e-5 * scale * sum_j |q_j k_j|  (the second term guards sums
    that cancel; fp32 accumulation error is bounded by a small multiple of that magnitude)."""
    if dtype == "bf16":
        q64, K64 = oracle.bf16_to_f64(q_imp_np), oracle.bf16_to_f64(Kimp_np)
    else:
        q64, K64 = q_imp_np.astype(np.float64), Kimp_np.astype(np.float64)
    mag = np.einsum("bhj,bhnj->bhn", np.abs(q64), np.repeat(np.abs(K64), g, axis=1))
    return 1e-5 * abs(scale) * mag
