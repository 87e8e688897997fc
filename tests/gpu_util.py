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


# --------------------------------------------------------------------------- the parity bars
# Stated once; every GPU test and the smoke check use these.
#
# index lists        bit-exact (both sides select on the same fp32 scores)
# scores             |gpu - ref| <= 1e-4 |ref| + 1e-5 * |scale| * sum_j |q_j k_j|
#                    (1e-4 relative is the bar of the benchmark definition; the second term
#                    covers sums that cancel: fp32 accumulation of d' <= 64 products errs by at
#                    most d' * 2^-24 = 3.8e-6 of that magnitude)
# attention output   1e-5 absolute (fp32 K/V), 2e-2 absolute (bf16 K/V): benchmark definition
# log-sum-exp        1e-4 * max(1, |ref|): fp32 evaluation of m ln 2 + log(sum) over up to ~1e4
#                    terms errs by a few 1e-6 relative; the bar leaves an order of magnitude
# projected keys     fp32 storage: 1e-5 * sum_d |K_d W_dj|  (fp32 accumulation of D <= 128
#                    products: at most D * 2^-24 = 7.6e-6 of that magnitude)
#                    bf16 storage: one unit in the last place of the oracle's value (fp32 and fp64
#                    sums can round to different neighbours) + 1e-6 * sum_d |K_d W_dj| (the
#                    accumulation error itself; random-walk size sqrt(D) * 2^-24 = 6.7e-7)
ATTN_TOL = {"f32": 1e-5, "bf16": 2e-2}
SCORE_RTOL, SCORE_GUARD = 1e-4, 1e-5
LSE_RTOL = 1e-4


def assert_attention(out, ref_out, dtype, lse=None, ref_lse=None, what="attention"):
    """out/lse: numpy arrays (or anything np.asarray takes) against the oracle's, to the bar above."""
    err = float(np.abs(np.asarray(out, dtype=np.float64) - np.asarray(ref_out, dtype=np.float64)).max(initial=0.0))
    assert err <= ATTN_TOL[dtype], f"{what}: max |out - oracle| = {err:.3e} > {ATTN_TOL[dtype]}"
    if lse is not None:
        l, r = np.asarray(lse, dtype=np.float64), np.asarray(ref_lse, dtype=np.float64)
        fin = np.isfinite(r)
        assert np.array_equal(fin, np.isfinite(l)), f"{what}: lse finiteness"
        assert np.all(np.abs(l[fin] - r[fin]) <= LSE_RTOL * np.maximum(1.0, np.abs(r[fin]))), f"{what}: lse"
    return err


def assert_scores(got, ref, mag, scale=1.0, what="scores"):
    """mag = sum_j |q_j k_j| (same shape as ref)."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    bad = np.abs(got - ref) > SCORE_RTOL * np.abs(ref) + SCORE_GUARD * abs(scale) * mag
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} beyond the bar"


def assert_projection(oracle, got, ref, mag, dtype, what="projection"):
    """got/ref: stored arrays (bf16 as uint16 bit patterns), mag = sum_d |K_d W_dj| in float64."""
    if dtype == "bf16":
        g64, r64 = oracle.bf16_to_f64(got), oracle.bf16_to_f64(ref)
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(r64), 2.0 ** -126))) - 7)
        bound = ulp * 1.0000001 + 1e-6 * mag
    else:
        g64, r64 = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
        bound = 1e-5 * mag + 1e-30
    bad = np.abs(g64 - r64) > bound
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} beyond the bar"


def projection_magnitude(oracle, K_np, W_np, dtype, Hkv):
    """sum_d |K[b,h,n,d]| |W[hw,d,j]| in float64; W [Hw][D][Dimp] with Hw == 1 or Hkv."""
    to64 = oracle.bf16_to_f64 if dtype == "bf16" else (lambda a: np.asarray(a, dtype=np.float64))
    W64 = np.abs(np.broadcast_to(to64(W_np), (Hkv,) + W_np.shape[1:]))
    return np.einsum("bhnd,hdj->bhnj", np.abs(to64(K_np)), W64)


def score_magnitude(oracle, q_imp_np, Kimp_np, dtype, g):
    """sum_j |q_imp[b,h,j]| |K_imp[b,h/g,n,j]| in float64."""
    to64 = oracle.bf16_to_f64 if dtype == "bf16" else (lambda a: np.asarray(a, dtype=np.float64))
    return np.einsum("bhj,bhnj->bhn", np.abs(to64(q_imp_np)), np.repeat(np.abs(to64(Kimp_np)), g, axis=1))


def score_tolerance(oracle, q_imp_np, Kimp_np, dtype, scale, g):
    """The guard term of the score bar (kept for callers that add 1e-4 |ref| themselves)."""
    return SCORE_GUARD * abs(scale) * score_magnitude(oracle, q_imp_np, Kimp_np, dtype, g)
