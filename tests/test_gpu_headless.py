"""Head-less selection (Appendix "Additional Efficiency Evaluation": one importance per token per
layer, no head dimension): scoring and selection run with one importance head, and every
attention head of the layer reads the one list.  Against the oracle, and against the per-head
entry point given the same list for every head (bit for bit without grouped queries, where both
run the same kernel; to rounding with them, where the work is split differently)."""
import math

import numpy as np
import pytest
import torch

from gpu_util import (DEV, assert_attention, assert_scores, dtype_name, gpu_attn, gpu_score, gpu_select, np_of,
                      score_magnitude)
from paper_2503_07518_amd import binding as tb

pytestmark = pytest.mark.gpu


def say(msg):
    print(f"[case] {msg}", flush=True)


def shared_attn(q, K, V, idx, cnt, N, sm_scale, max_count, tail=(0, 0)):
    B, Hq, D = q.shape
    d = tb.make_desc(N, Hq, K=K, V=V)
    ws = tb.new_workspace(tb.TB_OP_ATTN, d, max_count + tail[1] - tail[0])
    out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
    tb.tb_sparse_decode_attn_shared(d, q, K, V, idx, cnt, max_count, sm_scale, out, lse, ws, tail[0], tail[1])
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("dtype,B,Hq,Hkv,D,N,k,sink,window", [
    # fewer than 32 KV groups: the per-head kernel reads the shared list
    (torch.bfloat16, 2, 32, 8, 128, 5000, 1024, 4, 64),   # grouped queries, per-XCD placement
    (torch.bfloat16, 3, 8, 2, 64, 1301, 200, 1, 17),      # ragged, 3 KV groups per XCD round
    (torch.float32, 1, 4, 4, 64, 333, 50, 0, 0),          # no grouping
    (torch.float32, 2, 8, 4, 128, 97, 200, 2, 3),         # budget beyond the candidates: everything
    (torch.bfloat16, 1, 16, 4, 128, 40000, 4096, 16, 256),  # several workgroups per head
    # 32 KV groups or more: one workgroup serves all heads of a KV group
    (torch.bfloat16, 4, 32, 8, 128, 5000, 1024, 4, 64),   # 4 heads per KV head, several splits
    (torch.bfloat16, 16, 16, 2, 64, 3000, 1000, 0, 5),    # 8 heads per KV head
    (torch.float32, 16, 4, 2, 128, 2500, 700, 3, 30),     # 2 heads per KV head, fp32 rows of 32 lanes
    (torch.float32, 16, 16, 2, 64, 1100, 300, 0, 0),      # 8 heads per KV head, fp32
    (torch.bfloat16, 40, 8, 1, 128, 200, 13, 1, 2),       # lists shorter than a tile, one split
    (torch.float32, 32, 2, 1, 64, 40, 100, 0, 0),         # everything selected
])
def test_headless_pipeline(oracle, dtype, B, Hq, Hkv, D, N, k, sink, window):
    say(f"head-less pipeline dtype={dtype} B={B} Hq={Hq} Hkv={Hkv} D={D} N={N} k={k}")
    g = torch.Generator().manual_seed(31)
    Dimp = 16
    K = torch.randn((B, Hkv, N, D), generator=g).to(dtype).to(DEV)
    V = torch.randn((B, Hkv, N, D), generator=g).to(dtype).to(DEV)
    q = torch.randn((B, Hq, D), generator=g).to(dtype).to(DEV)
    Kimp = torch.randn((B, 1, N, Dimp), generator=g).to(dtype).to(DEV)   # one importance head
    q_imp = torch.randn((B, 1, Dimp), generator=g).to(dtype).to(DEV)
    sm = 1.0 / math.sqrt(D)

    scores = gpu_score(q_imp, Kimp, N)
    idx, cnt = gpu_select(scores, N, k, sink, window)          # [B][1][cap], [B][1]
    torch.cuda.synchronize()
    r_scores = oracle.score(np_of(q_imp), np_of(Kimp), dtype_name(Kimp), 1.0)
    assert_scores(np_of(scores)[..., :N], r_scores, score_magnitude(oracle, np_of(q_imp), np_of(Kimp), dtype_name(Kimp), 1))
    # the list is checked on the GPU's own scores, so that fp32 rounding decides nothing
    r_idx, r_cnt = oracle.select_topk(np_of(scores)[..., :N], k, sink, window)
    assert np.array_equal(np_of(cnt), r_cnt)
    need = int(r_cnt.max())
    assert np.array_equal(np_of(idx)[..., :need], r_idx[..., :need])

    out, lse = shared_attn(q, K, V, idx, cnt.reshape(B), N, sm, idx.shape[-1])
    r_out, r_lse = oracle.sparse_decode_attn_shared(np_of(q), np_of(K), np_of(V), r_idx.reshape(B, -1),
                                                    r_cnt.reshape(B), dtype_name(K), sm)
    assert_attention(np_of(out), r_out, dtype_name(K), np_of(lse), r_lse)

    # same rows in the same order through the per-head entry point
    rep_idx = idx.expand(B, Hq, idx.shape[-1]).contiguous()
    rep_cnt = cnt.expand(B, Hq).contiguous()
    out2, lse2 = gpu_attn(q, K, V, rep_idx, rep_cnt, N, sm)
    torch.cuda.synchronize()
    if Hq == Hkv:
        assert torch.equal(out, out2) and torch.equal(lse, lse2)
    else:
        assert torch.allclose(out, out2, atol=1e-5, rtol=1e-5) and torch.allclose(lse, lse2, atol=1e-5, rtol=1e-5)


@pytest.mark.parametrize("B", [3, 8])  # 12 KV groups: per-head kernel; 32: one workgroup per KV group
def test_headless_tail_and_ragged_counts(oracle, B):
    """A list reused across a prediction interval: ragged counts per batch element (one empty),
    a count above max_count (truncated), and the dense tail of appended tokens."""
    say(f"head-less attention with tail and ragged counts B={B}")
    g = torch.Generator().manual_seed(32)
    Hq, Hkv, D, N, cap = 8, 4, 128, 900, 300
    K = torch.randn((B, Hkv, N, D), generator=g).to(torch.bfloat16).to(DEV)
    V = torch.randn((B, Hkv, N, D), generator=g).to(torch.bfloat16).to(DEV)
    q = torch.randn((B, Hq, D), generator=g).to(torch.bfloat16).to(DEV)
    idx = torch.stack([torch.randperm(N - 10, generator=g)[:cap].sort().values for _ in range(B)]).to(torch.int32).to(DEV)
    cnt = torch.tensor(([cap + 50, 0, 123] * B)[:B], dtype=torch.int32, device=DEV)
    max_count, tail = 280, (N - 10, N - 3)
    out, lse = shared_attn(q, K, V, idx, cnt, N, 0.09, max_count, tail)
    eff = np.minimum(np_of(cnt), max_count)
    r_idx = np.full((B, max_count + 7), 0, np.int32)
    for b in range(B):
        r_idx[b, :eff[b]] = np_of(idx)[b, :eff[b]]
        r_idx[b, eff[b]:eff[b] + 7] = np.arange(tail[0], tail[1])
    r_out, r_lse = oracle.sparse_decode_attn_shared(np_of(q), np_of(K), np_of(V), r_idx, eff + 7, "bf16", 0.09)
    assert_attention(np_of(out), r_out, "bf16", np_of(lse), r_lse)


@pytest.mark.parametrize("name", ["C2_llama3_8b_32k", "C3_batched_depth", "C5_long_context"])
def test_headless_full_size_configs(oracle, name):
    """The benchmark shapes with one importance head (the first KV head's projected keys):
    selection bit-exact on the GPU's scores for every batch element, attention on sampled heads
    (the oracle is given one batch element, one query head and its KV head at a time)."""
    from paper_2503_07518_amd import workloads
    cfg = workloads.CONFIGS[name]
    say(f"head-less full size {name}")
    data = workloads.make_layer(cfg, layer=3, device=DEV)
    K, V, W = data["K"], data["V"], data["W"]
    q, q_imp = data["q"][0].contiguous(), data["q_imp"][0][:, :1].contiguous()
    B, Hq, Hkv, N, D, g = cfg.B, cfg.Hq, cfg.Hkv, cfg.N, cfg.D, cfg.g
    Kimp = torch.zeros((B, Hkv, N, cfg.Dimp), dtype=K.dtype, device=DEV)
    tb.tb_project_keys(tb.make_desc(N, Hq, K=K, V=V, Kimp=Kimp), K, W, Kimp, 0, N)
    workloads.apply_kimp_row_scale(Kimp, data["kimp_row_scale"])
    Kimp1 = Kimp[:, :1]                                    # [B][1][N][d'], strided view
    scores = gpu_score(q_imp, Kimp1, N)
    idx, cnt = gpu_select(scores, N, cfg.k)
    torch.cuda.synchronize()
    r_idx, r_cnt = oracle.select_topk(np_of(scores)[..., :N], cfg.k, 0, 0)
    assert np.array_equal(np_of(cnt), r_cnt) and np.array_equal(np_of(idx), r_idx)
    out, lse = shared_attn(q, K, V, idx, cnt.reshape(B), N, cfg.sm_scale, idx.shape[-1])
    rng = np.random.default_rng(5)
    units = [(b, h) for b in range(B) for h in range(Hq)]
    if len(units) > 64:
        units = [units[i] for i in rng.choice(len(units), 64, replace=False)]
    for b, h in units:
        hk = h // g
        ro, rl = oracle.sparse_decode_attn_shared(np_of(q[b:b + 1, h:h + 1]), np_of(K[b:b + 1, hk:hk + 1]),
                                                  np_of(V[b:b + 1, hk:hk + 1]), r_idx[b], r_cnt[b], cfg.dtype,
                                                  cfg.sm_scale)
        assert_attention(np_of(out[b, h]), ro[0, 0], cfg.dtype, np_of(lse[b, h]), rl[0, 0])


@pytest.mark.parametrize("B", [1, 8])  # per-head kernel / one workgroup per KV group
def test_headless_degenerate_lists(oracle, B):
    """No list at all (only the dense tail is attended), and nothing to attend (out = 0,
    lse = -inf), through both kernels that serve a shared list."""
    say(f"head-less degenerate lists B={B}")
    g = torch.Generator().manual_seed(33)
    Hq, Hkv, D, N = 8, 4, 64, 300
    K = torch.randn((B, Hkv, N, D), generator=g).to(torch.bfloat16).to(DEV)
    V = torch.randn((B, Hkv, N, D), generator=g).to(torch.bfloat16).to(DEV)
    q = torch.randn((B, Hq, D), generator=g).to(torch.bfloat16).to(DEV)
    idx = torch.zeros((B, 4), dtype=torch.int32, device=DEV)
    cnt = torch.zeros((B,), dtype=torch.int32, device=DEV)
    out, lse = shared_attn(q, K, V, idx, cnt, N, 0.2, 0, tail=(N - 5, N))
    r_idx = np.tile(np.arange(N - 5, N, dtype=np.int32), (B, 1))
    r_out, r_lse = oracle.sparse_decode_attn_shared(np_of(q), np_of(K), np_of(V), r_idx, np.full(B, 5, np.int32), "bf16", 0.2)
    assert_attention(np_of(out), r_out, "bf16", np_of(lse), r_lse)
    out, lse = shared_attn(q, K, V, idx, cnt, N, 0.2, 4)
    assert torch.all(out == 0) and torch.all(torch.isinf(lse) & (lse < 0))


@pytest.mark.parametrize("B,mode", [(2, 0), (8, 1)])  # 8 x 4 KV heads: the grouped kernel; cluster-aware neighbours
def test_headless_interval_loop(oracle, B, mode):
    """Prediction interval with neighbour fetching on one list per batch element: every step
    against the oracle's driver (selection on the GPU's scores, expansion on the GPU's
    selection, attention over the widened list plus the rows appended since)."""
    from paper_2503_07518_amd import interval, workloads
    say(f"head-less interval loop B={B} mode={mode}")
    cfg = workloads.C4.scaled(name="C4_headless_small", B=B, Hq=8, Hkv=4, N=3000, k=200, steps=10, P=4,
                              heavy_per_kv_head=8)
    data = workloads.make_layer(cfg, device=DEV)
    K, V, W = data["K"], data["V"], data["W"]
    Hq, N0, steps = cfg.Hq, cfg.N, 10
    Ncap = K.shape[2]
    Kimp_all = torch.zeros((B, cfg.Hkv, Ncap, cfg.Dimp), dtype=K.dtype, device=DEV)
    tb.tb_project_keys(tb.make_desc(Ncap, Hq, K=K, V=V, Kimp=Kimp_all), K, W, Kimp_all, 0, Ncap)
    Kimp = Kimp_all[:, :1].contiguous()  # the importance head; rows of future tokens are there but not visible
    dec = interval.IntervalDecoder(K, V, W, Kimp, Hq, cfg.k, cfg.P, cfg.radius, sm_scale=cfg.sm_scale, mode=mode,
                                   headless=True)
    drv = oracle.IntervalDriver(cfg.dtype, cfg.k, cfg.P, cfg.radius, sm_scale=cfg.sm_scale, mode=mode, headless=True)
    Kn, Vn, Kin = np_of(K), np_of(V), np_of(Kimp)
    for t in range(steps):
        N_t = N0 + t
        q, q_imp = data["q"][t].contiguous(), data["q_imp"][t][:, :1].contiguous()
        out, lse = dec.step(t, N_t, q, q_imp)
        torch.cuda.synchronize()
        if t % cfg.P == 0:
            drv.step(t, N_t, np_of(q), np_of(q_imp), Kn, Vn, Kin)  # sets N_pred
            s_idx, s_cnt = oracle.select_topk(np_of(dec.scores)[:, :, :N_t], cfg.k, 0, 0)
            g_idx, g_cnt = np_of(dec.idx), np_of(dec.cnt)
            assert np.array_equal(s_cnt, g_cnt) and np.array_equal(s_idx, g_idx[..., : s_idx.shape[-1]])
            e_idx, e_cnt = oracle.expand_neighbors(g_idx, g_cnt, N_t, cfg.radius, cap_out=dec.exp_idx.shape[-1], mode=mode)
            assert np.array_equal(np_of(dec.exp_cnt), e_cnt)
            mask = np.arange(e_idx.shape[-1])[None, None] < e_cnt[..., None]
            assert np.array_equal(np.where(mask, np_of(dec.exp_idx), -1), np.where(mask, e_idx, -1))
            drv.exp_idx, drv.exp_cnt = e_idx, e_cnt  # continue the oracle from the GPU's selection
            ro, rl = oracle.sparse_decode_attn_shared(np_of(q), Kn[:, :, :N_t], Vn[:, :, :N_t], g_idx[:, 0], g_cnt[:, 0],
                                                      cfg.dtype, cfg.sm_scale)
        else:
            ro, rl, _, ucnt = drv.step(t, N_t, np_of(q), np_of(q_imp), Kn, Vn, Kin)
            assert np.array_equal(ucnt, drv.exp_cnt + (N_t - drv.N_pred))
        assert_attention(np_of(out), ro, cfg.dtype, np_of(lse), rl, what=f"step {t}")
