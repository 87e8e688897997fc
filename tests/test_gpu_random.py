"""Seeded random shapes and policies for every operation against the oracle: the corner
combinations (ragged sizes, tiny budgets, sink/window overlapping the candidates, GQA groups,
empty lists) that the hand-picked cases do not enumerate."""
import math

import numpy as np
import pytest
import torch

from gpu_util import (DEV, dtype_name, gpu_attn, gpu_decode_step, gpu_expand, gpu_project, gpu_score, gpu_select,
                      np_of, score_magnitude, assert_attention, assert_scores)

pytestmark = pytest.mark.gpu


def rng_of(seed):
    return np.random.default_rng(seed)


def pick(r, xs):
    return xs[int(r.integers(len(xs)))]


@pytest.mark.parametrize("seed", range(24))
def test_random_select(oracle, seed):
    r = rng_of(1000 + seed)
    N = int(pick(r, [1, 3, 17, 255, 256, 257, 1023, 4095, 4099, 9000, 16384, 33001, 65537, 70000]))
    B, Hq = int(r.integers(1, 3)), int(pick(r, [1, 2, 5]))
    k = int(pick(r, [0, 1, 2, max(1, N // 50), max(1, N // 3), N - 1, N, N + 7]))
    sink = int(pick(r, [0, 0, 1, 4, N // 2, N + 1]))
    window = int(pick(r, [0, 0, 1, 64, N // 2, N + 1]))
    kind = pick(r, ["normal", "few_values", "constant", "sorted", "specials"])
    print(f"[case] random select seed={seed} N={N} B={B} Hq={Hq} k={k} sink={sink} window={window} kind={kind}", flush=True)
    stride = (N + 3) // 4 * 4
    g = torch.Generator().manual_seed(seed)
    if kind == "normal":
        s = torch.randn((B, Hq, stride), generator=g) * 10
    elif kind == "few_values":
        s = torch.randint(-3, 4, (B, Hq, stride), generator=g).float()
    elif kind == "constant":
        s = torch.full((B, Hq, stride), -2.5)
    elif kind == "sorted":
        s = torch.arange(stride, dtype=torch.float32).repeat(B, Hq, 1) * (1 if seed % 2 else -1)
    else:
        s = torch.randn((B, Hq, stride), generator=g)
        vals = torch.tensor([float("nan"), float("inf"), float("-inf"), -0.0, 0.0, 1e-45, -1e-45, 3.4e38])
        s[torch.rand((B, Hq, stride), generator=g) < 0.3] = 0
        sel = torch.rand((B, Hq, stride), generator=g) < 0.2
        s[sel] = vals[torch.randint(0, len(vals), (int(sel.sum()),), generator=g)]
    s = s.to(DEV)
    idx, cnt = gpu_select(s, N, k, sink, window)
    torch.cuda.synchronize()
    ridx, rcnt = oracle.select_topk(np_of(s)[:, :, :N], k, sink, window)
    assert np.array_equal(np_of(cnt), rcnt)
    w = ridx.shape[-1]
    mask = np.arange(w)[None, None, :] < rcnt[..., None]
    assert np.array_equal(np.where(mask, np_of(idx)[..., :w], -1), np.where(mask, ridx, -1))


@pytest.mark.parametrize("seed", range(16))
def test_random_select_long_rows(oracle, seed):
    """Rows beyond what one workgroup holds: the selection by pieces under random row counts,
    budgets, sink / window ranges and score patterns (among them a dense block of large scores)."""
    r = rng_of(5000 + seed)
    N = int(pick(r, [65537, 65540, 70000, 81921, 100001, 131072, 131075, 200000, 262147]))
    B, Hq = int(r.integers(1, 4)), int(pick(r, [1, 2, 5, 8, 13]))
    k = int(pick(r, [1, 2, 100, 4096, N // 50, N // 9, N // 8, N // 7, N // 3]))
    sink = int(pick(r, [0, 0, 1, 4, 128, 20000]))
    window = int(pick(r, [0, 0, 1, 64, 256, 30000]))
    kind = pick(r, ["normal", "normal", "few_values", "constant", "sorted", "specials", "cluster"])
    print(f"[case] random long select seed={seed} N={N} B={B} Hq={Hq} k={k} sink={sink} window={window} kind={kind}", flush=True)
    stride = (N + 3) // 4 * 4
    g = torch.Generator().manual_seed(seed)
    if kind == "normal":
        s = torch.randn((B, Hq, stride), generator=g) * 10
    elif kind == "few_values":
        s = torch.randint(-3, 4, (B, Hq, stride), generator=g).float()
    elif kind == "constant":
        s = torch.full((B, Hq, stride), -2.5)
    elif kind == "sorted":
        s = torch.arange(stride, dtype=torch.float32).repeat(B, Hq, 1) * (1 if seed % 2 else -1)
    elif kind == "cluster":
        s = torch.randn((B, Hq, stride), generator=g)
        a0 = int(r.integers(0, N - 5000))
        s[:, :, a0:a0 + int(r.integers(500, 5000))] += 50
    else:
        s = torch.randn((B, Hq, stride), generator=g)
        vals = torch.tensor([float("nan"), float("inf"), float("-inf"), -0.0, 0.0, 1e-45, -1e-45, 3.4e38])
        s[torch.rand((B, Hq, stride), generator=g) < 0.3] = 0
        sel = torch.rand((B, Hq, stride), generator=g) < 0.2
        s[sel] = vals[torch.randint(0, len(vals), (int(sel.sum()),), generator=g)]
    s = s.to(DEV)
    idx, cnt = gpu_select(s, N, k, sink, window)
    torch.cuda.synchronize()
    ridx, rcnt = oracle.select_topk(np_of(s)[:, :, :N], k, sink, window)
    assert np.array_equal(np_of(cnt), rcnt)
    w = ridx.shape[-1]
    mask = np.arange(w)[None, None, :] < rcnt[..., None]
    assert np.array_equal(np.where(mask, np_of(idx)[..., :w], -1), np.where(mask, ridx, -1))


@pytest.mark.parametrize("seed", range(12))
def test_random_decode_step(oracle, seed):
    r = rng_of(2000 + seed)
    dtype = pick(r, [torch.bfloat16, torch.bfloat16, torch.float32])
    D, Dimp = int(pick(r, [64, 128])), int(pick(r, [16, 32, 64]))
    Hkv = int(pick(r, [1, 2, 3]))
    gq = int(pick(r, [1, 2, 4, 8]))
    Hq, B = Hkv * gq, int(r.integers(1, 3))
    N = int(pick(r, [5, 130, 1000, 2049, 5000]))
    k = int(pick(r, [1, max(1, N // 10), N // 2, N]))
    sink, window = int(pick(r, [0, 2, 16])), int(pick(r, [0, 3, 32]))
    print(f"[case] random step seed={seed} dtype={dtype} B={B} Hq={Hq} Hkv={Hkv} D={D} Dimp={Dimp} N={N} k={k} "
          f"sink={sink} window={window}", flush=True)
    g = torch.Generator().manual_seed(seed)
    mk = lambda *shape, sc=1.0: (torch.randn(shape, generator=g) * sc).to(dtype).to(DEV)
    K, V, W = mk(B, Hkv, N + 2, D), mk(B, Hkv, N + 2, D), mk(1, D, Dimp, sc=D ** -0.5)
    q, q_imp = mk(B, Hq, D), mk(B, Hq, Dimp)
    Kimp = gpu_project(K, W, N)
    sm = 1.0 / math.sqrt(D)
    scores, idx, cnt, out, lse = gpu_decode_step(q, q_imp, K, V, Kimp, N, k, sink, window, sm, scale=0.5)
    torch.cuda.synchronize()
    dn = dtype_name(K)
    ref_s = oracle.score(np_of(q_imp), np_of(Kimp)[:, :, :N], dn, 0.5)
    assert_scores(np_of(scores)[:, :, :N], ref_s, score_magnitude(oracle, np_of(q_imp), np_of(Kimp)[:, :, :N], dn, gq), 0.5)
    ridx, rcnt = oracle.select_topk(np_of(scores)[:, :, :N], k, sink, window)
    assert np.array_equal(np_of(cnt), rcnt) and np.array_equal(np_of(idx)[..., : ridx.shape[-1]], ridx)
    ro, rl = oracle.sparse_decode_attn(np_of(q), np_of(K)[:, :, :N], np_of(V)[:, :, :N], np_of(idx), np_of(cnt), dn, sm)
    assert_attention(np_of(out), ro, dn, np_of(lse), rl)


@pytest.mark.parametrize("seed", range(12))
def test_random_expand_and_attention(oracle, seed):
    r = rng_of(3000 + seed)
    dtype = pick(r, [torch.bfloat16, torch.float32])
    D = int(pick(r, [64, 128]))
    Hkv, gq = int(pick(r, [1, 2])), int(pick(r, [1, 4]))
    Hq, B = Hkv * gq, int(r.integers(1, 3))
    N = int(pick(r, [40, 700, 3000, 9000]))
    cap = int(pick(r, [1, 7, N // 8 + 1, N // 3 + 1]))
    radius, mode = int(pick(r, [0, 1, 2, 5])), int(pick(r, [0, 0, 1]))
    tail = int(pick(r, [0, 1, 9]))
    print(f"[case] random expand+attn seed={seed} dtype={dtype} B={B} Hq={Hq} Hkv={Hkv} D={D} N={N} cap={cap} "
          f"radius={radius} mode={mode} tail={tail}", flush=True)
    g = torch.Generator().manual_seed(seed)
    Nc = N - tail  # the lists live in [0, Nc); the last `tail` rows are the dense tail
    idx = torch.stack([torch.stack([torch.randperm(Nc, generator=g)[:cap].sort().values for _ in range(Hq)])
                       for _ in range(B)]).to(torch.int32).to(DEV)
    cnt = torch.randint(0, cap + 1, (B, Hq), generator=g).to(torch.int32).to(DEV)
    eidx, ecnt = gpu_expand(idx, cnt, Nc, radius, mode)
    torch.cuda.synchronize()
    ridx, rcnt = oracle.expand_neighbors(np_of(idx), np_of(cnt), Nc, radius, cap_out=eidx.shape[-1], mode=mode)
    assert np.array_equal(np_of(ecnt), rcnt)
    mask = np.arange(ridx.shape[-1])[None, None, :] < rcnt[..., None]
    assert np.array_equal(np.where(mask, np_of(eidx), -1), np.where(mask, ridx, -1))
    mk = lambda *shape: torch.randn(shape, generator=g).to(dtype).to(DEV)
    K, V, q = mk(B, Hkv, N, D), mk(B, Hkv, N, D), mk(B, Hq, D)
    sm = 1.0 / math.sqrt(D)
    out, lse = gpu_attn(q, K, V, eidx, ecnt, N, sm, tail=(Nc, N))
    torch.cuda.synchronize()
    cn = np_of(ecnt)
    full = np.zeros((B, Hq, eidx.shape[-1] + tail), dtype=np.int32)
    for b in range(B):
        for h in range(Hq):
            c = cn[b, h]
            full[b, h, :c] = np_of(eidx)[b, h, :c]
            full[b, h, c:c + tail] = np.arange(Nc, N)
    ro, rl = oracle.sparse_decode_attn(np_of(q), np_of(K), np_of(V), full, cn + tail, dtype_name(K), sm)
    assert_attention(np_of(out), ro, dtype_name(K), np_of(lse), rl)
