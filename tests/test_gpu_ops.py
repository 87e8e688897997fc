"""GPU parity: every exported operation, called through the C ABI, against the CPU oracle on
the same bytes.  Sizes span several tiles and ragged tails; edge cases are listed per op.

The bars (index lists bit-exact; scores, attention, log-sum-exp and projected keys within the
tolerances of the benchmark definition) are stated once, in gpu_util.py."""
import math

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from gpu_util import (ATTN_TOL, DEV, assert_attention, assert_projection, assert_scores, dtype_name, gpu_attn,
                      gpu_decode_step, gpu_expand, gpu_project, gpu_score, gpu_select, np_of, projection_magnitude,
                      score_magnitude)


def say(msg):
    print(f"[case] {msg}", flush=True)


def randn(shape, dtype, seed, scale=1.0):
    g = torch.Generator(device="cpu").manual_seed(seed)
    return (torch.randn(shape, generator=g) * scale).to(dtype).to(DEV)


# --------------------------------------------------------------------------- projection

@pytest.mark.parametrize("dtype,D,Dimp,N,Hw", [
    (torch.float32, 64, 16, 1000, 1),
    (torch.bfloat16, 128, 32, 1037, 1),
    (torch.bfloat16, 128, 32, 300, 3),
    (torch.bfloat16, 64, 64, 129, 1),
    (torch.float32, 128, 64, 65, 3),
    (torch.bfloat16, 128, 16, 1, 1),
    # up to four rows: the one-wave-per-row form of the decode-step append
    (torch.float32, 64, 64, 3, 3),
    (torch.bfloat16, 128, 32, 2, 1),
    (torch.bfloat16, 64, 16, 4, 3),
    (torch.float32, 128, 32, 5, 1),
    # enough rows for the matrix-core form (bf16, Dimp 32), ragged last tile
    (torch.bfloat16, 128, 32, 4133, 1),
    (torch.bfloat16, 64, 32, 2501, 3),
    (torch.bfloat16, 128, 32, 2048, 3),
    (torch.bfloat16, 128, 16, 3000, 1),   # the paper's interaction dimension, on the same tile
    (torch.bfloat16, 64, 16, 2111, 3),
])
def test_project_keys(oracle, dtype, D, Dimp, N, Hw):
    say(f"project dtype={dtype} D={D} Dimp={Dimp} N={N} Hw={Hw}")
    B, Hkv = 2, 3
    K = randn((B, Hkv, N + 5, D), dtype, 1)
    W = randn((Hw, D, Dimp), dtype, 2, 1 / math.sqrt(D))
    Kimp = gpu_project(K, W, N)
    torch.cuda.synchronize()
    dn = dtype_name(K)
    ref = oracle.project_keys(np_of(K)[:, :, :N], np_of(W), dn)
    got = np_of(Kimp)
    assert not got[:, :, N:].any(), "rows beyond N must stay untouched"
    mag = projection_magnitude(oracle, np_of(K)[:, :, :N], np_of(W), dn, Hkv)
    assert_projection(oracle, got[:, :, :N], ref, mag, dn)
    if dn == "bf16":
        assert np.mean(got[:, :, :N] == ref) > 0.99  # and nearly always the same bits


@pytest.mark.parametrize("N,n_begin,n_end", [(500, 70, 391), (5000, 70, 4391)])
def test_project_identity_and_row_range(oracle, N, n_begin, n_end):
    say(f"project identity W, row range [{n_begin}, {n_end}) of {N}")
    B, Hkv, D, Dimp = 1, 2, 128, 32
    K = randn((B, Hkv, N, D), torch.bfloat16, 3)
    W = torch.zeros((1, D, Dimp), dtype=torch.bfloat16, device=DEV)
    W[0, 3:3 + Dimp, :] = torch.eye(Dimp, dtype=torch.bfloat16)
    Kimp = torch.full((B, Hkv, N, Dimp), 7.0, dtype=torch.bfloat16, device=DEV)
    gpu_project(K, W, N, n_begin=n_begin, n_end=n_end, Kimp=Kimp)
    torch.cuda.synchronize()
    assert torch.equal(Kimp[:, :, n_begin:n_end], K[:, :, n_begin:n_end, 3:3 + Dimp])
    assert torch.all(Kimp[:, :, :n_begin] == 7.0) and torch.all(Kimp[:, :, n_end:] == 7.0)


def test_project_strided_cache(oracle):
    say("project into a strided (over-allocated) cache")
    B, Hkv, N, D, Dimp = 2, 2, 200, 128, 32
    Kbig = randn((B, Hkv, 256, D + 8), torch.bfloat16, 4)
    K = Kbig[:, :, :, :D]  # row stride D+8
    W = randn((1, D, Dimp), torch.bfloat16, 5, 0.1)
    Kimp_big = torch.zeros((B, Hkv, 256, Dimp + 8), dtype=torch.bfloat16, device=DEV)
    Kimp = Kimp_big[:, :, :, :Dimp]
    gpu_project(K, W, N, Kimp=Kimp)
    torch.cuda.synchronize()
    ref = oracle.project_keys(np_of(K)[:, :, :N], np_of(W), "bf16")
    mag = projection_magnitude(oracle, np_of(K)[:, :, :N], np_of(W), "bf16", Hkv)
    assert_projection(oracle, np_of(Kimp)[:, :, :N], ref, mag, "bf16")
    assert not np_of(Kimp_big)[..., Dimp:].any()


# --------------------------------------------------------------------------- scoring

@pytest.mark.parametrize("dtype,B,Hq,Hkv,Dimp,N", [
    (torch.float32, 1, 8, 8, 16, 1024),
    (torch.bfloat16, 1, 32, 8, 32, 5000),
    (torch.bfloat16, 2, 16, 2, 32, 1025),
    (torch.bfloat16, 1, 4, 2, 16, 63),
    (torch.float32, 1, 2, 2, 64, 300),
    (torch.bfloat16, 1, 4, 4, 64, 1),
    (torch.float32, 2, 8, 2, 32, 4097),
    (torch.bfloat16, 1, 4, 4, 32, 257),    # the matrix-core form (bf16, 32 projected dims): one query head per KV head
    (torch.bfloat16, 3, 6, 3, 32, 70),     # ... two, a ragged single workgroup
    (torch.bfloat16, 1, 8, 1, 32, 9),      # ... eight, fewer rows than one matrix tile
])
def test_score(oracle, dtype, B, Hq, Hkv, Dimp, N):
    say(f"score dtype={dtype} B={B} Hq={Hq} Hkv={Hkv} Dimp={Dimp} N={N}")
    q_imp = randn((B, Hq, Dimp), dtype, 6)
    Kimp = randn((B, Hkv, N + 3, Dimp), dtype, 7)
    scale = 0.7
    s = gpu_score(q_imp, Kimp, N, scale)
    torch.cuda.synchronize()
    dn = dtype_name(Kimp)
    ref = oracle.score(np_of(q_imp), np_of(Kimp)[:, :, :N], dn, scale)
    got = np_of(s)
    assert_scores(got[:, :, :N], ref, score_magnitude(oracle, np_of(q_imp), np_of(Kimp)[:, :, :N], dn, Hq // Hkv), scale)
    assert np.isnan(got[:, :, N:]).all(), "padding beyond N must stay untouched"


# --------------------------------------------------------------------------- selection

def check_select(oracle, scores_t, N, k, sink, window, ws=None):
    idx, cnt = gpu_select(scores_t, N, k, sink, window, ws=ws)
    torch.cuda.synchronize()
    s_np = np_of(scores_t)[:, :, :N]
    ridx, rcnt = oracle.select_topk(s_np, k, sink, window)
    gi, gc = np_of(idx), np_of(cnt)
    assert np.array_equal(gc, rcnt)
    width = ridx.shape[-1]
    mask = np.arange(width)[None, None, :] < rcnt[..., None]
    assert np.array_equal(np.where(mask, gi[..., :width], -1), np.where(mask, ridx, -1))
    assert np.all(gi[..., :width][~mask] == -7), "entries beyond count must stay untouched"
    return gi, gc


@pytest.mark.parametrize("N", [1, 2, 63, 64, 65, 1000, 1025, 4096, 4097, 8192, 20000, 40000, 65536, 70001])
def test_select_sizes_random_scores(oracle, N):
    say(f"select random N={N}")
    B, Hq = 2, 3
    scores = randn((B, Hq, (N + 3) // 4 * 4), torch.float32, 100 + N)
    for k in sorted({1, max(1, N // 10), N - 1, N, N + 5} - {0}):
        check_select(oracle, scores, N, k, 0, 0)
    if N > 20:
        check_select(oracle, scores, N, max(1, N // 7), 5, 9)
        check_select(oracle, scores, N, 0, 3, 4)


@pytest.mark.parametrize("N,ks", [
    (65537, (1, 4096, 8192)),            # one score more than a workgroup holds in registers
    (70001, (4096, 8000, 35000)),        # a short last piece
    (131072, (4096, 13000, 65536)),      # streamed rows: the bracket's keys fit the LDS list
    (300001, (1, 4096, 30000, 150000)),  # ... and overflow it for the larger budgets
    (1 << 20, (4096, 104857)),           # longest supported row
])
def test_select_streamed_rows(oracle, N, ks):
    say(f"select streamed N={N}")
    from paper_2503_07518_amd import binding as tb
    scores = randn((1, 2, (N + 3) // 4 * 4), torch.float32, 200 + N % 1000)
    d = tb.tb_cache_desc()
    d.B, d.Hq, d.Hkv, d.D, d.Dimp, d.dtype, d.N = 1, 2, 2, 128, 32, tb.TB_F32, N
    d.k_stride_n = d.v_stride_n = 128
    d.ki_stride_n = 32
    assert tb.tb_workspace_bytes(tb.TB_OP_SELECT, d, ks[0]) > 0, "a long row on two heads is cut into pieces"
    # with the workspace that tb_workspace_bytes asks for, the row is selected piecewise by
    # several workgroups; with a smaller one, a single workgroup streams the whole row
    small = torch.zeros(256, dtype=torch.uint8, device=DEV)
    g = torch.Generator().manual_seed(N)
    tied = torch.randint(0, 50, scores.shape, generator=g).to(torch.float32).to(DEV)  # heavy ties at the threshold
    asc = torch.arange(scores.shape[-1], dtype=torch.float32).view(1, 1, -1).to(DEV)  # every kept key in one span
    for ws in (None, small):
        for k in ks:
            check_select(oracle, scores, N, k, 0, 0, ws=ws)
        check_select(oracle, scores, N, ks[0], 128, 256, ws=ws)
        check_select(oracle, tied, N, ks[0], 0, 0, ws=ws)
        check_select(oracle, tied, N, ks[-1], 3, 5, ws=ws)
        check_select(oracle, asc, N, ks[0], 0, 0, ws=ws)
        check_select(oracle, -asc, N, ks[0], 2, 0, ws=ws)
    # rows whose sample misleads the first stage: huge values exactly where it looks -> the pieces
    # keep fewer keys than the budget; hugely negative ones exactly there -> the pieces keep far
    # more than they have room for.  Both must end in the same lists (the second stage then
    # selects on the whole row).
    pos = sample_positions(N)
    huge = scores.clone()
    huge[:, :, pos.to(DEV)] = 1e30
    check_select(oracle, huge, N, min(N // 8, 3 * len(pos)), 0, 0)
    low = scores.clone()
    low[:, :, pos.to(DEV)] = -1e30
    check_select(oracle, low, N, ks[0], 0, 0)


def sample_positions(N, lo=0, hi=None):
    """Positions that the first stage of a selection by pieces may sample: four adjacent scores at
    each of up to 1024 places spread evenly over the candidates (a workgroup of T threads looks at
    the places t * span / T, T = 256, 512 or 1024: all on this grid)."""
    hi = N if hi is None else hi
    span = hi - lo
    start = torch.tensor([(lo + (t * span) // 1024) & ~3 for t in range(1024)])
    pos = (start[:, None] + torch.arange(4)[None, :]).reshape(-1)
    return torch.unique(pos[pos < N])


def test_select_pieces_row_count_not_a_multiple_of_eight(oracle):
    """The first stage places the pieces of a row on one XCD and pads its launch to a multiple of
    eight rows: 6 and 11 rows, sink and window, a ragged last piece."""
    say("select by pieces, 6 and 11 rows")
    for B, Hq, N in ((2, 3, 66003), (1, 11, 81925)):
        scores = randn((B, Hq, (N + 3) // 4 * 4), torch.float32, 300 + Hq)
        check_select(oracle, scores, N, 4096, 0, 0)
        check_select(oracle, scores, N, 2000, 64, 100)


def test_select_pieces_many_rows(oracle):
    """Enough long rows that the pieces take their widest form (512 threads, 16384 scores)."""
    say("select by pieces, 128 rows")
    N, k = 70001, 4096
    stride = (N + 3) // 4 * 4
    scores = randn((2, 64, stride), torch.float32, 77)
    check_select(oracle, scores, N, k, 0, 0)
    check_select(oracle, scores, N, 7000, 128, 256)
    # every kept score in one wave's span: its LDS region overflows and the piece takes the slower path
    asc = torch.arange(stride, dtype=torch.float32).view(1, 1, -1).expand(2, 64, stride).contiguous().to(DEV)
    check_select(oracle, asc, N, k, 0, 0)
    mixed = scores.clone()
    mixed[:, ::2, 20000:23000] += 100.0  # a dense block of large scores in every other row
    check_select(oracle, mixed, N, k, 3, 9)
    pos = sample_positions(N)
    low = scores.clone()
    low[:, :, pos.to(DEV)] = -1e30
    check_select(oracle, low, N, k, 0, 0)
    # flat distributions put several budgets' worth of scores into one coarse bin around the
    # threshold (the kept scores are cut inside that bin), a ramp towards recent positions puts
    # nearly all kept scores into the last piece (its waves' LDS regions overflow)
    g = torch.Generator().manual_seed(5)
    flat = (1.0 + torch.rand((2, 64, stride), generator=g)).to(DEV)
    check_select(oracle, flat, N, k, 0, 0)
    ramp = (torch.arange(stride, dtype=torch.float32).view(1, 1, -1) * (8.0 / N) + torch.randn((2, 64, stride), generator=g)).to(DEV)
    check_select(oracle, ramp, N, k, 16, 32)
    nan = scores.clone()
    nan[:, :, ::5] = float("nan")
    nan[:, :, 1::5] = float("-inf")
    check_select(oracle, nan, N, 60000, 0, 0)  # the threshold falls among the NaN / -inf ties


@pytest.mark.parametrize("N", [777, 9000, 66000])
def test_select_ties_and_special_values(oracle, N):
    say(f"select ties/specials N={N}")
    g = torch.Generator(device="cpu").manual_seed(N)
    stride = (N + 3) // 4 * 4
    # heavy ties: scores quantised to a handful of values, threshold lands inside a tie block
    q = torch.randint(-3, 4, (1, 4, stride), generator=g).float() * 0.5
    for k in (1, N // 3, N // 2, N - 1):
        check_select(oracle, q.to(DEV), N, k, 0, 0)
    check_select(oracle, q.to(DEV), N, N // 3, 17, 33)
    # all equal
    same = torch.full((1, 2, stride), 1.25)
    check_select(oracle, same.to(DEV), N, N // 5, 0, 0)
    check_select(oracle, same.to(DEV), N, N // 5, 11, 7)
    # special values: +-inf, NaN (ranks with -inf), -0 / +0, denormals, huge and tiny magnitudes
    sp = torch.randn((1, 3, stride), generator=g)
    pos = torch.randperm(N, generator=g)
    vals = [float("inf"), float("-inf"), float("nan"), -0.0, 0.0, 1e-42, -1e-42, 3e38, -3e38, 1e-30]
    for i, v in enumerate(vals):
        sp[:, :, pos[i::len(vals)][: max(1, N // 40)]] = v
    for k in (1, N // 20, N // 2, N - 2):
        check_select(oracle, sp.to(DEV), N, k, 0, 0)
    # all NaN / all -inf mixture: index order decides
    nn = torch.full((1, 1, stride), float("nan"))
    nn[0, 0, ::3] = float("-inf")
    check_select(oracle, nn.to(DEV), N, N // 2, 0, 0)
    # sorted ascending and descending
    asc = torch.arange(stride, dtype=torch.float32).view(1, 1, stride)
    check_select(oracle, asc.to(DEV), N, N // 4, 0, 0)
    check_select(oracle, (-asc).to(DEV), N, N // 4, 2, 2)
    # values that agree in the top 11 and top 22 key bits: every radix level has to refine
    base = torch.full((1, 2, stride), 1.0)
    base = (base.view(torch.int32) + torch.randint(0, 700, (1, 2, stride), generator=g, dtype=torch.int32)).view(torch.float32)
    check_select(oracle, base.to(DEV), N, N // 3, 0, 0)


def test_select_sink_window_cover_everything(oracle):
    say("select sink+window >= N")
    N = 300
    scores = randn((1, 2, 300), torch.float32, 9)
    gi, gc = check_select(oracle, scores, N, 10, 200, 200)
    assert np.all(gc == N)
    gi, gc = check_select(oracle, scores, N, 10, 400, 0)
    assert np.all(gc == N)


def test_select_repeatable_and_workspace_reuse(oracle):
    say("select repeated calls share one workspace")
    from paper_2503_07518_amd import binding as tb
    N, k = 30000, 3000
    scores = randn((2, 8, N), torch.float32, 10)
    d = tb.tb_cache_desc()
    d.B, d.Hq, d.Hkv, d.D, d.Dimp, d.dtype, d.N = 2, 8, 8, 128, 32, tb.TB_F32, N
    d.k_stride_n = d.v_stride_n = 128
    d.ki_stride_n = 32
    ws = tb.new_workspace(tb.TB_OP_SELECT, d)
    first = None
    for _ in range(4):
        idx, cnt = gpu_select(scores, N, k, ws=ws)
        torch.cuda.synchronize()
        if first is None:
            first = (idx.clone(), cnt.clone())
        assert torch.equal(idx, first[0]) and torch.equal(cnt, first[1])
    ridx, rcnt = oracle.select_topk(np_of(scores), k)
    assert np.array_equal(np_of(first[0]), ridx) and np.array_equal(np_of(first[1]), rcnt)
    assert not ws.any(), "the workspace is left zeroed"


# --------------------------------------------------------------------------- neighbours

def random_lists(B, Hq, N, count_max, seed, cap=None):
    rng = np.random.default_rng(seed)
    cap = cap or max(count_max, 1)
    idx = np.full((B, Hq, cap), -1, np.int32)
    cnt = np.zeros((B, Hq), np.int32)
    for b in range(B):
        for h in range(Hq):
            c = int(rng.integers(0, count_max + 1)) if (b + h) % 3 else count_max
            c = min(c, N)
            idx[b, h, :c] = np.sort(rng.choice(N, c, replace=False))
            cnt[b, h] = c
    return idx, cnt


@pytest.mark.parametrize("N,count_max,radius", [(50, 20, 1), (1000, 300, 1), (1000, 999, 2), (70000, 5000, 1),
                                                (4096, 4096, 3), (10, 0, 1), (100000, 7, 5), (5000, 2500, 0)])
@pytest.mark.parametrize("mode", [0, 1])
def test_expand_neighbors(oracle, N, count_max, radius, mode):
    say(f"expand N={N} count_max={count_max} r={radius} mode={mode}")
    idx, cnt = random_lists(2, 3, N, count_max, seed=N + radius)
    # clustered input as well: runs of consecutive positions and picks at both ends
    if count_max >= 8 and N > 64:
        run = np.arange(N - 6, N, dtype=np.int32)
        idx[0, 0, :] = -1
        head = np.array([0, 1, 2], np.int32)
        mid = np.arange(N // 2, N // 2 + min(count_max - 9, 40), dtype=np.int32)
        lst = np.concatenate([head, mid, run])
        idx[0, 0, : len(lst)] = lst
        cnt[0, 0] = len(lst)
    out, oc = gpu_expand(torch.from_numpy(idx).to(DEV), torch.from_numpy(cnt).to(DEV), N, radius, mode)
    torch.cuda.synchronize()
    ro, rc = oracle.expand_neighbors(idx, cnt, N, radius, cap_out=out.shape[-1], mode=mode)
    go, gc = np_of(out), np_of(oc)
    assert np.array_equal(gc, rc)
    mask = np.arange(go.shape[-1])[None, None, :] < rc[..., None]
    assert np.array_equal(np.where(mask, go, -1), np.where(mask, ro, -1))
    assert np.all(go[~mask] == -7)


# --------------------------------------------------------------------------- attention

@pytest.mark.parametrize("dtype,B,Hq,Hkv,D,N,count_max", [
    (torch.float32, 1, 8, 8, 64, 1024, 128),
    (torch.bfloat16, 1, 32, 8, 128, 5000, 700),
    (torch.bfloat16, 2, 8, 2, 128, 3000, 3000),
    (torch.float32, 1, 4, 2, 128, 777, 333),
    (torch.bfloat16, 1, 4, 4, 64, 900, 65),
    (torch.bfloat16, 1, 2, 2, 128, 40, 1),
    (torch.bfloat16, 3, 16, 2, 128, 9000, 2049),
])
def test_sparse_decode_attn(oracle, dtype, B, Hq, Hkv, D, N, count_max):
    say(f"attn dtype={dtype} B={B} Hq={Hq} Hkv={Hkv} D={D} N={N} count_max={count_max}")
    q = randn((B, Hq, D), dtype, 11)
    K = randn((B, Hkv, N + 2, D), dtype, 12)
    V = randn((B, Hkv, N + 2, D), dtype, 13)
    idx, cnt = random_lists(B, Hq, N, count_max, seed=14)
    cnt[0, 0] = 0  # an empty list
    sm = 1 / math.sqrt(D)
    out, lse = gpu_attn(q, K, V, torch.from_numpy(idx).to(DEV), torch.from_numpy(cnt).to(DEV), N, sm)
    torch.cuda.synchronize()
    dn = dtype_name(K)
    ro, rl = oracle.sparse_decode_attn(np_of(q), np_of(K)[:, :, :N], np_of(V)[:, :, :N], idx, cnt, dn, sm)
    go, gl = np_of(out), np_of(lse)
    assert_attention(go, ro, dn, gl, rl)
    assert not go[0, 0].any() and gl[0, 0] == -np.inf


def test_attn_full_budget_equals_dense_and_tail(oracle):
    say("attn full list == dense; list + dense tail")
    B, Hq, Hkv, D, N = 1, 8, 2, 128, 2500
    q = randn((B, Hq, D), torch.bfloat16, 15)
    K = randn((B, Hkv, N, D), torch.bfloat16, 16)
    V = randn((B, Hkv, N, D), torch.bfloat16, 17)
    sm = 1 / math.sqrt(D)
    full = torch.arange(N, dtype=torch.int32, device=DEV).expand(B, Hq, N).contiguous()
    cnt = torch.full((B, Hq), N, dtype=torch.int32, device=DEV)
    out, _ = gpu_attn(q, K, V, full, cnt, N, sm)
    torch.cuda.synchronize()
    dense = oracle.dense_decode_attn(np_of(q), np_of(K), np_of(V), "bf16", sm)
    assert_attention(np_of(out), dense, "bf16", what="full list against dense attention")
    # a list over the first part plus the rest as a dense tail gives the same result
    idx, c = random_lists(B, Hq, 2000, 300, seed=18)
    out_t, lse_t = gpu_attn(q, K, V, torch.from_numpy(idx).to(DEV), torch.from_numpy(c).to(DEV), N, sm,
                            tail=(2000, N))
    torch.cuda.synchronize()
    cap = idx.shape[-1] + (N - 2000)
    joined = np.full((B, Hq, cap), -1, np.int32)
    for h in range(Hq):
        joined[0, h, : c[0, h]] = idx[0, h, : c[0, h]]
        joined[0, h, c[0, h]: c[0, h] + N - 2000] = np.arange(2000, N)
    ro, rl = oracle.sparse_decode_attn(np_of(q), np_of(K), np_of(V), joined, c + (N - 2000), "bf16", sm)
    assert_attention(np_of(out_t), ro, "bf16", np_of(lse_t), rl)


def test_attn_strided_cache_and_max_count_truncation(oracle):
    say("attn on a strided cache view; max_count truncates longer lists")
    B, Hq, Hkv, D, N = 2, 4, 2, 128, 1200
    q = randn((B, Hq, D), torch.bfloat16, 19)
    Kbig = randn((B, Hkv, N, 2 * D), torch.bfloat16, 20)
    K, V = Kbig[..., :D], Kbig[..., D:]  # interleaved K|V rows, stride 2D
    idx, cnt = random_lists(B, Hq, N, 500, seed=21)
    sm = 0.1
    out, lse = gpu_attn(q, K, V, torch.from_numpy(idx).to(DEV), torch.from_numpy(cnt).to(DEV), N, sm, max_count=260)
    torch.cuda.synchronize()
    ro, rl = oracle.sparse_decode_attn(np_of(q), np_of(K), np_of(V), idx, np.minimum(cnt, 260), "bf16", sm)
    assert_attention(np_of(out), ro, "bf16", np_of(lse), rl)


@pytest.mark.parametrize("B,Hq,Hkv,N,k", [(1, 32, 8, 32768, 3277), (16, 32, 8, 16384, 2048)])
def test_attn_split_handover_repeatable(oracle, B, Hq, Hkv, N, k):
    """The split attention hands partial results from workgroup to workgroup (last arriver
    combines): 200 launches on the shapes of the single-sequence and the batched benchmark
    configuration, each compared bit for bit with the first, which is checked against the
    oracle.  Stops at the first mismatch."""
    say(f"attn hand-over: 200 launches, B={B} Hq={Hq} N={N} k={k}")
    D = 128
    q = randn((B, Hq, D), torch.bfloat16, 22)
    K = randn((B, Hkv, N, D), torch.bfloat16, 23)
    V = randn((B, Hkv, N, D), torch.bfloat16, 24)
    rng = np.random.default_rng(25)  # full lists: the largest number of splits
    idx = np.stack([np.stack([np.sort(rng.choice(N, k, replace=False)).astype(np.int32) for _ in range(Hq)])
                    for _ in range(B)])
    cnt = np.full((B, Hq), k, np.int32)
    ti, tc = torch.from_numpy(idx).to(DEV), torch.from_numpy(cnt).to(DEV)
    from paper_2503_07518_amd import binding as tb
    d = tb.make_desc(N, Hq, K=K, V=V)
    ws = tb.new_workspace(tb.TB_OP_ATTN, d, k)
    sm = 1 / math.sqrt(D)
    out, lse = gpu_attn(q, K, V, ti, tc, N, sm, ws=ws)
    torch.cuda.synchronize()
    ref = (out.clone(), lse.clone())
    # the oracle on a sample of units (all of them for the single sequence)
    rng = np.random.default_rng(7)
    units = [(b, h) for b in range(B) for h in range(Hq)] if B == 1 else [
        (int(rng.integers(B)), int(rng.integers(Hq))) for _ in range(64)]
    g = Hq // Hkv
    for b, h in units:
        ro, rl = oracle.sparse_decode_attn(np_of(q[b:b + 1, h:h + 1]), np_of(K[b:b + 1, h // g:h // g + 1]),
                                           np_of(V[b:b + 1, h // g:h // g + 1]), idx[b:b + 1, h:h + 1],
                                           cnt[b:b + 1, h:h + 1], "bf16", sm)
        assert_attention(np_of(out[b, h]), ro[0, 0], "bf16", np_of(lse[b, h]), rl[0, 0])
    for it in range(200):
        out, lse = gpu_attn(q, K, V, ti, tc, N, sm, ws=ws)
        if it % 20 == 19:
            print(f"[case]   launch {it + 1}", flush=True)
        torch.cuda.synchronize()
        assert torch.equal(out, ref[0]) and torch.equal(lse, ref[1]), f"launch {it} differs from the first"


# --------------------------------------------------------------------------- fused step

@pytest.mark.parametrize("dtype,B,Hq,Hkv,D,Dimp,N,k,sink,window", [
    (torch.float32, 1, 8, 8, 64, 16, 1024, 128, 0, 0),
    (torch.bfloat16, 1, 32, 8, 128, 32, 6000, 600, 0, 0),
    (torch.bfloat16, 2, 16, 2, 128, 32, 3001, 300, 16, 32),
    (torch.bfloat16, 1, 8, 2, 128, 32, 500, 500, 0, 0),
    (torch.bfloat16, 1, 8, 2, 128, 32, 500, 0, 4, 4),
])
def test_decode_step_matches_separate_calls_and_oracle(oracle, dtype, B, Hq, Hkv, D, Dimp, N, k, sink, window):
    say(f"decode_step dtype={dtype} B={B} Hq={Hq} Hkv={Hkv} D={D} Dimp={Dimp} N={N} k={k} S={sink} W={window}")
    q = randn((B, Hq, D), dtype, 26)
    q_imp = randn((B, Hq, Dimp), dtype, 27)
    K = randn((B, Hkv, N, D), dtype, 28)
    V = randn((B, Hkv, N, D), dtype, 29)
    W = randn((1, D, Dimp), dtype, 30, 1 / math.sqrt(D))
    Kimp = gpu_project(K, W, N)
    sm = 1 / math.sqrt(D)
    s, idx, cnt, out, lse = gpu_decode_step(q, q_imp, K, V, Kimp, N, k, sink, window, sm)
    s2 = gpu_score(q_imp, Kimp, N)
    idx2, cnt2 = gpu_select(s2, N, k, sink, window, Hkv=Hkv)
    out2, lse2 = gpu_attn(q, K, V, idx2, cnt2, N, sm, max_count=idx2.shape[-1])
    torch.cuda.synchronize()
    assert torch.equal(s[:, :, :N], s2[:, :, :N])
    assert torch.equal(cnt, cnt2) and torch.equal(idx, idx2)
    assert torch.equal(out, out2) and torch.equal(lse, lse2)
    dn = dtype_name(K)
    ridx, rcnt = oracle.select_topk(np_of(s)[:, :, :N], k, sink, window)
    assert np.array_equal(np_of(cnt), rcnt)
    assert np.array_equal(np_of(idx)[..., : ridx.shape[-1]], ridx)
    ro, rl = oracle.sparse_decode_attn(np_of(q), np_of(K), np_of(V), np_of(idx), np_of(cnt), dn, sm)
    assert_attention(np_of(out), ro, dn, np_of(lse), rl)


def test_read_stream_probe_reads_and_writes_nothing():
    """The bandwidth calibration kernel: any size (also below one vector, and ragged), the
    source and the sink word stay as they were."""
    from paper_2503_07518_amd import binding as tb
    print("[case] read-stream probe", flush=True)
    for nbytes in (8, 16, 100, 4096 * 33 + 16, 1 << 22):
        src = torch.arange(max(nbytes, 16), dtype=torch.int64, device=DEV).to(torch.uint8)[:max(nbytes, 16)].contiguous()
        before = src.clone()
        sink = torch.full((4,), 7, dtype=torch.int32, device=DEV)
        tb.tb_read_stream_probe(src[:nbytes], sink)
        torch.cuda.synchronize()
        assert torch.equal(src, before) and torch.all(sink == 7)
