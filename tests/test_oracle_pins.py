"""Pins for the CPU oracle: every check compares it with something other than itself --
a library fp64 routine, a closed form, a hand-worked fixture, brute force on tiny inputs or
an invariant of the definition.  No GPU involved."""
import math
import os

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


def f32_to_bf16_bits_trunc_pair(x64):
    """The two bf16 neighbours (as float64) around each double, by bit manipulation."""
    f = np.asarray(x64, dtype=np.float64)
    lo = (f.astype(np.float32).view(np.uint32) & 0xFFFF0000).view(np.float32).astype(np.float64)
    return lo


def bf16_bits(x):
    """fp32-representable values -> bf16 bit patterns by truncation (caller guarantees exactness)."""
    return (np.asarray(x, dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


def rand_bf16(rng, shape, scale=1.0):
    x = (rng.standard_normal(shape) * scale).astype(np.float32)
    bits = (x.view(np.uint32) >> 16).astype(np.uint16)  # truncation is fine for drawing inputs
    return bits


# ------------------------------------------------------------------------------ rounding


def test_bf16_rounding_enumerated(oracle):
    """Round-to-nearest-even at every kind of boundary, from the bit layout of bf16."""
    for bits in [0x3F80, 0x3F81, 0x3FFF, 0x4000, 0x0001, 0x007F, 0x0080, 0x7F7E, 0x0000, 0x4049]:
        a = float(oracle.bf16_to_f64(np.array([bits], dtype=np.uint16))[0])
        b = float(oracle.bf16_to_f64(np.array([bits + 1], dtype=np.uint16))[0])
        mid = (a + b) / 2.0
        even = bits if bits % 2 == 0 else bits + 1
        assert oracle.round_bf16(a) == bits
        assert oracle.round_bf16(mid) == even
        assert oracle.round_bf16(np.nextafter(mid, b)) == bits + 1
        assert oracle.round_bf16(np.nextafter(mid, a)) == bits
        assert oracle.round_bf16(-mid) == (even | 0x8000)
    assert oracle.round_bf16(float("inf")) == 0x7F80
    assert oracle.round_bf16(3.4e38) == 0x7F80  # beyond the largest bf16 (0x7F7F ~ 3.39e38) -> inf
    assert oracle.round_bf16(-0.0) == 0x8000
    assert oracle.round_bf16(float("nan")) & 0x7FC0 == 0x7FC0


# ------------------------------------------------------------------------------ projection


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_project_identity_selects_columns_bit_exact(oracle, dtype):
    """W = [I; 0] makes the projection a column slice (Sec. 3.1 equation with that W)."""
    rng = np.random.default_rng(1)
    B, Hkv, N, D, d = 2, 3, 17, 16, 8
    if dtype == "f32":
        K = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
        W = np.zeros((1, D, d), np.float32)
        W[0, :d, :] = np.eye(d)
    else:
        K = rand_bf16(rng, (B, Hkv, N, D))
        W = np.zeros((1, D, d), np.uint16)
        W[0, np.arange(d), np.arange(d)] = 0x3F80
    out = oracle.project_keys(K, W, dtype)
    assert np.array_equal(out, K[..., :d])
    Wz = np.zeros_like(W)
    assert not oracle.project_keys(K, Wz, dtype).any()


def test_project_matches_fp64_matmul_f32(oracle):
    rng = np.random.default_rng(2)
    B, Hkv, N, D, d = 2, 2, 33, 64, 16
    K = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    W = (rng.standard_normal((1, D, d)) / 8).astype(np.float32)
    ref = np.einsum("bhnd,dj->bhnj", K.astype(np.float64), W[0].astype(np.float64))
    out = oracle.project_keys(K, W, "f32")
    # one rounding from an fp64 sum: at most half an fp32 ulp from the fp64 value
    assert np.all(np.abs(out.astype(np.float64) - ref) <= np.spacing(np.abs(ref).astype(np.float32)) * 0.5 + 1e-300)


def test_project_bf16_is_nearest_bf16_of_fp64_matmul(oracle):
    rng = np.random.default_rng(3)
    B, Hkv, N, D, d = 1, 2, 40, 128, 32
    K = rand_bf16(rng, (B, Hkv, N, D))
    W = rand_bf16(rng, (1, D, d), 1 / math.sqrt(D))
    ref = np.einsum("bhnd,dj->bhnj", oracle.bf16_to_f64(K), oracle.bf16_to_f64(W)[0])
    out = oracle.bf16_to_f64(oracle.project_keys(K, W, "bf16"))
    # nearest bf16: error at most half the bf16 spacing (2^-8 relative) at the value
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - 7)
    assert np.all(np.abs(out - ref) <= 0.5 * ulp * (1 + 1e-12))


def test_project_per_head_matrices_and_row_range(oracle):
    rng = np.random.default_rng(4)
    B, Hkv, N, D, d = 2, 3, 12, 8, 4
    K = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    W = rng.standard_normal((Hkv, D, d)).astype(np.float32)
    ref = np.einsum("bhnd,hdj->bhnj", K.astype(np.float64), W.astype(np.float64)).astype(np.float32)
    out = np.full((B, Hkv, N, d), 7.0, np.float32)
    oracle.project_keys(K, W, "f32", n_begin=3, n_end=9, out=out)
    assert np.allclose(out[:, :, 3:9], ref[:, :, 3:9], rtol=1e-6, atol=1e-6)
    assert np.all(out[:, :, :3] == 7.0) and np.all(out[:, :, 9:] == 7.0)


# ------------------------------------------------------------------------------ scoring


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_score_matches_fp64_einsum_and_gqa_mapping(oracle, dtype):
    rng = np.random.default_rng(5)
    B, Hq, Hkv, N, d = 2, 8, 2, 50, 16
    g = Hq // Hkv
    if dtype == "f32":
        qi = rng.standard_normal((B, Hq, d)).astype(np.float32)
        Ki = rng.standard_normal((B, Hkv, N, d)).astype(np.float32)
        q64, K64 = qi.astype(np.float64), Ki.astype(np.float64)
    else:
        qi, Ki = rand_bf16(rng, (B, Hq, d)), rand_bf16(rng, (B, Hkv, N, d))
        q64, K64 = oracle.bf16_to_f64(qi), oracle.bf16_to_f64(Ki)
    ref = 0.37 * np.einsum("bhj,bhnj->bhn", q64, np.repeat(K64, g, axis=1))  # consecutive heads share
    out = oracle.score(qi, Ki, dtype, scale=0.37)
    assert out.dtype == np.float32
    assert np.allclose(out, ref, rtol=2e-7, atol=1e-7)


def test_score_with_identity_projection_is_the_attention_logit(oracle):
    """d' = D and W = I: the importance score is q.k, i.e. the logit of real attention; checked
    through the attention oracle (lse over a single selected row equals sm_scale * q.k)."""
    rng = np.random.default_rng(6)
    B, H, N, D = 1, 2, 9, 8
    K = rng.standard_normal((B, H, N, D)).astype(np.float32)
    V = rng.standard_normal((B, H, N, D)).astype(np.float32)
    q = rng.standard_normal((B, H, D)).astype(np.float32)
    W = np.eye(D, dtype=np.float32)[None]
    Kimp = oracle.project_keys(K, W, "f32")
    s = oracle.score(q, Kimp, "f32", scale=1.0)
    for n in range(N):
        idx = np.full((B, H, 1), n, np.int32)
        cnt = np.ones((B, H), np.int32)
        _, lse = oracle.sparse_decode_attn(q, K, V, idx, cnt, "f32", sm_scale=0.5)
        assert np.allclose(lse, 0.5 * s[:, :, n], rtol=1e-6, atol=1e-6)


# ------------------------------------------------------------------------------ selection


def numpy_select(scores, k, sink, window):
    """Independent statement of the policy with a stable library sort."""
    s = np.asarray(scores, np.float32).copy()
    N = len(s)
    lo = min(sink, N)
    hi = max(lo, N - window)
    s = np.where(np.isnan(s), -np.inf, s)
    cand = np.arange(lo, hi)
    order = cand[np.argsort(-s[lo:hi].astype(np.float64), kind="stable")]
    picked = np.sort(order[: min(k, hi - lo)])
    return np.concatenate([np.arange(lo), picked, np.arange(hi, N)]).astype(np.int32)


def test_select_golden_ties(oracle):
    g = read_golden("select_ties.txt")
    idx, cnt = oracle.select_topk(np.array(g["scores"], np.float32), int(g["k"][0]), int(g["sink"][0]),
                                  int(g["window"][0]))
    assert idx[: int(cnt)].tolist() == [int(v) for v in g["idx"]]


@settings(max_examples=300, deadline=None)
@given(st.data())
def test_select_vs_bruteforce_and_sort(oracle, data):
    N = data.draw(st.integers(1, 40))
    vals = data.draw(st.lists(st.sampled_from([-np.inf, -2.0, -0.0, 0.0, 1.0, 1.5, 3.0, np.inf, np.nan]),
                              min_size=N, max_size=N))
    k = data.draw(st.integers(0, N + 3))
    sink = data.draw(st.integers(0, N + 2))
    window = data.draw(st.integers(0, N + 2))
    s = np.array(vals, np.float32)
    idx, cnt = oracle.select_topk(s, k, sink, window)
    got = idx[: int(cnt)]
    assert np.array_equal(got, oracle.select_topk_bruteforce(s, k, sink, window))
    assert np.array_equal(got, numpy_select(s, k, sink, window))


def test_select_invariants_medium(oracle):
    rng = np.random.default_rng(7)
    N, k, sink, window = 5000, 500, 16, 64
    s = np.round(rng.standard_normal((3, N)) * 20).astype(np.float32) / 4  # many exact ties
    idx, cnt = oracle.select_topk(s, k, sink, window)
    for u in range(3):
        got = idx[u, : cnt[u]]
        assert cnt[u] == sink + k + window
        assert np.all(np.diff(got) > 0)
        assert np.array_equal(got, numpy_select(s[u], k, sink, window))
        sel = np.zeros(N, bool)
        sel[got] = True
        cand = np.zeros(N, bool)
        cand[sink:N - window] = True
        inn, out = s[u][sel & cand], s[u][~sel & cand]
        assert inn.min() >= out.max()
        thr = inn.min()
        # among candidates tied at the threshold the kept ones come first by index
        tied = np.nonzero(cand & (s[u] == thr))[0]
        kept = sel[tied]
        assert np.all(kept[:-1] >= kept[1:])
        # invariance under positive scaling and shifts that are exact in fp32 (multiples of 1/4)
        idx2, _ = oracle.select_topk(s[u] * 4.0 + 3.0, k, sink, window)
        assert np.array_equal(idx2[: cnt[u]], got)


def test_select_degenerate_cases(oracle):
    N = 37
    s = np.full(N, 2.5, np.float32)
    idx, cnt = oracle.select_topk(s, 5, 3, 4)
    assert idx[:cnt].tolist() == [0, 1, 2] + [3, 4, 5, 6, 7] + [33, 34, 35, 36]
    idx, cnt = oracle.select_topk(s, N + 5, 0, 0)
    assert idx[:cnt].tolist() == list(range(N))
    idx, cnt = oracle.select_topk(s, 5, 30, 30)  # sink + window cover everything
    assert idx[:cnt].tolist() == list(range(N))
    idx, cnt = oracle.select_topk(s, 0, 2, 2)
    assert idx[:cnt].tolist() == [0, 1, 35, 36]
    t = np.array([np.nan, -np.inf, np.nan, -np.inf], np.float32)  # NaN ranks with -inf: index decides
    idx, cnt = oracle.select_topk(t, 2, 0, 0)
    assert idx[:cnt].tolist() == [0, 1]
    z = np.array([-0.0, 0.0, -0.0, 1.0], np.float32)  # -0 == +0
    idx, cnt = oracle.select_topk(z, 2, 0, 0)
    assert idx[:cnt].tolist() == [0, 3]


# ------------------------------------------------------------------------------ neighbours


def numpy_expand(idx, N, r):
    if len(idx) == 0:
        return np.zeros(0, np.int32)
    allp = (np.asarray(idx)[:, None] + np.arange(-r, r + 1)[None, :]).ravel()
    return np.unique(allp[(allp >= 0) & (allp < N)]).astype(np.int32)


def test_expand_golden(oracle):
    g = read_golden("expand_radius1.txt")
    idx = np.array(g["idx_in"], np.int32)[None]
    cnt = np.array([idx.shape[1]], np.int32)
    out, c = oracle.expand_neighbors(idx, cnt, int(g["N"][0]), int(g["radius"][0]))
    assert out[0, : c[0]].tolist() == [int(v) for v in g["idx_out"]]
    out, c = oracle.expand_neighbors(idx, cnt, int(g["N"][0]), 1, mode=1)
    assert out[0, : c[0]].tolist() == [int(v) for v in g["cluster_out"]]


@settings(max_examples=200, deadline=None)
@given(st.data())
def test_expand_vs_numpy_union(oracle, data):
    N = data.draw(st.integers(1, 60))
    r = data.draw(st.integers(0, 4))
    picks = sorted(data.draw(st.sets(st.integers(0, N - 1), max_size=N)))
    idx = np.array(picks + [0], np.int32)[None]  # one slot of padding beyond count
    cnt = np.array([len(picks)], np.int32)
    out, c = oracle.expand_neighbors(idx, cnt, N, r, cap_out=N)
    got = out[0, : c[0]]
    assert np.array_equal(got, numpy_expand(picks, N, r))
    assert set(picks) <= set(got.tolist())
    if r == 0:
        assert got.tolist() == picks


def test_expand_closed_forms(oracle):
    N, r = 1000, 2
    iso = np.arange(10, 900, 20, dtype=np.int32)  # gaps > 2r, away from the edges
    out, c = oracle.expand_neighbors(iso[None], np.array([len(iso)], np.int32), N, r)
    assert c[0] == (2 * r + 1) * len(iso)
    run = np.arange(400, 450, dtype=np.int32)  # one contiguous run of m -> m + 2r
    out, c = oracle.expand_neighbors(run[None], np.array([len(run)], np.int32), N, r)
    assert c[0] == len(run) + 2 * r and out[0, 0] == 398 and out[0, c[0] - 1] == 451
    edge = np.array([0, N - 1], np.int32)  # clipping at both ends
    out, c = oracle.expand_neighbors(edge[None], np.array([2], np.int32), N, r)
    assert out[0, : c[0]].tolist() == [0, 1, 2, N - 3, N - 2, N - 1]


def test_expand_cluster_mode_properties(oracle):
    """Cluster-aware reading: 2*count unique positions whenever the sweep does not run off the
    end; every selected token kept; added slots are exactly the first free ones after clusters."""
    rng = np.random.default_rng(8)
    N = 400
    for _ in range(20):
        picks = np.sort(rng.choice(N - 150, size=60, replace=False)).astype(np.int32)
        out, c = oracle.expand_neighbors(picks[None], np.array([60], np.int32), N, 1, mode=1)
        got = out[0, : c[0]]
        assert c[0] == 120 and np.all(np.diff(got) > 0)
        assert set(picks.tolist()) <= set(got.tolist())
        # independent check: simulate with a python set, filling the nearest free slot to the right
        taken = set(picks.tolist())
        ref = set(taken)
        for p in picks.tolist():
            j = p + 1
            while j in ref:
                j += 1
            ref.add(j)
        assert sorted(ref) == got.tolist()


# ------------------------------------------------------------------------------ attention


def numpy_attention(q64, K64, V64, idx, sm_scale):
    logit = sm_scale * (K64[idx] @ q64)
    w = np.exp(logit - logit.max())
    w /= w.sum()
    return w @ V64[idx], logit.max() + np.log(np.exp(logit - logit.max()).sum())


def test_attention_golden_two_tokens(oracle):
    g = read_golden("attn_two_tokens.txt")
    K = np.array([g["K0"], g["K1"], g["K2"], g["K3"]], np.float32)[None, None]
    V = np.array([g["V0"], g["V1"], g["V2"], g["V3"]], np.float32)[None, None]
    q = np.array(g["q"], np.float32)[None, None]
    idx = np.array(g["idx"], np.int32)[None, None]
    out, lse = oracle.sparse_decode_attn(q, K, V, idx, np.array([[2]], np.int32), "f32", 1.0)
    assert np.allclose(out[0, 0], g["out"], atol=1e-6)
    assert np.allclose(lse[0, 0], g["lse"][0], atol=1e-6)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_attention_full_budget_is_dense(oracle, dtype):
    """budget = N: the sparse path equals dense decode attention (two separately written
    routines and a library fp64 softmax)."""
    rng = np.random.default_rng(9)
    B, Hq, Hkv, N, D = 2, 4, 2, 70, 16
    if dtype == "f32":
        q = rng.standard_normal((B, Hq, D)).astype(np.float32)
        K = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
        V = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
        q64, K64, V64 = q.astype(np.float64), K.astype(np.float64), V.astype(np.float64)
    else:
        q, K, V = rand_bf16(rng, (B, Hq, D)), rand_bf16(rng, (B, Hkv, N, D)), rand_bf16(rng, (B, Hkv, N, D))
        q64, K64, V64 = oracle.bf16_to_f64(q), oracle.bf16_to_f64(K), oracle.bf16_to_f64(V)
    s = rng.standard_normal((B, Hq, N)).astype(np.float32)
    idx, cnt = oracle.select_topk(s, N, 0, 0)
    assert np.all(cnt == N)
    out, lse = oracle.sparse_decode_attn(q, K, V, idx, cnt, dtype, 0.25)
    dense = oracle.dense_decode_attn(q, K, V, dtype, 0.25)
    assert np.allclose(out, dense, rtol=1e-6, atol=1e-7)
    for b in range(B):
        for h in range(Hq):
            ref, ref_lse = numpy_attention(q64[b, h], K64[b, h // 2], V64[b, h // 2], np.arange(N), 0.25)
            assert np.allclose(out[b, h], ref, rtol=1e-6, atol=1e-7)
            assert np.allclose(lse[b, h], ref_lse, rtol=1e-6)


def test_attention_closed_forms(oracle):
    rng = np.random.default_rng(10)
    B, H, N, D = 1, 3, 64, 8
    q = rng.standard_normal((B, H, D)).astype(np.float32)
    K = rng.standard_normal((B, H, N, D)).astype(np.float32)
    V = rng.standard_normal((B, H, N, D)).astype(np.float32)
    idx = np.stack([np.sort(rng.choice(N, 20, replace=False)) for _ in range(H)])[None].astype(np.int32)
    cnt = np.full((B, H), 20, np.int32)
    # weights sum to one: V = 1 gives out = 1
    out, _ = oracle.sparse_decode_attn(q, K, np.ones_like(V), idx, cnt, "f32", 0.3)
    assert np.allclose(out, 1.0, atol=1e-6)
    # identical keys: uniform weights, out = mean of the selected V rows
    Ksame = np.broadcast_to(K[:, :, :1], K.shape).copy()
    out, lse = oracle.sparse_decode_attn(q, Ksame, V, idx, cnt, "f32", 0.3)
    for h in range(H):
        assert np.allclose(out[0, h], V[0, h, idx[0, h]].mean(axis=0), atol=1e-6)
        assert np.isclose(lse[0, h], 0.3 * float(q[0, h] @ Ksame[0, h, 0]) + math.log(20), rtol=1e-5, atol=1e-5)
    # one dominant logit: out = that V row
    Kdom = K.copy()
    for h in range(H):
        Kdom[0, h, idx[0, h, 7]] = 100.0 * q[0, h]
    out, _ = oracle.sparse_decode_attn(q, Kdom, V, idx, cnt, "f32", 1.0)
    for h in range(H):
        assert np.allclose(out[0, h], V[0, h, idx[0, h, 7]], atol=1e-6)
    # order of the list does not matter
    out_a, lse_a = oracle.sparse_decode_attn(q, K, V, idx, cnt, "f32", 0.3)
    out_b, lse_b = oracle.sparse_decode_attn(q, K, V, idx[:, :, ::-1].copy(), cnt, "f32", 0.3)
    assert np.allclose(out_a, out_b, atol=1e-6) and np.allclose(lse_a, lse_b, atol=1e-6)
    # entries beyond count are ignored; count = 0 gives zeros and -inf
    cnt0 = np.array([[0, 20, 5]], np.int32)
    out, lse = oracle.sparse_decode_attn(q, K, V, idx, cnt0, "f32", 0.3)
    assert not out[0, 0].any() and lse[0, 0] == -np.inf
    ref, _ = numpy_attention(q[0, 2].astype(np.float64), K[0, 2].astype(np.float64), V[0, 2].astype(np.float64),
                             idx[0, 2, :5], 0.3)
    assert np.allclose(out[0, 2], ref, atol=1e-6)


def test_attention_lse_merges_over_disjoint_parts(oracle):
    """Partial results over disjoint parts of the list combine to the result over the union."""
    rng = np.random.default_rng(11)
    B, H, N, D = 1, 2, 90, 8
    q = rng.standard_normal((B, H, D)).astype(np.float32)
    K = rng.standard_normal((B, H, N, D)).astype(np.float32) * 2
    V = rng.standard_normal((B, H, N, D)).astype(np.float32)
    full = np.broadcast_to(np.arange(N, dtype=np.int32), (B, H, N)).copy()
    o, l = oracle.sparse_decode_attn(q, K, V, full, np.full((B, H), N, np.int32), "f32", 0.4)
    o1, l1 = oracle.sparse_decode_attn(q, K, V, full[:, :, :37].copy(), np.full((B, H), 37, np.int32), "f32", 0.4)
    o2, l2 = oracle.sparse_decode_attn(q, K, V, full[:, :, 37:].copy(), np.full((B, H), N - 37, np.int32), "f32", 0.4)
    m = np.maximum(l1, l2)
    w1, w2 = np.exp(l1 - m), np.exp(l2 - m)
    merged = (o1 * w1[..., None] + o2 * w2[..., None]) / (w1 + w2)[..., None]
    assert np.allclose(merged, o, atol=1e-6)
    assert np.allclose(m + np.log(w1 + w2), l, atol=1e-6)


def test_attention_dropped_mass_bound(oracle):
    """|out_S - out_dense|_inf <= 2 (1 - mass_S) max|V| for any subset S."""
    rng = np.random.default_rng(12)
    B, H, N, D = 1, 4, 200, 16
    q = rng.standard_normal((B, H, D)).astype(np.float32)
    K = rng.standard_normal((B, H, N, D)).astype(np.float32)
    V = rng.standard_normal((B, H, N, D)).astype(np.float32)
    dense = oracle.dense_decode_attn(q, K, V, "f32", 0.5)
    logits = 0.5 * np.einsum("bhd,bhnd->bhn", q.astype(np.float64), K.astype(np.float64))
    idx, cnt = oracle.select_topk(logits.astype(np.float32), 40, 0, 0)
    out, _ = oracle.sparse_decode_attn(q, K, V, idx, cnt, "f32", 0.5)
    p = np.exp(logits - logits.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    for h in range(H):
        mass = p[0, h, idx[0, h, :40]].sum()
        assert np.abs(out[0, h] - dense[0, h]).max() <= 2 * (1 - mass) * np.abs(V[0, h]).max() + 1e-6


def test_attention_gqa_head_mapping(oracle):
    """Query head h reads KV head h // g: make each KV head's V constant = its index."""
    B, Hq, Hkv, N, D = 1, 8, 2, 10, 4
    rng = np.random.default_rng(13)
    q = rng.standard_normal((B, Hq, D)).astype(np.float32)
    K = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    V = np.zeros((B, Hkv, N, D), np.float32)
    V[:, 1] = 1.0
    idx = np.broadcast_to(np.arange(N, dtype=np.int32), (B, Hq, N)).copy()
    out, _ = oracle.sparse_decode_attn(q, K, V, idx, np.full((B, Hq), N, np.int32), "f32", 1.0)
    assert np.allclose(out[0, :4], 0.0) and np.allclose(out[0, 4:], 1.0)


# ------------------------------------------------------------------------------ interval driver


def test_attention_shared_list_serves_every_head(oracle):
    """Head-less selection: all heads of a batch element attend over one list; checked against a
    library fp64 softmax per head (each head with its own query and its KV group's rows)."""
    rng = np.random.default_rng(21)
    B, Hq, Hkv, N, D = 2, 6, 2, 50, 16
    q = rng.standard_normal((B, Hq, D)).astype(np.float32)
    K = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    idx = np.full((B, 20), -1, np.int32)
    cnt = np.array([13, 20], np.int32)
    for b in range(B):
        idx[b, :cnt[b]] = np.sort(rng.choice(N, cnt[b], replace=False))
    out, lse = oracle.sparse_decode_attn_shared(q, K, V, idx, cnt, "f32", 0.3)
    for b in range(B):
        for h in range(Hq):
            ref, ref_lse = numpy_attention(q[b, h].astype(np.float64), K[b, h // 3].astype(np.float64),
                                           V[b, h // 3].astype(np.float64), idx[b, :cnt[b]], 0.3)
            assert np.allclose(out[b, h], ref, rtol=1e-6, atol=1e-7)
            assert np.allclose(lse[b, h], ref_lse, rtol=1e-6)


def test_interval_driver_headless_equals_per_head_path_with_one_importance_head_repeated(oracle):
    """Head-less loop: one importance head, one list for all heads.  With that importance head
    (its keys and its query) handed to every head of the per-head loop, every head selects the
    same list, so both loops must attend over the same rows: equal outputs, step by step,
    through prediction and reuse steps with neighbours."""
    rng = np.random.default_rng(15)
    B, Hq, Hkv, N0, D, d, k, steps = 2, 4, 2, 90, 16, 8, 10, 7
    Ncap = N0 + steps
    K = rng.standard_normal((B, Hkv, Ncap, D)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, Ncap, D)).astype(np.float32)
    Kimp1 = rng.standard_normal((B, 1, Ncap, d)).astype(np.float32)
    qs = rng.standard_normal((steps, B, Hq, D)).astype(np.float32)
    qi1 = rng.standard_normal((steps, B, 1, d)).astype(np.float32)
    hl = oracle.IntervalDriver("f32", k, P=3, radius=1, sink=1, window=2, sm_scale=0.25, headless=True)
    ph = oracle.IntervalDriver("f32", k, P=3, radius=1, sink=1, window=2, sm_scale=0.25)
    for t in range(steps):
        N_t = N0 + t
        o1, l1, i1, c1 = hl.step(t, N_t, qs[t], qi1[t], K, V, Kimp1)
        o2, l2, i2, c2 = ph.step(t, N_t, qs[t], np.repeat(qi1[t], Hq, axis=1), K, V, np.repeat(Kimp1, Hkv, axis=1))
        assert i1.shape[1] == 1 and np.array_equal(np.repeat(c1, Hq, axis=1), c2)
        assert all(np.array_equal(i1[:, 0, : c1[:, 0].max()], i2[:, h, : c1[:, 0].max()]) for h in range(Hq))
        assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_interval_driver_reduces_to_per_step_path_and_set_sizes(oracle):
    rng = np.random.default_rng(14)
    B, Hq, Hkv, N0, D, d, k, steps = 1, 4, 2, 120, 16, 8, 12, 9
    Ncap = N0 + steps
    K = rng.standard_normal((B, Hkv, Ncap, D)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, Ncap, D)).astype(np.float32)
    W = (rng.standard_normal((1, D, d)) / 4).astype(np.float32)
    Kimp = oracle.project_keys(K, W, "f32")
    qs = rng.standard_normal((steps, B, Hq, D)).astype(np.float32)
    qis = rng.standard_normal((steps, B, Hq, d)).astype(np.float32)
    # P = 1, r = 0: identical to score -> select -> attend every step
    drv = oracle.IntervalDriver("f32", k, P=1, radius=0, sink=2, window=3, sm_scale=0.25)
    for t in range(steps):
        N_t = N0 + t
        out, lse, idx, cnt = drv.step(t, N_t, qs[t], qis[t], K, V, Kimp)
        _, idx2, cnt2, out2, lse2 = oracle.decode_step(qs[t], qis[t], K[:, :, :N_t], V[:, :, :N_t], Kimp[:, :, :N_t],
                                                       "f32", k, 2, 3, 0.25)
        assert np.array_equal(cnt, cnt2) and np.array_equal(idx, idx2)
        assert np.array_equal(out, out2) and np.array_equal(lse, lse2)
    # P = 4, r = 1: reuse steps attend on expand(sel) plus the tokens appended since the prediction
    drv = oracle.IntervalDriver("f32", k, P=4, radius=1, sm_scale=0.25)
    for t in range(steps):
        N_t = N0 + t
        out, lse, idx, cnt = drv.step(t, N_t, qs[t], qis[t], K, V, Kimp)
        if t % 4 == 0:
            assert np.all(cnt == k)
            pred_N, exp_cnt = N_t, drv.exp_cnt.copy()
            assert np.all(exp_cnt >= k) and np.all(exp_cnt <= 3 * k)
        else:
            assert np.array_equal(cnt, exp_cnt + (N_t - pred_N))
            for h in range(Hq):
                got = idx[0, h, : cnt[0, h]]
                assert np.all(np.diff(got) > 0) and got[-1] == N_t - 1


def test_interval_driver_expand_on_predict(oracle):
    """Sec. 3.4, neighbour fetching "per prediction step": with expand_on_predict the prediction
    step itself attends over the widened selection.  Pins: the list it uses is exactly
    expand(select(scores)); its length is |expand(sel)| (between k and (2r+1)k, and 2k for the
    cluster rule away from the end of the cache); with P = 1 every step is such a step and the
    output equals attention over the widened set computed by hand from the separate calls; the
    reuse steps are unchanged by the flag."""
    rng = np.random.default_rng(21)
    B, Hq, Hkv, N0, D, d, k, steps = 2, 4, 2, 150, 16, 8, 10, 7
    Ncap = N0 + steps
    K = rng.standard_normal((B, Hkv, Ncap, D)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, Ncap, D)).astype(np.float32)
    W = (rng.standard_normal((1, D, d)) / 4).astype(np.float32)
    Kimp = oracle.project_keys(K, W, "f32")
    qs = rng.standard_normal((steps, B, Hq, D)).astype(np.float32)
    qis = rng.standard_normal((steps, B, Hq, d)).astype(np.float32)
    for mode, radius in ((0, 1), (0, 2), (1, 1)):
        # P = 1: every step predicts, widens and attends over the widened set
        drv = oracle.IntervalDriver("f32", k, P=1, radius=radius, sink=1, window=2, sm_scale=0.25,
                                    expand_on_predict=True, mode=mode)
        for t in range(steps):
            N_t = N0 + t
            out, lse, idx, cnt = drv.step(t, N_t, qs[t], qis[t], K, V, Kimp)
            s = oracle.score(qis[t], Kimp[:, :, :N_t], "f32", 1.0)
            sel, scnt = oracle.select_topk(s, k, 1, 2)
            eidx, ecnt = oracle.expand_neighbors(sel, scnt, N_t, radius, mode=mode)
            assert np.array_equal(cnt, ecnt)
            m = np.arange(eidx.shape[-1])[None, None] < ecnt[..., None]
            assert np.array_equal(np.where(m, idx, -1), np.where(m, eidx, -1))
            out2, lse2 = oracle.sparse_decode_attn(qs[t], K[:, :, :N_t], V[:, :, :N_t], eidx, ecnt, "f32", 0.25)
            assert np.array_equal(out, out2) and np.array_equal(lse, lse2)
            n_sel = int(scnt[0, 0])
            if mode == 0:
                assert np.all(ecnt >= n_sel) and np.all(ecnt <= (2 * radius + 1) * n_sel)
            else:
                assert np.all(ecnt <= 2 * n_sel) and np.all(ecnt >= n_sel)
            # every selected token is in the widened list
            for b in range(B):
                for h in range(Hq):
                    assert set(sel[b, h, : scnt[b, h]]) <= set(idx[b, h, : cnt[b, h]])
    # P = 3: the flag changes the prediction steps only
    a = oracle.IntervalDriver("f32", k, P=3, radius=1, sm_scale=0.25, expand_on_predict=True)
    c = oracle.IntervalDriver("f32", k, P=3, radius=1, sm_scale=0.25, expand_on_predict=False)
    for t in range(steps):
        N_t = N0 + t
        oa, la, ia, ca = a.step(t, N_t, qs[t], qis[t], K, V, Kimp)
        oc, lc, ic, cc = c.step(t, N_t, qs[t], qis[t], K, V, Kimp)
        if t % 3 == 0:
            assert np.array_equal(ca, a.exp_cnt) and np.all(ca >= cc) and np.all(cc == k)
            assert not np.array_equal(oa, oc)  # more rows attended: a different output
        else:
            assert np.array_equal(ca, cc) and np.array_equal(oa, oc) and np.array_equal(la, lc)


def test_interval_driver_ring_layout(oracle):
    """Sec. 3.3 "Inference Setup" (Sink Buffer, Local Window ring, Important Buffer) as the
    driver's ring mode.  Pins: with P = 1 every step is decode attention over the widened
    selection made with the window that has filled so far (min(ring, t) tokens), computed here
    from the separate calls; with P > 1 a reuse step attends over exactly the plain driver's set
    minus the rows that have left the window since the prediction, and its length is
    |widened list| - W_pred + W_t."""
    rng = np.random.default_rng(33)
    B, Hq, Hkv, N0, D, d, k, steps, S, W = 1, 4, 2, 140, 16, 8, 9, 14, 3, 5
    Ncap = N0 + steps
    K = rng.standard_normal((B, Hkv, Ncap, D)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, Ncap, D)).astype(np.float32)
    Wm = (rng.standard_normal((1, D, d)) / 4).astype(np.float32)
    Kimp = oracle.project_keys(K, Wm, "f32")
    qs = rng.standard_normal((steps, B, Hq, D)).astype(np.float32)
    qis = rng.standard_normal((steps, B, Hq, d)).astype(np.float32)
    # P = 1: per-step path with the window that has filled so far, attention over the widened list
    drv = oracle.IntervalDriver("f32", k, P=1, radius=1, sink=S, sm_scale=0.25, ring=W)
    for t in range(steps):
        N_t = N0 + t
        out, lse, idx, cnt = drv.step(t, N_t, qs[t], qis[t], K, V, Kimp)
        s = oracle.score(qis[t], Kimp[:, :, :N_t], "f32", 1.0)
        sel, scnt = oracle.select_topk(s, k, S, min(W, t))
        assert np.all(scnt == S + k + min(W, t))
        eidx, ecnt = oracle.expand_neighbors(sel, scnt, N_t, 1)
        out2, lse2 = oracle.sparse_decode_attn(qs[t], K[:, :, :N_t], V[:, :, :N_t], eidx, ecnt, "f32", 0.25)
        assert np.array_equal(cnt, ecnt) and np.array_equal(out, out2) and np.array_equal(lse, lse2)
        # the unprojected tail is never looked at: garbage projected keys there change nothing
        Kbad = Kimp.copy()
        Kbad[:, :, N_t - min(W, t):] = 1e30
        drv2 = oracle.IntervalDriver("f32", k, P=1, radius=1, sink=S, sm_scale=0.25, ring=W)
        drv2.N0 = N0
        o3, _, _, c3 = drv2.step(0, N_t, qs[t], qis[t], K, V, Kbad)
        assert np.array_equal(o3, out) and np.array_equal(c3, cnt)
    # P = 4 <= W: reuse steps against the plain driver that is given the same window at the
    # prediction steps (fixed window W once the ring is full: compare from the first prediction
    # step with a full ring on)
    P = 4
    ring = oracle.IntervalDriver("f32", k, P=P, radius=1, sink=S, sm_scale=0.25, ring=W)
    plain = oracle.IntervalDriver("f32", k, P=P, radius=1, sink=S, window=W, sm_scale=0.25, expand_on_predict=True)
    for t in range(steps):
        N_t = N0 + t
        ri, rc = ring.lists(t, N_t, qis[t], Kimp)
        pi, pc = plain.lists(t, N_t, qis[t], Kimp)
        W_t = min(W, t)
        if t % P == 0:
            N_p, W_p, e_cnt = N_t, W_t, ring.exp_cnt.copy()
            assert np.array_equal(rc, e_cnt)
            for h in range(Hq):  # sink first, the window last
                assert np.array_equal(ri[0, h, :S], np.arange(S)) and np.array_equal(ri[0, h, rc[0, h] - W_t: rc[0, h]], np.arange(N_t - W_t, N_t))
        else:
            assert np.array_equal(rc, e_cnt - W_p + W_t)
        if t >= 2 * P:  # both drivers predicted with a full ring
            for h in range(Hq):
                a = set(ri[0, h, : rc[0, h]].tolist())
                b = set(pi[0, h, : pc[0, h]].tolist())
                assert a == b - set(range(N_p - W_p, N_t - W_t)), (t, h)
                assert len(a) == rc[0, h], "no position twice"


# --------------------------------------------------------------------------- buffer migration

def test_gather_kv_rows_are_copies_in_list_order(oracle):
    """Sec. 3.3 (Important Buffer): the migrated rows are the cache rows the list names, in list
    order, per query head through the GQA map; attention over the buffer (identity list) equals
    attention over the cache with the list."""
    rng = np.random.default_rng(3)
    B, Hq, Hkv, N, D = 2, 4, 2, 50, 8
    K = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    V = rng.standard_normal((B, Hkv, N, D)).astype(np.float32)
    q = rng.standard_normal((B, Hq, D)).astype(np.float32)
    idx = np.stack([np.stack([np.sort(rng.choice(N, 9, replace=False)) for _ in range(Hq)]) for _ in range(B)]).astype(np.int32)
    cnt = rng.integers(0, 10, size=(B, Hq)).astype(np.int32)
    Kb, Vb = oracle.gather_kv(K, V, idx, cnt, 12)
    for b in range(B):
        for h in range(Hq):
            for i in range(12):
                want = K[b, h // 2, idx[b, h, i]] if i < cnt[b, h] else np.zeros(D, np.float32)
                assert np.array_equal(Kb[b, h, i], want)
            assert np.array_equal(Vb[b, h, : cnt[b, h]], V[b, h // 2][idx[b, h, : cnt[b, h]]])
    ident = np.broadcast_to(np.arange(12, dtype=np.int32), (B, Hq, 12)).copy()
    o1, l1 = oracle.sparse_decode_attn(q, K, V, idx, cnt, "f32", 0.3)
    o2, l2 = oracle.sparse_decode_attn(q, Kb, Vb, ident, cnt, "f32", 0.3)  # buffers: one "kv head" per query head
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


# --------------------------------------------------------------------------- query predictor

def test_predict_queries_against_library_layers_and_closed_forms(oracle):
    """Sec. 3.1 "Query prediction": LN + two-layer MLP.  Pinned to torch's own layer_norm /
    linear / gelu in fp64, to the slot-outermost output layout, and to closed forms (a constant
    hidden state normalises to beta; zero first-layer weights give gelu(b1) for every row)."""
    import torch
    import torch.nn.functional as F

    rng = np.random.default_rng(7)
    B, E, hidden, G, Hq, Dimp = 3, 64, 24, 2, 4, 8
    h = rng.standard_normal((B, E)).astype(np.float32) * 3 + 1
    gamma = rng.standard_normal(E).astype(np.float32)
    beta = rng.standard_normal(E).astype(np.float32)
    W1 = rng.standard_normal((hidden, E)).astype(np.float32) / 8
    b1 = rng.standard_normal(hidden).astype(np.float32)
    W2 = rng.standard_normal((G * Hq * Dimp, hidden)).astype(np.float32) / 5
    b2 = rng.standard_normal(G * Hq * Dimp).astype(np.float32)
    q, z = oracle.predict_queries(h, gamma, beta, W1, b1, W2, b2, G, Hq, Dimp, "f32")
    t = lambda a: torch.from_numpy(a).double()
    x = F.layer_norm(t(h), (E,), t(gamma), t(beta), 1e-5)
    zt = F.gelu(F.linear(x, t(W1), t(b1)))
    yt = F.linear(zt, t(W2), t(b2)).reshape(B, G, Hq, Dimp).permute(1, 0, 2, 3)
    assert np.allclose(z, zt.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(q, yt.numpy().astype(np.float32), rtol=1e-6, atol=1e-6)
    # layout: output row (s*Hq + hq)*Dimp + j lands in q[s, b, hq, j]
    W2m = np.zeros_like(W2)
    b2m = np.arange(G * Hq * Dimp, dtype=np.float32)
    qm, _ = oracle.predict_queries(h, gamma, beta, W1, b1, W2m, b2m, G, Hq, Dimp, "f32")
    assert np.array_equal(qm[1, 2, 3], (1 * Hq + 3) * Dimp + np.arange(Dimp, dtype=np.float32))
    # constant hidden state: variance 0, LN gives beta exactly
    hc = np.full((1, E), 2.5, dtype=np.float32)
    _, zc = oracle.predict_queries(hc, gamma, beta, W1, b1, W2, b2, G, Hq, Dimp, "f32")
    pre = beta.astype(np.float64) @ W1.astype(np.float64).T + b1
    assert np.allclose(zc[0], 0.5 * pre * (1 + np.array([math.erf(v / math.sqrt(2)) for v in pre])), atol=1e-12)
    # bf16 storage: the stored value is the nearest bf16 of the fp64 result
    qb, _ = oracle.predict_queries(*(oracle.to_numpy(torch.from_numpy(a).bfloat16()) for a in (h, gamma, beta, W1, b1, W2, b2)),
                                   G, Hq, Dimp, "bf16")
    assert qb.dtype == np.uint16 and qb.shape == (G, B, Hq, Dimp)
    # ... checked value by value against torch's own fp64 layers on the bf16-rounded inputs and
    # torch's own fp64 -> bf16 conversion (round to nearest even): identical bit patterns, except
    # where the fp64 result lies within 1e-9 (relative) of the midpoint between two bf16 values
    # and the two fp64 evaluations may fall on different sides of it
    tb16 = lambda a: torch.from_numpy(a).bfloat16().double()
    xb = F.layer_norm(tb16(h), (E,), tb16(gamma), tb16(beta), 1e-5)
    yb = F.linear(F.gelu(F.linear(xb, tb16(W1), tb16(b1))), tb16(W2), tb16(b2))
    yb = yb.reshape(B, G, Hq, Dimp).permute(1, 0, 2, 3).contiguous()
    want = yb.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    diff = qb != want
    if diff.any():
        lo64 = np.minimum(oracle.bf16_to_f64(qb), oracle.bf16_to_f64(want))
        hi64 = np.maximum(oracle.bf16_to_f64(qb), oracle.bf16_to_f64(want))
        mid = 0.5 * (lo64 + hi64)
        assert np.all(np.abs(yb.numpy() - mid)[diff] <= 1e-9 * np.abs(mid)[diff]), "bf16 predictor output off by more than a tie"
    assert diff.mean() < 0.01
    # a planted mistake must show: a wrong slot order or a dropped bias changes most values
    assert (oracle.bf16_to_f64(qb) != oracle.bf16_to_f64(qb[::-1])).mean() > 0.9
