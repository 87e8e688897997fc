"""GPU parity at the full sizes of the five benchmark configurations, in the launch
configuration bench.py times (tb_decode_step on seeded synthetic inputs generated on the GPU).

The oracle is fed a host copy of exactly the bytes the GPU buffers hold.  Selection is checked
bit-exactly on every (batch, head) unit against the oracle run on the GPU's own scores; scores
and attention are checked on every unit of the single-sequence configurations and on at least
64 sampled units of the batched ones; the batched-depth configuration runs all of its 32 layers
and the interval configuration all of its 64 steps.  The bars are those of gpu_util.py."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from gpu_util import (DEV, assert_attention, assert_projection, assert_scores, np_of, projection_magnitude,
                      score_magnitude)
from paper_2503_07518_amd import binding as tb
from paper_2503_07518_amd import interval, workloads


def say(msg):
    print(f"[case] {msg}", flush=True)


def run_config(oracle, cfg, layer, sample_units=None, sink=0, window=0, projection_windows=2):
    """One prediction step of `cfg` on layer `layer`'s inputs.  sample_units: None = scores and
    attention on every (batch, head) unit, 0 = selection only, n = n sampled units."""
    data = workloads.make_layer(cfg, layer=layer, device=DEV)
    K, V, W = data["K"], data["V"], data["W"]
    q, q_imp = data["q"][0].contiguous(), data["q_imp"][0].contiguous()
    B, Hq, Hkv, N, D, g = cfg.B, cfg.Hq, cfg.Hkv, cfg.N, cfg.D, cfg.g
    Kimp = torch.zeros((B, Hkv, N, cfg.Dimp), dtype=K.dtype, device=DEV)
    d = tb.make_desc(N, Hq, K=K, V=V, Kimp=Kimp)
    tb.tb_project_keys(d, K, W, Kimp, 0, N)
    torch.cuda.synchronize()

    # projection parity on sampled (b, kv-head) units and row windows (before any rescaling)
    rng = np.random.default_rng(layer + 17)
    for _ in range(projection_windows):
        b, h = int(rng.integers(B)), int(rng.integers(Hkv))
        r0 = int(rng.integers(0, max(1, N - 2048)))
        r1 = min(N, r0 + 2048)
        Ks = np_of(K[b:b + 1, h:h + 1, r0:r1])
        ref = oracle.project_keys(Ks, np_of(W), cfg.dtype)
        got = np_of(Kimp[b:b + 1, h:h + 1, r0:r1])
        assert_projection(oracle, got, ref, projection_magnitude(oracle, Ks, np_of(W), cfg.dtype, 1), cfg.dtype)

    workloads.apply_kimp_row_scale(Kimp, data["kimp_row_scale"])
    need = tb.policy_count(N, cfg.k, sink, window)
    stride = (N + 3) // 4 * 4
    scores = torch.empty((B, Hq, stride), dtype=torch.float32, device=DEV)
    idx = torch.full((B, Hq, need), -7, dtype=torch.int32, device=DEV)
    cnt = torch.zeros((B, Hq), dtype=torch.int32, device=DEV)
    out = torch.empty((B, Hq, D), dtype=torch.float32, device=DEV)
    lse = torch.empty((B, Hq), dtype=torch.float32, device=DEV)
    ws = tb.new_workspace(tb.TB_OP_DECODE_STEP, d, need)
    for rep in range(2):  # second run on the same workspace must reproduce the first bit for bit
        tb.tb_decode_step(d, q_imp, Kimp, 1.0, q, K, V, cfg.k, sink, window, cfg.sm_scale, scores, idx, cnt, out, lse, ws)
        torch.cuda.synchronize()
        if rep == 0:
            first = (idx.clone(), cnt.clone(), out.clone(), lse.clone())
    assert torch.equal(first[0], idx) and torch.equal(first[1], cnt)
    assert torch.equal(first[2], out) and torch.equal(first[3], lse)

    s_np, idx_np, cnt_np = np_of(scores)[:, :, :N], np_of(idx), np_of(cnt)
    # selection: every unit, bit-exact, on the GPU's scores
    ridx, rcnt = oracle.select_topk(s_np, cfg.k, sink, window)
    assert np.array_equal(cnt_np, rcnt), "count"
    assert np.array_equal(idx_np, ridx), "selection"
    if sample_units == 0:
        return 0.0

    if sample_units is None:
        # scores and attention on every unit, whole arrays at once
        qi, Ki = np_of(q_imp), np_of(Kimp)
        assert_scores(s_np, oracle.score(qi, Ki, cfg.dtype, 1.0), score_magnitude(oracle, qi, Ki, cfg.dtype, g))
        ro, rl = oracle.sparse_decode_attn(np_of(q), np_of(K)[:, :, :N], np_of(V)[:, :, :N], idx_np, cnt_np, cfg.dtype,
                                           cfg.sm_scale)
        worst_attn = assert_attention(np_of(out), ro, cfg.dtype, np_of(lse), rl)
        units = [(b, h) for b in range(B) for h in range(Hq)]
    else:
        # sampled units (one unit = one query head with its KV head), without repetition
        pick = rng.choice(B * Hq, size=min(sample_units, B * Hq), replace=False)
        units = [(int(u) // Hq, int(u) % Hq) for u in pick]
        worst_attn = 0.0
        for b, h in units:
            hk = h // g
            qi = np_of(q_imp[b:b + 1, h:h + 1])
            Ki = np_of(Kimp[b:b + 1, hk:hk + 1])
            assert_scores(s_np[b:b + 1, h:h + 1], oracle.score(qi, Ki, cfg.dtype, 1.0),
                          score_magnitude(oracle, qi, Ki, cfg.dtype, 1), what=f"scores of unit ({b},{h})")
            ro, rl = oracle.sparse_decode_attn(np_of(q[b:b + 1, h:h + 1]), np_of(K[b:b + 1, hk:hk + 1, :N]),
                                               np_of(V[b:b + 1, hk:hk + 1, :N]), idx_np[b:b + 1, h:h + 1],
                                               cnt_np[b:b + 1, h:h + 1], cfg.dtype, cfg.sm_scale)
            worst_attn = max(worst_attn, assert_attention(np_of(out[b, h]), ro[0, 0], cfg.dtype, np_of(lse[b, h]),
                                                          rl[0, 0], what=f"attention of unit ({b},{h})"))
    # sanity (not parity): the planted heavy tokens are found by the importance scores
    if cfg.correlated_q_imp and not cfg.zipf_kimp:
        heavy = data["heavy"]
        hits = tot = 0
        for b, h in units:
            hk = h // g
            mine = heavy[b, hk][torch.arange(heavy.shape[-1]) % g == h % g].numpy()
            sel = set(idx_np[b, h, : cnt_np[b, h]].tolist())
            hits += sum(int(p) in sel for p in mine)
            tot += len(mine)
        assert hits / max(tot, 1) > 0.3, f"planted-token recall {hits}/{tot} (a random 10% pick would give 0.1)"
    return worst_attn


def test_c1_tiny_fp32(oracle):
    say("C1 tiny fp32, every unit")
    run_config(oracle, workloads.C1, 0)


def test_c2_llama3_8b_32k(oracle):
    say("C2 32k bf16, every unit")
    run_config(oracle, workloads.C2, 0)


def test_c2_with_sink_and_window(oracle):
    say("C2 with 128 sink + 256 window tokens, budget 8K total of 64K-style split, every unit")
    run_config(oracle, workloads.C2.scaled(k=3277 - 384), 1, sink=128, window=256)


def test_c3_batched_depth_all_layers(oracle):
    """All 32 layers (independent seeds per layer): the selection of every one of the 512 units
    of every layer bit-exact; projection, scores and attention on 8 sampled units of every
    fourth layer and of the last (9 layers, 72 units)."""
    cfg = workloads.C3
    for layer in range(cfg.layers):
        full = layer % 4 == 0 or layer == cfg.layers - 1
        say(f"C3 layer {layer}: selection on all units" + (", scores and attention on 8 units" if full else ""))
        run_config(oracle, cfg, layer, sample_units=8 if full else 0, projection_windows=2 if full else 0)
        torch.cuda.empty_cache()


def test_c5_long_context_zipf(oracle):
    say("C5 128k, 64 q heads, Zipf-scaled projected keys: selection on all 256 units, 64 units in full")
    run_config(oracle, workloads.C5, 0, sample_units=64)


def interval_case(oracle, cfg, steps, full_reuse_steps=None, expand_on_predict=False, mode=0):
    """The prediction-interval loop on the GPU against the oracle's driver on the same bytes.
    Every prediction step: selection and widened list bit-exact, attention on every unit.
    Every reuse step: the length of the list it attends over.  Reuse steps in
    `full_reuse_steps` (None: all of them): attention on every unit."""
    data = workloads.make_layer(cfg, device=DEV)
    K, V, W = data["K"], data["V"], data["W"]
    B, Hq, Hkv, N0, D = cfg.B, cfg.Hq, cfg.Hkv, cfg.N, cfg.D
    Ncap = K.shape[2]
    Kimp = torch.zeros((B, Hkv, Ncap, cfg.Dimp), dtype=K.dtype, device=DEV)
    tb.tb_project_keys(tb.make_desc(N0, Hq, K=K, V=V, Kimp=Kimp), K, W, Kimp, 0, N0)  # post-prefill state
    dec = interval.IntervalDecoder(K, V, W, Kimp, Hq, cfg.k, cfg.P, cfg.radius, sm_scale=cfg.sm_scale,
                                   expand_on_predict=expand_on_predict, mode=mode)
    outs = []
    for t in range(steps):
        out, lse = dec.step(t, N0 + t, data["q"][t].contiguous(), data["q_imp"][t].contiguous())
        if t % cfg.P == 0:
            rec = (out.clone(), lse.clone(), dec.idx.clone(), dec.cnt.clone(), dec.exp_idx.clone(), dec.exp_cnt.clone(),
                   dec.scores[:, :, : N0 + t].clone())
        else:
            rec = (out.clone(), lse.clone(), None, None, None, dec.exp_cnt.clone(), None)
        outs.append(rec)
    torch.cuda.synchronize()
    # oracle on the same bytes (the projected keys the GPU produced, rows appended included)
    Kn, Vn, Kin = np_of(K), np_of(V), np_of(Kimp)
    drv = oracle.IntervalDriver(cfg.dtype, cfg.k, cfg.P, cfg.radius, sm_scale=cfg.sm_scale,
                                expand_on_predict=expand_on_predict, mode=mode)
    n_full = 0
    for t in range(steps):
        N_t = N0 + t
        q_t, qi_t = np_of(data["q"][t]), np_of(data["q_imp"][t])
        if t % cfg.P == 0:
            say(f"  step {t}: prediction")
            ridx, rcnt = drv.lists(t, N_t, qi_t, Kin)
            # the selection is bit-exact against the oracle's rule on the GPU's own fp32 scores
            # (the oracle's fp64-accumulated scores may order near-ties differently: that set is
            # only required to agree almost everywhere); the expansion is bit-exact on the GPU's
            # selection, from which the oracle then continues
            g_idx, g_cnt = np_of(outs[t][2]), np_of(outs[t][3])
            s_idx, s_cnt = oracle.select_topk(np_of(outs[t][6]), cfg.k, 0, 0)
            assert np.array_equal(s_cnt, g_cnt) and np.array_equal(s_idx, g_idx[..., : s_idx.shape[-1]])
            e_idx, e_cnt = oracle.expand_neighbors(g_idx, g_cnt, N_t, cfg.radius, cap_out=outs[t][4].shape[-1], mode=mode)
            assert np.array_equal(np_of(outs[t][5]), e_cnt)
            mask = np.arange(e_idx.shape[-1])[None, None] < e_cnt[..., None]
            assert np.array_equal(np.where(mask, np_of(outs[t][4]), -1), np.where(mask, e_idx, -1))
            drv.exp_idx, drv.exp_cnt = e_idx, e_cnt  # continue the oracle from the GPU's selection
            u_idx, u_cnt = (e_idx, e_cnt) if expand_on_predict else (g_idx, g_cnt)
            ro, rl = oracle.sparse_decode_attn(q_t, Kn[:, :, :N_t], Vn[:, :, :N_t], u_idx, u_cnt, cfg.dtype, cfg.sm_scale)
            if not expand_on_predict:
                same = np.mean([len(set(ridx[b, h, :rcnt[b, h]]) & set(g_idx[b, h, :g_cnt[b, h]])) / max(1, rcnt[b, h])
                                for b in range(B) for h in range(0, Hq, 7)])
                assert same > 0.98, f"fp32 vs fp64 scores select nearly the same set ({same})"
        else:
            # the list of a reuse step: the stored widened list followed by the rows appended since
            u_idx, u_cnt = drv.lists(t, N_t, qi_t, Kin)
            assert np.array_equal(u_cnt, np_of(outs[t][5]) + (N_t - drv.N_pred)), f"step {t}: list length"
            if full_reuse_steps is not None and t not in full_reuse_steps:
                continue
            say(f"  step {t}: reuse, attention on every unit")
            ro, rl = oracle.sparse_decode_attn(q_t, Kn[:, :, :N_t], Vn[:, :, :N_t], u_idx, u_cnt, cfg.dtype, cfg.sm_scale)
            n_full += 1
        assert_attention(np_of(outs[t][0]), ro, cfg.dtype, np_of(outs[t][1]), rl, what=f"step {t}")
    return n_full


def test_interval_neighbors_small(oracle):
    say("interval + neighbours, scaled-down C4, every step checked")
    cfg = workloads.C4.scaled(name="C4_small", B=2, N=4096, k=256, steps=20, P=4, heavy_per_kv_head=8)
    interval_case(oracle, cfg, steps=20)


@pytest.mark.parametrize("mode", [0, 1])
def test_interval_expand_on_predict_small(oracle, mode):
    """The variant in which the prediction step itself attends over the widened selection
    (Sec. 3.4: neighbours are fetched per prediction step), both neighbour rules, every step."""
    say(f"interval, widened list on the prediction step too, neighbour rule {mode}, every step checked")
    cfg = workloads.C4.scaled(name="C4_small_eop", B=2, N=4096, k=256, steps=13, P=4, heavy_per_kv_head=8)
    interval_case(oracle, cfg, steps=13, expand_on_predict=True, mode=mode)


def test_c4_interval_neighbors_full_size(oracle):
    """All 64 steps at full size: the 8 prediction steps in full (selection, widened list,
    attention on all 128 units), the list length of all 56 reuse steps, and one reuse step per
    interval in full (a different offset into the interval each time)."""
    cfg = workloads.C4
    say(f"C4 full size: {cfg.N} tokens growing over {cfg.steps} steps, P={cfg.P}, r={cfg.radius}")
    full = {p + 1 + (p // cfg.P) % (cfg.P - 1) for p in range(0, cfg.steps, cfg.P)}
    n_full = interval_case(oracle, cfg, steps=cfg.steps, full_reuse_steps=full)
    assert n_full == cfg.steps // cfg.P


def test_producer_group_batched_scoring_and_selection(oracle):
    """Sec. 3.3 batches the predictor operations of a producer's consumer layers: the projected-key
    caches of 4 layers stacked along the batch axis of one descriptor, one scoring and one
    selection call for all of them, then one attention call per layer on its slice of the lists.
    Same lists and outputs as per-layer calls, and the lists are the oracle's."""
    say("producer group: 4 layers scored and selected in one call each (C2 shape, N = 32768)")
    cfg = workloads.C2
    G, B, Hq, N, D = 4, cfg.B, cfg.Hq, cfg.N, cfg.D
    layers = []
    for layer in range(G):
        data = workloads.make_layer(cfg, layer=layer, device=DEV)
        K, V = data["K"], data["V"]
        Kimp = torch.zeros((B, cfg.Hkv, N, cfg.Dimp), dtype=K.dtype, device=DEV)
        d = tb.make_desc(N, Hq, K=K, V=V, Kimp=Kimp)
        tb.tb_project_keys(d, K, data["W"], Kimp, 0, N)
        workloads.apply_kimp_row_scale(Kimp, data["kimp_row_scale"])
        layers.append((d, K, V, Kimp, data["q"][0].contiguous(), data["q_imp"][0].contiguous()))
    need = tb.policy_count(N, cfg.k, 0, 0)
    stride = (N + 3) // 4 * 4
    gKimp = torch.cat([l[3] for l in layers], dim=0)
    gq_imp = torch.cat([l[5] for l in layers], dim=0)
    gd = tb.make_desc(N, Hq, Kimp=gKimp)
    gscores = torch.empty((G * B, Hq, stride), dtype=torch.float32, device=DEV)
    gidx = torch.full((G * B, Hq, need), -7, dtype=torch.int32, device=DEV)
    gcnt = torch.zeros((G * B, Hq), dtype=torch.int32, device=DEV)
    tb.tb_score(gd, gq_imp, gKimp, 1.0, gscores)
    tb.tb_select_topk(gd, gscores, cfg.k, 0, 0, gidx, gcnt, tb.new_workspace(tb.TB_OP_SELECT, gd, need))
    torch.cuda.synchronize()
    ridx, rcnt = oracle.select_topk(np_of(gscores)[:, :, :N], cfg.k, 0, 0)
    assert np.array_equal(np_of(gcnt), rcnt) and np.array_equal(np_of(gidx)[:, :, :need], ridx[:, :, :need])
    for li, (d, K, V, Kimp, q, q_imp) in enumerate(layers):
        scores = torch.empty((B, Hq, stride), dtype=torch.float32, device=DEV)
        idx = torch.full((B, Hq, need), -7, dtype=torch.int32, device=DEV)
        cnt = torch.zeros((B, Hq), dtype=torch.int32, device=DEV)
        out = torch.empty((B, Hq, D), dtype=torch.float32, device=DEV)
        lse = torch.empty((B, Hq), dtype=torch.float32, device=DEV)
        ws = tb.new_workspace(tb.TB_OP_DECODE_STEP, d, need)
        tb.tb_decode_step(d, q_imp, Kimp, 1.0, q, K, V, cfg.k, 0, 0, cfg.sm_scale, scores, idx, cnt, out, lse, ws)
        out2 = torch.empty_like(out)
        lse2 = torch.empty_like(lse)
        tb.tb_sparse_decode_attn(d, q, K, V, gidx[li * B:(li + 1) * B], gcnt[li * B:(li + 1) * B], need, cfg.sm_scale, out2, lse2, ws)
        torch.cuda.synchronize()
        assert torch.equal(scores, gscores[li * B:(li + 1) * B]), f"layer {li}: scores of the batched call differ"
        assert torch.equal(idx, gidx[li * B:(li + 1) * B]) and torch.equal(cnt, gcnt[li * B:(li + 1) * B])
        assert torch.equal(out, out2) and torch.equal(lse, lse2), f"layer {li}: attention on the batched lists differs"
