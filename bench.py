#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

A step is one prediction step of one layer: importance scoring over the whole projected-key
cache, top-k selection per query head, decode attention over the gathered K/V rows
(tb_decode_step).  Inputs are seeded synthetic tensors already resident in HBM; the step
cycles through several distinct copies of the layer's buffers so that no step finds its cache
in the 256 MB last-level cache.

Prints ONE JSON line; its main fields:
  value          microseconds per step (lower is better)
  roofline       achieved HBM GB/s of the dominant kernel (gather attention) against 8 TB/s,
                 timed live with events on the launch stream
  cpu_baseline   the CPU oracle timed on the same bytes on the host cores of this machine
"""
from __future__ import annotations

import argparse
import types
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X datasheet HBM3E bandwidth
PRODUCER_GROUP = 4       # consumer layers per producer layer (Sec. 4, predictor architecture)
GRAPH_MIN_STEPS = 32     # steps that one HIP graph of the timed loop holds at least: the layers of the modelled network



def measured_traffic(cfg_name, kernel, what="decode_step"):
    """HBM bytes per launch of `kernel` on this configuration, as measured with rocprofv3 PMC
    counters (FETCH_SIZE + WRITE_SIZE, each scaled by what the same counter reads for a 256 MiB
    device copy): read from the summary of those runs under profiles/, None when there is none."""
    path = os.path.join(ROOT, "profiles", f"{what}_{cfg_name.split('_')[0]}_hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel:
                return float(f[2])
    except OSError:
        pass
    return None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", default="C2_llama3_8b_32k")
    ap.add_argument("--copies", type=int, default=0, help="rotating buffer copies (0: enough for >= 1 GiB)")
    ap.add_argument("--no-graph", action="store_true", help="launch every step eagerly instead of replaying a HIP graph")
    ap.add_argument("--kv-layout", choices=("separate", "interleaved"), default="separate",
                    help="K and V as two arrays, or one array [B][Hkv][N][2][D] (a token's K and V rows adjacent)")
    ap.add_argument("--kv-host", action="store_true",
                    help="offloaded cache: K and V in pinned host memory, projected keys on the GPU; "
                         "only the selected rows cross the host link")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-group", action="store_true", help="skip the producer-group (batched scoring and selection of 4 layers) timing")
    ap.add_argument("--no-headless", action="store_true",
                    help="skip the timings of the head-less variant (keeps a profile of the per-head kernels clean)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--only-reuse-step", action="store_true",
                    help="interval configurations: run the loop once, then time (and, under a profiler, expose) only "
                         "the attention launch of a reuse step; prints that record and exits")
    return ap.parse_args()


class LayerBuffers:
    """One copy of a layer's inputs and outputs in HBM."""

    def __init__(self, cfg, seed, tb, workloads, torch, kv_layout="separate", kv_host=False, layer=0):
        data = workloads.make_layer(cfg, layer=layer, seed=seed, device="cuda")
        self.K, self.V, self.W = data["K"], data["V"], data["W"]
        if kv_layout == "interleaved":
            kv = torch.stack((self.K, self.V), dim=3)  # [B][Hkv][N][2][D]
            self.K, self.V = kv[:, :, :, 0, :], kv[:, :, :, 1, :]
        self.q = data["q"][0].contiguous()
        self.q_imp = data["q_imp"][0].contiguous()
        B, Hq, Hkv, N, D = cfg.B, cfg.Hq, cfg.Hkv, cfg.N, cfg.D
        self.Kimp = torch.zeros((B, Hkv, N, cfg.Dimp), dtype=self.K.dtype, device="cuda")
        self.desc = tb.make_desc(N, Hq, K=self.K, V=self.V, Kimp=self.Kimp)
        tb.tb_project_keys(self.desc, self.K, self.W, self.Kimp, 0, N)
        workloads.apply_kimp_row_scale(self.Kimp, data["kimp_row_scale"])
        self.need = tb.policy_count(N, cfg.k, cfg.sink, cfg.window)
        self.scores = torch.empty((B, Hq, (N + 3) // 4 * 4), dtype=torch.float32, device="cuda")
        self.idx = torch.zeros((B, Hq, self.need), dtype=torch.int32, device="cuda")
        self.cnt = torch.zeros((B, Hq), dtype=torch.int32, device="cuda")
        self.out = torch.empty((B, Hq, D), dtype=torch.float32, device="cuda")
        self.lse = torch.empty((B, Hq), dtype=torch.float32, device="cuda")
        self.ws = tb.new_workspace(tb.TB_OP_DECODE_STEP, self.desc, self.need)
        if kv_host:  # the projected keys are made; now the cache itself moves to pinned host memory
            torch.cuda.synchronize()
            self.K = torch.empty(self.K.shape, dtype=self.K.dtype, pin_memory=True).copy_(self.K)
            self.V = torch.empty(self.V.shape, dtype=self.V.dtype, pin_memory=True).copy_(self.V)
            self.desc = tb.make_desc(N, Hq, K=self.K, V=self.V, Kimp=self.Kimp)
        # target of the timed batched projection (the cache that the step reads stays as it is)
        self.Kimp_bulk = torch.empty_like(self.Kimp)
        self.desc_bulk = tb.make_desc(N, Hq, K=self.K, V=self.V, Kimp=self.Kimp_bulk)

    def nbytes(self):
        return sum(t.numel() * t.element_size() for t in (self.K, self.V, self.Kimp, self.scores, self.idx))


def time_interval_loop(cfg, tb, workloads, torch, replays=5, buffered=False, mode=0, reuse_launches=20,
                       ring=0, sink=None, window=None, expand_on_predict=False):
    """The prediction-interval loop of the config (cfg.steps decode steps, a prediction every
    cfg.P steps, neighbours of radius cfg.radius on the steps in between) as one HIP graph:
    mean time per step, and the rows that attention gathers on the two kinds of step.
    buffered: the widened selection is migrated into per-query-head buffers on prediction steps
    (the paper's Important Buffer) and the other steps read the buffers instead of gathering."""
    from paper_2503_07518_amd import interval

    data = workloads.make_layer(cfg, layer=1, seed=0, device="cuda")
    K, V, W = data["K"], data["V"], data["W"]
    Kimp = torch.zeros((cfg.B, cfg.Hkv, K.shape[2], cfg.Dimp), dtype=K.dtype, device="cuda")
    tb.tb_project_keys(tb.make_desc(cfg.N, cfg.Hq, K=K, V=V, Kimp=Kimp), K, W, Kimp, 0, cfg.N)
    qs = [data["q"][t].contiguous() for t in range(cfg.steps)]
    qis = [data["q_imp"][t].contiguous() for t in range(cfg.steps)]

    sink = cfg.sink if sink is None else sink
    window = cfg.window if window is None else window
    if ring:
        # the paper's three physical buffers (sink, local-window ring, important buffer) with the
        # projection deferred to the wraps of the ring
        dec = interval.RingLayoutDecoder(K, V, W, Kimp, cfg.Hq, cfg.k, cfg.P, cfg.radius, ring, sink=sink,
                                         sm_scale=cfg.sm_scale, mode=mode)
    else:
        dec = interval.IntervalDecoder(K, V, W, Kimp, cfg.Hq, cfg.k, cfg.P, cfg.radius, sink=sink, window=window,
                                       sm_scale=cfg.sm_scale, buffered=buffered, mode=mode,
                                       expand_on_predict=expand_on_predict)

    def loop():
        if not ring:
            dec.N_pred = dec.projected_upto = None  # the cache is back at its post-prefill length
        for t in range(cfg.steps):
            dec.step(t, cfg.N + t, qs[t], qis[t])

    loop()  # eager once: first touch, and the list sizes for the byte counts
    torch.cuda.synchronize()
    sel_rows = int(dec.cnt.sum().item())
    exp_rows = int(dec.exp_cnt.sum().item())
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            loop()
    torch.cuda.current_stream().wait_stream(side)
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    cur = torch.cuda.current_stream()
    e0.record(cur)
    for _ in range(replays):
        g.replay()
    e1.record(cur)
    torch.cuda.synchronize()
    us_loop = e0.elapsed_time(e1) * 1e3 / replays
    n_pred = -(-cfg.steps // cfg.P)
    if ring:
        return {"attention_reads": "sink buffer + local-window ring + important buffer", "ring": ring, "sink": sink,
                "steps": cfg.steps, "P": cfg.P, "radius": cfg.radius, "prediction_steps": n_pred,
                "batched_projections": dec.projections // 2,  # (the loop ran twice on the host: eagerly and under capture)
                "us_per_step_mean": round(us_loop / cfg.steps, 3), "us_loop": round(us_loop, 1),
                "rows_in_important_buffers": int(dec.imp_cnt.sum().item())}
    # one reuse step on its own (attention over the widened list + the rows appended since)
    t_last = cfg.steps - 1
    N_last = cfg.N + t_last
    desc = tb.make_desc(N_last, cfg.Hq, K=K, V=V, Kimp=Kimp)
    e0.record(cur)
    for _ in range(reuse_launches):
        if buffered:
            tb.tb_buffered_decode_attn(desc, qs[t_last], dec.Kbuf, dec.Vbuf, dec.exp_cnt, dec.exp_cap, K, V,
                                       cfg.sm_scale, dec.out, dec.lse, dec.ws, tail_begin=dec.N_pred, tail_end=N_last)
        else:
            tb.tb_sparse_decode_attn(desc, qs[t_last], K, V, dec.exp_idx, dec.exp_cnt, dec.exp_cap, cfg.sm_scale,
                                     dec.out, dec.lse, dec.ws, tail_begin=dec.N_pred, tail_end=N_last)
    e1.record(cur)
    torch.cuda.synchronize()
    us_reuse = e0.elapsed_time(e1) * 1e3 / reuse_launches
    reuse_bytes = (exp_rows + cfg.B * cfg.Hq * (N_last - dec.N_pred)) * 2 * cfg.D * cfg.elt_bytes
    us_migrate = None
    if buffered:
        e0.record(cur)
        for _ in range(10):
            tb.tb_gather_kv(desc, K, V, dec.exp_idx, dec.exp_cnt, dec.exp_cap, dec.Kbuf, dec.Vbuf)
        e1.record(cur)
        torch.cuda.synchronize()
        us_migrate = e0.elapsed_time(e1) * 1e3 / 10
    return {
        "attention_reads": "migrated buffers" if buffered else "cache rows (fused gather)",
        "neighbours": "union of +-radius" if mode == 0 else "cluster-aware (one free position per selected token)",
        "migration_us": None if us_migrate is None else round(us_migrate, 3),
        "steps": cfg.steps, "P": cfg.P, "radius": cfg.radius, "prediction_steps": n_pred,
        "reuse_steps": cfg.steps - n_pred, "us_per_step_mean": round(us_loop / cfg.steps, 3),
        "us_loop": round(us_loop, 1),
        "rows_gathered_last_prediction_step": sel_rows, "rows_in_widened_list": exp_rows,
        "reuse_step": {"us": round(us_reuse, 3), "algorithmic_bytes": reuse_bytes,
                       "achieved": round(reuse_bytes / us_reuse / 1e3, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                       "frac": round(reuse_bytes / us_reuse / 1e3 / HBM_PEAK_GBPS, 4)},
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2503_07518_amd import binding as tb
    from paper_2503_07518_amd import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    tb.load_library()
    cfg = {**workloads.CONFIGS, **workloads.EXTRA_CONFIGS}[args.config]
    if args.only_reuse_step:
        assert cfg.P > 1, "--only-reuse-step needs a configuration with a prediction interval"
        rec = time_interval_loop(cfg, tb, workloads, torch, replays=1, reuse_launches=40)
        rec["reuse_step"]["traffic"] = measured_traffic(cfg.name, "attn_kernel", what="reuse_step")
        print(json.dumps({"metric": "reuse_step_attention_latency", "value": rec["reuse_step"]["us"], "unit": "us/step",
                          "n_gpus": 1, "config": {"workload": cfg.name + " (reuse step)"}, "interval_loop": rec}))
        return

    # ---- buffers: enough distinct copies that a step never finds its data in the last-level cache
    probe = LayerBuffers(cfg, 0, tb, workloads, torch, args.kv_layout, args.kv_host)
    copies = args.copies or (2 if args.kv_host else max(2, -(-(1 << 30) // probe.nbytes())))
    bufs = [probe] + [LayerBuffers(cfg, s, tb, workloads, torch, args.kv_layout, args.kv_host)
                      for s in range(1, copies)]
    torch.cuda.synchronize()

    def step(b):
        tb.tb_decode_step(b.desc, b.q_imp, b.Kimp, 1.0, b.q, b.K, b.V, cfg.k, cfg.sink, cfg.window, cfg.sm_scale,
                          b.scores, b.idx, b.cnt, b.out, b.lse, b.ws)

    def stage_score(b):
        tb.tb_score(b.desc, b.q_imp, b.Kimp, 1.0, b.scores)

    def stage_select(b):
        tb.tb_select_topk(b.desc, b.scores, cfg.k, cfg.sink, cfg.window, b.idx, b.cnt, b.ws)

    def stage_attn(b):
        tb.tb_sparse_decode_attn(b.desc, b.q, b.K, b.V, b.idx, b.cnt, b.need, cfg.sm_scale, b.out, b.lse, b.ws)

    def stage_project_append(b):
        tb.tb_project_keys(b.desc, b.K, b.W, b.Kimp, cfg.N - 1, cfg.N)

    def stage_project_bulk(b):
        tb.tb_project_keys(b.desc_bulk, b.K, b.W, b.Kimp_bulk, 0, cfg.N)

    # a plain device copy of known size: the reference dispatch that HBM byte counters of a
    # profiler run are scaled by (256 MiB read + 256 MiB written)
    cal_src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        cal_dst.copy_(cal_src)
    # the same copy timed: what a plain streaming kernel reaches on this machine, next to the 8 TB/s of the data sheet
    torch.cuda.synchronize()
    ce0, ce1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ce0.record()
    for _ in range(5):
        cal_dst.copy_(cal_src)
    ce1.record()
    torch.cuda.synchronize()
    copy_gbps = 5 * 2 * (256 << 20) / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    del cal_src, cal_dst
    # a plain 128-bit read stream over 1 GiB: the read ceiling of this machine for bandwidth-bound
    # kernels, quoted next to the data-sheet figure
    rd_src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    rd_sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    rd_src.zero_()
    for _ in range(2):
        tb.tb_read_stream_probe(rd_src, rd_sink)
    torch.cuda.synchronize()
    ce0.record()
    for _ in range(5):
        tb.tb_read_stream_probe(rd_src, rd_sink)
    ce1.record()
    torch.cuda.synchronize()
    read_gbps = 5 * (1 << 30) / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    del rd_src, rd_sink

    for b in bufs:  # first touch, also fills idx/cnt for the per-stage timings
        step(b)
    torch.cuda.synchronize()
    selected_rows = int(sum(int(b.cnt.sum().item()) for b in bufs) / len(bufs))

    stream = torch.cuda.current_stream()

    def time_eager(fn, n_steps, warmup):
        for i in range(warmup):
            fn(bufs[i % copies])
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(n_steps):
            fn(bufs[i % copies])
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n_steps  # us per call

    # calls per graph: one per buffer copy, repeated until the graph holds at least as many steps
    # as the model has layers (a serving loop captures a whole forward pass: one step per layer)
    per_graph = copies * max(1, -(-GRAPH_MIN_STEPS // copies))

    def time_graph(fn, n_steps, warmup):
        """Replay a HIP graph of `per_graph` calls that go round the buffer copies.  Exactly n_steps
        calls are timed: whole replays of that graph plus one replay of a shorter graph for the
        remainder."""
        def capture(n_calls):
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    for i in range(n_calls):
                        fn(bufs[i % copies])
            torch.cuda.current_stream().wait_stream(side)
            return g

        reps, rest = divmod(n_steps, per_graph)
        g_full = capture(per_graph) if reps or warmup >= per_graph else None
        g_rest = capture(rest) if rest else None
        for _ in range(warmup // per_graph):
            g_full.replay()
        if warmup % per_graph:
            capture(warmup % per_graph).replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        cur = torch.cuda.current_stream()
        e0.record(cur)
        for _ in range(reps):
            g_full.replay()
        if g_rest is not None:
            g_rest.replay()
        e1.record(cur)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / n_steps, n_steps

    use_graph = not args.no_graph
    steps_done = args.steps
    t_wall0 = time.perf_counter()
    if use_graph:
        try:
            us_step, steps_done = time_graph(step, args.steps, args.warmup)
        except Exception as e:  # graph capture unavailable: fall back to eager launches, say so
            print(f"[bench] graph replay failed ({e}); timing eager launches", file=sys.stderr)
            use_graph = False
    if not use_graph:
        us_step = time_eager(step, args.steps, args.warmup)
    wall_s = time.perf_counter() - t_wall0

    # spread of the step time: every replay of the full graph timed on its own
    pct = None
    if use_graph:
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for i in range(per_graph):
                    step(bufs[i % copies])
        torch.cuda.current_stream().wait_stream(side)
        n_rep = max(20, min(200, args.steps // per_graph))
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_rep + 1)]
        g.replay()
        evs[0].record()
        for i in range(n_rep):
            g.replay()
            evs[i + 1].record()
        torch.cuda.synchronize()
        per = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 / per_graph for i in range(n_rep))
        pct = {"p10": round(per[n_rep // 10], 3), "median": round(per[n_rep // 2], 3), "p90": round(per[(n_rep * 9) // 10], 3),
               "replays": n_rep, "steps_per_replay": per_graph}

    timer = (lambda fn: time_graph(fn, args.steps, args.warmup)[0]) if use_graph else (
        lambda fn: time_eager(fn, args.steps, args.warmup))
    us_score = timer(stage_score)
    us_select = timer(stage_select)
    us_attn = timer(stage_attn)

    # The attention kernel as it runs inside the step: step time minus the time of the step
    # without it.  Launched back to back on its own (us_attn) it finds part of its rows in the
    # 256 MB last-level cache again when the working set of all buffer copies is small enough
    # (13.7 against 14.4 us on C2, 77 against 92 us on C3 under the profiler); inside the step the
    # scoring pass streams the projected keys through that cache in between.
    def stage_score_select(b):
        stage_score(b)
        stage_select(b)

    us_pre = timer(stage_score_select)
    us_attn_step = max(us_step - us_pre, 1e-3)  # (a nonsensical difference is flagged as roofline.suspect)
    us_proj = timer(stage_project_append)
    # (with the cache in host memory the batched projection would time the host link, not the kernel)
    us_proj_bulk = timer(stage_project_bulk) if not args.kv_host else float("inf")
    us_step_eager = time_eager(step, args.steps, args.warmup) if use_graph else us_step

    # query predictor of a producer layer (LN + two-layer MLP, hidden 512, 4 consumer slots; runs
    # once per 4 layers, before the steps of its consumer layers): random weights, speed only
    E, hidden, G = cfg.Hq * cfg.D, 512, 4
    td = probe.K.dtype
    pw = {
        "h": torch.randn((cfg.B, E), device="cuda").to(td), "gamma": torch.ones(E, device="cuda").to(td),
        "beta": torch.zeros(E, device="cuda").to(td), "W1": (torch.randn((hidden, E), device="cuda") * E ** -0.5).to(td),
        "b1": torch.zeros(hidden, device="cuda").to(td),
        "W2": (torch.randn((G * cfg.Hq * cfg.Dimp, hidden), device="cuda") * hidden ** -0.5).to(td),
        "b2": torch.zeros(G * cfg.Hq * cfg.Dimp, device="cuda").to(td),
        "z": torch.empty((cfg.B, hidden), dtype=torch.float32, device="cuda"),
        "xln": torch.empty((cfg.B, E), dtype=torch.float32, device="cuda"),
        "q": torch.empty((G, cfg.B, cfg.Hq, cfg.Dimp), dtype=td, device="cuda"),
    }

    def stage_predict(b):
        tb.tb_predict_queries(pw["h"], pw["gamma"], pw["beta"], pw["W1"], pw["b1"], pw["W2"], pw["b2"], G, cfg.Hq,
                              cfg.Dimp, pw["z"], pw["xln"], pw["q"])

    us_predict = timer(stage_predict)
    bytes_predict = (pw["W1"].numel() + pw["W2"].numel()) * cfg.elt_bytes

    us_hl_step = us_hl_attn = None
    if not args.no_headless:
        # head-less variant: one importance head per layer (here the first KV head's projected keys),
        # one token list per batch element that every attention head reads
        for b in bufs:
            b.hl_Kimp = b.Kimp[:, :1]
            b.hl_qimp = b.q_imp[:, :1].contiguous()
            b.hl_desc = tb.make_desc(cfg.N, 1, Kimp=b.hl_Kimp)
            b.hl_scores = torch.empty((cfg.B, 1, (cfg.N + 3) // 4 * 4), dtype=torch.float32, device="cuda")
            b.hl_idx = torch.zeros((cfg.B, 1, b.need), dtype=torch.int32, device="cuda")
            b.hl_cnt = torch.zeros((cfg.B,), dtype=torch.int32, device="cuda")
            b.hl_ws = tb.new_workspace(tb.TB_OP_SELECT, b.hl_desc, b.need)

        def headless_attn(b):
            tb.tb_sparse_decode_attn_shared(b.desc, b.q, b.K, b.V, b.hl_idx, b.hl_cnt, b.need, cfg.sm_scale, b.out,
                                            b.lse, b.ws)

        def headless_step(b):
            tb.tb_score(b.hl_desc, b.hl_qimp, b.hl_Kimp, 1.0, b.hl_scores)
            tb.tb_select_topk(b.hl_desc, b.hl_scores, cfg.k, cfg.sink, cfg.window, b.hl_idx, b.hl_cnt, b.hl_ws)
            headless_attn(b)

        for b in bufs:
            headless_step(b)
        torch.cuda.synchronize()
        us_hl_step = timer(headless_step)
        us_hl_attn = timer(headless_attn)
        step(bufs[0])       # restore copy 0's per-head outputs, which the parity check reads
        torch.cuda.synchronize()

    # Producer groups (Sec. 3.3, batching of the predictor operations): the importance queries of
    # the G = 4 consumer layers of a producer are known together, so their scoring and selection
    # run as one batched call each (the layers' projected-key caches stacked along the batch axis
    # of one descriptor), followed by the layers' attention calls one after the other.
    group = None
    if use_graph and not args.kv_host and not args.no_group and copies >= 2 and cfg.B * PRODUCER_GROUP * probe.nbytes() < (24 << 30):
        G4 = PRODUCER_GROUP
        n_groups = max(2, -(-copies // G4))
        layers = list(bufs)
        while len(layers) < n_groups * G4:  # whole groups of distinct layers
            layers.append(LayerBuffers(cfg, len(layers), tb, workloads, torch, args.kv_layout, False))
        groups = []
        for gi in range(n_groups):
            ls = layers[gi * G4:(gi + 1) * G4]
            gb = types.SimpleNamespace(layers=ls)
            gb.Kimp = torch.cat([b.Kimp for b in ls], dim=0)  # [G*B][Hkv][N][d']
            gb.q_imp = torch.cat([b.q_imp for b in ls], dim=0)
            gb.desc = tb.make_desc(cfg.N, cfg.Hq, Kimp=gb.Kimp)
            gb.scores = torch.empty((G4 * cfg.B, cfg.Hq, (cfg.N + 3) // 4 * 4), dtype=torch.float32, device="cuda")
            gb.idx = torch.zeros((G4 * cfg.B, cfg.Hq, probe.need), dtype=torch.int32, device="cuda")
            gb.cnt = torch.zeros((G4 * cfg.B, cfg.Hq), dtype=torch.int32, device="cuda")
            gb.ws = tb.new_workspace(tb.TB_OP_SELECT, gb.desc, probe.need)
            groups.append(gb)

        def group_step(gb):
            tb.tb_score(gb.desc, gb.q_imp, gb.Kimp, 1.0, gb.scores)
            tb.tb_select_topk(gb.desc, gb.scores, cfg.k, cfg.sink, cfg.window, gb.idx, gb.cnt, gb.ws)
            for li, b in enumerate(gb.layers):
                tb.tb_sparse_decode_attn(b.desc, b.q, b.K, b.V, gb.idx[li * cfg.B:(li + 1) * cfg.B],
                                         gb.cnt[li * cfg.B:(li + 1) * cfg.B], probe.need, cfg.sm_scale, b.out, b.lse, b.ws)

        for gb in groups:
            group_step(gb)
        torch.cuda.synchronize()
        # the batched calls select what the per-layer calls select (same kernels, same scores)
        same = all(torch.equal(gb.idx[li * cfg.B:(li + 1) * cfg.B], b.idx) and torch.equal(gb.cnt[li * cfg.B:(li + 1) * cfg.B], b.cnt)
                   for gb in groups for li, b in enumerate(gb.layers) if b in bufs)
        gg = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        n_calls = n_groups * max(1, -(-GRAPH_MIN_STEPS // (n_groups * G4)))
        with torch.cuda.stream(side):
            with torch.cuda.graph(gg, stream=side):
                for i in range(n_calls):
                    group_step(groups[i % n_groups])
        torch.cuda.current_stream().wait_stream(side)
        gg.replay()
        torch.cuda.synchronize()
        n_rep = max(3, args.steps // (n_calls * G4))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n_rep):
            gg.replay()
        e1.record()
        torch.cuda.synchronize()
        us_layer = e0.elapsed_time(e1) * 1e3 / (n_rep * n_calls * G4)
        group = {"layers_per_group": G4, "us_per_layer": round(us_layer, 3), "groups_of_buffers": n_groups,
                 "layer_steps_timed": n_rep * n_calls * G4, "lists_equal_per_layer_calls": bool(same),
                 "note": "scoring and selection of a producer's 4 consumer layers as one batched call each, then 4 attention calls"}
        step(bufs[0])       # restore copy 0's outputs, which the parity check reads
        torch.cuda.synchronize()
        del groups, layers

    elt = cfg.elt_bytes
    bytes_kimp = cfg.B * cfg.Hkv * cfg.N * cfg.Dimp * elt
    bytes_gather = selected_rows * 2 * cfg.D * elt
    bytes_step = bytes_kimp + bytes_gather
    step_gbps = bytes_step / us_step / 1e3
    bytes_proj_bulk = cfg.B * cfg.Hkv * cfg.N * (cfg.D + cfg.Dimp) * elt
    proj_gbps = bytes_proj_bulk / us_proj_bulk / 1e3
    attn_gbps = bytes_gather / us_attn_step / 1e3

    result = {
        "metric": "decode_step_latency_score_topk_sparse_attn",
        "value": round(us_step, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": steps_done,
        "warmup": args.warmup,
        "ms_per_step": round(us_step / 1e3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {
            "workload": cfg.name, "B": cfg.B, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "D": cfg.D, "N": cfg.N,
            "d_imp": cfg.Dimp, "k": cfg.k, "sink": cfg.sink, "window": cfg.window,
            "buffer_copies": copies, "kv_layout": args.kv_layout,
            "kv_memory": "pinned host" if args.kv_host else "hbm", "launch": "hipgraph" if use_graph else "eager",
            "steps_per_graph": per_graph if use_graph else None,
        },
        "step_hbm": {
            "algorithmic_bytes": bytes_step, "achieved": round(step_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": round(step_gbps / HBM_PEAK_GBPS, 4),
        },
        "stages_us": {
            "score": round(us_score, 3), "select_topk": round(us_select, 3), "sparse_attn": round(us_attn, 3),
            "score_then_select": round(us_pre, 3), "sparse_attn_inside_step": round(us_attn_step, 3),
            "project_append_1row": round(us_proj, 3), "step_eager_launch": round(us_step_eager, 3),
            "predict_queries_4slots": round(us_predict, 3),
        },
        "predictor": {"E": E, "hidden": hidden, "slots": G, "weight_bytes": bytes_predict, "us": round(us_predict, 3),
                      "note": "two launches that read 8 MiB of weights: a latency figure"},
        # the batched projection of the whole key cache (done once per window of appended tokens,
        # not per step): read K, write K_imp
        "project_bulk": {
            "us": round(us_proj_bulk, 3), "algorithmic_bytes": bytes_proj_bulk, "achieved": round(proj_gbps, 1),
            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(proj_gbps / HBM_PEAK_GBPS, 4),
            "tflops": round(2.0 * cfg.B * cfg.Hkv * cfg.N * cfg.D * cfg.Dimp / us_proj_bulk / 1e6, 1),
        },
        # the dominant kernel of the step.  `us` is its duration inside the step (step minus the
        # step without it), which is what the profiler's in-step duration shows; launched back to
        # back on its own it can be faster (rows found again in the last-level cache).  The whole
        # step against the same peak is in `step` (and in step_hbm above).
        "roofline": {
            "kernel": "attn_kernel (tb_sparse_decode_attn)", "bound": "hbm", "achieved": round(attn_gbps, 1),
            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(attn_gbps / HBM_PEAK_GBPS, 4),
            "algorithmic_bytes": bytes_gather, "us": round(us_attn_step, 3),
            "us_back_to_back": round(us_attn, 3),
            "frac_back_to_back": round(bytes_gather / us_attn / 1e3 / HBM_PEAK_GBPS, 4),
            "timing": "us: inside the step (step minus score + select); us_back_to_back: launched on its own",
            "traffic": measured_traffic(cfg.name, "attn_kernel"),
            "step": {"us": round(us_step, 3), "algorithmic_bytes": bytes_step, "achieved": round(step_gbps, 1),
                     "frac": round(step_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic(cfg.name, "step")},
            # a difference of two noisy timings: flagged when it cannot be right
            "suspect": bool(us_attn_step <= 0.5 * us_attn or attn_gbps > HBM_PEAK_GBPS),
        },
        # head-less selection (one list per batch element for all heads): scoring and selection
        # of one importance head, attention over the shared list
        "headless": None if us_hl_step is None else {"us_step": round(us_hl_step, 3), "attn_us": round(us_hl_attn, 3)},
        "producer_group": None if group is None else dict(
            group, algorithmic_bytes_per_layer=bytes_step, achieved=round(bytes_step / group["us_per_layer"] / 1e3, 1),
            unit="GB/s", frac=round(bytes_step / group["us_per_layer"] / 1e3 / HBM_PEAK_GBPS, 4)),
        "step_us_spread": pct,
        "device_copy_256MiB_GBps": round(copy_gbps, 1),
        # measured read ceiling of this machine, and the same kernels' rates against it
        "read_stream_1GiB_GBps": round(read_gbps, 1),
        "frac_of_read_stream": {"step": round(step_gbps / read_gbps, 4), "attn_kernel": round(attn_gbps / read_gbps, 4)},
        "timed_wall_s": round(wall_s, 3),
    }

    if args.kv_host:
        # the gathered rows cross the host link (PCIe 5.0 x16: 64 GB/s per direction); HBM is not the bound
        result["roofline"].update({"bound": "host_link", "peak": 64.0, "frac": round(attn_gbps / 64.0, 4),
                                   "traffic": None})
        result.pop("project_bulk")
    if cfg.layers > 1 and not args.kv_host:
        # the whole stack of layers, every layer with its own cache, queries and lists: one decode
        # step of the model as far as this path goes (one graph, one step per layer)
        del bufs[1:]
        stack = [probe] + [LayerBuffers(cfg, 0, tb, workloads, torch, args.kv_layout, False, layer=l)
                           for l in range(1, cfg.layers)]
        for b in stack:
            step(b)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for b in stack:
                    step(b)
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(2):
            g.replay()
        torch.cuda.synchronize()
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_rep = 10
        d0.record()
        for _ in range(n_rep):
            g.replay()
        d1.record()
        torch.cuda.synchronize()
        us_stack = d0.elapsed_time(d1) * 1e3 / n_rep
        rows = sum(int(b.cnt.sum().item()) for b in stack)
        stack_bytes = cfg.layers * bytes_kimp + rows * 2 * cfg.D * elt
        result["depth_loop"] = {
            "layers": cfg.layers, "us_all_layers": round(us_stack, 1), "us_per_layer": round(us_stack / cfg.layers, 3),
            "algorithmic_bytes": stack_bytes, "achieved": round(stack_bytes / us_stack / 1e3, 1), "peak": HBM_PEAK_GBPS,
            "unit": "GB/s", "frac": round(stack_bytes / us_stack / 1e3 / HBM_PEAK_GBPS, 4),
            "resident_bytes": sum(b.nbytes() for b in stack),
        }
        del stack
    if cfg.P > 1:
        result["interval_loop"] = time_interval_loop(cfg, tb, workloads, torch)
        result["interval_loop"]["reuse_step"]["traffic"] = measured_traffic(cfg.name, "attn_kernel", what="reuse_step")
        result["interval_loop_buffered"] = time_interval_loop(cfg, tb, workloads, torch, buffered=True)
        result["interval_loop_cluster_neighbours"] = time_interval_loop(cfg, tb, workloads, torch, mode=1)
        # the paper's layout in full (128 sink tokens, a ring of 256) against the fused gather under
        # the same policy (sink 128, window 256, the widened list attended on prediction steps too)
        result["interval_loop_ring_layout"] = time_interval_loop(cfg, tb, workloads, torch, ring=256, sink=128)
        result["interval_loop_fused_same_policy"] = time_interval_loop(cfg, tb, workloads, torch, sink=128, window=256,
                                                                       expand_on_predict=True)

    if not args.no_cpu_baseline:
        import numpy as np

        import oracle

        b = bufs[0]
        to_np = oracle.to_numpy
        host = {k: to_np(getattr(b, k)) for k in ("q", "q_imp", "K", "V", "Kimp")}
        reps, t_total = 0, 0.0
        while reps < 3 or (t_total < args.cpu_seconds and reps < 200):
            t0 = time.perf_counter()
            s, ridx, rcnt, rout, rlse = oracle.decode_step(host["q"], host["q_imp"], host["K"], host["V"],
                                                           host["Kimp"], cfg.dtype, cfg.k, cfg.sink, cfg.window,
                                                           cfg.sm_scale)
            t_total += time.perf_counter() - t0
            reps += 1
        # the same run doubles as a parity check of the benchmarked buffers (selection on the
        # GPU's own scores must be bit-exact; attention within the bf16/fp32 bar)
        gidx, gcnt = oracle.select_topk(to_np(b.scores)[:, :, : cfg.N], cfg.k, cfg.sink, cfg.window)
        sel_ok = bool(np.array_equal(gidx, to_np(b.idx)) and np.array_equal(gcnt, to_np(b.cnt)))
        gout, _ = oracle.sparse_decode_attn(host["q"], host["K"], host["V"], to_np(b.idx), to_np(b.cnt), cfg.dtype,
                                            cfg.sm_scale)
        attn_err = float(np.abs(gout - to_np(b.out)).max())
        n_threads = oracle.num_threads()
        oracle.set_num_threads(1)  # the same step on one core, once
        t0 = time.perf_counter()
        oracle.decode_step(host["q"], host["q_imp"], host["K"], host["V"], host["Kimp"], cfg.dtype, cfg.k, cfg.sink,
                           cfg.window, cfg.sm_scale)
        t_single = time.perf_counter() - t0
        oracle.set_num_threads(n_threads)
        result["cpu_baseline"] = {
            "value": round(t_total / reps * 1e6, 1), "unit": "us/step", "cores": n_threads,
            "kind": "oracle", "sample": f"{reps} full {cfg.name} steps (score+select+attention) on copy 0's bytes",
            "single_thread_us": round(t_single * 1e6, 1),
        }
        result["parity_in_bench"] = {"selection_bit_exact": sel_ok, "attn_max_abs_err": attn_err}

    print(json.dumps(result))


if __name__ == "__main__":
    main()
