"""The entry points under HIP graph capture: a captured call, replayed several times with the
program's own eager work and synchronisations between the replays, must reproduce the eager
result bit for bit on every replay (the library clears its counters and scratch with kernels of
its own, never with memset nodes)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from gpu_util import DEV, np_of
from paper_2503_07518_amd import binding as tb
from paper_2503_07518_amd import workloads


def _capture(fn):
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    return g


def _layer(cfg, layer):
    data = workloads.make_layer(cfg, layer=layer, device=DEV)
    K, V = data["K"], data["V"]
    Kimp = torch.zeros((cfg.B, cfg.Hkv, cfg.N, cfg.Dimp), dtype=K.dtype, device=DEV)
    d = tb.make_desc(cfg.N, cfg.Hq, K=K, V=V, Kimp=Kimp)
    tb.tb_project_keys(d, K, data["W"], Kimp, 0, cfg.N)
    need = tb.policy_count(cfg.N, cfg.k, 0, 0)
    stride = (cfg.N + 3) // 4 * 4
    bufs = dict(
        d=d, K=K, V=V, Kimp=Kimp, q=data["q"][0].contiguous(), q_imp=data["q_imp"][0].contiguous(), need=need,
        scores=torch.zeros((cfg.B, cfg.Hq, stride), dtype=torch.float32, device=DEV),
        idx=torch.zeros((cfg.B, cfg.Hq, need), dtype=torch.int32, device=DEV),
        cnt=torch.zeros((cfg.B, cfg.Hq), dtype=torch.int32, device=DEV),
        out=torch.zeros((cfg.B, cfg.Hq, cfg.D), dtype=torch.float32, device=DEV),
        lse=torch.zeros((cfg.B, cfg.Hq), dtype=torch.float32, device=DEV),
        ws=tb.new_workspace(tb.TB_OP_DECODE_STEP, d, need))
    return bufs


def _step(cfg, b):
    tb.tb_decode_step(b["d"], b["q_imp"], b["Kimp"], 1.0, b["q"], b["K"], b["V"], cfg.k, 0, 0, cfg.sm_scale,
                      b["scores"], b["idx"], b["cnt"], b["out"], b["lse"], b["ws"])


@pytest.mark.parametrize("name,kw", [
    ("split attention, one selection workgroup per row", dict(B=1, N=8192, k=800)),
    ("selection by pieces (workspace scratch in the graph)", dict(B=2, N=70001, k=4096, heavy_per_kv_head=64)),
])
def test_decode_step_graph_replays_match_eager(name, kw):
    print(f"[case] graph replay: {name}", flush=True)
    cfg = workloads.C2.scaled(name="C2_graph", **kw)
    a, other = _layer(cfg, 0), _layer(cfg, 1)
    _step(cfg, a)
    torch.cuda.synchronize()
    ref = {k: a[k].clone() for k in ("scores", "idx", "cnt", "out", "lse")}
    assert int(ref["cnt"].min()) == a["need"]
    g = _capture(lambda: _step(cfg, a))
    for r in range(4):
        for k in ("scores", "out", "lse"):
            a[k].fill_(float("nan"))
        a["idx"].fill_(-1)
        a["cnt"].fill_(-1)
        _step(cfg, other)            # eager work of the same library between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k, v in ref.items():
            got = a[k][..., :cfg.N] if k == "scores" else a[k]      # (the padding of a score row is not written)
            want = v[..., :cfg.N] if k == "scores" else v
            assert torch.equal(got, want), f"replay {r}: {k} differs from the eager call"


def test_static_scratch_attention_in_a_graph():
    """The entry point for callers that cannot allocate, used the way such a caller would: captured."""
    print("[case] graph replay: attention on the library's own scratch", flush=True)
    cfg = workloads.C2.scaled(name="C2_graph_static", B=1, N=8192, k=800)
    a = _layer(cfg, 0)
    _step(cfg, a)
    torch.cuda.synchronize()
    ref_out, ref_lse = a["out"].clone(), a["lse"].clone()

    def call():
        tb.tb_sparse_decode_attn_static(a["d"], a["q"], a["K"], a["V"], a["idx"], a["cnt"], a["need"], cfg.sm_scale,
                                        a["out"], a["lse"])
    g = _capture(call)
    for r in range(3):
        a["out"].fill_(float("nan"))
        a["lse"].fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(a["out"], ref_out) and torch.equal(a["lse"], ref_lse), f"replay {r} differs"
        call()                       # and an eager call on the same scratch in between
        torch.cuda.synchronize()
        assert torch.equal(a["out"], ref_out)
