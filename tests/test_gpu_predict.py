"""Query predictor (LN + two-layer MLP, Sec. 3.1) through the C ABI against the fp64 oracle."""
import numpy as np
import pytest
import torch

from gpu_util import DEV, dtype_name, np_of
from paper_2503_07518_amd import binding as tb

pytestmark = pytest.mark.gpu


def make(B, E, hidden, G, Hq, Dimp, dtype, seed):
    g = torch.Generator().manual_seed(seed)
    r = lambda *shape, scale=1.0, shift=0.0: ((torch.randn(shape, generator=g) * scale + shift).to(dtype).to(DEV))
    return dict(h=r(B, E, scale=2.0, shift=0.5), gamma=r(E, shift=1.0, scale=0.2), beta=r(E, scale=0.2),
                W1=r(hidden, E, scale=E ** -0.5), b1=r(hidden, scale=0.3),
                W2=r(G * Hq * Dimp, hidden, scale=hidden ** -0.5), b2=r(G * Hq * Dimp, scale=0.3))


@pytest.mark.parametrize("dtype,B,E,hidden,G,Hq,Dimp", [
    (torch.bfloat16, 1, 4096, 512, 4, 32, 32),   # Llama-3-8B shape, the paper's predictor
    (torch.bfloat16, 5, 4096, 512, 4, 32, 16),   # odd batch: a half-filled batch chunk
    (torch.float32, 3, 1024, 256, 2, 8, 16),
    (torch.float32, 1, 8192, 2048, 1, 4, 8),     # largest supported sizes
    (torch.bfloat16, 2, 64, 8, 3, 2, 8),         # rows shorter than one pass of a wave
    # batches of 8 or more in bf16: the matrix-core form
    (torch.bfloat16, 16, 4096, 512, 4, 32, 32),  # one full tile of sequences
    (torch.bfloat16, 8, 4096, 512, 4, 32, 32),   # half a tile
    (torch.bfloat16, 20, 1024, 256, 2, 8, 16),   # two tiles per workgroup, the second ragged
    (torch.bfloat16, 45, 512, 64, 1, 4, 16),     # two workgroup groups along the batch
    (torch.bfloat16, 9, 96, 32, 3, 2, 8),        # smallest sizes the tiles divide
    (torch.bfloat16, 16, 4096, 520, 4, 32, 32),  # hidden size not a multiple of 32: the FMA form
    (torch.float32, 16, 1024, 256, 2, 8, 16),    # fp32 batches stay on the FMA form
])
def test_predict_queries(oracle, dtype, B, E, hidden, G, Hq, Dimp):
    print(f"[case] predictor dtype={dtype} B={B} E={E} hidden={hidden} G={G} Hq={Hq} Dimp={Dimp}", flush=True)
    p = make(B, E, hidden, G, Hq, Dimp, dtype, 21)
    z = torch.full((B, hidden), float("nan"), dtype=torch.float32, device=DEV)
    q_imp = torch.zeros((G, B, Hq, Dimp), dtype=dtype, device=DEV)
    xln = torch.empty((B, E), dtype=torch.float32, device=DEV)
    tb.tb_predict_queries(p["h"], p["gamma"], p["beta"], p["W1"], p["b1"], p["W2"], p["b2"], G, Hq, Dimp, z, xln, q_imp)
    torch.cuda.synchronize()
    dn = dtype_name(p["h"])
    rq, rz = oracle.predict_queries(*(np_of(p[k]) for k in ("h", "gamma", "beta", "W1", "b1", "W2", "b2")), G, Hq, Dimp, dn)
    # hidden activations: fp32 sums of E products after an fp32 LayerNorm
    assert np.abs(np_of(z) - rz).max() <= 2e-4 * max(1.0, np.abs(rz).max())
    got = np_of(q_imp)
    if dn == "bf16":
        g64, r64 = oracle.bf16_to_f64(got), oracle.bf16_to_f64(rq)
        assert np.all(np.abs(g64 - r64) <= 2.0 ** -7 * np.abs(r64) + 2e-3)
        assert np.mean(got == rq) > 0.97  # and nearly always the same bits
    else:
        assert np.abs(got - rq).max() <= 2e-4 * max(1.0, np.abs(rq).max())


def test_predicted_slot_feeds_scoring(oracle):
    """Slot s of the predictor's output is laid out as tb_score's q_imp."""
    print("[case] predictor slot -> tb_score", flush=True)
    from gpu_util import gpu_score, score_tolerance
    B, E, hidden, G, Hq, Hkv, Dimp, N = 2, 512, 64, 4, 8, 2, 32, 3000
    p = make(B, E, hidden, G, Hq, Dimp, torch.bfloat16, 22)
    z = torch.empty((B, hidden), dtype=torch.float32, device=DEV)
    q_imp = torch.zeros((G, B, Hq, Dimp), dtype=torch.bfloat16, device=DEV)
    xln = torch.empty((B, E), dtype=torch.float32, device=DEV)
    tb.tb_predict_queries(p["h"], p["gamma"], p["beta"], p["W1"], p["b1"], p["W2"], p["b2"], G, Hq, Dimp, z, xln, q_imp)
    Kimp = (torch.randn((B, Hkv, N, Dimp), generator=torch.Generator().manual_seed(23))).to(torch.bfloat16).to(DEV)
    s = gpu_score(q_imp[2], Kimp, N)
    torch.cuda.synchronize()
    ref = oracle.score(np_of(q_imp[2]), np_of(Kimp), "bf16", 1.0)
    guard = score_tolerance(oracle, np_of(q_imp[2]), np_of(Kimp), "bf16", 1.0, Hq // Hkv)
    assert np.all(np.abs(np_of(s)[:, :, :N] - ref) <= 1e-4 * np.abs(ref) + guard)
