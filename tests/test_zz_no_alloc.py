"""The allocation-free attention entry point against the workspace form: same kernels, so the
results must be bit-identical; two calls in a row on the library's scratch, the second smaller."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from gpu_util import DEV, gpu_attn, np_of
from paper_2503_07518_amd import binding as tb


def _case(seed, B, Hq, Hkv, N, D, k, dtype):
    g = torch.Generator(device="cpu").manual_seed(seed)
    K = torch.randn((B, Hkv, N, D), generator=g).to(dtype).to(DEV)
    V = torch.randn((B, Hkv, N, D), generator=g).to(dtype).to(DEV)
    q = torch.randn((B, Hq, D), generator=g).to(dtype).to(DEV)
    idx = torch.stack([torch.stack([torch.randperm(N, generator=g)[:k].sort().values for _ in range(Hq)])
                       for _ in range(B)]).to(torch.int32).to(DEV)
    cnt = torch.full((B, Hq), k, dtype=torch.int32, device=DEV)
    cnt[0, 0] = k // 2  # a shorter list among them
    return q, K, V, idx, cnt


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_static_scratch_matches_workspace_form(oracle, dtype):
    for seed, (B, Hq, Hkv, N, D, k) in enumerate([(2, 8, 2, 6000, 128, 2500), (1, 4, 4, 700, 64, 300)]):
        print(f"[case] static scratch dtype={dtype} B={B} Hq={Hq} N={N} k={k}", flush=True)
        q, K, V, idx, cnt = _case(seed, B, Hq, Hkv, N, D, k, dtype)
        sm = D ** -0.5
        ref_out, ref_lse = gpu_attn(q, K, V, idx, cnt, N, sm, tail=(N - 5, N))
        d = tb.make_desc(N, Hq, K=K, V=V)
        out = torch.full((B, Hq, D), float("nan"), dtype=torch.float32, device=DEV)
        lse = torch.full((B, Hq), float("nan"), dtype=torch.float32, device=DEV)
        tb.tb_sparse_decode_attn_static(d, q, K, V, idx, cnt, k, sm, out, lse, tail_begin=N - 5, tail_end=N)
        torch.cuda.synchronize()
        assert np.array_equal(np_of(out), np_of(ref_out)) and np.array_equal(np_of(lse), np_of(ref_lse))
        # and against the oracle, to the bar of the attention tests
        ci, cc = np_of(idx), np_of(cnt)
        ext = np.zeros((B, Hq, k + 5), dtype=np.int32)
        for b in range(B):
            for h in range(Hq):
                n = int(cc[b, h])
                ext[b, h, :n] = ci[b, h, :n]
                ext[b, h, n:n + 5] = np.arange(N - 5, N)  # the dense tail follows the list
        o_ref, _ = oracle.sparse_decode_attn(np_of(q), np_of(K), np_of(V), ext, cc + 5,
                                             "bf16" if dtype == torch.bfloat16 else "f32", sm)
        assert np.abs(np_of(out) - o_ref).max() <= (2e-2 if dtype == torch.bfloat16 else 1e-5)


def test_static_scratch_rejects_oversized_shapes():
    d = tb.tb_cache_desc()
    d.B, d.Hq, d.Hkv, d.D, d.Dimp, d.dtype, d.N = 256, 64, 8, 128, 32, tb.TB_BF16, 1 << 20
    d.k_stride_n = d.v_stride_n = 128
    d.k_stride_h = d.v_stride_h = 128 << 20
    d.k_stride_b = d.v_stride_b = 8 * (128 << 20)
    d.ki_stride_n = 32
    assert tb.tb_workspace_bytes(tb.TB_OP_ATTN, d, 8192) > (4 << 20)
    t = torch.zeros((1, 1, 8192), dtype=torch.int32, device=DEV)  # never read: the call must fail on the host
    with pytest.raises(tb.TbError) as e:
        tb.tb_sparse_decode_attn_static(d, t, t, t, t, t, 8192, 1.0, t.float(), None)
    assert e.value.code == tb.TB_ERR_WORKSPACE
