"""Offloaded cache (the paper's efficiency section, contexts beyond GPU memory): K and V live in
pinned host memory that is mapped into the device address space, the projected keys stay on
the GPU, and only the rows that the selection picks cross the host link.  The library needs
nothing special for it -- the kernels read through whatever device-accessible pointers they are
given -- so this checks exactly that, against the oracle, on the same bytes."""
import ctypes
import math

import numpy as np
import pytest
import torch

from gpu_util import DEV, assert_attention, assert_projection, gpu_decode_step, gpu_project, np_of, projection_magnitude
from paper_2503_07518_amd import binding as tb

pytestmark = pytest.mark.gpu


def device_address(t: torch.Tensor) -> int:
    """Device-side address of a pinned host tensor, asked from the HIP runtime (0 if the
    allocation is not mapped for the device)."""
    hip = ctypes.CDLL("libamdhip64.so")
    hip.hipHostGetDevicePointer.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_uint]
    hip.hipHostGetDevicePointer.restype = ctypes.c_int
    out = ctypes.c_void_p(0)
    rc = hip.hipHostGetDevicePointer(ctypes.byref(out), ctypes.c_void_p(t.data_ptr()), 0)
    return int(out.value or 0) if rc == 0 else 0


def test_decode_step_with_kv_in_pinned_host_memory(oracle):
    print("[case] offloaded K/V: pinned host memory, B=1 Hq=8 Hkv=2 N=8192 k=300", flush=True)
    B, Hq, Hkv, N, D, Dimp, k = 1, 8, 2, 8192, 128, 32, 300
    g = torch.Generator().manual_seed(5)
    K = torch.empty((B, Hkv, N, D), dtype=torch.bfloat16, pin_memory=True).copy_(torch.randn((B, Hkv, N, D), generator=g))
    V = torch.empty((B, Hkv, N, D), dtype=torch.bfloat16, pin_memory=True).copy_(torch.randn((B, Hkv, N, D), generator=g))
    assert K.is_pinned() and V.is_pinned()
    if device_address(K) != K.data_ptr() or device_address(V) != V.data_ptr():
        pytest.skip("pinned host memory is not mapped at the same address for the device on this box")
    W = (torch.randn((1, D, Dimp), generator=g) / math.sqrt(D)).to(torch.bfloat16).to(DEV)
    q = torch.randn((B, Hq, D), generator=g).to(torch.bfloat16).to(DEV)
    q_imp = torch.randn((B, Hq, Dimp), generator=g).to(torch.bfloat16).to(DEV)
    Kimp = torch.zeros((B, Hkv, N, Dimp), dtype=torch.bfloat16, device=DEV)  # stays on the GPU
    gpu_project(K, W, N, Kimp=Kimp)  # the batched projection reads the host-resident keys once
    scores, idx, cnt, out, lse = gpu_decode_step(q, q_imp, K, V, Kimp, N, k, 4, 16, 1.0 / math.sqrt(D))
    torch.cuda.synchronize()
    Kn, Vn, Kin = np_of(K), np_of(V), np_of(Kimp)
    ref_kimp = oracle.project_keys(Kn, np_of(W), "bf16")
    assert_projection(oracle, Kin, ref_kimp, projection_magnitude(oracle, Kn, np_of(W), "bf16", Hkv), "bf16")
    assert np.mean(Kin == ref_kimp) > 0.99
    ridx, rcnt = oracle.select_topk(np_of(scores)[:, :, :N], k, 4, 16)
    assert np.array_equal(rcnt, np_of(cnt)) and np.array_equal(ridx, np_of(idx)[..., : ridx.shape[-1]])
    rout, rlse = oracle.sparse_decode_attn(np_of(q), Kn, Vn, np_of(idx), np_of(cnt), "bf16", 1.0 / math.sqrt(D))
    assert_attention(np_of(out), rout, "bf16", np_of(lse), rlse)
