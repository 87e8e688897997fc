"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments on the host before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tb():
    from paper_2503_07518_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        from paper_2503_07518_amd import build

        build.build(force=True)
    binding.load_library()
    return binding


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "tokenbutler.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tb_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(tb):
    names = declared_symbols()
    assert set(names) == set(tb.EXPORTS), (names, tb.EXPORTS)
    lib = tb.load_library()
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_status_strings(tb):
    assert tb.tb_version() >= 100
    assert tb.status_string(0) == "ok"
    for code in (1, 2, 3, 4):
        assert tb.status_string(code) not in ("ok", "unknown status")
    assert tb.status_string(99) == "unknown status"


def desc(tb, **kw):
    d = tb.tb_cache_desc()
    base = dict(B=1, Hq=8, Hkv=2, D=128, Dimp=32, dtype=tb.TB_BF16, N=1000,
                k_stride_b=2 * 1024 * 128, k_stride_h=1024 * 128, k_stride_n=128,
                v_stride_b=2 * 1024 * 128, v_stride_h=1024 * 128, v_stride_n=128,
                ki_stride_b=2 * 1024 * 32, ki_stride_h=1024 * 32, ki_stride_n=32)
    base.update(kw)
    for k, v in base.items():
        setattr(d, k, v)
    return d


P = ctypes.c_void_p(0x10000)  # never dereferenced: every call below must fail validation first
NULL = None


def test_workspace_sizes(tb):
    d = desc(tb)
    sel = tb.tb_workspace_bytes(tb.TB_OP_SELECT, d, 0)
    att = tb.tb_workspace_bytes(tb.TB_OP_ATTN, d, 500)
    step = tb.tb_workspace_bytes(tb.TB_OP_DECODE_STEP, d, 500)
    assert sel == 0 and att >= 8 * 256 and step == att
    assert tb.tb_workspace_bytes(99, d, 0) == 0
    assert tb.tb_workspace_bytes(tb.TB_OP_ATTN, desc(tb, D=96), 10) == 0
    assert tb.tb_workspace_bytes(tb.TB_OP_ATTN, d, -1) == 0
    # long rows on few heads are selected in two stages and need room for the candidates
    long_row = desc(tb, N=1 << 20)
    need = tb.tb_workspace_bytes(tb.TB_OP_SELECT, long_row, 8192)
    assert need >= 8 * 8 * 8192 * 8 and tb.tb_workspace_bytes(tb.TB_OP_DECODE_STEP, long_row, 8192) >= need
    assert tb.tb_workspace_bytes(tb.TB_OP_SELECT, long_row, 0) == 0


def test_rejects_bad_arguments_without_launching(tb):
    L = tb.load_library()
    d = desc(tb)
    r = ctypes.byref
    # null pointers
    assert L.tb_score(r(d), NULL, P, 1.0, P, 1000, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_project_keys(r(d), P, NULL, 1, P, 0, 10, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_select_topk(r(d), P, 1000, 10, 0, 0, NULL, P, 100, P, 1 << 20, None) == tb.TB_ERR_INVALID_ARG
    # inconsistent shapes
    assert L.tb_score(r(desc(tb, Hq=7)), P, P, 1.0, P, 1000, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_score(r(desc(tb, N=-1)), P, P, 1.0, P, 1000, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_score(r(d), P, P, 1.0, P, 996, None) == tb.TB_ERR_INVALID_ARG  # stride < N
    # unsupported shapes / alignment
    assert L.tb_score(r(desc(tb, Dimp=24)), P, P, 1.0, P, 1000, None) == tb.TB_ERR_UNSUPPORTED
    assert L.tb_score(r(desc(tb, D=96)), P, P, 1.0, P, 1000, None) == tb.TB_ERR_UNSUPPORTED
    assert L.tb_score(r(desc(tb, Hq=6, Hkv=2)), P, P, 1.0, P, 1000, None) == tb.TB_ERR_UNSUPPORTED
    assert L.tb_score(r(d), P, P, 1.0, P, 1002, None) == tb.TB_ERR_UNSUPPORTED  # stride % 4
    assert L.tb_score(r(d), ctypes.c_void_p(0x10004), P, 1.0, P, 1000, None) == tb.TB_ERR_UNSUPPORTED
    assert L.tb_score(r(desc(tb, ki_stride_n=36)), P, P, 1.0, P, 1000, None) == tb.TB_ERR_UNSUPPORTED
    # projection ranges
    assert L.tb_project_keys(r(d), P, P, 1, P, 5, 4, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_project_keys(r(d), P, P, 1, P, 0, 1001, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_project_keys(r(d), P, P, 3, P, 0, 10, None) == tb.TB_ERR_INVALID_ARG  # Hw not 1 or Hkv
    assert L.tb_project_keys(r(d), P, P, 1, P, 7, 7, None) == tb.TB_OK  # empty range: no-op
    # selection: negative budget, capacity too small, missing workspace, N too large
    assert L.tb_select_topk(r(d), P, 1000, -1, 0, 0, P, P, 100, P, 1 << 20, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_select_topk(r(d), P, 1000, 10, 4, 4, P, P, 17, P, 1 << 20, None) == tb.TB_ERR_INVALID_ARG
    big = desc(tb, N=(1 << 20) + 4)
    assert L.tb_select_topk(r(big), P, (1 << 20) + 4, 10, 0, 0, P, P, 10, P, 1 << 20, None) == tb.TB_ERR_UNSUPPORTED
    # neighbours: output capacity, mode, aliasing
    assert L.tb_expand_neighbors(1, 8, 1000, 1, 0, P, P, 100, ctypes.c_void_p(0x20000), P, 299, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_expand_neighbors(1, 8, 1000, 1, 2, P, P, 100, ctypes.c_void_p(0x20000), P, 300, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_expand_neighbors(1, 8, 1000, 1, 0, P, P, 100, P, P, 300, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_expand_neighbors(1, 8, 1000, -1, 0, P, P, 100, ctypes.c_void_p(0x20000), P, 300, None) == tb.TB_ERR_INVALID_ARG
    # attention: max_count beyond capacity, tail outside the cache, workspace too small
    assert L.tb_sparse_decode_attn(r(d), P, P, P, P, P, 100, 101, 0, 0, 1.0, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_sparse_decode_attn(r(d), P, P, P, P, P, 100, 100, 990, 1001, 1.0, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_sparse_decode_attn(r(d), P, P, P, P, P, 100, 100, 0, 0, 1.0, P, NULL, P, 64, None) == tb.TB_ERR_WORKSPACE
    assert L.tb_sparse_decode_attn(r(desc(tb, k_stride_n=100)), P, P, P, P, P, 100, 100, 0, 0, 1.0, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    # the head-less form takes the same checks
    assert L.tb_sparse_decode_attn_shared(r(d), P, P, P, P, P, 100, 101, 0, 0, 1.0, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_sparse_decode_attn_shared(r(d), P, P, P, NULL, P, 100, 100, 0, 0, 1.0, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_sparse_decode_attn_shared(r(d), P, P, P, P, P, 100, 100, 0, 0, 1.0, P, NULL, P, 64, None) == tb.TB_ERR_WORKSPACE
    # fused step inherits all of the above
    assert L.tb_decode_step(r(d), P, P, 1.0, P, P, P, 10, 0, 0, 1.0, P, 1000, P, P, 9, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_decode_step(r(d), P, P, 1.0, P, P, P, 10, 0, 0, 1.0, P, 1000, P, P, 10, P, NULL, P, 64, None) == tb.TB_ERR_WORKSPACE
    # buffer migration and buffered attention: capacities, null buffers, workspace
    assert L.tb_gather_kv(r(d), P, P, P, P, 100, 101, P, P, 200, None) == tb.TB_ERR_INVALID_ARG  # max_count > idx_cap
    assert L.tb_gather_kv(r(d), P, P, P, P, 100, 100, P, P, 99, None) == tb.TB_ERR_INVALID_ARG   # buffer too small
    assert L.tb_gather_kv(r(d), P, P, P, P, 100, 100, NULL, P, 100, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_gather_kv(r(d), P, P, P, P, 100, 100, ctypes.c_void_p(0x10008), P, 100, None) == tb.TB_ERR_UNSUPPORTED
    assert L.tb_buffered_decode_attn(r(d), P, NULL, P, 100, P, 100, P, P, 0, 0, 1.0, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_buffered_decode_attn(r(d), P, P, P, 100, P, 101, P, P, 0, 0, 1.0, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_buffered_decode_attn(r(d), P, P, P, 100, P, 100, P, P, 0, 1001, 1.0, P, NULL, P, 1 << 24, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_buffered_decode_attn(r(d), P, P, P, 100, P, 100, P, P, 0, 0, 1.0, P, NULL, P, 64, None) == tb.TB_ERR_WORKSPACE
    # query predictor: shapes, null pointers, sizes outside the supported range
    pd = tb.tb_predictor_desc(4096, 512, 4, 32, 32, tb.TB_BF16, 1e-5)
    args = (P, P, P, P, P, P, P, P, P, P)
    assert L.tb_predict_queries(r(pd), 1, NULL, *args[1:], None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_predict_queries(r(pd), -1, *args, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_predict_queries(r(tb.tb_predictor_desc(4100, 512, 4, 32, 32, tb.TB_BF16, 1e-5)), 1, *args, None) == tb.TB_ERR_UNSUPPORTED
    assert L.tb_predict_queries(r(tb.tb_predictor_desc(16384, 512, 4, 32, 32, tb.TB_BF16, 1e-5)), 1, *args, None) == tb.TB_ERR_UNSUPPORTED
    assert L.tb_predict_queries(r(tb.tb_predictor_desc(4096, 512, 0, 32, 32, tb.TB_BF16, 1e-5)), 1, *args, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_predict_queries(r(tb.tb_predictor_desc(4096, 512, 4, 32, 32, 7, 1e-5)), 1, *args, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_predict_queries(r(pd), 0, *args, None) == tb.TB_OK  # empty batch: no-op
    # workspace init
    assert L.tb_workspace_init(NULL, 16, None) == tb.TB_ERR_INVALID_ARG
    assert L.tb_workspace_init(P, 6, None) == tb.TB_ERR_INVALID_ARG


def test_missing_library_is_an_error(tb, monkeypatch, tmp_path):
    """The product path has no fallback: without the HIP library the ops raise."""
    monkeypatch.setattr(tb, "_lib", None)
    monkeypatch.setattr(tb, "LIB_PATH", str(tmp_path / "libtokenbutler.so"))
    with pytest.raises(ImportError):
        tb.tb_version()
