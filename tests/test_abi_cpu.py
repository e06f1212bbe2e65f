"""C-ABI checks that need no GPU: the library loads, exports every declared symbol, and rejects bad
arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2502_03805_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(P.binding.LIB_PATH):
        from paper_2502_03805_amd.build import build
        build()
    return P.load()


def good_desc(**over):
    kw = dict(batch=1, n_q_heads=8, n_kv_heads=2, head_dim=128, d_model=256, n_ctx=1000, window=16, pool_kernel=7,
              dtype=P.CKV_BF16)
    kw.update(over)
    return P.make_desc(**kw)


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "criticalkv.h")).read()
    declared = set(re.findall(r"CKV_API[^;(]*?\b(criticalkv_\w+)\s*\(", header))
    assert declared == set(P.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_descriptor_struct_matches_header_layout():
    # 12 x int32 + 2 x float + 6 x int64, no padding surprises
    assert ctypes.sizeof(P.LayerDesc) == 12 * 4 + 2 * 4 + 6 * 8
    assert P.LayerDesc.k_stride.offset == 56 and P.LayerDesc.v_stride.offset == 80


def test_strerror_is_static_text(lib):
    for code in (0, -1, -2, -3, -4, -99):
        s = P.strerror(code)
        assert isinstance(s, str) and len(s) > 3


def test_workspace_bytes_is_positive_and_monotone(lib):
    a = P.workspace_bytes(good_desc(n_ctx=1000), 100)
    b = P.workspace_bytes(good_desc(n_ctx=2000), 100)
    assert 0 < a < b and a % 256 == 0
    assert P.workspace_bytes(good_desc(n_ctx=0), 1) == 0


@pytest.mark.parametrize("over,code", [
    (dict(batch=0), P.CKV_E_INVALID_ARG),
    (dict(n_q_heads=7), P.CKV_E_INVALID_ARG),          # H % Hkv != 0
    (dict(window=0), P.CKV_E_INVALID_ARG),
    (dict(window=2000), P.CKV_E_INVALID_ARG),          # W > n
    (dict(pool_kernel=4), P.CKV_E_INVALID_ARG),        # even pooling width
    (dict(dtype=5), P.CKV_E_INVALID_ARG),
    (dict(window_reduce=3), P.CKV_E_INVALID_ARG),
    (dict(flags=64), P.CKV_E_INVALID_ARG),
    (dict(softmax_scale=-1.0), P.CKV_E_INVALID_ARG),
    (dict(eps=float("nan")), P.CKV_E_INVALID_ARG),
    (dict(head_dim=96), P.CKV_E_UNSUPPORTED),
    (dict(d_model=100), P.CKV_E_UNSUPPORTED),
    (dict(norm=3), P.CKV_E_INVALID_ARG),
    (dict(k_stride=(128000, 64000, 100)), P.CKV_E_INVALID_ARG),   # token stride below head_dim
    (dict(k_stride=(128004, 64004, 132)), P.CKV_E_UNSUPPORTED),   # rows not 16-byte aligned
])
def test_bad_descriptors_are_rejected_without_a_device(lib, over, code):
    d = good_desc(**over)
    buf = ctypes.create_string_buffer(512)  # never dereferenced: validation fails first
    p = ctypes.addressof(buf)
    p = (p + 255) & ~255
    rc = lib.criticalkv_score(ctypes.byref(d), p, p, p, p, p, p, None, p, 1 << 40, None)
    assert rc == code
    rc = lib.criticalkv_compact(ctypes.byref(d), p, p, p, p, 10, p, p, None)
    assert rc == code


def test_null_pointers_workspace_and_ranges(lib):
    d = good_desc()
    need = P.workspace_bytes(d, 100)
    buf = ctypes.create_string_buffer(1024)
    p = (ctypes.addressof(buf) + 255) & ~255
    # null tensor
    assert lib.criticalkv_score(ctypes.byref(d), None, p, p, p, p, p, None, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_score(None, p, p, p, p, p, p, None, p, need, None) == P.CKV_E_INVALID_ARG
    # a tensor that does not start on a 16-byte boundary
    assert lib.criticalkv_score(ctypes.byref(d), p, p + 8, p, p, p, p, None, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_compact(ctypes.byref(d), p, p + 2, p, p, 10, p, p, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_select(ctypes.byref(d), p + 4, p, p, 0.5, 100, p, p, p, need, None) == P.CKV_E_INVALID_ARG
    # workspace missing / misaligned / too small
    assert lib.criticalkv_score(ctypes.byref(d), p, p, p, p, p, p, None, None, need, None) == P.CKV_E_WORKSPACE
    assert lib.criticalkv_score(ctypes.byref(d), p, p, p, p, p, p, None, p + 8, need, None) == P.CKV_E_WORKSPACE
    assert lib.criticalkv_score(ctypes.byref(d), p, p, p, p, p, p, None, p, 4096, None) == P.CKV_E_WORKSPACE
    # select: alpha and max_budget ranges
    assert lib.criticalkv_select(ctypes.byref(d), p, p, p, 1.5, 100, p, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_select(ctypes.byref(d), p, p, p, float("nan"), 100, p, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_select(ctypes.byref(d), p, p, p, 0.5, 0, p, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_select(ctypes.byref(d), p, p, p, 0.5, 1001, p, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_select(ctypes.byref(d), p, p, None, 0.5, 100, p, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_select(ctypes.byref(d), p, p, p, 0.5, 100, p, p, p, 16, None) == P.CKV_E_WORKSPACE
    # allocate: total and floor ranges, workspace sized for the pooled list
    assert lib.criticalkv_allocate(ctypes.byref(d), p, -1, 0.5, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_allocate(ctypes.byref(d), p, 100, 1.5, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_allocate(ctypes.byref(d), None, 100, 0.5, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_allocate(ctypes.byref(d), p, d.n_kv_heads * d.n_ctx + 1, 0.5, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_allocate(ctypes.byref(d), p, d.n_kv_heads * 1000, 0.0, p, p, 4096, None) == P.CKV_E_WORKSPACE
    assert P.workspace_bytes(d, 1000) > need
    # diagnostics: pointers, budget range, modes without magnitudes or without the projection
    assert lib.criticalkv_diagnostics(ctypes.byref(d), p, None, None, p, p, 100, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_diagnostics(ctypes.byref(d), p, p, None, p, p, 0, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_diagnostics(ctypes.byref(d), p, p, None, p, p, 1001, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_diagnostics(ctypes.byref(d), p, p, None, p, p, 100, p, p, 4096, None) == P.CKV_E_WORKSPACE
    d_attn_only = good_desc(flags=P.CKV_ATTN_ONLY)
    assert lib.criticalkv_diagnostics(ctypes.byref(d_attn_only), p, p, None, p, p, 100, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_compact(ctypes.byref(d), p, p, p, p, 0, p, p, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_compact(ctypes.byref(d), p, p, p, None, 10, p, p, None) == P.CKV_E_INVALID_ARG


def test_noalloc_select_and_prepared_wo_validate_before_any_device_call(lib):
    d = good_desc()
    buf = ctypes.create_string_buffer(1024)
    p = (ctypes.addressof(buf) + 255) & ~255
    f = lib.criticalkv_select_noalloc
    assert f(ctypes.byref(d), None, p, p, 0.5, 100, p, p, None) == P.CKV_E_INVALID_ARG
    assert f(ctypes.byref(d), p, p, p, 1.5, 100, p, p, None) == P.CKV_E_INVALID_ARG
    assert f(ctypes.byref(d), p, p, p, 0.5, 1001, p, p, None) == P.CKV_E_INVALID_ARG
    assert f(ctypes.byref(d), p + 4, p, p, 0.5, 100, p, p, None) == P.CKV_E_INVALID_ARG
    # more entries than the static buffer covers: refused with its own code, nothing launched
    big = good_desc(n_ctx=1 << 20, n_q_heads=8, n_kv_heads=8)
    assert f(ctypes.byref(big), p, p, p, 0.5, 100, p, p, None) == P.CKV_E_STATIC_LIMIT
    assert "static" in P.strerror(P.CKV_E_STATIC_LIMIT)
    # the workloads' largest shapes fit: 8 heads x 128K and 32 heads x 32K entries
    assert P.CKV_STATIC_SCRATCH_BYTES == 12 << 20
    header = open(os.path.join(ROOT, "include", "criticalkv.h")).read()
    assert "#define CKV_STATIC_SCRATCH_BYTES ((size_t)12 << 20)" in header
    # prepared projection
    assert P.prepared_wo_bytes(d) == 8 * 128 * 256 * 2
    g = lib.criticalkv_prepare_wo
    assert g(ctypes.byref(d), None, p, None) == P.CKV_E_INVALID_ARG
    assert g(ctypes.byref(d), p, p, None) == P.CKV_E_INVALID_ARG                      # in place
    assert g(ctypes.byref(good_desc(flags=P.CKV_WO_OUT_IN)), p, p + 256, None) == P.CKV_E_INVALID_ARG


def test_gram_entry_points_validate(lib):
    d = good_desc(d_model=512, norm=P.CKV_NORM_L2)
    assert P.gram_bytes(d) == 8 * 2 * 128 * 128 * 2
    assert P.gram_bytes(good_desc(d_model=256, norm=P.CKV_NORM_L2)) == 0          # d_model not a multiple of 512
    assert P.gram_bytes(good_desc(d_model=512, dtype=P.CKV_F32)) == 0
    buf = ctypes.create_string_buffer(1024)
    p = (ctypes.addressof(buf) + 255) & ~255
    need = P.workspace_bytes(d, 10)
    assert lib.criticalkv_prepare_gram(ctypes.byref(d), None, p, p, need, None) == P.CKV_E_INVALID_ARG
    assert lib.criticalkv_prepare_gram(ctypes.byref(d), p, p, p, 64, None) == P.CKV_E_WORKSPACE
    d2 = good_desc(d_model=256)
    assert lib.criticalkv_prepare_gram(ctypes.byref(d2), p, p, p, need, None) == P.CKV_E_UNSUPPORTED
    # the prepared-Gram flag needs the L2 norm and the matrix-core path
    d3 = good_desc(d_model=512, norm=P.CKV_NORM_L1, flags=P.CKV_WO_IS_GRAM)
    assert lib.criticalkv_score(ctypes.byref(d3), p, p, p, p, p, p, None, p, need, None) == P.CKV_E_INVALID_ARG
    d4 = good_desc(d_model=512, norm=P.CKV_NORM_L2, flags=P.CKV_WO_IS_GRAM | P.CKV_NO_MFMA)
    assert lib.criticalkv_score(ctypes.byref(d4), p, p, p, p, p, p, None, p, need, None) == P.CKV_E_INVALID_ARG


def test_binding_raises_with_code():
    d = good_desc(head_dim=96)

    class Fake:
        def data_ptr(self): return 256
        def numel(self): return 1 << 30
        def element_size(self): return 1

    class FakeStream:
        cuda_stream = 0

    f = Fake()
    with pytest.raises(P.CriticalKVError) as e:
        P.criticalkv_score(d, f, f, f, f, f, f, None, workspace=f, stream=FakeStream())
    assert e.value.code == P.CKV_E_UNSUPPORTED
    # every wrapper reports its library's code (each fails validation before any device call)
    ok = good_desc()
    calls = {
        "criticalkv_allocate": lambda: P.criticalkv_allocate(ok, f, 100, 1.5, f, workspace=f, stream=FakeStream()),
        "criticalkv_select": lambda: P.criticalkv_select(ok, f, f, f, 2.0, 10, f, f, workspace=f, stream=FakeStream()),
        "criticalkv_select_noalloc": lambda: P.criticalkv_select_noalloc(ok, f, f, f, 2.0, 10, f, f, stream=FakeStream()),
        "criticalkv_compact": lambda: P.criticalkv_compact(ok, f, f, f, f, 0, f, f, stream=FakeStream()),
        "criticalkv_diagnostics": lambda: P.criticalkv_diagnostics(ok, f, f, None, f, f, 0, f, workspace=f, stream=FakeStream()),
        "criticalkv_prepare_gram": lambda: P.criticalkv_prepare_gram(good_desc(d_model=512), None, f, workspace=f, stream=FakeStream()),
        "criticalkv_prepare_wo": lambda: P.criticalkv_prepare_wo(ok, None, f, stream=FakeStream()),
    }
    for name, call in calls.items():
        with pytest.raises(P.CriticalKVError) as e:
            call()
        assert e.value.code == P.CKV_E_INVALID_ARG and name in str(e.value), name
    # too small a workspace for the allocation's pooled list
    class Small(Fake):
        def numel(self): return 4096
    with pytest.raises(P.CriticalKVError) as e:
        P.criticalkv_allocate(ok, f, 2000, 0.0, f, workspace=Small(), stream=FakeStream())
    assert e.value.code == P.CKV_E_WORKSPACE
