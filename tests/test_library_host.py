"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes workspaces, and rejects invalid arguments before touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "larosa.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2507_01299_amd import api, build
    if not os.path.exists(api.LIB_PATH):
        build.build_library()
    return api.lib()


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(larosa_[a-z_0-9]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"larosa_rotate", "larosa_topk", "larosa_sparse_gemv", "larosa_layer_forward"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings_and_version(lib):
    from paper_2507_01299_amd import api
    assert api.version() >= 100
    seen = {api.status_string(s) for s in (0, -1, -2, -3, -4, -99)}
    assert len(seen) == 6 and api.status_string(0) == "ok"


def test_workspace_bytes_is_pure_and_monotone(lib):
    a = lib.larosa_workspace_bytes(1, 4096, 4096, 2457)
    b = lib.larosa_workspace_bytes(1, 4096, 22016, 2457)
    c = lib.larosa_workspace_bytes(4, 4096, 22016, 2457)
    assert 0 < a <= b < c and a % 256 == 0
    assert lib.larosa_workspace_bytes(0, 1, 1, 1) == 0


def test_invalid_arguments_are_rejected_on_the_host(lib):
    from paper_2507_01299_amd import api
    null = None
    fake = ctypes.c_void_p(0x1000)        # never dereferenced: checks fail first
    odd = ctypes.c_void_p(0x1004)
    assert lib.larosa_sparse_gemv(null, fake, fake, fake, 1, 64, 64, 8, 0, fake, 1 << 20, null) == api.EINVAL
    assert lib.larosa_sparse_gemv(fake, fake, fake, fake, 1, 64, 64, 0, 0, fake, 1 << 20, null) == api.EINVAL
    assert lib.larosa_sparse_gemv(fake, fake, fake, fake, 1, 64, 64, 65, 0, fake, 1 << 20, null) == api.EINVAL
    assert lib.larosa_sparse_gemv(fake, fake, fake, fake, 1, 64, 60, 8, 0, fake, 1 << 20, null) == api.EINVAL
    assert lib.larosa_sparse_gemv(odd, fake, fake, fake, 1, 64, 64, 8, 0, fake, 1 << 20, null) == api.EINVAL
    assert lib.larosa_sparse_gemv(fake, fake, fake, fake, 1, 64, 64, 8, 7, fake, 1 << 20, null) == api.EINVAL
    assert lib.larosa_sparse_gemv(fake, fake, fake, fake, 1, 64, 64, 8, 0, fake, 16, null) == api.EWORKSPACE
    assert lib.larosa_sparse_gemv(fake, fake, fake, fake, 1, 64, 64, 8, 0, null, 0, null) == api.EWORKSPACE
    assert lib.larosa_topk(fake, 1, 64, 0, fake, null, 0, null, 0, null) == api.EINVAL
    assert lib.larosa_topk(fake, 1, 64, 65, fake, null, 0, null, 0, null) == api.EINVAL
    assert lib.larosa_topk(fake, 1, 65536, 8, fake, null, 0, null, 0, null) == api.EUNSUPPORTED
    assert lib.larosa_rotate(fake, null, fake, 1, 64, 0, fake, 1 << 20, null) == api.EINVAL
    assert lib.larosa_workspace_init(null, 1 << 20, null) == api.EWORKSPACE
    assert lib.larosa_set_tuning(99, 1) == api.EINVAL
    assert lib.larosa_set_tuning(4, 8) == api.EINVAL          # a key that no longer exists
    # every documented key accepts its default and rejects a value out of range
    for key, good, bad in ((0, 0, -1), (1, 112, 0), (2, 0, 3), (3, 1, 2), (5, 0, 4), (6, 0, 4),
                           (7, 32768, 100), (8, 16384, 4), (9, 1, 2), (10, 0, 3)):
        assert lib.larosa_set_tuning(key, bad) == api.EINVAL
        assert lib.larosa_set_tuning(key, good) == api.OK


def test_layer_struct_validation(lib):
    from paper_2507_01299_amd import api
    L = api._Layer(256, 256, 128, 704, 32, 100, 100, 100, 300, 0x1000, 0x1000, 0x1000, 0x1000,
                   None, None, None, None, None, -1.0, 0, 0, None, None)
    n = lib.larosa_layer_workspace_bytes(ctypes.byref(L), 2)
    assert n > 0
    L.K4 = 705
    assert lib.larosa_layer_workspace_bytes(ctypes.byref(L), 2) == 0
    L.K4 = 300
    L.head_dim = 48
    assert lib.larosa_layer_workspace_bytes(ctypes.byref(L), 2) == 0
    L.head_dim = 32
    L.shortcut_mlp = 0x1004                      # misaligned adapter
    assert lib.larosa_layer_workspace_bytes(ctypes.byref(L), 2) == 0
    L.shortcut_mlp = 0x3000
    assert lib.larosa_layer_workspace_bytes(ctypes.byref(L), 2) >= n       # two more stage buffers
    L.shortcut_mlp = None
    fake = ctypes.c_void_p(0x1000)
    assert lib.larosa_layer_forward(ctypes.byref(L), fake, fake, 1, None, fake, n, None) == api.EINVAL  # x_out aliases x
    assert lib.larosa_layer_forward(ctypes.byref(L), fake, ctypes.c_void_p(0x2000), 1, None, fake, 16, None) == api.EWORKSPACE
    # the layer split around a caller's attention core
    other = ctypes.c_void_p(0x2000)
    assert lib.larosa_layer_qkv(ctypes.byref(L), fake, None, None, 1, None, fake, n, None) == api.EINVAL          # no qkv
    assert lib.larosa_layer_qkv(ctypes.byref(L), None, other, None, 1, None, fake, n, None) == api.EINVAL
    assert lib.larosa_layer_qkv(ctypes.byref(L), fake, other, None, 1, None, fake, 16, None) == api.EWORKSPACE
    L.shortcut_attn = 0x3000
    n2 = lib.larosa_layer_workspace_bytes(ctypes.byref(L), 2)
    assert lib.larosa_layer_qkv(ctypes.byref(L), fake, other, None, 1, None, fake, n2, None) == api.EINVAL        # s1 required
    L.shortcut_attn = None
    assert lib.larosa_layer_after_attention(ctypes.byref(L), fake, None, other, 1, None, fake, n, None) == api.EINVAL
    assert lib.larosa_layer_after_attention(ctypes.byref(L), fake, other, fake, 1, None, fake, n, None) == api.EINVAL  # aliasing
    assert lib.larosa_layer_after_attention(ctypes.byref(L), fake, other, ctypes.c_void_p(0x4000), 1, None, fake, 16,
                                            None) == api.EWORKSPACE
    L.attn_mode = 1
    assert lib.larosa_layer_forward(ctypes.byref(L), fake, other, 1, None, fake, n, None) == api.EUNSUPPORTED
    L.attn_mode = 0


def test_offline_calls_reject_invalid_arguments(lib):
    from paper_2507_01299_amd import api
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1004)
    big = 1 << 30
    assert lib.larosa_offline_workspace_bytes(4096, 0) == 2 * 2 * 4096 * 4096 * 2
    assert lib.larosa_offline_workspace_bytes(4096, 1) == 2 * 3 * 4096 * 4096 * 2
    assert lib.larosa_offline_workspace_bytes(4096, 5) == 0
    assert lib.larosa_second_moment(None, 16, 64, 0, fake, 0, None) == api.EINVAL
    assert lib.larosa_second_moment(fake, 0, 64, 0, fake, 0, None) == api.EINVAL
    assert lib.larosa_second_moment(fake, 16, 60, 0, fake, 0, None) == api.EINVAL
    assert lib.larosa_second_moment(odd, 16, 64, 0, fake, 0, None) == api.EINVAL
    assert lib.larosa_fold_input(fake, fake, 64, 64, 0, fake, fake, big, None) == api.EINVAL      # aliasing
    assert lib.larosa_fold_input(fake, fake, 64, 60, 0, odd, fake, big, None) == api.EINVAL
    other = ctypes.c_void_p(0x2000)
    assert lib.larosa_fold_input(fake, fake, 64, 64, 0, other, fake, 16, None) == api.EWORKSPACE
    assert lib.larosa_fold_output(fake, fake, 64, 64, 0, other, None, big, None) == api.EWORKSPACE
    assert lib.larosa_fold_output(fake, fake, 12, 64, 0, other, fake, big, None) == api.EINVAL
    assert lib.larosa_residual_adapter(fake, fake, 64, 2, other, fake, big, None) == api.EINVAL
    assert lib.larosa_residual_adapter(fake, fake, 64, 1, other, fake, 3 * 64 * 64 * 2, None) == api.EWORKSPACE


def test_w4_and_threshold_calls_reject_invalid_arguments(lib):
    from paper_2507_01299_amd import api
    fake = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1002)
    big = 1 << 24
    assert lib.larosa_quantize_w4(None, 8, 64, 0, fake, fake, None) == api.EINVAL
    assert lib.larosa_quantize_w4(fake, 8, 60, 0, fake, fake, None) == api.EINVAL
    assert lib.larosa_quantize_w4(fake, 0, 64, 0, fake, fake, None) == api.EINVAL
    assert lib.larosa_quantize_w4(fake, 8, 64, 3, fake, fake, None) == api.EINVAL
    assert lib.larosa_sparse_gemv_w4(fake, None, fake, fake, fake, 1, 64, 64, 8, 0, fake, big, None) == api.EINVAL
    assert lib.larosa_sparse_gemv_w4(fake, fake, fake, None, fake, 1, 64, 64, 8, 0, fake, big, None) == api.EINVAL
    assert lib.larosa_sparse_gemv_w4(fake, fake, fake, fake, fake, 1, 64, 64, 65, 0, fake, big, None) == api.EINVAL
    assert lib.larosa_sparse_gemv_w4(fake, fake, odd, fake, fake, 1, 64, 64, 8, 0, fake, big, None) == api.EINVAL
    assert lib.larosa_sparse_gemv_w4(fake, fake, fake, fake, fake, 1, 64, 64, 8, 0, fake, 16, None) == api.EWORKSPACE
    f = ctypes.c_float
    assert lib.larosa_threshold_select(None, 1, 64, f(0.1), 0, fake, fake, None) == api.EINVAL
    assert lib.larosa_threshold_select(fake, 1, 60, f(0.1), 0, fake, fake, None) == api.EINVAL
    assert lib.larosa_threshold_select(fake, 1, 64, f(-1.0), 0, fake, fake, None) == api.EINVAL
    assert lib.larosa_threshold_select(fake, 1, 64, f(float("nan")), 0, fake, fake, None) == api.EINVAL
    assert lib.larosa_threshold_select(fake, 1, 65536, f(0.1), 0, fake, fake, None) == api.EUNSUPPORTED
