"""Host-only checks of the C ABI: the built library loads, exports every function
the public header declares, and its size queries behave.  No GPU call is made."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mpcpipe.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2209_13643_amd import mpc
    if not os.path.exists(mpc.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return mpc.lib()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mpc_[a-z0-9_]+)\s*\(", text)))


def test_header_functions_are_exported(lib):
    names = declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mpcpipe.h but not exported"


def test_binding_lists_every_declared_function():
    from paper_2209_13643_amd import mpc
    assert sorted(mpc.EXPORTS) == declared_functions()


def test_strerror(lib):
    assert lib.mpc_strerror(0) == b"success"
    for code in (-1, -2, -3, -4):
        assert len(lib.mpc_strerror(code)) > 10
    assert b"unknown" in lib.mpc_strerror(-99)


def test_workspace_queries(lib):
    # digit planes alone: 3 left + 3 right operands, 8 bytes per (padded) element
    M, K, N = 256, 64, 128
    ws = lib.mpc_matmul_workspace_bytes(M, K, N, 1)
    assert ws >= 3 * 8 * M * K + 3 * 8 * K * N + 4 * 8 * M * K + 4 * 8 * K * N
    assert lib.mpc_matmul_workspace_bytes(M, K, N, 2) > ws
    assert lib.mpc_matmul_workspace_bytes(0, K, N, 1) == 0
    assert lib.mpc_matmul_workspace_bytes(M, 1 << 20, N, 1) > ws          # long contractions are cut into exact slices
    assert lib.mpc_matmul_workspace_bytes(M, (1 << 22) + 1, N, 1) == 0    # beyond MPC_MAX_K_TOTAL
    assert lib.mpc_conv2d_workspace_bytes(2, 8, 8, 3, 16, 3, 3, 1, 1) > 0
    assert lib.mpc_conv2d_workspace_bytes(2, 8, 8, 3, 16, 3, 3, 1, 0) == 0
    assert lib.mpc_relu_workspace_bytes(1000) >= 2 * (8 * 1000 * 8 + 2 * 1000 * 8)
    assert lib.mpc_relu_workspace_bytes(0) == 0
    assert lib.mpc_maxpool_workspace_bytes(1, 4, 4, 2) > lib.mpc_relu_workspace_bytes(16)
    assert lib.mpc_maxpool_workspace_bytes(1, 3, 4, 2) == 0               # odd height


def test_null_context_is_rejected(lib):
    # argument validation happens before any device work
    assert lib.mpc_ctx_sync(None) == -1
    assert lib.mpc_ctx_destroy(None) == -1
    assert lib.mpc_ctx_create(None, 0, 16) == -1
    h = ctypes.c_void_p()
    assert lib.mpc_ctx_create(ctypes.byref(h), 0, 99) == -1              # frac_bits out of range
