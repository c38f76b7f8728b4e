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
    assert lib.mpc_ctx_create_single_queue(None, 0, 16) == -1
    assert lib.mpc_ctx_create_single_queue(ctypes.byref(h), 0, -1) == -1
    r = ctypes.c_double()
    assert lib.mpc_mfma_rate(None, 1, 100, 1, ctypes.byref(r)) == -1


def test_packed_triple_layout_size(lib):
    """mpc_relu_packed_words against the layout as the header states it: triple 0 on plain
    words, triple t = 1..11 on ceil64(n) / 2^(l+1) words with l = (t-1)/2, every segment
    padded to a multiple of four words."""
    r4 = lambda v: (v + 3) // 4 * 4
    for n in (1, 2, 63, 64, 65, 1000, 4096, 4097, 1 << 20, (1 << 21) + 5):
        n64 = (n + 63) // 64 * 64
        want = r4(n) + sum(r4(n64 >> ((t - 1) // 2 + 1)) for t in range(1, 12))
        assert lib.mpc_relu_packed_words(n) == want, n
    assert lib.mpc_relu_packed_words(0) == 0
    assert lib.mpc_relu_msb_workspace_bytes(1 << 20) > 0 and lib.mpc_relu_msb_workspace_bytes(0) == 0
    assert lib.mpc_maxpool_msb_workspace_bytes(1, 3, 4, 2) == 0


def test_prepared_plane_sizes(lib):
    """Three right and two left plane tensors, eight digit planes of [rows][K padded to 32] bytes each."""
    r, l = ctypes.c_size_t(), ctypes.c_size_t()
    M, K, N = 96, 100, 40
    assert lib.mpc_matmul_prepared_bytes(M, K, N, 1, ctypes.byref(r), ctypes.byref(l)) == 0
    kpad = (K + 31) // 32 * 32
    up = lambda v: (v + 255) // 256 * 256
    assert r.value == 3 * up(8 * N * kpad) and l.value == 2 * up(8 * M * kpad)
    assert lib.mpc_matmul_prepared_bytes(M, K, N, 3, ctypes.byref(r), None) == 0 and r.value == 3 * up(3 * 8 * N * kpad)
    assert lib.mpc_matmul_prepared_bytes(0, K, N, 1, ctypes.byref(r), ctypes.byref(l)) == -1
    # conv: activation planes are not expanded by the filter taps (plus one zero row)
    assert lib.mpc_conv2d_prepared_bytes(2, 8, 8, 16, 32, 3, 3, 1, 1, ctypes.byref(r), ctypes.byref(l)) == 0
    assert l.value == 2 * up(8 * (2 * 8 * 8 + 1) * 16)
    assert lib.mpc_conv2d_prepared_bytes(2, 8, 8, 16, 32, 3, 3, 1, 0, ctypes.byref(r), ctypes.byref(l)) == -1


def test_filter_window_larger_than_the_padded_image_is_rejected(lib):
    """H + 2 pad < KH (or the same in W): no output pixel exists; every query and prepare-size call says so,
    whatever the stride (integer division would otherwise round the negative extent up to one pixel)."""
    r, l = ctypes.c_size_t(), ctypes.c_size_t()
    for (H, W, KH, KW, pad, stride) in [(2, 8, 3, 3, 0, 2), (8, 2, 3, 3, 0, 2), (1, 1, 5, 5, 1, 3), (2, 2, 3, 3, 0, 1)]:
        assert lib.mpc_conv2d_workspace_bytes(1, H, W, 4, 4, KH, KW, pad, stride) == 0, (H, W, KH, KW, pad, stride)
        assert lib.mpc_conv2d3_workspace_bytes(1, H, W, 4, 4, KH, KW, pad, stride) == 0
        assert lib.mpc_conv2d_prepared_bytes(1, H, W, 4, 4, KH, KW, pad, stride, ctypes.byref(r), ctypes.byref(l)) == -1
    assert lib.mpc_conv2d_workspace_bytes(1, 3, 3, 4, 4, 3, 3, 0, 2) > 0          # the window just fits


def test_gradient_and_elementwise_workspace_queries(lib):
    assert lib.mpc_conv2d_grad_x_workspace_bytes(2, 8, 8, 3, 16, 3, 3, 1, 1) > 0
    assert lib.mpc_conv2d_grad_x_workspace_bytes(2, 8, 8, 3, 16, 3, 3, 1, 2) > 0       # strided: plus the dilated gradient
    assert lib.mpc_conv2d_grad_x_workspace_bytes(2, 8, 8, 3, 16, 3, 5, 1, 1) == 0      # non-square filter
    assert lib.mpc_conv2d_grad_w_workspace_bytes(2, 8, 8, 3, 16, 3, 3, 1, 2) > 0
    assert lib.mpc_mul_workspace_bytes(1000) >= 8 * 1000 * 8
    assert lib.mpc_maxpool_backward_workspace_bytes(1, 4, 4, 2) > lib.mpc_mul_workspace_bytes(16)
    assert lib.mpc_maxpool_backward_workspace_bytes(1, 4, 5, 2) == 0


def test_three_party_workspace_queries(lib):
    M, K, N = 96, 100, 40
    assert lib.mpc_matmul3_workspace_bytes(M, K, N, 1) > lib.mpc_matmul_workspace_bytes(M, K, N, 1)
    assert lib.mpc_matmul3_workspace_bytes(0, K, N, 1) == 0
    assert lib.mpc_conv2d3_workspace_bytes(2, 8, 8, 3, 16, 3, 3, 1, 1) > lib.mpc_conv2d_workspace_bytes(2, 8, 8, 3, 16, 3, 3, 1, 1)
    assert lib.mpc_conv2d3_workspace_bytes(2, 8, 8, 3, 16, 3, 3, 1, 0) == 0
    up = lambda v: (v + 255) // 256 * 256
    assert lib.mpc_truncate3_workspace_bytes(1000) == 4 * up(8000) and lib.mpc_truncate3_workspace_bytes(0) == 0
    # per party: 18 word arrays (two received A2B words, S, W, P, G, 4 sent and 2 x 4 received words) and 4 byte
    # arrays; then the second set of receive buffers of the remote-store exchange (2 x 4 words per party)
    n = 1000
    assert lib.mpc_relu3_workspace_bytes(n) == 3 * (6 * up(8 * n) + 3 * up(32 * n) + 4 * up(n)) + 6 * up(32 * n)
    assert lib.mpc_relu3_workspace_bytes(0) == 0
    assert lib.mpc_maxpool3_workspace_bytes(1, 4, 4, 2) > lib.mpc_relu3_workspace_bytes(16)
    assert lib.mpc_maxpool3_workspace_bytes(1, 3, 4, 2) == 0               # odd height
    # sign-only chain: two whole-word triples, then eleven packed ones (64, 64, 32, 32, ... words at n = 128,
    # each padded to four: 64+64+32+32+16+16+8+8+4+4+4 = 252)
    assert lib.mpc_relu3_packed_words(128) == 2 * 128 + 252
    assert lib.mpc_relu3_packed_words(1) == 2 * 4 + 32 + 32 + 16 + 16 + 8 + 8 + 4 + 4 + 4 + 4 + 4
    assert lib.mpc_relu3_packed_words(0) == 0
    big = 1 << 20
    assert lib.mpc_relu3_packed_words(big) < 13 * big // 3                 # against 13 n words unpacked
    # one pass over the whole call: the whole-word words of the first two rounds and a block per level
    assert 3 * 11 * 8 * big < lib.mpc_relu3_msb_workspace_bytes(big) < 3 * 30 * 8 * big
    assert lib.mpc_relu3_msb_workspace_bytes(0) == 0
    assert lib.mpc_maxpool3_msb_workspace_bytes(1, 4, 4, 2) > lib.mpc_relu3_msb_workspace_bytes(16)
    assert lib.mpc_maxpool3_msb_workspace_bytes(1, 3, 4, 2) == 0
    # null arguments are rejected before any device work
    assert lib.mpc_open3(None, mpc_null3(), None, 4) == -1


def mpc_null3():
    from paper_2209_13643_amd import mpc
    return mpc.CShare3()


def test_gemm_kernel_leaves_room_for_a_streaming_wave():
    """The digit-plane GEMM owns all 256 accumulator registers of a SIMD; it must stay at or below 120
    vector registers, so that 136 of the SIMD's 512 remain and a wave of another lane's streaming
    kernel (the secure-ReLU stages use up to 134) fits beside it: the inter-batch pipeline overlaps
    MFMA-bound and HBM-bound work that way.  Compiled here with the resource-usage remarks on (no GPU
    needed)."""
    import subprocess
    import __graft_entry__ as ge
    src = os.path.join(ge.CSRC, "limb_gemm.hip")
    out = subprocess.run([ge.HIPCC, *ge.HIP_FLAGS, "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage",
                          "-c", src, "-o", os.devnull], capture_output=True, text=True)
    assert out.returncode == 0, out.stderr[-2000:]
    rows = re.findall(r"Function Name: (\S+).*?VGPRs: (\d+).*?AGPRs: (\d+).*?VGPRs Spill: (\d+)", out.stderr, flags=re.S)
    gemm = [(n, int(v), int(a), int(sp)) for n, v, a, sp in rows if "k_limb_gemm" in n]
    assert len(gemm) == 6, [r[0] for r in gemm]
    full = [r for r in gemm if r[2] == 256]
    half = [r for r in gemm if r[2] == 128]          # the half-width wave tile of short contractions: two waves per SIMD
    assert len(full) == 4 and len(half) == 2, gemm
    for name, vgprs, agprs, spill in full:
        assert spill == 0 and vgprs <= 120, (name, vgprs, agprs, spill)
    for name, vgprs, agprs, spill in half:
        assert spill == 0 and vgprs <= 128, (name, vgprs, agprs, spill)


def test_relu_stage_kernels_fit_beside_the_gemm():
    """... and the other half of that budget: every secure-ReLU stage kernel stays within 136 vector registers."""
    import subprocess
    import __graft_entry__ as ge
    out = subprocess.run([ge.HIPCC, *ge.HIP_FLAGS, "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage",
                          "-c", os.path.join(ge.CSRC, "relu.hip"), "-o", os.devnull], capture_output=True, text=True)
    assert out.returncode == 0, out.stderr[-2000:]
    rows = re.findall(r"Function Name: (\S+).*?VGPRs: (\d+).*?AGPRs: (\d+)", out.stderr, flags=re.S)
    stages = [(n, int(v) + int(a)) for n, v, a in rows if "k_relu_stage" in n or "k_relu_msb_stage" in n]
    assert len(stages) > 50
    worst = max(stages, key=lambda r: r[1])
    assert worst[1] <= 136, worst
    # the three-party kernels: the same budget, and nothing spilled
    out = subprocess.run([ge.HIPCC, *ge.HIP_FLAGS, "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage",
                          "-c", os.path.join(ge.CSRC, "three_party.hip"), "-o", os.devnull], capture_output=True, text=True)
    assert out.returncode == 0, out.stderr[-2000:]
    rows = re.findall(r"Function Name: (\S+).*?VGPRs: (\d+).*?AGPRs: (\d+).*?ScratchSize \[bytes/lane\]: (\d+)", out.stderr, flags=re.S)
    assert len(rows) > 40
    for name, v, a, scratch in rows:
        assert int(v) + int(a) <= 136 and int(scratch) == 0, (name, v, a, scratch)
