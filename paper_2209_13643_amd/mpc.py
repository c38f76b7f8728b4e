"""ctypes binding over libmpcpipe (the C ABI in include/mpcpipe.h).

Argument marshalling only: every protocol step runs in the library's HIP
kernels.  torch is used for device memory (int64 tensors carry the uint64 ring
elements bit for bit) and nothing else.  There is no CPU fallback: if the
library is missing or the device is absent, calls raise.
"""
from __future__ import annotations

import ctypes
import threading
import os
from ctypes import POINTER, byref, c_int, c_size_t, c_uint8, c_uint64, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmpcpipe.so")

MPC_TRUNCATE = 1
MPC_TRANS_X = 4
MPC_TRANS_Y = 8
MPC_FOLDED = 16
MPC_TWO_PHASE = 2
PROF_GEMM_KERNEL, PROF_LINEAR, PROF_RELU = 0, 1, 2
N_AND_TRIPLES = 12

_P64 = POINTER(c_uint64)
_P8 = POINTER(c_uint8)


class CShare(ctypes.Structure):
    _fields_ = [("p", _P64 * 2)]


class ReluMaterial(ctypes.Structure):
    _fields_ = [("r", CShare), ("and_a", CShare), ("and_b", CShare), ("and_c", CShare),
                ("rb", _P8 * 2), ("ra", CShare), ("ma", CShare), ("mb", CShare), ("mc", CShare)]


class CShare3(ctypes.Structure):
    _fields_ = [("p", _P64 * 3)]


class Relu3Material(ctypes.Structure):
    _fields_ = [("r0", CShare3), ("r1", CShare3), ("and_a", CShare3), ("and_b", CShare3), ("and_c", CShare3),
                ("rb", _P8 * 3), ("ra", CShare3), ("ma", CShare3), ("mb", CShare3), ("mc", CShare3)]


N_AND_TRIPLES3 = 13

EXPORTS = [
    "mpc_ctx_create", "mpc_ctx_destroy", "mpc_ctx_set_streams", "mpc_ctx_stream", "mpc_ctx_set_workspace",
    "mpc_ctx_create_single_queue", "mpc_ctx_sync", "mpc_ctx_wait", "mpc_last_hip_error", "mpc_strerror",
    "mpc_ctx_set_profiling", "mpc_ctx_profile", "mpc_ctx_profile_reset",
    "mpc_matmul_workspace_bytes", "mpc_conv2d_workspace_bytes", "mpc_relu_workspace_bytes",
    "mpc_maxpool_workspace_bytes", "mpc_open", "mpc_sub", "mpc_beaver_matmul", "mpc_conv2d", "mpc_truncate",
    "mpc_relu", "mpc_maxpool2x2", "mpc_ring_matmul", "mpc_ring_conv2d", "mpc_relu_static", "mpc_relu_static_max_n",
    "mpc_relu_msb_workspace_bytes", "mpc_maxpool_msb_workspace_bytes", "mpc_relu_packed_words",
    "mpc_relu_pack_triples", "mpc_relu_msb", "mpc_maxpool2x2_msb",
    "mpc_conv2d_grad_x_workspace_bytes", "mpc_conv2d_grad_w_workspace_bytes", "mpc_conv2d_grad_x",
    "mpc_conv2d_grad_w", "mpc_mul_workspace_bytes", "mpc_mul", "mpc_relu_backward",
    "mpc_ring_conv2d_grad_x", "mpc_ring_conv2d_grad_w",
    "mpc_maxpool2x2_signs", "mpc_maxpool_backward_workspace_bytes", "mpc_maxpool2x2_backward",
    "mpc_ctx_set_adder", "mpc_ctx_set_exchange", "mpc_ctx_profile_samples", "mpc_add",
    "mpc_matmul_prepared_bytes", "mpc_conv2d_prepared_bytes", "mpc_matmul_prepare", "mpc_conv2d_prepare",
    "mpc_beaver_matmul_prepared", "mpc_conv2d_prepared", "mpc_beaver_matmul_folded", "mpc_matmul_fold", "mpc_conv2d_fold", "mpc_set_gemm_small_tile", "mpc_mfma_rate", "mpc_ctx_set_relu_chunk",
    "mpc_ctx_capture_begin", "mpc_ctx_capture_end", "mpc_graph_launch", "mpc_graph_destroy",
    "mpc_open3", "mpc_matmul3_workspace_bytes", "mpc_beaver_matmul3", "mpc_conv2d3_workspace_bytes", "mpc_conv2d3",
    "mpc_truncate3_workspace_bytes", "mpc_truncate3", "mpc_relu3_workspace_bytes", "mpc_relu3",
    "mpc_maxpool3_workspace_bytes", "mpc_maxpool3",
    "mpc_relu3_packed_words", "mpc_relu3_pack_triples", "mpc_relu3_msb_workspace_bytes", "mpc_relu3_msb",
    "mpc_maxpool3_msb_workspace_bytes", "mpc_maxpool3_msb",
    "mpc_matmul3_prepared_bytes", "mpc_conv2d3_prepared_bytes", "mpc_matmul3_prepare", "mpc_conv2d3_prepare",
    "mpc_beaver_matmul3_prepared", "mpc_conv2d3_prepared",
    "mpc_conv2d3_grad_x_workspace_bytes", "mpc_conv2d3_grad_w_workspace_bytes", "mpc_conv2d3_grad_x", "mpc_conv2d3_grad_w",
    "mpc_add3", "mpc_sub3", "mpc_mul3_workspace_bytes", "mpc_mul3", "mpc_relu3_backward", "mpc_maxpool3_signs",
    "mpc_maxpool3_backward_workspace_bytes", "mpc_maxpool3_backward",
]

_lib = None


def lib():
    """Load the shared library (built by __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'`")
    L = ctypes.CDLL(LIB_PATH)
    L.mpc_ctx_create.argtypes = [POINTER(c_void_p), c_int, c_int]
    L.mpc_ctx_create_single_queue.argtypes = [POINTER(c_void_p), c_int, c_int]
    L.mpc_ctx_destroy.argtypes = [c_void_p]
    L.mpc_ctx_set_adder.argtypes = [c_void_p, c_int]
    L.mpc_add.argtypes = [c_void_p, CShare, CShare, CShare, c_size_t]
    L.mpc_ctx_capture_begin.argtypes = [c_void_p]
    L.mpc_ctx_capture_end.argtypes = [c_void_p, POINTER(c_void_p)]
    L.mpc_graph_launch.argtypes = [c_void_p, c_void_p]
    L.mpc_graph_destroy.argtypes = [c_void_p]
    L.mpc_matmul_prepared_bytes.argtypes = [c_int] * 4 + [POINTER(c_size_t)] * 2
    L.mpc_conv2d_prepared_bytes.argtypes = [c_int] * 9 + [POINTER(c_size_t)] * 2
    L.mpc_matmul_prepare.argtypes = [c_void_p, CShare, CShare, _P64, c_void_p, c_void_p] + [c_int] * 5
    L.mpc_conv2d_prepare.argtypes = [c_void_p, CShare, CShare, _P64, c_void_p, c_void_p] + [c_int] * 9
    L.mpc_beaver_matmul_prepared.argtypes = [c_void_p, CShare, CShare, CShare, CShare, c_void_p, c_void_p] + [c_int] * 6
    L.mpc_conv2d_prepared.argtypes = [c_void_p, CShare, CShare, CShare, CShare, c_void_p, c_void_p] + [c_int] * 11
    L.mpc_beaver_matmul_folded.argtypes = [c_void_p] + [CShare] * 6 + [c_void_p, c_void_p] + [c_int] * 6
    L.mpc_set_gemm_small_tile.argtypes = [c_int, c_int]
    L.mpc_ctx_set_relu_chunk.argtypes = [c_void_p, c_size_t, c_size_t]
    L.mpc_mfma_rate.argtypes = [c_void_p, c_int, c_int, c_int, POINTER(ctypes.c_double)]
    L.mpc_matmul_fold.argtypes = [c_void_p, _P64, _P64, _P64, _P64] + [c_int] * 5
    L.mpc_conv2d_fold.argtypes = [c_void_p, _P64, _P64, _P64, _P64] + [c_int] * 9
    L.mpc_ctx_profile_samples.argtypes = [c_void_p, c_int, POINTER(ctypes.c_double), c_int, POINTER(c_int)]
    L.mpc_ctx_set_exchange.argtypes = [c_void_p, c_int]
    L.mpc_ctx_set_streams.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    L.mpc_ctx_stream.argtypes = [c_void_p, c_int]; L.mpc_ctx_stream.restype = c_void_p
    L.mpc_ctx_set_workspace.argtypes = [c_void_p, c_void_p, c_size_t]
    L.mpc_ctx_sync.argtypes = [c_void_p]
    L.mpc_ctx_wait.argtypes = [c_void_p, c_void_p]
    L.mpc_ctx_set_profiling.argtypes = [c_void_p, c_int]
    L.mpc_ctx_profile.argtypes = [c_void_p, c_int, POINTER(ctypes.c_double), POINTER(c_int)]
    L.mpc_ctx_profile_reset.argtypes = [c_void_p]
    L.mpc_last_hip_error.argtypes = [c_void_p]
    L.mpc_strerror.argtypes = [c_int]; L.mpc_strerror.restype = ctypes.c_char_p
    L.mpc_matmul_workspace_bytes.argtypes = [c_int] * 4; L.mpc_matmul_workspace_bytes.restype = c_size_t
    L.mpc_conv2d_workspace_bytes.argtypes = [c_int] * 9; L.mpc_conv2d_workspace_bytes.restype = c_size_t
    L.mpc_relu_workspace_bytes.argtypes = [c_size_t]; L.mpc_relu_workspace_bytes.restype = c_size_t
    L.mpc_maxpool_workspace_bytes.argtypes = [c_int] * 4; L.mpc_maxpool_workspace_bytes.restype = c_size_t
    L.mpc_relu_msb_workspace_bytes.argtypes = [c_size_t]; L.mpc_relu_msb_workspace_bytes.restype = c_size_t
    L.mpc_maxpool_msb_workspace_bytes.argtypes = [c_int] * 4; L.mpc_maxpool_msb_workspace_bytes.restype = c_size_t
    L.mpc_relu_packed_words.argtypes = [c_size_t]; L.mpc_relu_packed_words.restype = c_size_t
    L.mpc_relu_pack_triples.argtypes = [c_void_p, CShare, CShare, c_size_t]
    L.mpc_open.argtypes = [c_void_p, CShare, _P64, c_size_t]
    L.mpc_sub.argtypes = [c_void_p, CShare, CShare, CShare, c_size_t]
    L.mpc_beaver_matmul.argtypes = [c_void_p] + [CShare] * 6 + [c_int] * 4 + [_P64, c_int, c_int]
    L.mpc_conv2d.argtypes = [c_void_p] + [CShare] * 6 + [c_int] * 9 + [_P64, c_int, c_int]
    L.mpc_truncate.argtypes = [c_void_p, CShare, c_size_t, c_int]
    for name in ("mpc_conv2d_grad_x_workspace_bytes", "mpc_conv2d_grad_w_workspace_bytes"):
        getattr(L, name).argtypes = [c_int] * 9; getattr(L, name).restype = c_size_t
    L.mpc_conv2d_grad_x.argtypes = L.mpc_conv2d.argtypes
    L.mpc_conv2d_grad_w.argtypes = L.mpc_conv2d.argtypes
    L.mpc_mul_workspace_bytes.argtypes = [c_size_t]; L.mpc_mul_workspace_bytes.restype = c_size_t
    L.mpc_ring_conv2d_grad_x.argtypes = [c_void_p, _P64, _P64, _P64] + [c_int] * 9
    L.mpc_ring_conv2d_grad_w.argtypes = [c_void_p, _P64, _P64, _P64] + [c_int] * 9
    L.mpc_mul.argtypes = [c_void_p] + [CShare] * 6 + [c_size_t, c_int]
    L.mpc_relu_backward.argtypes = [c_void_p] + [CShare] * 6 + [c_size_t]
    L.mpc_relu.argtypes = [c_void_p, CShare, POINTER(ReluMaterial), CShare, c_size_t, c_int,
                           POINTER(_P8 * 2), POINTER(_P64 * 2)]
    L.mpc_maxpool2x2.argtypes = [c_void_p, CShare, POINTER(ReluMaterial), POINTER(ReluMaterial), CShare,
                                 c_int, c_int, c_int, c_int, c_int]
    L.mpc_relu_msb.argtypes = L.mpc_relu.argtypes
    L.mpc_relu_static.argtypes = L.mpc_relu.argtypes
    L.mpc_relu_static_max_n.argtypes = []; L.mpc_relu_static_max_n.restype = c_size_t
    L.mpc_maxpool2x2_signs.argtypes = [c_void_p, CShare, POINTER(ReluMaterial), POINTER(ReluMaterial), CShare,
                                       POINTER(_P64 * 2), POINTER(_P64 * 2)] + [c_int] * 6
    L.mpc_maxpool_backward_workspace_bytes.argtypes = [c_int] * 4
    L.mpc_maxpool_backward_workspace_bytes.restype = c_size_t
    L.mpc_maxpool2x2_backward.argtypes = [c_void_p] + [CShare] * 10 + [c_int] * 4
    L.mpc_maxpool2x2_msb.argtypes = L.mpc_maxpool2x2.argtypes
    L.mpc_ring_matmul.argtypes = [c_void_p, _P64, _P64, _P64] + [c_int] * 4
    L.mpc_ring_conv2d.argtypes = [c_void_p, _P64, _P64, _P64] + [c_int] * 9
    L.mpc_open3.argtypes = [c_void_p, CShare3, _P64, c_size_t]
    L.mpc_matmul3_workspace_bytes.argtypes = [c_int] * 4; L.mpc_matmul3_workspace_bytes.restype = c_size_t
    L.mpc_conv2d3_workspace_bytes.argtypes = [c_int] * 9; L.mpc_conv2d3_workspace_bytes.restype = c_size_t
    L.mpc_beaver_matmul3.argtypes = [c_void_p] + [CShare3] * 6 + [c_int] * 4 + [_P64, c_int]
    L.mpc_conv2d3.argtypes = [c_void_p] + [CShare3] * 6 + [c_int] * 9 + [_P64]
    L.mpc_truncate3_workspace_bytes.argtypes = [c_size_t]; L.mpc_truncate3_workspace_bytes.restype = c_size_t
    L.mpc_truncate3.argtypes = [c_void_p, CShare3, CShare3, CShare3, c_size_t, c_int]
    L.mpc_relu3_workspace_bytes.argtypes = [c_size_t]; L.mpc_relu3_workspace_bytes.restype = c_size_t
    L.mpc_relu3.argtypes = [c_void_p, CShare3, POINTER(Relu3Material), CShare3, c_size_t,
                            POINTER(_P8 * 3), POINTER(_P64 * 3)]
    L.mpc_maxpool3_workspace_bytes.argtypes = [c_int] * 4; L.mpc_maxpool3_workspace_bytes.restype = c_size_t
    L.mpc_maxpool3.argtypes = [c_void_p, CShare3, POINTER(Relu3Material), POINTER(Relu3Material), CShare3] + [c_int] * 4
    L.mpc_relu3_packed_words.argtypes = [c_size_t]; L.mpc_relu3_packed_words.restype = c_size_t
    L.mpc_relu3_pack_triples.argtypes = [c_void_p, CShare3, CShare3, c_size_t]
    L.mpc_relu3_msb_workspace_bytes.argtypes = [c_size_t]; L.mpc_relu3_msb_workspace_bytes.restype = c_size_t
    L.mpc_relu3_msb.argtypes = L.mpc_relu3.argtypes
    L.mpc_maxpool3_msb_workspace_bytes.argtypes = [c_int] * 4; L.mpc_maxpool3_msb_workspace_bytes.restype = c_size_t
    L.mpc_maxpool3_msb.argtypes = L.mpc_maxpool3.argtypes
    L.mpc_matmul3_prepared_bytes.argtypes = [c_int] * 4 + [POINTER(c_size_t)] * 2
    L.mpc_conv2d3_prepared_bytes.argtypes = [c_int] * 9 + [POINTER(c_size_t)] * 2
    L.mpc_matmul3_prepare.argtypes = [c_void_p, CShare3, CShare3, _P64, c_void_p, c_void_p] + [c_int] * 5
    L.mpc_conv2d3_prepare.argtypes = [c_void_p, CShare3, CShare3, _P64, c_void_p, c_void_p] + [c_int] * 9
    L.mpc_beaver_matmul3_prepared.argtypes = [c_void_p, CShare3, CShare3, CShare3, CShare3, c_void_p, c_void_p] + [c_int] * 5
    L.mpc_conv2d3_prepared.argtypes = [c_void_p, CShare3, CShare3, CShare3, CShare3, c_void_p, c_void_p] + [c_int] * 9
    for fn in (L.mpc_conv2d3_grad_x_workspace_bytes, L.mpc_conv2d3_grad_w_workspace_bytes):
        fn.argtypes = [c_int] * 9; fn.restype = c_size_t
    L.mpc_conv2d3_grad_x.argtypes = [c_void_p] + [CShare3] * 6 + [c_int] * 9 + [_P64]
    L.mpc_conv2d3_grad_w.argtypes = [c_void_p] + [CShare3] * 6 + [c_int] * 9
    L.mpc_add3.argtypes = [c_void_p, CShare3, CShare3, CShare3, c_size_t]
    L.mpc_sub3.argtypes = [c_void_p, CShare3, CShare3, CShare3, c_size_t]
    L.mpc_mul3_workspace_bytes.argtypes = [c_size_t]; L.mpc_mul3_workspace_bytes.restype = c_size_t
    L.mpc_mul3.argtypes = [c_void_p] + [CShare3] * 6 + [c_size_t]
    L.mpc_relu3_backward.argtypes = [c_void_p] + [CShare3] * 6 + [c_size_t]
    L.mpc_maxpool3_signs.argtypes = [c_void_p, CShare3, POINTER(Relu3Material), POINTER(Relu3Material), CShare3,
                                     POINTER(_P64 * 3), POINTER(_P64 * 3)] + [c_int] * 5
    L.mpc_maxpool3_backward_workspace_bytes.argtypes = [c_int] * 4; L.mpc_maxpool3_backward_workspace_bytes.restype = c_size_t
    L.mpc_maxpool3_backward.argtypes = [c_void_p] + [CShare3] * 10 + [c_int] * 4
    _lib = L
    return L


class MpcError(RuntimeError):
    pass


# Argument lifetime.  The calls only enqueue work, and torch's allocator knows nothing about a lane's queues: a
# tensor passed as a temporary would go back to the allocator when the call returns and could be handed out (and
# overwritten) while the enqueued kernels still read it.  Every tensor whose pointer is marshalled is therefore
# noted here and kept by the lane (Lane._check) until the lane is next synchronised.
_marshalled = threading.local()


def _note(t):
    lst = getattr(_marshalled, "tensors", None)
    if lst is None:
        lst = _marshalled.tensors = []
    lst.append(t)


def _take_noted():
    lst = getattr(_marshalled, "tensors", None)
    _marshalled.tensors = []
    return lst or []


def _p64(t):
    if t is None:
        return ctypes.cast(None, _P64)
    assert t.is_cuda and t.is_contiguous() and t.dtype == torch.int64, "int64 contiguous device tensor expected"
    _note(t)
    return ctypes.cast(t.data_ptr(), _P64)


def _p8(t):
    if t is None:
        return ctypes.cast(None, _P8)
    assert t.is_cuda and t.is_contiguous() and t.dtype == torch.uint8
    _note(t)
    return ctypes.cast(t.data_ptr(), _P8)


def _share(pair):
    s = CShare()
    if pair is None:
        pair = (None, None)
    s.p[0], s.p[1] = _p64(pair[0]), _p64(pair[1])
    return s


def _share3(tri):
    s = CShare3()
    if tri is None:
        tri = (None, None, None)
    if len(tri) != 3:
        raise ValueError("a three-party sharing is a triple of tensors")
    for i in range(3):
        s.p[i] = _p64(tri[i])
    return s


def _material3(mat: dict, n: int, packed: bool = False) -> Relu3Material:
    m = Relu3Material()
    tw = lib().mpc_relu3_packed_words(n) if packed else N_AND_TRIPLES3 * n
    for key in ("r0", "r1", "ra", "ma", "mb", "mc"):
        if any(t.numel() != n for t in mat[key]):
            raise ValueError(f"material '{key}': {n} words per party expected")
        setattr(m, key, _share3(mat[key]))
    for key in ("and_a", "and_b", "and_c"):
        if any(t.numel() != tw for t in mat[key]):
            raise ValueError(f"material '{key}': {tw} words per party expected ({'packed' if packed else '[13][n]'} layout)")
        setattr(m, key, _share3(mat[key]))
    if any(t.numel() != n for t in mat["rb"]):
        raise ValueError("material 'rb': one byte per element and party expected")
    for i in range(3):
        m.rb[i] = _p8(mat["rb"][i])
    return m


def to_device(arr, device="cuda:0"):
    """numpy uint64 / uint8 array -> device tensor with the same bits."""
    import numpy as np
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(a).to(device)


def to_host(t):
    """device int64 tensor -> numpy uint64 (uint8 stays uint8)."""
    import numpy as np
    a = t.cpu().numpy()
    return a.view(np.uint64) if a.dtype == np.int64 else a


def material_to_device(mat: dict, device="cuda:0") -> dict:
    return {k: tuple(to_device(q, device) for q in v) for k, v in mat.items()}


def _material(mat: dict, n: int, packed: bool = False) -> ReluMaterial:
    """Marshal a material dict; `packed`: and_a/b/c hold the packed layout of mpc_relu_msb."""
    m = ReluMaterial()
    n_and = lib().mpc_relu_packed_words(n) if packed else N_AND_TRIPLES * n
    for key in ("r", "ra", "ma", "mb", "mc"):
        assert mat[key][0].numel() == n and mat[key][1].numel() == n, key
        setattr(m, key, _share(mat[key]))
    for key in ("and_a", "and_b", "and_c"):
        assert mat[key][0].numel() == n_and and mat[key][1].numel() == n_and, key
        setattr(m, key, _share(mat[key]))
    assert mat["rb"][0].numel() == n and mat["rb"][1].numel() == n
    m.rb[0], m.rb[1] = _p8(mat["rb"][0]), _p8(mat["rb"][1])
    return m


class Graph:
    """A recorded sequence of lane calls (Lane.capture); launch() enqueues one replay."""

    def __init__(self, handle, keep):
        self._h = handle
        self._keep = keep          # tensors the recorded calls allocated: must stay in place

    def launch(self, lane: "Lane"):
        lane._check(lib().mpc_graph_launch(self._h, lane._h))

    def close(self):
        if self._h:
            lib().mpc_graph_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class _Capture:
    def __init__(self, lane):
        self.lane = lane; self.graph = None

    def __enter__(self):
        self.lane._check(lib().mpc_ctx_capture_begin(self.lane._h))
        return self

    def __exit__(self, exc_type, exc, tb):
        h = c_void_p()
        rc = lib().mpc_ctx_capture_end(self.lane._h, byref(h))
        if exc_type is None:
            self.lane._check(rc)
            self.graph = Graph(h, [self.lane._ws])
        return False


def set_gemm_small_tile(max_steps: int = 16, min_tiles: int = 512):
    """Process-wide tuning of the GEMM's tile choice (mpc_set_gemm_small_tile); the defaults restore the library's."""
    rc = lib().mpc_set_gemm_small_tile(max_steps, min_tiles)
    if rc != 0:
        raise MpcError(f"mpcpipe error {rc}: {lib().mpc_strerror(rc).decode()}")


class Lane:
    """One execution lane: a library context plus a grow-only workspace."""

    def __init__(self, device: int = 0, frac_bits: int = 16, single_queue: bool = False):
        if not torch.cuda.is_available():
            raise RuntimeError("mpcpipe needs a GPU: no HIP device is visible")
        self.device = torch.device("cuda", device)
        self._h = c_void_p()
        self._pending = []           # tensors the enqueued calls still use (see _note); released by sync()
        create = lib().mpc_ctx_create_single_queue if single_queue else lib().mpc_ctx_create
        self._check(create(byref(self._h), device, frac_bits))
        self._ws = None
        self._ws_bytes = 0

    # -- plumbing
    def _check(self, rc: int):
        self._pending.extend(_take_noted())
        if len(self._pending) > (1 << 17):       # a queue this deep without a sync: let the oldest half go
            del self._pending[: 1 << 16]
        if rc != 0:
            msg = lib().mpc_strerror(rc).decode()
            hip = lib().mpc_last_hip_error(self._h) if self._h else 0
            raise MpcError(f"mpcpipe error {rc}: {msg}" + (f" (hipError {hip})" if rc == -3 else ""))

    def close(self):
        if self._h:
            lib().mpc_ctx_destroy(self._h)
            self._h = c_void_p()
            self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def sync(self):
        self._check(lib().mpc_ctx_sync(self._h))
        self._pending.clear()

    def set_profiling(self, on: bool):
        self._check(lib().mpc_ctx_set_profiling(self._h, 1 if on else 0))

    def profile(self, which: int):
        """(total milliseconds, region count) for PROF_GEMM_KERNEL / PROF_LINEAR / PROF_RELU."""
        ms, cnt = ctypes.c_double(), c_int()
        self._check(lib().mpc_ctx_profile(self._h, which, byref(ms), byref(cnt)))
        return ms.value, cnt.value

    def profile_samples(self, which: int):
        """Every recorded region's duration in milliseconds, in recording order."""
        cnt = c_int()
        self._check(lib().mpc_ctx_profile_samples(self._h, which, None, 0, byref(cnt)))
        buf = (ctypes.c_double * max(cnt.value, 1))()
        self._check(lib().mpc_ctx_profile_samples(self._h, which, buf, cnt.value, byref(cnt)))
        return list(buf)[:cnt.value]

    def profile_reset(self):
        self._check(lib().mpc_ctx_profile_reset(self._h))

    def wait_for(self, other: "Lane"):
        self._check(lib().mpc_ctx_wait(self._h, other._h))

    def wait_torch(self):
        """Order the lane after the work torch has enqueued on its current stream
        (inputs produced by torch ops are otherwise not ordered with the lane's queues)."""
        cur = torch.cuda.current_stream(self.device)
        for s in {self.stream(0), self.stream(1), self.stream(2)}:
            torch.cuda.ExternalStream(s, device=self.device).wait_stream(cur)

    def capture(self):
        """Context manager: record the lane calls made inside it into a Graph (`.graph` afterwards).
        Single-queue lanes only; run the sequence once eagerly first and pass `out=` buffers, since
        a replay reuses the very tensors the recorded calls touched."""
        return _Capture(self)

    def set_exchange(self, mode: str):
        """Secure-ReLU exchange: "copy" (copy kernels on the wire stream) or "put" (the producing
        kernel stores into the peer's receive buffer; single-queue lanes only)."""
        self._check(lib().mpc_ctx_set_exchange(self._h, {"copy": 0, "put": 1}[mode]))

    def set_adder(self, name: str):
        """Carry network of relu / maxpool2x2: "kogge-stone" (default) or "tree" (the listing of Sec. 4.2)."""
        self._check(lib().mpc_ctx_set_adder(self._h, {"kogge-stone": 0, "tree": 1}[name]))

    def set_relu_chunk(self, whole_word_elems: int = 0, packed_elems: int = 0):
        """Elements per chunk of this lane's secure ReLU / max-pool when n_chunks = 0 (0: the library's default)."""
        self._check(lib().mpc_ctx_set_relu_chunk(self._h, whole_word_elems, packed_elems))

    def use_single_queue(self):
        """Issue both parties and the wire on party 0's stream (one in-order queue)."""
        s0 = self.stream(0)
        self._check(lib().mpc_ctx_set_streams(self._h, c_void_p(s0), c_void_p(s0), c_void_p(s0)))

    def stream(self, which: int) -> int:
        return lib().mpc_ctx_stream(self._h, which) or 0

    def reserve(self, nbytes: int):
        """Make the workspace at least nbytes large (syncs the lane if it has to grow)."""
        if nbytes <= 0:
            raise MpcError("workspace query rejected the shape")
        if self._ws is None or self._ws_bytes < nbytes:
            if self._ws is not None:
                self.sync()
            self._ws = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            base = self._ws.data_ptr()
            off = (-base) % 256
            self._check(lib().mpc_ctx_set_workspace(self._h, c_void_p(base + off), nbytes))
            self._ws_bytes = nbytes          # what the library was told, not the tensor's padded size

    # -- protocol calls
    def open(self, s):
        n = s[0].numel()
        self.reserve(2 * (n * 8 + 256))
        out = torch.empty_like(s[0])
        self._check(lib().mpc_open(self._h, _share(s), _p64(out), n))
        return out

    def add(self, x, y, out=None):
        """Local sum of two sharings."""
        if out is None:
            out = (torch.empty_like(x[0]), torch.empty_like(x[1]))
        self._check(lib().mpc_add(self._h, _share(x), _share(y), _share(out), x[0].numel()))
        return out

    def sub(self, x, a, out=None):
        if out is None:
            out = (torch.empty_like(x[0]), torch.empty_like(x[1]))
        self._check(lib().mpc_sub(self._h, _share(x), _share(a), _share(out), x[0].numel()))
        return out

    def beaver_matmul(self, x, y, a, b, c, f_public=None, n_chunks=1, flags=MPC_TRUNCATE, out=None):
        """x, a: [.., M, K] ([.., K, M] with MPC_TRANS_X); y, b: [.., K, N] ([.., N, K] with MPC_TRANS_Y)."""
        shp = a[0].shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = (shp[-1], shp[-2]) if flags & MPC_TRANS_X else (shp[-2], shp[-1])
        K2, N = (b[0].shape[-1], b[0].shape[-2]) if flags & MPC_TRANS_Y else (b[0].shape[-2], b[0].shape[-1])
        assert K2 == K and c[0].shape[-2:] == (M, N)
        self.reserve(lib().mpc_matmul_workspace_bytes(M, K, N, batch))
        z = out if out is not None else (torch.empty_like(c[0]), torch.empty_like(c[1]))
        self._check(lib().mpc_beaver_matmul(self._h, _share(x), _share(y), _share(a), _share(b), _share(c),
                                            _share(z), M, K, N, batch, _p64(f_public), n_chunks, flags))
        return z

    def conv2d(self, x, w, a, b, c, pad, stride, f_public=None, n_chunks=1, flags=MPC_TRUNCATE, out=None):
        B, H, W, Cin = a[0].shape
        KH, KW, Cin2, Cout = b[0].shape
        assert Cin == Cin2
        self.reserve(lib().mpc_conv2d_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        z = out if out is not None else (torch.empty_like(c[0]), torch.empty_like(c[1]))
        self._check(lib().mpc_conv2d(self._h, _share(x), _share(w), _share(a), _share(b), _share(c), _share(z),
                                     B, H, W, Cin, Cout, KH, KW, pad, stride, _p64(f_public), n_chunks, flags))
        return z

    # -- prepared layers: digit planes of the input-independent operands, recoded once
    def _planes(self, nbytes):
        return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=self.device)

    def prepare_matmul(self, a, b, f_public, flags=0, left=True, right=True):
        """Returns (right_planes or None, left_planes or None) for beaver_matmul_prepared."""
        shp = a[0].shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = (shp[-1], shp[-2]) if flags & MPC_TRANS_X else (shp[-2], shp[-1])
        N = b[0].shape[-2] if flags & MPC_TRANS_Y else b[0].shape[-1]
        r, l = c_size_t(), c_size_t()
        self._check(lib().mpc_matmul_prepared_bytes(M, K, N, batch, byref(r), byref(l)))
        rp = self._planes(r.value) if right else None; lp = self._planes(l.value) if left else None
        self._check(lib().mpc_matmul_prepare(self._h, _share(a), _share(b), _p64(f_public), rp.data_ptr() if right else None,
                                             lp.data_ptr() if left else None, M, K, N, batch, flags))
        return rp, lp

    def beaver_matmul_prepared(self, x, a, c, right, left=None, n_chunks=1, flags=MPC_TRUNCATE, out=None):
        shp = a[0].shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = (shp[-1], shp[-2]) if flags & MPC_TRANS_X else (shp[-2], shp[-1])
        N = c[0].shape[-1]
        self.reserve(lib().mpc_matmul_workspace_bytes(M, K, N, batch))
        z = out if out is not None else (torch.empty_like(c[0]), torch.empty_like(c[1]))
        self._check(lib().mpc_beaver_matmul_prepared(self._h, _share(x), _share(a), _share(c), _share(z), right.data_ptr(),
                                                     left.data_ptr() if left is not None else None,
                                                     M, K, N, batch, n_chunks, flags))
        return z

    def beaver_matmul_folded(self, x, y, a, b, c, right, left, n_chunks=1, flags=MPC_TRUNCATE, out=None):
        """Folded product of two shared operands: c = (fold_matmul(a, b, c), c_1); right, left from
        prepare_matmul(a, b, None)."""
        shp = a[0].shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = (shp[-1], shp[-2]) if flags & MPC_TRANS_X else (shp[-2], shp[-1])
        N = c[0].shape[-1]
        self.reserve(lib().mpc_matmul_workspace_bytes(M, K, N, batch))
        z = out if out is not None else (torch.empty_like(c[0]), torch.empty_like(c[1]))
        self._check(lib().mpc_beaver_matmul_folded(self._h, _share(x), _share(y), _share(a), _share(b), _share(c), _share(z),
                                                   right.data_ptr(), left.data_ptr(), M, K, N, batch, n_chunks, flags))
        return z

    def fold_matmul(self, a, b, c, flags=0):
        """Party 0's folded addend c_0 - a_0 b_0 for beaver_matmul_prepared(..., flags | MPC_FOLDED)."""
        shp = a[0].shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = (shp[-1], shp[-2]) if flags & MPC_TRANS_X else (shp[-2], shp[-1])
        N = c[0].shape[-1]
        self.reserve(lib().mpc_matmul_workspace_bytes(M, K, N, batch))
        out = torch.empty_like(c[0])
        self._check(lib().mpc_matmul_fold(self._h, _p64(a[0]), _p64(b[0]), _p64(c[0]), _p64(out), M, K, N, batch, flags))
        return out

    def mfma_rate(self, random_operands: bool, iters: int = 2000, launches: int = 10) -> float:
        """int8 matrix-core operations per second on register-resident operands (mpc_mfma_rate); blocks."""
        self.reserve(1 << 20)
        r = ctypes.c_double()
        self._check(lib().mpc_mfma_rate(self._h, 1 if random_operands else 0, iters, launches, byref(r)))
        return r.value

    def fold_conv2d(self, a, b, c, pad, stride):
        """Party 0's folded addend c_0 - conv(a_0, b_0) for conv2d_prepared(..., flags | MPC_FOLDED)."""
        B, H, W, Cin = a[0].shape; KH, KW, _, Cout = b[0].shape
        self.reserve(lib().mpc_conv2d_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        out = torch.empty_like(c[0])
        self._check(lib().mpc_conv2d_fold(self._h, _p64(a[0]), _p64(b[0]), _p64(c[0]), _p64(out),
                                          B, H, W, Cin, Cout, KH, KW, pad, stride))
        return out

    def prepare_conv2d(self, a, b, f_public, pad, stride, left=True, right=True):
        B, H, W, Cin = a[0].shape; KH, KW, _, Cout = b[0].shape
        r, l = c_size_t(), c_size_t()
        self._check(lib().mpc_conv2d_prepared_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride, byref(r), byref(l)))
        rp = self._planes(r.value) if right else None; lp = self._planes(l.value) if left else None
        self._check(lib().mpc_conv2d_prepare(self._h, _share(a), _share(b), _p64(f_public), rp.data_ptr() if right else None,
                                             lp.data_ptr() if left else None, B, H, W, Cin, Cout, KH, KW, pad, stride))
        return rp, lp

    def conv2d_prepared(self, x, a, c, right, left, KH, KW, pad, stride, n_chunks=1, flags=MPC_TRUNCATE, out=None):
        B, H, W, Cin = a[0].shape; Cout = c[0].shape[-1]
        self.reserve(lib().mpc_conv2d_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        z = out if out is not None else (torch.empty_like(c[0]), torch.empty_like(c[1]))
        self._check(lib().mpc_conv2d_prepared(self._h, _share(x), _share(a), _share(c), _share(z), right.data_ptr(),
                                              left.data_ptr() if left is not None else None,
                                              B, H, W, Cin, Cout, KH, KW, pad, stride, n_chunks, flags))
        return z

    def conv2d_grad_x(self, g, w, a, b, c, pad, stride=1, f_public=None, n_chunks=1, flags=MPC_TRUNCATE, out=None):
        """Input gradient of conv2d: g, a [B,Ho,Wo,Cout]; w, b [KH,KW,Cin,Cout]; c and result [B,H,W,Cin]."""
        B, H, W, Cin = c[0].shape
        KH, KW, Cin2, Cout = b[0].shape
        assert Cin == Cin2 and a[0].shape[-1] == Cout
        self.reserve(lib().mpc_conv2d_grad_x_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        gx = out if out is not None else (torch.empty_like(c[0]), torch.empty_like(c[1]))
        self._check(lib().mpc_conv2d_grad_x(self._h, _share(g), _share(w), _share(a), _share(b), _share(c), _share(gx),
                                            B, H, W, Cin, Cout, KH, KW, pad, stride, _p64(f_public), n_chunks, flags))
        return gx

    def conv2d_grad_w(self, x, g, a, b, c, pad, stride, e_public=None, n_chunks=1, flags=MPC_TRUNCATE, out=None):
        """Filter gradient of conv2d: x, a [B,H,W,Cin]; g, b [B,Ho,Wo,Cout]; c and result [KH,KW,Cin,Cout]."""
        B, H, W, Cin = a[0].shape
        KH, KW, Cin2, Cout = c[0].shape
        assert Cin == Cin2 and b[0].shape[-1] == Cout
        self.reserve(lib().mpc_conv2d_grad_w_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        gw = out if out is not None else (torch.empty_like(c[0]), torch.empty_like(c[1]))
        self._check(lib().mpc_conv2d_grad_w(self._h, _share(x), _share(g), _share(a), _share(b), _share(c), _share(gw),
                                            B, H, W, Cin, Cout, KH, KW, pad, stride, _p64(e_public), n_chunks, flags))
        return gw

    def mul(self, x, y, a, b, c, flags=0, out=None):
        """Element-wise Alg. 1."""
        n = x[0].numel()
        self.reserve(lib().mpc_mul_workspace_bytes(n))
        z = out if out is not None else (torch.empty_like(x[0]), torch.empty_like(x[1]))
        self._check(lib().mpc_mul(self._h, _share(x), _share(y), _share(a), _share(b), _share(c), _share(z), n, flags))
        return z

    def relu_backward(self, g, s_arith, a, b, c, out=None):
        """Output gradient times the ReLU input mask 1 - s (s_arith from the forward relu)."""
        n = g[0].numel()
        self.reserve(lib().mpc_mul_workspace_bytes(n))
        gx = out if out is not None else (torch.empty_like(g[0]), torch.empty_like(g[1]))
        self._check(lib().mpc_relu_backward(self._h, _share(g), _share(s_arith), _share(a), _share(b), _share(c),
                                            _share(gx), n))
        return gx

    def maxpool2x2_backward(self, g, s1, s2, t1, t2, x_shape):
        """Gradient of maxpool2x2 w.r.t. its input; t1 / t2: element-wise triples (a, b, c) on 2*n_out / n_out words."""
        B, H, W, C = x_shape
        self.reserve(lib().mpc_maxpool_backward_workspace_bytes(B, H, W, C))
        gx = tuple(torch.empty(tuple(x_shape), dtype=torch.int64, device=self.device) for _ in range(2))
        self._check(lib().mpc_maxpool2x2_backward(self._h, _share(g), _share(s1), _share(s2),
                                                  _share(t1[0]), _share(t1[1]), _share(t1[2]),
                                                  _share(t2[0]), _share(t2[1]), _share(t2[2]), _share(gx), B, H, W, C))
        return gx

    # -- three parties (every argument a triple of tensors, one per party)
    def _empty3(self, like):
        return tuple(torch.empty_like(like) for _ in range(3))

    def open3(self, s):
        n = s[0].numel()
        self.reserve(3 * (n * 8 + 256))
        out = torch.empty_like(s[0])
        self._check(lib().mpc_open3(self._h, _share3(s), _p64(out), n))
        return out

    def beaver_matmul3(self, x, y, a, b, c, f_public=None, flags=0, out=None):
        shp = a[0].shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = (shp[-1], shp[-2]) if flags & MPC_TRANS_X else (shp[-2], shp[-1])
        K2, N = (b[0].shape[-1], b[0].shape[-2]) if flags & MPC_TRANS_Y else (b[0].shape[-2], b[0].shape[-1])
        if K2 != K or tuple(c[0].shape[-2:]) != (M, N):
            raise ValueError("operand shapes do not match")
        self.reserve(lib().mpc_matmul3_workspace_bytes(M, K, N, batch))
        z = out if out is not None else self._empty3(c[0])
        self._check(lib().mpc_beaver_matmul3(self._h, _share3(x), _share3(y), _share3(a), _share3(b), _share3(c),
                                             _share3(z), M, K, N, batch, _p64(f_public), flags))
        return z

    def conv2d3(self, x, w, a, b, c, pad, stride, f_public=None, out=None):
        B, H, W, Cin = a[0].shape
        KH, KW, Cin2, Cout = b[0].shape
        if Cin != Cin2:
            raise ValueError("operand shapes do not match")
        self.reserve(lib().mpc_conv2d3_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        z = out if out is not None else self._empty3(c[0])
        self._check(lib().mpc_conv2d3(self._h, _share3(x), _share3(w), _share3(a), _share3(b), _share3(c), _share3(z),
                                      B, H, W, Cin, Cout, KH, KW, pad, stride, _p64(f_public)))
        return z

    def prepare_matmul3(self, a, b, f_public, left=True):
        """Returns (right_planes, left_planes or None) for beaver_matmul3_prepared."""
        shp = a[0].shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = shp[-2], shp[-1]; N = b[0].shape[-1]
        r, l = c_size_t(), c_size_t()
        self._check(lib().mpc_matmul3_prepared_bytes(M, K, N, batch, byref(r), byref(l)))
        right = self._planes(r.value); lp = self._planes(l.value) if left else None
        self._check(lib().mpc_matmul3_prepare(self._h, _share3(a), _share3(b), _p64(f_public), right.data_ptr(),
                                              lp.data_ptr() if left else None, M, K, N, batch, 0))
        return right, lp

    def beaver_matmul3_prepared(self, x, a, c, right, left=None, out=None):
        shp = a[0].shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = shp[-2], shp[-1]; N = c[0].shape[-1]
        self.reserve(lib().mpc_matmul3_workspace_bytes(M, K, N, batch))
        z = out if out is not None else self._empty3(c[0])
        self._check(lib().mpc_beaver_matmul3_prepared(self._h, _share3(x), _share3(a), _share3(c), _share3(z), right.data_ptr(),
                                                      left.data_ptr() if left is not None else None, M, K, N, batch, 0))
        return z

    def prepare_conv2d3(self, a, b, f_public, pad, stride, left=True):
        B, H, W, Cin = a[0].shape; KH, KW, _, Cout = b[0].shape
        r, l = c_size_t(), c_size_t()
        self._check(lib().mpc_conv2d3_prepared_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride, byref(r), byref(l)))
        right = self._planes(r.value); lp = self._planes(l.value) if left else None
        self._check(lib().mpc_conv2d3_prepare(self._h, _share3(a), _share3(b), _p64(f_public), right.data_ptr(),
                                              lp.data_ptr() if left else None, B, H, W, Cin, Cout, KH, KW, pad, stride))
        return right, lp

    def conv2d3_prepared(self, x, a, c, right, left, KH, KW, pad, stride, out=None):
        B, H, W, Cin = a[0].shape; Cout = c[0].shape[-1]
        self.reserve(lib().mpc_conv2d3_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        z = out if out is not None else self._empty3(c[0])
        self._check(lib().mpc_conv2d3_prepared(self._h, _share3(x), _share3(a), _share3(c), _share3(z), right.data_ptr(),
                                               left.data_ptr() if left is not None else None,
                                               B, H, W, Cin, Cout, KH, KW, pad, stride))
        return z

    def truncate3(self, z, r, rt, bits=16):
        """Masked rescale in place with the offline pair (r, r >> bits)."""
        n = z[0].numel()
        self.reserve(lib().mpc_truncate3_workspace_bytes(n))
        self._check(lib().mpc_truncate3(self._h, _share3(z), _share3(r), _share3(rt), n, bits))
        return z

    def pack_material3(self, mat: dict) -> dict:
        """Offline helper: three-party material with and_a/b/c in the packed layout of relu3(packed=True)."""
        n = mat["r0"][0].numel()
        words = lib().mpc_relu3_packed_words(n)
        out = dict(mat)
        for key in ("and_a", "and_b", "and_c"):
            pk = tuple(torch.empty(words, dtype=torch.int64, device=self.device) for _ in range(3))
            self._check(lib().mpc_relu3_pack_triples(self._h, _share3(mat[key]), _share3(pk), n))
            out[key] = pk
        self.sync()
        return out

    def relu3(self, x, mat, want_sign=False, out=None, packed=False):
        """Three-party secure ReLU; packed=True runs the sign-only carry chain on packed material (mpc_relu3_msb)."""
        n = x[0].numel()
        fn = lib().mpc_relu3_msb if packed else lib().mpc_relu3
        self.reserve(lib().mpc_relu3_msb_workspace_bytes(n) if packed else lib().mpc_relu3_workspace_bytes(n))
        y = out if out is not None else self._empty3(x[0])
        m = _material3(mat, n, packed)
        if want_sign:
            sb = tuple(torch.empty(n, dtype=torch.uint8, device=self.device) for _ in range(3))
            sa = tuple(torch.empty(n, dtype=torch.int64, device=self.device) for _ in range(3))
            sbp = (_P8 * 3)(*[_p8(t) for t in sb]); sap = (_P64 * 3)(*[_p64(t) for t in sa])
            self._check(fn(self._h, _share3(x), byref(m), _share3(y), n, byref(sbp), byref(sap)))
            return y, sb, sa
        self._check(fn(self._h, _share3(x), byref(m), _share3(y), n, None, None))
        return y

    def maxpool3(self, x, mat1, mat2, packed=False, want_signs=False):
        """Three-party 2x2 max-pool; want_signs=True also returns the sign shares (s1, s2) the backward pass needs."""
        B, H, W, C = x[0].shape
        n_out = B * (H // 2) * (W // 2) * C
        ws = lib().mpc_maxpool3_msb_workspace_bytes if packed else lib().mpc_maxpool3_workspace_bytes
        self.reserve(ws(B, H, W, C))
        y = tuple(torch.empty((B, H // 2, W // 2, C), dtype=torch.int64, device=self.device) for _ in range(3))
        m1, m2 = _material3(mat1, 2 * n_out, packed), _material3(mat2, n_out, packed)
        if want_signs:
            s1 = tuple(torch.empty(2 * n_out, dtype=torch.int64, device=self.device) for _ in range(3))
            s2 = tuple(torch.empty(n_out, dtype=torch.int64, device=self.device) for _ in range(3))
            p1 = (_P64 * 3)(*[_p64(t) for t in s1]); p2 = (_P64 * 3)(*[_p64(t) for t in s2])
            self._check(lib().mpc_maxpool3_signs(self._h, _share3(x), byref(m1), byref(m2), _share3(y), byref(p1), byref(p2),
                                                 B, H, W, C, 1 if packed else 0))
            return y, s1, s2
        fn = lib().mpc_maxpool3_msb if packed else lib().mpc_maxpool3
        self._check(fn(self._h, _share3(x), byref(m1), byref(m2), _share3(y), B, H, W, C))
        return y

    def conv2d3_grad_x(self, g, w, a, b, c, pad, stride=1, f_public=None, out=None):
        """Input gradient of conv2d3 (no rescale): g, a [B,Ho,Wo,Cout]; w, b [KH,KW,Cin,Cout]; c and result [B,H,W,Cin]."""
        B, H, W, Cin = c[0].shape
        KH, KW, Cin2, Cout = b[0].shape
        if Cin != Cin2 or a[0].shape[-1] != Cout:
            raise ValueError("operand shapes do not match")
        self.reserve(lib().mpc_conv2d3_grad_x_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        gx = out if out is not None else self._empty3(c[0])
        self._check(lib().mpc_conv2d3_grad_x(self._h, _share3(g), _share3(w), _share3(a), _share3(b), _share3(c), _share3(gx),
                                             B, H, W, Cin, Cout, KH, KW, pad, stride, _p64(f_public)))
        return gx

    def conv2d3_grad_w(self, x, g, a, b, c, pad, stride, out=None):
        """Filter gradient of conv2d3 (no rescale): x, a [B,H,W,Cin]; g, b [B,Ho,Wo,Cout]; c and result [KH,KW,Cin,Cout]."""
        B, H, W, Cin = a[0].shape
        KH, KW, Cin2, Cout = c[0].shape
        if Cin != Cin2 or b[0].shape[-1] != Cout:
            raise ValueError("operand shapes do not match")
        self.reserve(lib().mpc_conv2d3_grad_w_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        gw = out if out is not None else self._empty3(c[0])
        self._check(lib().mpc_conv2d3_grad_w(self._h, _share3(x), _share3(g), _share3(a), _share3(b), _share3(c), _share3(gw),
                                             B, H, W, Cin, Cout, KH, KW, pad, stride))
        return gw

    def add3(self, x, y, out=None):
        z = out if out is not None else self._empty3(x[0])
        self._check(lib().mpc_add3(self._h, _share3(x), _share3(y), _share3(z), x[0].numel()))
        return z

    def sub3(self, x, y, out=None):
        z = out if out is not None else self._empty3(x[0])
        self._check(lib().mpc_sub3(self._h, _share3(x), _share3(y), _share3(z), x[0].numel()))
        return z

    def mul3(self, x, y, a, b, c, out=None):
        """Element-wise Alg. 1 with three parties (no rescale)."""
        n = x[0].numel()
        self.reserve(lib().mpc_mul3_workspace_bytes(n))
        z = out if out is not None else self._empty3(x[0])
        self._check(lib().mpc_mul3(self._h, _share3(x), _share3(y), _share3(a), _share3(b), _share3(c), _share3(z), n))
        return z

    def relu3_backward(self, g, s_arith, a, b, c, out=None):
        """Output gradient times the ReLU input mask 1 - s (s_arith from the forward relu3)."""
        n = g[0].numel()
        self.reserve(lib().mpc_mul3_workspace_bytes(n))
        gx = out if out is not None else self._empty3(g[0])
        self._check(lib().mpc_relu3_backward(self._h, _share3(g), _share3(s_arith), _share3(a), _share3(b), _share3(c),
                                             _share3(gx), n))
        return gx

    def maxpool3_backward(self, g, s1, s2, t1, t2, x_shape):
        """Gradient of maxpool3 w.r.t. its input; t1 / t2: element-wise triples (a, b, c) on 2*n_out / n_out words."""
        B, H, W, C = x_shape
        self.reserve(lib().mpc_maxpool3_backward_workspace_bytes(B, H, W, C))
        gx = tuple(torch.empty(tuple(x_shape), dtype=torch.int64, device=self.device) for _ in range(3))
        self._check(lib().mpc_maxpool3_backward(self._h, _share3(g), _share3(s1), _share3(s2),
                                                _share3(t1[0]), _share3(t1[1]), _share3(t1[2]),
                                                _share3(t2[0]), _share3(t2[1]), _share3(t2[2]), _share3(gx), B, H, W, C))
        return gx

    def truncate(self, z, bits=16):
        self._check(lib().mpc_truncate(self._h, _share(z), z[0].numel(), bits))
        return z

    def pack_material(self, mat: dict) -> dict:
        """Offline helper: the same material with and_a/b/c in the packed layout of relu_msb."""
        n = mat["r"][0].numel()
        words = lib().mpc_relu_packed_words(n)
        out = dict(mat)
        for key in ("and_a", "and_b", "and_c"):
            pk = tuple(torch.empty(words, dtype=torch.int64, device=self.device) for _ in range(2))
            self._check(lib().mpc_relu_pack_triples(self._h, _share(mat[key]), _share(pk), n))
            out[key] = pk
        self.sync()
        return out

    def relu(self, x, mat, n_chunks=0, want_sign=False, out=None, packed=False):
        """Secure ReLU; packed=True runs the sign-only carry chain on packed material (mpc_relu_msb)."""
        n = x[0].numel()
        fn = lib().mpc_relu_msb if packed else lib().mpc_relu
        self.reserve(lib().mpc_relu_msb_workspace_bytes(n) if packed else lib().mpc_relu_workspace_bytes(n))
        y = out if out is not None else (torch.empty_like(x[0]), torch.empty_like(x[1]))
        m = _material(mat, n, packed)
        if want_sign:
            sb = tuple(torch.empty(n, dtype=torch.uint8, device=self.device) for _ in range(2))
            sa = tuple(torch.empty(n, dtype=torch.int64, device=self.device) for _ in range(2))
            sbp = (_P8 * 2)(_p8(sb[0]), _p8(sb[1])); sap = (_P64 * 2)(_p64(sa[0]), _p64(sa[1]))
            self._check(fn(self._h, _share(x), byref(m), _share(y), n, n_chunks, byref(sbp), byref(sap)))
            return y, sb, sa
        self._check(fn(self._h, _share(x), byref(m), _share(y), n, n_chunks, None, None))
        return y

    def relu_static(self, x, mat, y, n_chunks=0, s_bit=None, s_arith=None):
        """mpc_relu_static: secure ReLU on the library's fixed scratch array; every buffer is the caller's."""
        n = x[0].numel()
        m = _material(mat, n, False)
        sbp = byref((_P8 * 2)(_p8(s_bit[0]), _p8(s_bit[1]))) if s_bit is not None else None
        sap = byref((_P64 * 2)(_p64(s_arith[0]), _p64(s_arith[1]))) if s_arith is not None else None
        self._check(lib().mpc_relu_static(self._h, _share(x), byref(m), _share(y), n, n_chunks, sbp, sap))
        return y

    def maxpool2x2(self, x, mat1, mat2, n_chunks=0, packed=False, want_signs=False, out=None):
        """2x2 max-pool; want_signs=True also returns the sign shares (s1, s2) the backward pass needs."""
        B, H, W, C = x[0].shape
        n_out = B * (H // 2) * (W // 2) * C
        ws = lib().mpc_maxpool_msb_workspace_bytes if packed else lib().mpc_maxpool_workspace_bytes
        self.reserve(ws(B, H, W, C))
        y = out if out is not None else \
            tuple(torch.empty((B, H // 2, W // 2, C), dtype=torch.int64, device=self.device) for _ in range(2))
        m1, m2 = _material(mat1, 2 * n_out, packed), _material(mat2, n_out, packed)
        if want_signs:
            s1 = tuple(torch.empty(2 * n_out, dtype=torch.int64, device=self.device) for _ in range(2))
            s2 = tuple(torch.empty(n_out, dtype=torch.int64, device=self.device) for _ in range(2))
            p1 = (_P64 * 2)(_p64(s1[0]), _p64(s1[1])); p2 = (_P64 * 2)(_p64(s2[0]), _p64(s2[1]))
            self._check(lib().mpc_maxpool2x2_signs(self._h, _share(x), byref(m1), byref(m2), _share(y), byref(p1), byref(p2),
                                                   B, H, W, C, n_chunks, int(packed)))
            return y, s1, s2
        fn = lib().mpc_maxpool2x2_msb if packed else lib().mpc_maxpool2x2
        self._check(fn(self._h, _share(x), byref(m1), byref(m2), _share(y), B, H, W, C, n_chunks))
        return y

    # -- dealer helpers (offline phase stand-in)
    def ring_matmul(self, L, R):
        shp = L.shape
        batch = 1 if len(shp) == 2 else shp[0]
        M, K = shp[-2], shp[-1]; N = R.shape[-1]
        self.reserve(lib().mpc_matmul_workspace_bytes(M, K, N, batch))
        Z = torch.empty(shp[:-1] + (N,), dtype=torch.int64, device=self.device)
        self._check(lib().mpc_ring_matmul(self._h, _p64(L), _p64(R), _p64(Z), M, K, N, batch))
        return Z

    def ring_conv2d_grad_x(self, g, w, x_shape, pad, stride=1):
        B, H, W, Cin = x_shape; KH, KW, _, Cout = w.shape
        self.reserve(lib().mpc_conv2d_grad_x_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        gx = torch.empty(tuple(x_shape), dtype=torch.int64, device=self.device)
        self._check(lib().mpc_ring_conv2d_grad_x(self._h, _p64(g), _p64(w), _p64(gx), B, H, W, Cin, Cout, KH, KW, pad, stride))
        return gx

    def ring_conv2d_grad_w(self, x, g, KH, KW, pad, stride):
        B, H, W, Cin = x.shape; Cout = g.shape[-1]
        self.reserve(lib().mpc_conv2d_grad_w_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        gw = torch.empty((KH, KW, Cin, Cout), dtype=torch.int64, device=self.device)
        self._check(lib().mpc_ring_conv2d_grad_w(self._h, _p64(x), _p64(g), _p64(gw), B, H, W, Cin, Cout, KH, KW, pad, stride))
        return gw

    def ring_conv2d(self, x, w, pad, stride):
        B, H, W, Cin = x.shape; KH, KW, _, Cout = w.shape
        Ho = (H + 2 * pad - KH) // stride + 1; Wo = (W + 2 * pad - KW) // stride + 1
        self.reserve(lib().mpc_conv2d_workspace_bytes(B, H, W, Cin, Cout, KH, KW, pad, stride))
        z = torch.empty((B, Ho, Wo, Cout), dtype=torch.int64, device=self.device)
        self._check(lib().mpc_ring_conv2d(self._h, _p64(x), _p64(w), _p64(z), B, H, W, Cin, Cout, KH, KW, pad, stride))
        return z
