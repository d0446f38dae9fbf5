"""ctypes binding of libdbf: the same entry points as include/dbf.h, argument
marshalling only.  Every step of the layer product runs inside the library's
HIP kernels; there is no Python or CPU fallback, and a missing library is an
error.

Device buffers are passed as integer addresses (for example
``tensor.data_ptr()``), streams as the integer value of a ``hipStream_t``
(``torch.cuda.current_stream().cuda_stream``) or 0 for the default stream.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdbf.so")

DBF_OK, DBF_EINVAL, DBF_ESHAPE, DBF_ENOTSIGN, DBF_ENOMEM, DBF_EHIP, DBF_EWORKSPACE = 0, -1, -2, -3, -4, -5, -6
GEMV_AUTO, GEMV_VALU, GEMV_MFMA, GEMV_MFMA_SPLIT = 0, 1, 2, 3
GEMM_AUTO, GEMM_I8 = 0, 2
(TUNE_COL_PIECES, TUNE_PIECE_TARGET, TUNE_PIECE_MIN_TILES, TUNE_PIECE_NEVER_TILES, TUNE_PIECE_MAX_ROW_TILES,
 TUNE_STACK_SPAN_B, TUNE_STACK_SPAN_A, TUNE_SHARED_Q, TUNE_SHARED_MIN_BATCH, TUNE_SHARED_LDS_KB,
 TUNE_WAIT_LIMIT_US, TUNE_LONG_ROWS, TUNE_GEMM_SPLITS, TUNE_FUSED_MIN_B_ITEMS, TUNE_WIDE_WG_MAX_ITEMS,
 TUNE_FP4_MAX_ITEMS) = range(16)
MAX_BATCH = 16
GEMM_STATIC_BYTES = 32 << 20  # DBF_GEMM_STATIC_BYTES

EXPORTS = [
    "dbf_pack", "dbf_pack_bits", "dbf_unpack_bits", "dbf_dims", "dbf_free",
    "dbf_tiled_bytes", "dbf_signs_to_bits_host", "dbf_tile_host", "dbf_untile_host",
    "dbf_gemv", "dbf_gemv_kind", "dbf_sync_timeouts", "dbf_gemm_workspace_bytes", "dbf_gemm", "dbf_gemm_kind",
    "dbf_gemm_static",
    "dbf_stack_create", "dbf_stack_create_grouped", "dbf_stack_offsets", "dbf_stack_gemv", "dbf_stack_gemv_timed",
    "dbf_stack_sync_timeouts", "dbf_stack_free",
    "dbf_prune_middle", "dbf_svid_workspace_bytes", "dbf_svid", "dbf_admm_workspace_bytes", "dbf_admm_step", "dbf_admm_prepare_workspace_bytes", "dbf_admm_prepare", "dbf_probe_read", "dbf_probe_mfma", "dbf_strerror",
    "dbf_tuning_set", "dbf_tuning_get", "dbf_tuning_reset",
]

_lib = None


class DbfError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (where, strerror(code), code))


def lib() -> C.CDLL:
    """Loads libdbf.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build(verbose=False)
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    pp = C.POINTER(C.c_void_p)
    L.dbf_pack.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, pp]
    L.dbf_pack_bits.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, pp]
    L.dbf_unpack_bits.argtypes = [vp, vp, vp, vp, vp, vp]
    L.dbf_dims.argtypes = [vp, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(sz)]
    L.dbf_free.argtypes = [vp]
    L.dbf_free.restype = None
    L.dbf_tiled_bytes.argtypes = [i32, i32]
    L.dbf_tiled_bytes.restype = sz
    L.dbf_signs_to_bits_host.argtypes = [i32, i32, vp, vp]
    L.dbf_tile_host.argtypes = [i32, i32, vp, vp]
    L.dbf_untile_host.argtypes = [i32, i32, vp, vp]
    L.dbf_gemv.argtypes = [vp, vp, vp, i32, vp]
    L.dbf_gemv_kind.argtypes = [vp, vp, vp, i32, i32, vp]
    L.dbf_sync_timeouts.argtypes = [vp, C.POINTER(i32)]
    L.dbf_stack_sync_timeouts.argtypes = [vp, C.POINTER(i32)]
    L.dbf_gemm_workspace_bytes.argtypes = [vp, i32]
    L.dbf_gemm_workspace_bytes.restype = sz
    L.dbf_gemm.argtypes = [vp, vp, vp, i32, vp, sz, vp]
    L.dbf_gemm_kind.argtypes = [vp, vp, vp, i32, vp, sz, i32, vp]
    L.dbf_gemm_static.argtypes = [vp, vp, vp, i32, vp]
    L.dbf_stack_create.argtypes = [pp, i32, pp]
    L.dbf_stack_create_grouped.argtypes = [pp, i32, C.POINTER(C.c_int), i32, pp]
    L.dbf_stack_offsets.argtypes = [vp, i32, i32, C.POINTER(sz), C.POINTER(sz)]
    L.dbf_stack_gemv.argtypes = [vp, vp, vp, i32, i32, vp]
    L.dbf_stack_gemv_timed.argtypes = [vp, vp, vp, i32, i32, vp, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    L.dbf_stack_free.argtypes = [vp]
    L.dbf_stack_free.restype = None
    L.dbf_prune_middle.argtypes = [vp, vp, i32, pp]
    L.dbf_svid_workspace_bytes.argtypes = [i32, i32]
    L.dbf_svid_workspace_bytes.restype = sz
    L.dbf_svid.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    L.dbf_admm_workspace_bytes.argtypes = [i32, i32]
    L.dbf_admm_workspace_bytes.restype = sz
    L.dbf_admm_step.argtypes = [vp, vp, i32, i32, C.c_float, i32, vp, vp, vp, vp, vp, sz, vp]
    L.dbf_admm_prepare_workspace_bytes.argtypes = [i32, i32, i32]
    L.dbf_admm_prepare_workspace_bytes.restype = sz
    L.dbf_admm_prepare.argtypes = [vp, vp, vp, vp, i32, i32, i32, C.c_float, vp, vp, vp, sz, vp, vp]
    L.dbf_probe_read.argtypes = [vp, sz, vp, vp]
    L.dbf_probe_mfma.argtypes = [i32, i32, i32, i32, vp, vp, C.POINTER(C.c_double)]
    L.dbf_tuning_set.argtypes = [i32, i32]
    L.dbf_tuning_get.argtypes = [i32]
    L.dbf_tuning_reset.argtypes = []
    L.dbf_tuning_reset.restype = None
    L.dbf_strerror.argtypes = [i32]
    L.dbf_strerror.restype = C.c_char_p
    for name in EXPORTS:
        getattr(L, name)  # every declared entry point must be exported
    _lib = L
    return L


def strerror(code: int) -> str:
    return lib().dbf_strerror(int(code)).decode()


def _check(code: int, where: str) -> None:
    if code != DBF_OK:
        raise DbfError(code, where)


def _host(arr, dtype) -> np.ndarray:
    out = np.ascontiguousarray(arr, dtype=dtype)
    return out


def _ptr(arr: np.ndarray) -> int:
    return arr.ctypes.data


# ---- host-side layout helpers ------------------------------------------------------------


def dbf_tiled_bytes(rows: int, cols: int) -> int:
    return int(lib().dbf_tiled_bytes(rows, cols))


def dbf_signs_to_bits_host(pm1) -> np.ndarray:
    pm1 = _host(pm1, np.int8)
    rows, cols = pm1.shape
    bits = np.empty((rows, (cols + 31) // 32), dtype=np.uint32)
    _check(lib().dbf_signs_to_bits_host(rows, cols, _ptr(pm1), _ptr(bits)), "dbf_signs_to_bits_host")
    return bits


def dbf_tile_host(rows: int, cols: int, bits) -> np.ndarray:
    bits = _host(bits, np.uint32)
    tiled = np.empty(dbf_tiled_bytes(rows, cols), dtype=np.uint8)
    _check(lib().dbf_tile_host(rows, cols, _ptr(bits), _ptr(tiled)), "dbf_tile_host")
    return tiled


def dbf_untile_host(rows: int, cols: int, tiled) -> np.ndarray:
    tiled = _host(tiled, np.uint8)
    bits = np.zeros((rows, (cols + 31) // 32), dtype=np.uint32)
    _check(lib().dbf_untile_host(rows, cols, _ptr(tiled), _ptr(bits)), "dbf_untile_host")
    return bits


# ---- layers --------------------------------------------------------------------------------


class Layer:
    """Owns one dbf_layer handle; freed on close() or garbage collection."""

    def __init__(self, handle: int, n_in: int, n_out: int, k: int):
        self.handle = handle
        self.n_in, self.n_out, self.k = n_in, n_out, k

    def close(self) -> None:
        if self.handle:
            lib().dbf_free(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def device_bytes(self) -> int:
        sz = C.c_size_t(0)
        _check(lib().dbf_dims(self.handle, None, None, None, C.byref(sz)), "dbf_dims")
        return int(sz.value)


def dbf_pack(n_in: int, n_out: int, k: int, A_pm1, B_pm1, a, m, b) -> Layer:
    A = _host(A_pm1, np.int8)
    B = _host(B_pm1, np.int8)
    a, m, b = _host(a, np.uint16), _host(m, np.uint16), _host(b, np.uint16)
    if A.size != n_out * k or B.size != k * n_in or a.size != n_out or m.size != k or b.size != n_in:
        raise DbfError(DBF_ESHAPE, "dbf_pack (host array sizes)")
    h = C.c_void_p(0)
    _check(lib().dbf_pack(n_in, n_out, k, _ptr(A), _ptr(B), _ptr(a), _ptr(m), _ptr(b), C.byref(h)), "dbf_pack")
    return Layer(h.value, n_in, n_out, k)


def dbf_pack_bits(n_in: int, n_out: int, k: int, A_bits, B_bits, a, m, b) -> Layer:
    A = _host(A_bits, np.uint32)
    B = _host(B_bits, np.uint32)
    a, m, b = _host(a, np.uint16), _host(m, np.uint16), _host(b, np.uint16)
    if (A.size != n_out * ((k + 31) // 32) or B.size != k * ((n_in + 31) // 32)
            or a.size != n_out or m.size != k or b.size != n_in):
        raise DbfError(DBF_ESHAPE, "dbf_pack_bits (host array sizes)")
    h = C.c_void_p(0)
    _check(lib().dbf_pack_bits(n_in, n_out, k, _ptr(A), _ptr(B), _ptr(a), _ptr(m), _ptr(b), C.byref(h)),
           "dbf_pack_bits")
    return Layer(h.value, n_in, n_out, k)


def dbf_prune_middle(layer: Layer, keep) -> Layer:
    """New layer that keeps the middle channels `keep` (strictly increasing indices) of `layer`."""
    idx = _host(keep, np.int32).reshape(-1)
    h = C.c_void_p(0)
    _check(lib().dbf_prune_middle(layer.handle, _ptr(idx), int(idx.size), C.byref(h)), "dbf_prune_middle")
    return Layer(h.value, layer.n_in, layer.n_out, int(idx.size))


def dbf_svid_workspace_bytes(rows: int, cols: int) -> int:
    return int(lib().dbf_svid_workspace_bytes(rows, cols))


def dbf_svid(z_ptr: int, rows: int, cols: int, iters: int, a_ptr: int, m_ptr: int, bits_ptr: int, ws_ptr: int,
             ws_bytes: int, stream: int = 0) -> None:
    _check(lib().dbf_svid(z_ptr, rows, cols, iters, a_ptr, m_ptr, bits_ptr, ws_ptr, ws_bytes, stream), "dbf_svid")


def dbf_admm_workspace_bytes(q: int, r: int) -> int:
    return int(lib().dbf_admm_workspace_bytes(q, r))


def dbf_admm_step(minv_ptr: int, c_ptr: int, q: int, r: int, rho: float, svid_iters: int, a_ptr: int, m_ptr: int,
                  bits_ptr: int, u_ptr: int, ws_ptr: int, ws_bytes: int, stream: int = 0) -> None:
    _check(lib().dbf_admm_step(minv_ptr, c_ptr, q, r, float(rho), svid_iters, a_ptr, m_ptr, bits_ptr, u_ptr,
                               ws_ptr, ws_bytes, stream), "dbf_admm_step")


def dbf_admm_prepare_workspace_bytes(p: int, q: int, r: int) -> int:
    return int(lib().dbf_admm_prepare_workspace_bytes(p, q, r))


def dbf_admm_prepare(bits_ptr: int, m2_ptr: int, b_ptr: int, w_ptr: int, p: int, q: int, r: int, rho: float,
                     minv_ptr: int, c_ptr: int, ws_ptr: int, ws_bytes: int, flag_ptr: int = 0, stream: int = 0) -> None:
    _check(lib().dbf_admm_prepare(bits_ptr, m2_ptr, b_ptr, w_ptr, p, q, r, float(rho), minv_ptr, c_ptr, ws_ptr,
                                  ws_bytes, flag_ptr, stream), "dbf_admm_prepare")


def dbf_unpack_bits(layer: Layer):
    A = np.zeros((layer.n_out, (layer.k + 31) // 32), dtype=np.uint32)
    B = np.zeros((layer.k, (layer.n_in + 31) // 32), dtype=np.uint32)
    a = np.zeros(layer.n_out, dtype=np.uint16)
    m = np.zeros(layer.k, dtype=np.uint16)
    b = np.zeros(layer.n_in, dtype=np.uint16)
    _check(lib().dbf_unpack_bits(layer.handle, _ptr(A), _ptr(B), _ptr(a), _ptr(m), _ptr(b)), "dbf_unpack_bits")
    return A, B, a, m, b


def dbf_dims(layer: Layer):
    n_in, n_out, k, sz = C.c_int(0), C.c_int(0), C.c_int(0), C.c_size_t(0)
    _check(lib().dbf_dims(layer.handle, C.byref(n_in), C.byref(n_out), C.byref(k), C.byref(sz)), "dbf_dims")
    return n_in.value, n_out.value, k.value, int(sz.value)


def dbf_gemv(layer: Layer, x_ptr: int, y_ptr: int, batch: int, stream: int = 0, kind: int = GEMV_AUTO) -> None:
    _check(lib().dbf_gemv_kind(layer.handle, x_ptr, y_ptr, batch, kind, stream), "dbf_gemv")


def dbf_gemm_workspace_bytes(layer: Layer, T: int) -> int:
    return int(lib().dbf_gemm_workspace_bytes(layer.handle, T))


def dbf_gemm(layer: Layer, X_ptr: int, Y_ptr: int, T: int, workspace_ptr: int, workspace_bytes: int,
             stream: int = 0, kind: int = GEMM_AUTO) -> None:
    _check(lib().dbf_gemm_kind(layer.handle, X_ptr, Y_ptr, T, workspace_ptr, workspace_bytes, kind, stream),
           "dbf_gemm")


def dbf_gemm_static(layer: Layer, X_ptr: int, Y_ptr: int, T: int, stream: int = 0) -> None:
    """dbf_gemm with the scratch in the library's static device array (allocates nothing)."""
    _check(lib().dbf_gemm_static(layer.handle, X_ptr, Y_ptr, T, stream), "dbf_gemm_static")


# ---- stacks --------------------------------------------------------------------------------


class Stack:
    def __init__(self, handle: int, layers):
        self.handle = handle
        self.layers = list(layers)  # keeps the layers alive

    def close(self) -> None:
        if self.handle:
            lib().dbf_stack_free(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def offsets(self, index: int, batch: int):
        xo, yo = C.c_size_t(0), C.c_size_t(0)
        _check(lib().dbf_stack_offsets(self.handle, index, batch, C.byref(xo), C.byref(yo)), "dbf_stack_offsets")
        return int(xo.value), int(yo.value)


def dbf_stack_create(layers) -> Stack:
    layers = list(layers)
    arr = (C.c_void_p * max(1, len(layers)))(*[l.handle for l in layers])
    h = C.c_void_p(0)
    _check(lib().dbf_stack_create(arr, len(layers), C.byref(h)), "dbf_stack_create")
    return Stack(h.value, layers)


def dbf_stack_create_grouped(layers, group_sizes) -> Stack:
    """Stack whose consecutive groups of layers (sizes in group_sizes) each read one shared x block."""
    layers = list(layers)
    sizes = [int(v) for v in group_sizes]
    arr = (C.c_void_p * max(1, len(layers)))(*[l.handle for l in layers])
    gs = (C.c_int * max(1, len(sizes)))(*sizes)
    h = C.c_void_p(0)
    _check(lib().dbf_stack_create_grouped(arr, len(layers), gs, len(sizes), C.byref(h)), "dbf_stack_create_grouped")
    return Stack(h.value, layers)


def dbf_stack_offsets(stack: Stack, layer_index: int, batch: int):
    """Element offsets (x, y) of a layer's blocks in the stack's x and y buffers; layer_index == number of
    layers gives the totals."""
    xo, yo = C.c_size_t(0), C.c_size_t(0)
    _check(lib().dbf_stack_offsets(stack.handle, layer_index, batch, C.byref(xo), C.byref(yo)), "dbf_stack_offsets")
    return int(xo.value), int(yo.value)


def dbf_stack_gemv(stack: Stack, x_ptr: int, y_ptr: int, batch: int, stream: int = 0,
                   kind: int = GEMV_AUTO) -> None:
    _check(lib().dbf_stack_gemv(stack.handle, x_ptr, y_ptr, batch, kind, stream), "dbf_stack_gemv")


def dbf_stack_gemv_timed(stack: Stack, x_ptr: int, y_ptr: int, batch: int, stream: int = 0,
                         kind: int = GEMV_AUTO):
    """Returns (ms of the B-stage kernel, ms of the A-stage kernel); blocks until done."""
    mb, ma = C.c_float(0), C.c_float(0)
    _check(lib().dbf_stack_gemv_timed(stack.handle, x_ptr, y_ptr, batch, kind, stream, C.byref(mb), C.byref(ma)),
           "dbf_stack_gemv_timed")
    return float(mb.value), float(ma.value)


def dbf_probe_read(src_ptr: int, nbytes: int, sink_ptr: int = 0, stream: int = 0) -> None:
    _check(lib().dbf_probe_read(src_ptr, nbytes, sink_ptr, stream), "dbf_probe_read")


def dbf_probe_mfma(wide: bool, with_ands: bool, wavefronts_per_simd: int, iters: int, sink_ptr: int = 0,
                   stream: int = 0) -> float:
    """Launches the matrix-pipe probe; returns the integer operations of the launch."""
    ops = C.c_double(0)
    _check(lib().dbf_probe_mfma(int(wide), int(with_ands), wavefronts_per_simd, iters, sink_ptr, stream,
                                C.byref(ops)), "dbf_probe_mfma")
    return float(ops.value)


def dbf_tuning_set(knob: int, value: int) -> None:
    _check(lib().dbf_tuning_set(int(knob), int(value)), "dbf_tuning_set")


def dbf_tuning_get(knob: int) -> int:
    return int(lib().dbf_tuning_get(int(knob)))


def dbf_tuning_reset() -> None:
    lib().dbf_tuning_reset()


def dbf_sync_timeouts(layer: Layer) -> int:
    n = C.c_int(0)
    _check(lib().dbf_sync_timeouts(layer.handle, C.byref(n)), "dbf_sync_timeouts")
    return int(n.value)


def dbf_stack_sync_timeouts(stack: Stack) -> int:
    n = C.c_int(0)
    _check(lib().dbf_stack_sync_timeouts(stack.handle, C.byref(n)), "dbf_stack_sync_timeouts")
    return int(n.value)
