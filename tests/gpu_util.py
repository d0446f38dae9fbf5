"""Helpers for the GPU parity tests: move seeded inputs to the device, call the
C-ABI through the binding, bring results back as float64."""
import sys

import numpy as np
import torch

from oracle import dbf_oracle as O
from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

TOL = 2e-3  # max gated relative error of fp16 outputs against the fp64 oracle


def say(msg):
    print("[gpu-case] " + msg, flush=True)
    sys.stdout.flush()


def f16_to_dev(bits_u16: np.ndarray) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16).copy())
    return t.cuda().view(torch.float16)


def dev_to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().view(torch.int16).numpy().view(np.float16).astype(np.float64)


def stream_handle() -> int:
    return torch.cuda.current_stream().cuda_stream


def pack(L: I.LayerInputs) -> B.Layer:
    return B.dbf_pack_bits(L.n_in, L.n_out, L.k, L.A_bits, L.B_bits, L.a, L.m, L.b)


def run_gemv(layer: B.Layer, X_bits: np.ndarray, kind: int) -> np.ndarray:
    batch = X_bits.shape[0]
    x = f16_to_dev(X_bits)
    y = torch.full((batch, layer.n_out), float("nan"), dtype=torch.float16, device="cuda")
    B.dbf_gemv(layer, x.data_ptr(), y.data_ptr(), batch, stream_handle(), kind)
    torch.cuda.synchronize()
    return dev_to_f64(y)


def run_gemm(layer: B.Layer, X_bits: np.ndarray, kind: int = B.GEMM_AUTO) -> np.ndarray:
    T = X_bits.shape[0]
    x = f16_to_dev(X_bits)
    y = torch.full((T, layer.n_out), float("nan"), dtype=torch.float16, device="cuda")
    ws_bytes = B.dbf_gemm_workspace_bytes(layer, T)
    # scratch pre-filled with a byte pattern: nothing may depend on its contents
    ws = torch.full((max(ws_bytes, 256),), 0xA5, dtype=torch.uint8, device="cuda")
    assert ws.data_ptr() % 256 == 0
    B.dbf_gemm(layer, x.data_ptr(), y.data_ptr(), T, ws.data_ptr(), ws_bytes, stream_handle(), kind)
    torch.cuda.synchronize()
    return dev_to_f64(y)


def check(y_gpu: np.ndarray, y_ref: np.ndarray, what: str, tol: float = TOL) -> float:
    assert y_gpu.shape == y_ref.shape, what
    assert np.all(np.isfinite(y_gpu)), what + ": non-finite output"
    # Outputs are fp16: below 2^-14 their spacing is the absolute 2^-24, so half of that
    # (one rounding of a subnormal result) is allowed on top of the relative gate.
    delta = np.abs(y_gpu - y_ref)
    y_adj = y_ref + np.sign(y_gpu - y_ref) * np.maximum(delta - 2.0 ** -25, 0.0)
    err = O.gated_relative_error(y_adj, y_ref)
    # (also the plain relative error over the outputs that are at least as large as their row's rms, where the gate
    #  and the plain definition coincide: reported, and bounded by the same assertion)
    ref2 = y_ref if y_ref.ndim > 1 else y_ref[None, :]
    adj2 = y_adj if y_adj.ndim > 1 else y_adj[None, :]
    big = np.abs(ref2) >= np.sqrt(np.mean(ref2 * ref2, axis=1, keepdims=True))
    big &= ref2 != 0.0
    plain = float(np.max(np.abs(adj2[big] - ref2[big]) / np.abs(ref2[big]))) if big.any() else 0.0
    say("%s: gated rel err %.3e, plain rel err over |y| >= rms %.3e (tol %.1e)" % (what, err, plain, tol))
    assert err <= tol, "%s: error %.3e > %.1e" % (what, err, tol)
    return err
