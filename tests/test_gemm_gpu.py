"""GPU parity of the prefill path (dbf_gemm: two matrix-core contractions) against
the fp64 dense-W' oracle on the same seeded inputs, for both variants: int8 matrix
cores with 16-bit fixed-point activations (the default) and fp16 matrix cores.
Gate as for decode: gated relative error <= 2e-3.
"""
import numpy as np
import pytest
import torch

from oracle import dbf_oracle as O
from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu


KINDS = [(B.GEMM_I8, "i8"), (B.GEMM_F16, "f16")]


def _case(n_in, n_out, k, T, seed, rows=None):
    L = I.make_layer(n_in, n_out, k, seed)
    X = I.make_activations(T, n_in, seed)
    layer = G.pack(L)
    try:
        ref = O.forward_from_packed(X if rows is None else X[rows], L, "dense")
        for kind, name in KINDS:
            what = "gemm[%s] n_in=%d n_out=%d k=%d T=%d seed=%d" % (name, n_in, n_out, k, T, seed)
            G.say("start " + what)
            y = G.run_gemm(layer, X, kind)
            if rows is None:
                G.check(y, ref, what)
            else:
                # large case: the oracle evaluates a sample of token rows (each output row one by one)
                G.check(y[rows], ref, what + " (sampled rows)")
    finally:
        layer.close()


@pytest.mark.parametrize("T", [1, 8, 64, 100, 130])
def test_config1_token_counts(T):
    _case(T=T, seed=I.seed_for(4, T), **I.CONFIG1)


@pytest.mark.parametrize("shape", [
    (1, 1, 1), (5, 3, 2), (64, 128, 64), (65, 129, 65), (100, 77, 33), (130, 300, 257),
    (1000, 50, 130), (72, 600, 520), (517, 513, 129)])
@pytest.mark.parametrize("T", [3, 70])
def test_ragged_shapes(shape, T):
    n_in, n_out, k = shape
    _case(n_in, n_out, k, T, seed=I.seed_for(4, 20 + T))


def test_gemm_agrees_with_gemv_rows():
    """Rows of X are independent: prefill of 16 tokens equals 16-token decode within rounding."""
    L = I.make_layer(seed=I.seed_for(4, 50), **I.CONFIG1)
    X = I.make_activations(16, 512, I.seed_for(4, 50))
    layer = G.pack(L)
    try:
        yv = G.run_gemv(layer, X, B.GEMV_VALU)
        for kind, name in KINDS:
            G.check(G.run_gemm(layer, X, kind), yv, "gemm[%s] vs gemv[valu]" % name)
        # the int8 variant quantises exactly as the matrix-core decode kernel does: same integers,
        # same scales, so the fp16 outputs are identical
        assert np.array_equal(G.run_gemm(layer, X, B.GEMM_I8), G.run_gemv(layer, X, B.GEMV_MFMA_SPLIT))
        # dbf_gemm (DBF_GEMM_AUTO) runs up to 16 tokens as a decode batch: the same bits again, also for T = 1 and 5
        for T in (1, 5, 16):
            assert np.array_equal(G.run_gemm(layer, X[:T], B.GEMM_AUTO), G.run_gemm(layer, X[:T], B.GEMM_I8)), T
    finally:
        layer.close()


def test_config4_square_prefill():
    cfg = I.CONFIG4[0]
    rows = np.arange(0, cfg["T"], 37)
    _case(cfg["n_in"], cfg["n_out"], cfg["k"], cfg["T"], seed=I.seed_for(4, 100), rows=rows)


def test_config4_down_projection_prefill():
    cfg = I.CONFIG4[1]
    rows = np.array([0, 1, 63, 64, 1000, 1023, 1024, 2047])
    _case(cfg["n_in"], cfg["n_out"], cfg["k"], cfg["T"], seed=I.seed_for(4, 101), rows=rows)


def test_gemm_argument_errors():
    L = I.make_layer(seed=I.seed_for(4, 60), **I.CONFIG1)
    layer = G.pack(L)
    lib = B.lib()
    try:
        T = 4
        x = torch.zeros((T, 512), dtype=torch.float16, device="cuda")
        y = torch.zeros((T, 512), dtype=torch.float16, device="cuda")
        need = B.dbf_gemm_workspace_bytes(layer, T)
        assert need >= T * 256 * 2 and need % 256 == 0
        ws = torch.zeros(need + 256, dtype=torch.uint8, device="cuda")
        h = layer.handle
        assert lib.dbf_gemm(h, x.data_ptr(), y.data_ptr(), 0, ws.data_ptr(), need, None) == B.DBF_EINVAL
        assert lib.dbf_gemm(h, None, y.data_ptr(), T, ws.data_ptr(), need, None) == B.DBF_EINVAL
        assert lib.dbf_gemm(h, x.data_ptr(), y.data_ptr(), T, None, need, None) == B.DBF_EWORKSPACE
        assert lib.dbf_gemm(h, x.data_ptr(), y.data_ptr(), T, ws.data_ptr(), need - 1, None) == B.DBF_EWORKSPACE
        assert lib.dbf_gemm(h, x.data_ptr(), y.data_ptr(), T, ws.data_ptr() + 16, need, None) == B.DBF_EWORKSPACE
        assert lib.dbf_gemm_workspace_bytes(h, 0) == 0
    finally:
        layer.close()
