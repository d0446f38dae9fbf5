"""GPU parity of the prefill path (dbf_gemm: two matrix-core contractions) against
the fp64 dense-W' oracle on the same seeded inputs, the int8 matrix cores as the adder
with 16-bit fixed-point activations.
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


KINDS = [(B.GEMM_I8, "i8"), (B.GEMM_AUTO, "auto")]


def _case(n_in, n_out, k, T, seed, mode="dense"):
    L = I.make_layer(n_in, n_out, k, seed)
    X = I.make_activations(T, n_in, seed)
    layer = G.pack(L)
    try:
        G.say("oracle (%s) n_in=%d n_out=%d k=%d T=%d" % (mode, n_in, n_out, k, T))
        ref = O.forward_from_packed(X, L, mode)
        for kind, name in KINDS:
            what = "gemm[%s] n_in=%d n_out=%d k=%d T=%d seed=%d" % (name, n_in, n_out, k, T, seed)
            G.say("start " + what)
            G.check(G.run_gemm(layer, X, kind), ref, what)
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


@pytest.mark.parametrize("shape", [(512, 512, 256), (1000, 130, 77), (4100, 333, 600)])
def test_up_to_32_tokens_run_as_decode_batches_with_the_same_bits(shape):
    """dbf_gemm hands 17 ... 32 tokens to the decode kernels as two batches (16 and the rest); 33 tokens and more take
    the prefill kernels.  Either way the outputs are those of the prefill kernels bit for bit, and within the gate of
    the oracle."""
    n_in, n_out, k = shape
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(4, 60 + k))
    X = I.make_activations(40, n_in, I.seed_for(4, 61 + k))
    ref = O.forward_from_packed(X, L, "staged")
    layer = G.pack(L)
    try:
        for T in (17, 24, 31, 32, 33, 40):
            what = "gemm[auto] n_in=%d n_out=%d k=%d T=%d" % (n_in, n_out, k, T)
            G.say("start " + what)
            y = G.run_gemm(layer, X[:T], B.GEMM_AUTO)
            G.check(y, ref[:T], what)
            assert np.array_equal(y, G.run_gemm(layer, X[:T], B.GEMM_I8)), what
    finally:
        layer.close()


def _decode_in_batches(layer, X):
    return np.concatenate([G.run_gemv(layer, X[t0:t0 + B.MAX_BATCH], B.GEMV_MFMA_SPLIT) for t0 in range(0, X.shape[0], B.MAX_BATCH)])


@pytest.mark.parametrize("shape", [(512, 512, 256), (1000, 130, 77), (4100, 333, 600), (700, 2600, 1500)])
def test_column_splits_of_calls_of_few_tokens(shape):
    """Up to 512 tokens, a stage that would start fewer than 256 workgroups cuts its column steps into shares over
    grid.z workgroups, which add exact integer sums and let the last to arrive finish (the sums and counters live in
    the workspace, cleared by the first quantiser launch: the workspace here is pre-filled with a byte pattern).
    Every token of every call equals the decode kernels' result bit for bit -- with the built-in number of shares,
    with 2, 5 and as many as there are column steps, and with none -- and is within the gate of the oracle; a second
    call on the same workspace finds what the first left."""
    n_in, n_out, k = shape
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(4, 80 + k))
    X = I.make_activations(513, n_in, I.seed_for(4, 81 + k))
    ref = O.forward_from_packed(X, L, "staged")
    layer = G.pack(L)
    try:
        want = _decode_in_batches(layer, X)
        for T in (33, 64, 100, 256, 512, 513):
            for splits in (-1, 1, 2, 5, 1024):
                B.dbf_tuning_set(B.TUNE_GEMM_SPLITS, splits)
                what = "gemm n_in=%d n_out=%d k=%d T=%d splits knob %d" % (n_in, n_out, k, T, splits)
                G.say("start " + what)
                y = G.run_gemm(layer, X[:T], B.GEMM_I8)
                assert np.array_equal(y, want[:T]), what
                if splits == -1:
                    G.check(y, ref[:T], what)
        # two calls in a row on ONE workspace, the second smaller: the sums and counters the first call left are zero
        B.dbf_tuning_set(B.TUNE_GEMM_SPLITS, 3)
        T1, T2 = 200, 70
        wsb = B.dbf_gemm_workspace_bytes(layer, T1)
        ws = torch.full((wsb,), 0x5A, dtype=torch.uint8, device="cuda")
        for T in (T1, T2):
            x = G.f16_to_dev(X[:T])
            y = torch.full((T, n_out), float("nan"), dtype=torch.float16, device="cuda")
            B.dbf_gemm(layer, x.data_ptr(), y.data_ptr(), T, ws.data_ptr(), wsb, G.stream_handle(), B.GEMM_I8)
            torch.cuda.synchronize()
            assert np.array_equal(G.dev_to_f64(y), want[:T]), (T1, T2, T)
    finally:
        B.dbf_tuning_reset()
        layer.close()


@pytest.mark.parametrize("T", [24, 64, 600])
def test_prefill_call_replayed_from_a_captured_graph(T):
    """dbf_gemm allocates nothing, synchronises nothing and clears what it needs with its own kernels (no memset), in all
    three regimes -- decode batches (24 tokens), column shares with their sums and counters in the workspace (64), the
    plain four launches (600) -- so a call can be captured into a HIP graph.  Every replay, with new inputs written and
    eager work in between, must give what the eager call gives for those inputs, bit for bit."""
    n_in, n_out, k = 1000, 390, 520
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(4, 90))
    layer = G.pack(L)
    try:
        wsb = B.dbf_gemm_workspace_bytes(layer, T)
        ws = torch.full((max(wsb, 256),), 0x3C, dtype=torch.uint8, device="cuda")
        x = G.f16_to_dev(I.make_activations(T, n_in, I.seed_for(4, 91)))
        y = torch.full((T, n_out), float("nan"), dtype=torch.float16, device="cuda")
        B.dbf_gemm(layer, x.data_ptr(), y.data_ptr(), T, ws.data_ptr(), wsb, G.stream_handle())   # (first call outside the capture)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            graph.capture_begin()
            B.dbf_gemm(layer, x.data_ptr(), y.data_ptr(), T, ws.data_ptr(), wsb, side.cuda_stream)
            graph.capture_end()
        torch.cuda.current_stream().wait_stream(side)
        for rep in range(4):
            X = I.make_activations(T, n_in, I.seed_for(4, 92 + rep))
            want = G.run_gemm(layer, X, B.GEMM_AUTO)          # eager, on a workspace of its own
            x.copy_(G.f16_to_dev(X))
            y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(G.dev_to_f64(y), want), (T, rep)
        del graph
    finally:
        layer.close()


@pytest.mark.parametrize("idx", [0, 1])
def test_config4_prefill_every_token(idx):
    """Both prefill shapes at T = 2048, every one of the 2048 x 4096 outputs against the oracle's staged
    mode (the forward-pass expression left to right in fp64, which the oracle's own pins tie to the dense
    product to 1e-12; forming W' densely first would cost 2.7e11 more multiply-adds at k = 5970)."""
    cfg = I.CONFIG4[idx]
    _case(cfg["n_in"], cfg["n_out"], cfg["k"], cfg["T"], seed=I.seed_for(4, 100 + idx), mode="staged")


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
        assert lib.dbf_gemm_kind(h, x.data_ptr(), y.data_ptr(), T, ws.data_ptr(), need, 1, None) == B.DBF_EINVAL  # withdrawn
    finally:
        layer.close()
