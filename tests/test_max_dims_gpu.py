"""GPU parity at the largest sizes the library accepts.

The largest dimension, 2^20, in each of the three places it can stand: the input length, the output length (8192
row tiles in the A stage) and the middle size (8192 row tiles in the B stage, rows of 16384 column tiles in the A
stage).  A stage input longer than DBF_INT_PATH_MAX_COLS = 65536 is beyond what the integer matrix-core paths can
add exactly in int32, so the default kind runs those layers on the vector-ALU kernel, the kinds that name the
matrix-core kernel and the prefill kernels (dbf_gemm beyond 32 tokens) refuse them (DBF_ESHAPE).

The longest stage input the integer paths do take, 65536: random inputs through every kind and the prefill, and
the adversarial input -- every product x_l b_l at the quantiser's full scale and a row of B with all signs equal,
so that one middle activation is the largest sum the path can meet, 65536 * 32512 = 2 130 706 432 < 2^31 -- which
must come out exact.

The other dimensions are kept small and ragged, so that the fp64 oracle (staged evaluation) still forms both sign
matrices.  Every output is compared.
"""
import numpy as np
import pytest
import torch

import gpu_util as G
from oracle import dbf_oracle as O
from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

pytestmark = pytest.mark.gpu

BIG = 1 << 20
SHAPES = {"n_in": (BIG, 130, 33), "n_out": (70, BIG, 33), "k": (24, 40, BIG)}  # (n_in, n_out, k)


LIMIT = 1 << 16


@pytest.mark.parametrize("which", ["n_in", "n_out", "k"])
def test_decode_at_the_largest_dimension(which):
    n_in, n_out, k = SHAPES[which]
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(1, 900 + len(which)))
    layer = G.pack(L)
    try:
        for batch in (1, 3, 16):
            X = I.make_activations(batch, n_in, seed=I.seed_for(1, 910 + batch))
            ref = O.forward_from_packed(X, L, "staged")
            what = "largest %s: n_in=%d n_out=%d k=%d batch=%d" % (which, n_in, n_out, k, batch)
            G.say("start " + what)
            G.check(G.run_gemv(layer, X, B.GEMV_AUTO), ref, what)
            if which == "n_out":   # no long stage input: the matrix-core kinds take it
                G.check(G.run_gemv(layer, X, B.GEMV_MFMA), ref, what + " (one launch)")
        if which != "n_out":
            x = G.f16_to_dev(I.make_activations(1, n_in, seed=1))
            y = torch.zeros((1, n_out), dtype=torch.float16, device="cuda")
            for kind in (B.GEMV_MFMA, B.GEMV_MFMA_SPLIT):
                rc = B.lib().dbf_gemv_kind(layer.handle, x.data_ptr(), y.data_ptr(), 1, kind, G.stream_handle())
                assert rc == B.DBF_ESHAPE, (kind, rc)
            # (up to 32 tokens dbf_gemm runs decode batches, which take such layers; beyond, the prefill kernels refuse)
            X33 = G.f16_to_dev(I.make_activations(33, n_in, seed=2))
            Y33 = torch.zeros((33, n_out), dtype=torch.float16, device="cuda")
            wsb = B.dbf_gemm_workspace_bytes(layer, 33)
            ws = torch.zeros(max(wsb, 256), dtype=torch.uint8, device="cuda")
            rc = B.lib().dbf_gemm(layer.handle, X33.data_ptr(), Y33.data_ptr(), 33, ws.data_ptr(), wsb, G.stream_handle())
            assert rc == B.DBF_ESHAPE, rc
            X20 = I.make_activations(20, n_in, seed=I.seed_for(1, 930))
            G.check(G.run_gemm(layer, X20, B.GEMM_AUTO), O.forward_from_packed(X20, L, "staged"), "20 tokens, largest " + which)
    finally:
        layer.close()


@pytest.mark.parametrize("which", ["n_in", "k"])
def test_longest_stage_input_of_the_integer_paths(which):
    """65536 inputs per stage: every kind and the prefill on random inputs; then the largest sum the integer path can
    meet, exactly."""
    n_in, n_out, k = (LIMIT, 130, 33) if which == "n_in" else (24, 40, LIMIT)
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(1, 950 + len(which)))
    layer = G.pack(L)
    try:
        for batch in (1, 2, 16):
            X = I.make_activations(batch, n_in, seed=I.seed_for(1, 960 + batch))
            ref = O.forward_from_packed(X, L, "staged")
            for kind, name in ((B.GEMV_AUTO, "auto"), (B.GEMV_MFMA, "one launch"), (B.GEMV_MFMA_SPLIT, "two launches")):
                what = "longest integer %s: n_in=%d n_out=%d k=%d batch=%d kind %s" % (which, n_in, n_out, k, batch, name)
                G.say("start " + what)
                G.check(G.run_gemv(layer, X, kind), ref, what)
        X = I.make_activations(70, n_in, seed=I.seed_for(4, 970))
        G.say("start prefill, longest integer %s" % which)
        G.check(G.run_gemm(layer, X, B.GEMM_AUTO), O.forward_from_packed(X, L, "staged"), "prefill, longest integer " + which)
    finally:
        layer.close()


def test_the_largest_sum_of_the_integer_path_is_exact():
    """n_in = 65536, x_l b_l = 2 for every l (so every q is 32512, the quantiser's full scale), row 5 of B all +1, row 6
    all -1, the other rows random: t_5 = +131072 m_5 and t_6 = -131072 m_6 exactly -- sums of 65536 * 32512 in int32.
    k = 8 and A = identity-like signs keep the A stage out of the way: y is compared with the oracle element by element,
    and t_5, t_6 are recovered from it."""
    n_in, n_out, k = LIMIT, 16, 8
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(1, 990))
    words = L.B_bits.reshape(k, -1).copy()
    words[5, :] = 0xFFFFFFFF
    words[6, :] = 0
    L.B_bits = words
    L.b = np.full(n_in, np.float16(1.0).view(np.uint16), dtype=np.uint16)
    X = np.full((2, n_in), np.float16(2.0).view(np.uint16), dtype=np.uint16)
    X[1, ::2] = np.float16(-2.0).view(np.uint16)     # second batch row: alternating signs, sums near zero
    ref = O.forward_from_packed(X, L, "staged")
    layer = G.pack(L)
    try:
        for kind, name in ((B.GEMV_AUTO, "auto"), (B.GEMV_MFMA, "one launch"), (B.GEMV_MFMA_SPLIT, "two launches"),
                           (B.GEMV_VALU, "vector ALU")):
            what = "largest int32 sum, kind %s" % name
            G.say("start " + what)
            G.check(G.run_gemv(layer, X, kind), ref, what)
        G.check(G.run_gemm(layer, np.repeat(X, 20, axis=0), B.GEMM_AUTO), np.repeat(ref, 20, axis=0), "largest int32 sum, prefill")
    finally:
        layer.close()
