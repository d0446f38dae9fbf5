"""GPU test of dbf_gemm_static, the prefill entry point that allocates nothing (its scratch is a static
device array of the library): called through the C ABI, its output must equal dbf_gemm's -- the same
kernels, so bit for bit, which is inside the 2e-3 gate a fortiori -- on two calls in a row, the second with
a smaller input (the array keeps the first call's contents), and once more against the fp64 oracle.
Sizes beyond the static array are refused before anything is launched."""
import numpy as np
import pytest
import torch

import gpu_util as G
from oracle import dbf_oracle as O
from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

pytestmark = pytest.mark.gpu


def _static(layer, X_bits):
    T = X_bits.shape[0]
    x = G.f16_to_dev(X_bits)
    y = torch.full((T, layer.n_out), float("nan"), dtype=torch.float16, device="cuda")
    B.dbf_gemm_static(layer, x.data_ptr(), y.data_ptr(), T, G.stream_handle())
    torch.cuda.synchronize()
    return G.dev_to_f64(y)


def test_static_scratch_prefill_equals_dbf_gemm_on_two_calls_in_a_row():
    big = I.make_layer(1100, 520, 700, seed=I.seed_for(4, 300))       # ragged in every dimension
    small = I.make_layer(260, 130, 97, seed=I.seed_for(4, 301))
    Xb = I.make_activations(300, big.n_in, I.seed_for(4, 300))
    Xs = I.make_activations(37, small.n_in, I.seed_for(4, 301))
    lb, ls = G.pack(big), G.pack(small)
    try:
        assert B.dbf_gemm_workspace_bytes(lb, 300) <= B.GEMM_STATIC_BYTES
        G.say("dbf_gemm_static: first call, T=300 on 1100->520, k=700")
        got_b = _static(lb, Xb)
        G.say("dbf_gemm_static: second call, T=37 on 260->130, k=97")
        got_s = _static(ls, Xs)
        want_b = G.run_gemm(lb, Xb, B.GEMM_I8)
        want_s = G.run_gemm(ls, Xs, B.GEMM_I8)
        assert np.array_equal(got_b, want_b) and np.array_equal(got_s, want_s)
        G.check(got_b, O.forward_from_packed(Xb, big, "dense"), "dbf_gemm_static T=300")
        G.check(got_s, O.forward_from_packed(Xs, small, "dense"), "dbf_gemm_static T=37")
        # the same layer again after the small one, and a decode-sized call (T <= 16 is no special case here)
        assert np.array_equal(_static(lb, Xb), want_b)
        assert np.array_equal(_static(ls, Xs[:5]), G.run_gemm(ls, Xs[:5], B.GEMM_I8))
    finally:
        lb.close()
        ls.close()


def test_static_scratch_prefill_refuses_what_does_not_fit_and_bad_arguments():
    L = I.make_layer(4096, 512, 4096, seed=I.seed_for(4, 302))
    layer = G.pack(L)
    lib = B.lib()
    try:
        T = 4096                                       # 4096 tokens x (2 x 4096 + 4 x 4096 + 2 x 4096) bytes = 128 MiB
        assert B.dbf_gemm_workspace_bytes(layer, T) > B.GEMM_STATIC_BYTES
        x = torch.zeros((T, 4096), dtype=torch.float16, device="cuda")
        y = torch.full((T, 512), 3.0, dtype=torch.float16, device="cuda")
        h = layer.handle
        assert lib.dbf_gemm_static(h, x.data_ptr(), y.data_ptr(), T, None) == B.DBF_EWORKSPACE
        torch.cuda.synchronize()
        assert bool((y == 3.0).all())                  # nothing was launched
        assert lib.dbf_gemm_static(None, x.data_ptr(), y.data_ptr(), 4, None) == B.DBF_EINVAL
        assert lib.dbf_gemm_static(h, None, y.data_ptr(), 4, None) == B.DBF_EINVAL
        assert lib.dbf_gemm_static(h, x.data_ptr(), None, 4, None) == B.DBF_EINVAL
        assert lib.dbf_gemm_static(h, x.data_ptr(), y.data_ptr(), 0, None) == B.DBF_EINVAL
    finally:
        layer.close()
