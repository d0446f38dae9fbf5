"""GPU parity at full size of the stacks that quantise their stage inputs once per call at batch 1 too (several
layers with one stage input longer than 6144 values and the other longer than 4096): short streams of the
down-projection of configuration 3 at 2 bits per weight and of the largest layer of the paper's Table 4, as
bench.py's `config3_mlp` and `table4` blocks launch them (default kind, one stack call).

Every layer bit for bit against a call of that layer alone in the two-launch kind (a plan of one layer never
takes the shared-input launches at batch 1, so launches, work lists and kernel instances all differ); one layer
per case element by element against the fp64 oracle.
"""
import numpy as np
import pytest
import torch

import gpu_util as G
from oracle import dbf_oracle as O
from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

pytestmark = pytest.mark.gpu

CASES = [((11008, 4096, 5970), 12, 1), ((11008, 4096, 5970), 12, 4), ((28672, 8192, 6371), 4, 1), ((28672, 8192, 6371), 4, 16)]


@pytest.mark.parametrize("shape,n_layers,batch", CASES)
def test_long_rows_stream_at_full_size(shape, n_layers, batch):
    n_in, n_out, k = shape
    G.say("long-rows stream: %d layers n_in=%d n_out=%d k=%d batch %d" % (n_layers, n_in, n_out, k, batch))
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(3, 7000 + n_in + i)) for i in range(n_layers)]
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        rng = np.random.default_rng(I.seed_for(3, 8000 + batch))
        X = I.random_activations_fp16(rng, n_layers * batch, n_in).reshape(n_layers, batch, n_in)
        x_all = G.f16_to_dev(X.reshape(-1, n_in)).reshape(-1)
        y_all = torch.full((n_layers * batch * n_out,), float("nan"), dtype=torch.float16, device="cuda")
        for rep in range(2):
            y_all.fill_(float("nan"))
            B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), B.GEMV_AUTO)
            torch.cuda.synchronize()
        got_bits = y_all.cpu().view(torch.int16).numpy().reshape(n_layers, batch, n_out)
        got = G.dev_to_f64(y_all).reshape(n_layers, batch, n_out)
        y_one = torch.empty(batch * n_out, dtype=torch.float16, device="cuda")
        for i, layer in enumerate(layers):
            xi = x_all[i * batch * n_in:(i + 1) * batch * n_in]
            B.dbf_gemv(layer, xi.data_ptr(), y_one.data_ptr(), batch, G.stream_handle(), B.GEMV_MFMA_SPLIT)
            torch.cuda.synchronize()
            assert np.array_equal(y_one.cpu().view(torch.int16).numpy().reshape(batch, n_out), got_bits[i]), i
        i = n_layers // 2
        G.check(got[i], O.forward_from_packed(X[i], Ls[i], "staged"), "long-rows stream layer %d" % i)
    finally:
        stack.close()
        for layer in layers:
            layer.close()
