"""GPU parity of the headline measurement itself: 512 distinct layers n_in = n_out = 4096, k = 2048
(configuration 2; 1 GiB of sign bits) run as ONE stack call of the default kind, which is the launch
configuration bench.py times -- at batch 1 (both stages of all layers in one launch), 4 and 16 (input
quantisers and work items with a row tile per wavefront).

What is unique is compared bit for bit: every layer's outputs must equal those of a call of that
layer alone in the two-launch kind, whose work lists, launches and kernels are different ones (integer
sums are exact, so the cut of the work must not show).  Eight sampled layers per batch are compared
element by element against the fp64 oracle (staged evaluation), as is the layer that deviates most from
the variance law of i.i.d. signs, against which every layer is checked (it holds at any size).
"""
import numpy as np
import pytest
import torch

import gpu_util as G
from oracle import dbf_oracle as O
from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

pytestmark = pytest.mark.gpu

N_LAYERS = 512


@pytest.fixture(scope="module")
def stream():
    cfg = I.CONFIG2
    G.say("config2 stream: generating and packing %d layers" % N_LAYERS)
    Ls = [I.make_layer(cfg["n_in"], cfg["n_out"], cfg["k"], seed=I.seed_for(2, 5000 + i)) for i in range(N_LAYERS)]
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    yield Ls, layers, stack
    stack.close()
    for layer in layers:
        layer.close()


@pytest.mark.parametrize("batch", [1, 4, 16])
def test_config2_stream_as_the_benchmark_launches_it(stream, batch):
    Ls, layers, stack = stream
    n_in, n_out = Ls[0].n_in, Ls[0].n_out
    rng = np.random.default_rng(I.seed_for(2, 6000 + batch))
    X = I.random_activations_fp16(rng, N_LAYERS * batch, n_in).reshape(N_LAYERS, batch, n_in)
    x_all = G.f16_to_dev(X.reshape(-1, n_in)).reshape(-1)
    y_all = torch.full((N_LAYERS * batch * n_out,), float("nan"), dtype=torch.float16, device="cuda")
    for rep in range(2):  # (the second call finds counters and scratch as the first left them)
        G.say("config2 stream: stack call %d, batch %d" % (rep, batch))
        y_all.fill_(float("nan"))
        B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), B.GEMV_AUTO)
        torch.cuda.synchronize()
    assert B.dbf_stack_sync_timeouts(stack) == 0
    got_bits = y_all.cpu().view(torch.int16).numpy().reshape(N_LAYERS, batch, n_out)
    got = G.dev_to_f64(y_all).reshape(N_LAYERS, batch, n_out)
    assert np.all(np.isfinite(got))

    G.say("  every layer against its own two-launch call, bit for bit")
    y_one = torch.empty(batch * n_out, dtype=torch.float16, device="cuda")
    for i, layer in enumerate(layers):
        xi = x_all[i * batch * n_in:(i + 1) * batch * n_in]
        B.dbf_gemv(layer, xi.data_ptr(), y_one.data_ptr(), batch, G.stream_handle(), B.GEMV_MFMA_SPLIT)
        torch.cuda.synchronize()
        assert np.array_equal(y_one.cpu().view(torch.int16).numpy().reshape(batch, n_out), got_bits[i]), i

    G.say("  every layer against the variance law; eight layers against the oracle")
    # (the law: given the middle activations t the outputs have variance a_i^2 sum_j m_j^2 t_j^2, whose mean over t is
    #  a_i^2 sum_j m_j^2 sum_l (b_l x_l)^2; with k = 2048 the measured rms scatters by 1.6 % around it, so over the
    #  8192 rows of the batch-16 case deviations of 7-8 % do occur: the bound is 12 %, and the layer that deviates most
    #  is one of those compared with the oracle)
    worst, worst_dev = 0, 0.0
    for i, L in enumerate(Ls):
        a, m, b = O.f16_bits_to_f64(L.a), O.f16_bits_to_f64(L.m), O.f16_bits_to_f64(L.b)
        x = O.f16_bits_to_f64(X[i]).reshape(batch, n_in)
        want = np.sqrt(np.mean(a ** 2) * np.sum((x * b[None, :]) ** 2, axis=1) * np.sum(m ** 2))
        rms = np.sqrt(np.mean(got[i] ** 2, axis=1))
        dev = float(np.max(np.abs(rms / want - 1.0)))
        assert dev < 0.12, (i, rms, want)
        if dev > worst_dev:
            worst, worst_dev = i, dev
    G.say("  largest deviation from the law: %.3f (layer %d)" % (worst_dev, worst))
    for i in sorted({0, 1, 63, 64, 255, 256, 300, 511, worst}):
        G.check(got[i], O.forward_from_packed(X[i], Ls[i], "staged"), "config2 stream layer %d batch %d" % (i, batch))
