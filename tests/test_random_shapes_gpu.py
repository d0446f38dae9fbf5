"""GPU parity on seeded random layer shapes: dimensions drawn from 1 ... 9000 (ragged, mostly no multiple of anything),
two random batches per layer through every decode kind, one random token count through the prefill entry point.

Every output is compared with the fp64 oracle (staged evaluation), the matrix-core kinds with each other bit for bit,
and the first 16 prefill tokens with the decode result bit for bit.

The gate of the other tests measures an error against max(|y_i|, rms of the output row).  A row of one or two
outputs, or a layer with a single middle channel (all outputs multiples of one sum), has no such scale: when that
sum cancels, the gate becomes the plain relative error of a value near zero.  Such layers are drawn here as well;
for them the error is measured against the statistical scale of an output instead, |a_i| * ||m|| * ||x . b|| (the
standard deviation of y_i over random signs, section 3's forward expression), with the same bound."""
import numpy as np
import pytest

import gpu_util as G
from oracle import dbf_oracle as O
from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

pytestmark = pytest.mark.gpu

KINDS = ((B.GEMV_AUTO, "auto"), (B.GEMV_MFMA, "one launch"), (B.GEMV_MFMA_SPLIT, "two launches"), (B.GEMV_VALU, "vector ALU"))


def _dim(rng):
    r = rng.random()
    if r < 0.3:
        return int(rng.integers(1, 200))
    if r < 0.8:
        return int(rng.integers(200, 3000))
    return int(rng.integers(3000, 9000))


def _statistical_scale(L, X):
    a, m, b = O.f16_bits_to_f64(L.a), O.f16_bits_to_f64(L.m), O.f16_bits_to_f64(L.b)
    x = O.f16_bits_to_f64(X).reshape(-1, L.n_in)
    return np.abs(a)[None, :] * np.sqrt(np.sum(m * m)) * np.sqrt(np.sum((x * b) ** 2, axis=1))[:, None]


def _check(y, ref, L, X, what):
    if L.n_out >= 8 and L.k >= 8:
        G.check(y, ref, what)
        return
    assert np.all(np.isfinite(y)), what
    scale = _statistical_scale(L, X)
    err = float(np.max((np.abs(y - ref) - 2.0 ** -25) / np.maximum(scale, np.abs(ref))))
    G.say("%s: error against the statistical scale %.3e" % (what, err))
    assert err <= G.TOL, "%s: error %.3e" % (what, err)


@pytest.mark.parametrize("block", range(6))
def test_random_layers(block):
    rng = np.random.default_rng(I.seed_for(7, 40 + block))
    for case in range(8):
        n_in, n_out, k = _dim(rng), _dim(rng), _dim(rng)
        if case == 0:      # one degenerate layer per block: very few outputs or middle channels
            n_out, k = ((1, k), (2, k), (n_out, 1))[block % 3]
        if rng.random() < 0.3:
            n_in = (n_in + 7) // 8 * 8     # (rows that can be read in 16-byte pieces take other input paths)
        L = I.make_layer(n_in, n_out, k, seed=int(rng.integers(1 << 30)))
        layer = G.pack(L)
        try:
            for _ in range(2):
                batch = int(rng.integers(1, B.MAX_BATCH + 1))
                X = I.make_activations(batch, n_in, seed=int(rng.integers(1 << 30)))
                ref = O.forward_from_packed(X, L, "staged")
                outs = {}
                for kind, name in KINDS:
                    what = "random layer n_in=%d n_out=%d k=%d batch=%d kind %s" % (n_in, n_out, k, batch, name)
                    G.say("start " + what)
                    outs[name] = G.run_gemv(layer, X, kind)
                    _check(outs[name], ref, L, X, what)
                assert np.array_equal(outs["auto"], outs["two launches"]), what
                assert np.array_equal(outs["one launch"], outs["two launches"]), what
            T = int(rng.integers(1, 130))
            X = I.make_activations(T, n_in, seed=int(rng.integers(1 << 30)))
            what = "random layer n_in=%d n_out=%d k=%d prefill T=%d" % (n_in, n_out, k, T)
            G.say("start " + what)
            y = G.run_gemm(layer, X, B.GEMM_AUTO)
            _check(y, O.forward_from_packed(X, L, "staged"), L, X, what)
            head = min(T, B.MAX_BATCH)
            assert np.array_equal(G.run_gemv(layer, X[:head], B.GEMV_MFMA_SPLIT), y[:head]), what + " (decode bits)"
        finally:
            layer.close()
