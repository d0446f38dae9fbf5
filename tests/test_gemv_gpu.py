"""GPU parity of the decode path (dbf_pack / dbf_gemv / dbf_stack_gemv) against
the fp64 dense-W' oracle, element by element, on the same seeded inputs.

Gate: max_i |y_gpu - y_ref| / max(|y_ref|, rms(y_ref)) <= 2e-3 per output row;
packing and indexing bit-exact.
"""
import numpy as np
import pytest
import torch

from oracle import dbf_oracle as O
from paper_2505_11076_amd import binding as B
from paper_2505_11076_amd import inputs as I

import gpu_util as G

pytestmark = pytest.mark.gpu

KINDS = [(B.GEMV_VALU, "valu"), (B.GEMV_MFMA, "mfma"), (B.GEMV_MFMA_SPLIT, "mfma_split"), (B.GEMV_AUTO, "auto")]


@pytest.fixture(autouse=True)
def _default_tuning():
    """Every test starts from, and leaves behind, the library's default tuning knobs."""
    B.dbf_tuning_reset()
    yield
    B.dbf_tuning_reset()


def _case(n_in, n_out, k, batch, seed, kinds=KINDS, mode="dense"):
    L = I.make_layer(n_in, n_out, k, seed)
    X = I.make_activations(batch, n_in, seed)
    ref = O.forward_from_packed(X, L, mode)
    layer = G.pack(L)
    errs = {}
    try:
        for kind, name in kinds:
            what = "gemv[%s] n_in=%d n_out=%d k=%d batch=%d seed=%d" % (name, n_in, n_out, k, batch, seed)
            G.say("start " + what)
            y = G.run_gemv(layer, X, kind)
            errs[name] = G.check(y, ref, what)
    finally:
        layer.close()
    return errs


# ---- packing ----------------------------------------------------------------------------------


@pytest.mark.parametrize("shape", [(512, 512, 256), (100, 77, 33), (1, 1, 1), (130, 129, 65), (97, 300, 2985)])
def test_pack_unpack_round_trip_bit_exact(shape):
    n_in, n_out, k = shape
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(1, 7))
    G.say("round trip n_in=%d n_out=%d k=%d" % shape)
    layer = G.pack(L)
    try:
        A, Bm, a, m, b = B.dbf_unpack_bits(layer)
        assert np.array_equal(A, L.A_bits) and np.array_equal(Bm, L.B_bits)
        assert np.array_equal(a, L.a) and np.array_equal(m, L.m) and np.array_equal(b, L.b)
        assert B.dbf_dims(layer)[:3] == (n_in, n_out, k)
        assert layer.device_bytes >= B.dbf_tiled_bytes(n_out, k) + B.dbf_tiled_bytes(k, n_in)
    finally:
        layer.close()


def test_pack_from_int8_signs_equals_pack_from_words():
    n_in, n_out, k = 70, 45, 37
    rng = np.random.default_rng(I.seed_for(1, 8))
    A = I.random_signs(rng, n_out, k)
    Bs = I.random_signs(rng, k, n_in)
    a = I.random_scale_fp16(rng, n_out)
    m = I.random_scale_fp16(rng, k)
    b = I.random_scale_fp16(rng, n_in)
    layer = B.dbf_pack(n_in, n_out, k, A, Bs, a, m, b)
    try:
        Ab, Bb, a2, m2, b2 = B.dbf_unpack_bits(layer)
        assert np.array_equal(Ab, O.pack_signs(A)) and np.array_equal(Bb, O.pack_signs(Bs))
        assert np.array_equal(a2, a) and np.array_equal(m2, m) and np.array_equal(b2, b)
    finally:
        layer.close()


# ---- decode parity ----------------------------------------------------------------------------


@pytest.mark.parametrize("batch", [1, 8])
def test_config1(batch):
    _case(batch=batch, seed=I.seed_for(1, batch), **I.CONFIG1)


@pytest.mark.parametrize("shape", [
    (1, 1, 1), (5, 3, 2), (64, 128, 64), (65, 129, 65), (100, 77, 33), (130, 300, 257), (1000, 50, 130)])
@pytest.mark.parametrize("batch", [1, 3])
def test_ragged_shapes(shape, batch):
    n_in, n_out, k = shape
    _case(n_in, n_out, k, batch, seed=I.seed_for(1, 20 + batch))


@pytest.mark.parametrize("batch", [2, 5, 9, 16])
def test_batches_and_column_groups(batch):
    _case(n_in=700, n_out=260, k=390, batch=batch, seed=I.seed_for(1, 40 + batch))


def test_many_column_chunks_at_batch_16():
    # 16 batch rows leave room for about 1024 staged columns, so 3000 columns take several chunks
    _case(n_in=3000, n_out=200, k=1500, batch=16, seed=I.seed_for(1, 60))


@pytest.mark.parametrize("batch", [1, 4, 16])
def test_config2(batch):
    _case(batch=batch, seed=I.seed_for(2, batch), **I.CONFIG2)


@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_config3(idx):
    cfg = I.CONFIG3[idx]
    _case(batch=1, seed=I.seed_for(3, idx), **cfg)


def test_special_inputs_zero_and_single_entry():
    """x = 0 gives y = 0 exactly; x = e_l gives column l of W' (one weight per output)."""
    L = I.make_layer(n_in=200, n_out=150, k=100, seed=I.seed_for(1, 70))
    layer = G.pack(L)
    try:
        X = np.zeros((2, 200), dtype=np.uint16)
        X[1, 137] = np.float16(1.0).view(np.uint16)
        ref = O.forward_from_packed(X, L, "dense")
        for kind, name in KINDS:
            G.say("special inputs [%s]" % name)
            y = G.run_gemv(layer, X, kind)
            assert np.all(y[0] == 0.0)
            G.check(y[1:], ref[1:], "single entry [%s]" % name)
    finally:
        layer.close()


def test_outlier_activation():
    """One activation 1000x larger than the rest: the fixed-point step of the matrix-core
    variant is set by the maximum, so this bounds its worst case."""
    n_in, n_out, k = 1024, 256, 512
    L = I.make_layer(n_in, n_out, k, seed=I.seed_for(1, 71))
    X = I.make_activations(1, n_in, I.seed_for(1, 71))
    Xf = X.view(np.float16).copy()
    Xf[0, 5] = np.float16(300.0)
    X = Xf.view(np.uint16)
    ref = O.forward_from_packed(X, L, "dense")
    layer = G.pack(L)
    try:
        for kind, name in KINDS:
            G.say("outlier [%s]" % name)
            G.check(G.run_gemv(layer, X, kind), ref, "outlier [%s]" % name)
    finally:
        layer.close()


def test_deterministic_across_runs():
    L = I.make_layer(seed=I.seed_for(1, 72), **I.CONFIG1)
    X = I.make_activations(4, 512, I.seed_for(1, 72))
    layer = G.pack(L)
    try:
        for kind, name in KINDS:
            y0 = G.run_gemv(layer, X, kind)
            for _ in range(3):
                assert np.array_equal(G.run_gemv(layer, X, kind), y0), name
    finally:
        layer.close()


def test_gemv_on_a_side_stream():
    L = I.make_layer(seed=I.seed_for(1, 73), **I.CONFIG1)
    X = I.make_activations(2, 512, I.seed_for(1, 73))
    ref = O.forward_from_packed(X, L, "dense")
    layer = G.pack(L)
    try:
        s = torch.cuda.Stream()
        x = G.f16_to_dev(X)
        y = torch.zeros((2, 512), dtype=torch.float16, device="cuda")
        torch.cuda.synchronize()
        with torch.cuda.stream(s):
            B.dbf_gemv(layer, x.data_ptr(), y.data_ptr(), 2, s.cuda_stream)
        s.synchronize()
        G.check(G.dev_to_f64(y), ref, "side stream")
    finally:
        layer.close()


# ---- stacks -----------------------------------------------------------------------------------


@pytest.mark.parametrize("batch", [1, 3, 16])
def test_stack_of_mixed_layers(batch):
    shapes = [(512, 512, 256), (100, 77, 33), (300, 640, 200), (512, 512, 256), (64, 128, 1)]
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 100 + i)) for i, L in enumerate(Ls)]
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
        n_y = sum(batch * L.n_out for L in Ls)
        for kind, name in KINDS:
            G.say("stack [%s] batch=%d" % (name, batch))
            y_all = torch.full((n_y,), float("nan"), dtype=torch.float16, device="cuda")
            B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), kind)
            torch.cuda.synchronize()
            xo_want = yo_want = 0
            for i, L in enumerate(Ls):
                xo, yo = stack.offsets(i, batch)
                assert (xo, yo) == (xo_want, yo_want)
                y = G.dev_to_f64(y_all[yo:yo + batch * L.n_out]).reshape(batch, L.n_out)
                G.check(y, O.forward_from_packed(Xs[i], L, "dense"), "stack[%s] layer %d" % (name, i))
                xo_want += batch * L.n_in
                yo_want += batch * L.n_out
    finally:
        stack.close()
        for l in layers:
            l.close()


def test_one_launch_equals_two_launches_bit_for_bit():
    """The fused launch (A-stage workgroups wait on the device for their layer's B stage) and
    the two-launch variant run the same integer arithmetic, so their fp16 outputs must be
    identical; repeated calls exercise the ever-growing counters (each launch waits for what it adds itself)."""
    shapes = [(512, 512, 256)] * 6 + [(1024, 384, 700), (64, 2048, 64), (2048, 64, 2048)]
    batch = 2
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 200 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 300 + i)) for i, L in enumerate(Ls)]
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
        n_y = sum(batch * L.n_out for L in Ls)
        outs = {}
        for kind, name in ((B.GEMV_MFMA_SPLIT, "split"), (B.GEMV_MFMA, "fused")):
            for rep in range(4):
                G.say("stack %s rep %d" % (name, rep))
                y_all = torch.full((n_y,), float("nan"), dtype=torch.float16, device="cuda")
                B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), kind)
                torch.cuda.synchronize()
                got = y_all.cpu().view(torch.int16).numpy().copy()
                if name in outs:
                    assert np.array_equal(got, outs[name]), (name, rep)
                outs[name] = got
        assert np.array_equal(outs["split"], outs["fused"])
        assert B.dbf_stack_sync_timeouts(stack) == 0
        # the same for single layers (their B and A workgroups are all resident at once)
        for i, layer in enumerate(layers[:3] + layers[-2:]):
            ys = []
            for kind in (B.GEMV_MFMA_SPLIT, B.GEMV_MFMA, B.GEMV_MFMA):
                ys.append(G.run_gemv(layer, Xs[layers.index(layer)], kind))
            assert np.array_equal(ys[0], ys[1]) and np.array_equal(ys[1], ys[2])
            assert B.dbf_sync_timeouts(layer) == 0
    finally:
        stack.close()
        for l in layers:
            l.close()


@pytest.mark.parametrize("batch", [12, 16])
def test_more_workgroups_than_compute_units_at_large_batch(batch):
    """Batches 9-16 use large LDS operands, so only two workgroups fit a compute unit; with more
    than 256 A-stage workgroups some of them share one, and with k = 1024 every A-stage
    workgroup walks two column chunks.  (Regression: placeholder loads of the tile prefetcher
    that were still in flight at a chunk restart used to overwrite reused registers in exactly
    this situation, which corrupted whole row tiles at random.)"""
    shapes = [(256, 4096, 1024)] * 12
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 800 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 900 + i)) for i, L in enumerate(Ls)]
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
        n_y = sum(batch * L.n_out for L in Ls)
        refs = [O.forward_from_packed(Xs[i], L, "staged") for i, L in enumerate(Ls)]
        for kind, name in ((B.GEMV_MFMA, "mfma"), (B.GEMV_MFMA_SPLIT, "mfma_split")):
            for rep in range(3):
                G.say("many workgroups, batch %d [%s] rep %d" % (batch, name, rep))
                y_all = torch.full((n_y,), float("nan"), dtype=torch.float16, device="cuda")
                B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), kind)
                torch.cuda.synchronize()
                yo = 0
                for i, L in enumerate(Ls):
                    y = G.dev_to_f64(y_all[yo:yo + batch * L.n_out]).reshape(batch, L.n_out)
                    G.check(y, refs[i], "many-wg[%s] rep %d layer %d" % (name, rep, i))
                    yo += batch * L.n_out
        assert B.dbf_stack_sync_timeouts(stack) == 0
    finally:
        stack.close()
        for l in layers:
            l.close()


def test_launch_errors_with_a_real_layer():
    L = I.make_layer(seed=I.seed_for(1, 74), **I.CONFIG1)
    layer = G.pack(L)
    lib = B.lib()
    try:
        x = torch.zeros(512, dtype=torch.float16, device="cuda")
        y = torch.zeros(512, dtype=torch.float16, device="cuda")
        h = layer.handle
        assert lib.dbf_gemv(h, None, y.data_ptr(), 1, None) == B.DBF_EINVAL
        assert lib.dbf_gemv(h, x.data_ptr(), None, 1, None) == B.DBF_EINVAL
        assert lib.dbf_gemv(h, x.data_ptr(), y.data_ptr(), 0, None) == B.DBF_EINVAL
        assert lib.dbf_gemv(h, x.data_ptr(), y.data_ptr(), 17, None) == B.DBF_EINVAL
        assert lib.dbf_gemv_kind(h, x.data_ptr(), y.data_ptr(), 1, 7, None) == B.DBF_EINVAL
        assert lib.dbf_gemv_kind(h, x.data_ptr(), y.data_ptr(), 1, 4, None) == B.DBF_EINVAL   # (a withdrawn kind)
        # a layer may appear only once in a stack
        with pytest.raises(B.DbfError) as err:
            B.dbf_stack_create([layer, layer])
        assert err.value.code == B.DBF_EINVAL
    finally:
        layer.close()


@pytest.mark.parametrize("batch", [1, 4])
def test_stack_call_replayed_from_a_captured_graph(batch):
    """The launch entry points allocate nothing, synchronise nothing and keep all state on the
    device (counters cleared by the last workgroup), so a stack call can be captured into a HIP
    graph and replayed.  Every replay, with eager work and synchronisations in between, must
    reproduce the eager result bit for bit.  (Batch 4 takes the four-launch path with the input quantisers.)
    The device-side counters of the one-launch kernel only ever grow and the kernel works out from them what
    the current launch must add, so a replayed launch needs no host-side state."""
    shapes = [(512, 512, 256), (1024, 384, 700), (256, 640, 1000), (512, 512, 256)]
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 950 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 960 + i)) for i, L in enumerate(Ls)]
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
        n_y = batch * sum(L.n_out for L in Ls)
        for kind, name in ((B.GEMV_AUTO, "auto"), (B.GEMV_MFMA, "mfma"), (B.GEMV_MFMA_SPLIT, "mfma_split")):
            G.say("graph capture [%s]" % name)
            y_eager = torch.full((n_y,), float("nan"), dtype=torch.float16, device="cuda")
            B.dbf_stack_gemv(stack, x_all.data_ptr(), y_eager.data_ptr(), batch, G.stream_handle(), kind)
            torch.cuda.synchronize()
            want = y_eager.cpu().view(torch.int16).numpy().copy()
            y_graph = torch.full((n_y,), float("nan"), dtype=torch.float16, device="cuda")
            graph = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                graph.capture_begin()
                B.dbf_stack_gemv(stack, x_all.data_ptr(), y_graph.data_ptr(), batch, side.cuda_stream, kind)
                graph.capture_end()
            torch.cuda.current_stream().wait_stream(side)
            for rep in range(4):
                y_graph.fill_(float("nan"))          # eager work between the replays
                torch.cuda.synchronize()
                graph.replay()
                torch.cuda.synchronize()
                got = y_graph.cpu().view(torch.int16).numpy()
                assert np.array_equal(got, want), (name, rep)
            del graph
        assert B.dbf_stack_sync_timeouts(stack) == 0
    finally:
        stack.close()
        for l in layers:
            l.close()


@pytest.mark.parametrize("batch", [1, 2])
def test_column_pieces_equal_whole_rows_bit_for_bit(batch):
    """Launches with few row tiles cut long rows into column pieces that add exact integer sums into
    per-row accumulators; the last piece scales and stores.  Every piece quantises with the scale of
    the whole row, so the result must equal the uncut launch bit for bit -- for a layer alone (two
    launches), for a short stack (one launch, the finishing piece publishes the row tile), with
    pieces forced onto short rows, and on repeated calls (accumulators and counters are left at zero)."""
    shapes = [(6000, 300, 520), (520, 700, 6000), (4100, 260, 4500)]
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 970 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 980 + i)) for i, L in enumerate(Ls)]

    def run(knobs):
        B.dbf_tuning_reset()
        for knob, val in knobs.items():
            B.dbf_tuning_set(knob, val)
        layers = [G.pack(L) for L in Ls]       # the plans are built here, under these knobs
        stack = B.dbf_stack_create(layers)
        outs = []
        try:
            for rep in range(2):
                for L, X, layer in zip(Ls, Xs, layers):
                    y = torch.full((batch, L.n_out), float("nan"), dtype=torch.float16, device="cuda")
                    B.dbf_gemv(layer, G.f16_to_dev(X).data_ptr(), y.data_ptr(), batch, G.stream_handle())
                    torch.cuda.synchronize()
                    outs.append(y.cpu().view(torch.int16).numpy().copy())
                x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
                y_all = torch.full((sum(batch * L.n_out for L in Ls),), float("nan"), dtype=torch.float16, device="cuda")
                B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle())
                torch.cuda.synchronize()
                outs.append(y_all.cpu().view(torch.int16).numpy().copy())
            assert B.dbf_stack_sync_timeouts(stack) == 0
            for layer in layers:
                assert B.dbf_sync_timeouts(layer) == 0
        finally:
            stack.close()
            for l in layers:
                l.close()
        return outs

    G.say("column pieces: whole rows")
    whole = run({B.TUNE_COL_PIECES: 0})
    for label, env in (("default rule", {}), ("3 pieces everywhere", {B.TUNE_COL_PIECES: 3}),
                       ("many small pieces", {B.TUNE_PIECE_NEVER_TILES: 0, B.TUNE_PIECE_MIN_TILES: 2,
                                              B.TUNE_PIECE_TARGET: 4096})):
        G.say("column pieces: " + label)
        got = run(env)
        assert len(got) == len(whole)
        for i, (g, w) in enumerate(zip(got, whole)):
            assert np.array_equal(g, w), (label, i)
    # and the whole-row result is the oracle's, within the gate
    for L, X, y_bits in zip(Ls, Xs, whole[:3]):
        G.check(O.f16_bits_to_f64(y_bits.view(np.uint16)).reshape(batch, L.n_out), O.forward_from_packed(X, L, "staged"),
                "whole rows %dx%d" % (L.n_out, L.n_in))


@pytest.mark.parametrize("batch", [1, 3, 4])
def test_eight_wavefront_workgroups_equal_four_bit_for_bit(batch):
    """A launch of few whole-row items over long stage inputs gives every workgroup eight wavefronts instead of
    four (wavefronts 4-7 only stream tiles; integer sums, so the order of the adds does not matter).  The results
    must not depend on the width: a layer alone and a stack of three, every workgroup quantising its own input
    (at batches 3 and 4 too, by the knob), rows in one pass and rows in the general two-pass prologue."""
    shapes = [(4096, 600, 2100), (2300, 520, 3100), (6500, 300, 2050)]
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 1200 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 1210 + i)) for i, L in enumerate(Ls)]

    def run(max_items):
        B.dbf_tuning_reset()
        B.dbf_tuning_set(B.TUNE_COL_PIECES, 0)
        B.dbf_tuning_set(B.TUNE_SHARED_MIN_BATCH, 17)
        B.dbf_tuning_set(B.TUNE_WIDE_WG_MAX_ITEMS, max_items)
        layers = [G.pack(L) for L in Ls]
        stack = B.dbf_stack_create(layers)
        outs = []
        try:
            for rep in range(2):
                for L, X, layer in zip(Ls, Xs, layers):
                    y = torch.full((batch, L.n_out), float("nan"), dtype=torch.float16, device="cuda")
                    B.dbf_gemv(layer, G.f16_to_dev(X).data_ptr(), y.data_ptr(), batch, G.stream_handle())
                    torch.cuda.synchronize()
                    outs.append(y.cpu().view(torch.int16).numpy().copy())
                x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
                y_all = torch.full((sum(batch * L.n_out for L in Ls),), float("nan"), dtype=torch.float16, device="cuda")
                for kind in (B.GEMV_AUTO, B.GEMV_MFMA):
                    B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), kind)
                    torch.cuda.synchronize()
                    outs.append(y_all.cpu().view(torch.int16).numpy().copy())
            assert B.dbf_stack_sync_timeouts(stack) == 0
        finally:
            stack.close()
            for l in layers:
                l.close()
            B.dbf_tuning_reset()
        return outs

    G.say("workgroup width: four wavefronts")
    four = run(0)
    G.say("workgroup width: eight wavefronts")
    eight = run(1 << 20)
    assert len(four) == len(eight)
    for i, (a, b) in enumerate(zip(four, eight)):
        assert np.array_equal(a, b), i
    for L, X, y_bits in zip(Ls, Xs, eight[:3]):
        G.check(O.f16_bits_to_f64(y_bits.view(np.uint16)).reshape(batch, L.n_out), O.forward_from_packed(X, L, "staged"),
                "eight wavefronts %dx%d" % (L.n_out, L.n_in))


def test_fp4_sign_operands_equal_the_int8_form_bit_for_bit():
    """Batch-1 launches of few items over stage inputs of 2048-4096 columns feed the matrix cores fp4 sign operands
    and the stage input as four signed hexadecimal digits in bf6; the sums are integers below 2^24 in fp32, so the
    result must be the int8 form's bit for bit: a layer alone, stacks in one launch and in two, launches larger than
    the rule would give this form (by the knob), repeated calls, and an x that cannot be read in 16-byte pieces
    (which takes the int8 form whatever the knob says)."""
    shapes = [(4096, 600, 2100), (2304, 520, 4096), (4096, 300, 2056), (2048, 1000, 3000)]
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 1300 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    Xs = [I.make_activations(1, L.n_in, I.seed_for(5, 1310 + i)) for i, L in enumerate(Ls)]
    # an outlier and exact zeros in one input: digits at both ends of their range
    Xs[0] = Xs[0].copy()
    Xs[0][0, 5] = np.array([60000.0], np.float16).view(np.uint16)[0]
    Xs[0][0, 100:200] = 0

    def run(max_items):
        B.dbf_tuning_reset()
        B.dbf_tuning_set(B.TUNE_FP4_MAX_ITEMS, max_items)
        layers = [G.pack(L) for L in Ls]
        stack = B.dbf_stack_create(layers)
        outs = []
        try:
            for rep in range(2):
                for L, X, layer in zip(Ls, Xs, layers):
                    y = torch.full((1, L.n_out), float("nan"), dtype=torch.float16, device="cuda")
                    B.dbf_gemv(layer, G.f16_to_dev(X).data_ptr(), y.data_ptr(), 1, G.stream_handle())
                    torch.cuda.synchronize()
                    outs.append(y.cpu().view(torch.int16).numpy().copy())
                x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
                y_all = torch.full((sum(L.n_out for L in Ls),), float("nan"), dtype=torch.float16, device="cuda")
                for kind in (B.GEMV_AUTO, B.GEMV_MFMA, B.GEMV_MFMA_SPLIT):
                    B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), 1, G.stream_handle(), kind)
                    torch.cuda.synchronize()
                    outs.append(y_all.cpu().view(torch.int16).numpy().copy())
            # x two bytes off a 16-byte boundary
            L, X, layer = Ls[0], Xs[0], layers[0]
            buf = torch.zeros(L.n_in + 8, dtype=torch.float16, device="cuda")
            buf[1:1 + L.n_in] = G.f16_to_dev(X).reshape(-1)
            y = torch.full((1, L.n_out), float("nan"), dtype=torch.float16, device="cuda")
            B.dbf_gemv(layer, buf.data_ptr() + 2, y.data_ptr(), 1, G.stream_handle())
            torch.cuda.synchronize()
            outs.append(y.cpu().view(torch.int16).numpy().copy())
            assert B.dbf_stack_sync_timeouts(stack) == 0
        finally:
            stack.close()
            for l in layers:
                l.close()
            B.dbf_tuning_reset()
        return outs

    G.say("sign operands: int8")
    int8 = run(0)
    G.say("sign operands: fp4, every eligible launch")
    fp4 = run(1 << 20)
    assert len(int8) == len(fp4)
    for i, (a, b) in enumerate(zip(int8, fp4)):
        assert np.array_equal(a, b), i
    assert np.array_equal(fp4[-1], fp4[0])  # the misaligned call gives what the aligned one gave
    for L, X, y_bits in zip(Ls, Xs, fp4[:4]):
        G.check(O.f16_bits_to_f64(y_bits.view(np.uint16)).reshape(1, L.n_out), O.forward_from_packed(X, L, "staged"),
                "fp4 operands %dx%d" % (L.n_out, L.n_in))


@pytest.mark.parametrize("batch", [1, 3])
def test_groups_of_layers_sharing_one_input(batch):
    """q, k, v read one activation vector, gate and up another: a grouped stack takes one x block
    per group.  Every layer's output must equal, bit for bit, its own dbf_gemv on that block, and
    the oracle's within the gate; the reported offsets follow the groups."""
    shapes = [(512, 512, 256), (512, 128, 200), (512, 128, 130),      # q, k, v
              (384, 1000, 300), (384, 1000, 310),                      # gate, up
              (1000, 384, 300)]                                        # down, alone
    groups = [3, 2, 1]
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 990 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    group_x = [I.make_activations(batch, n_in, I.seed_for(5, 996 + g)) for g, n_in in enumerate((512, 384, 1000))]
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create_grouped(layers, groups)
    try:
        owner = [0, 0, 0, 1, 1, 2]
        x_starts = [0, batch * 512, batch * (512 + 384)]
        yo = 0
        for i, L in enumerate(Ls):
            assert B.dbf_stack_offsets(stack, i, batch) == (x_starts[owner[i]], yo)
            yo += batch * L.n_out
        assert B.dbf_stack_offsets(stack, len(Ls), batch) == (batch * (512 + 384 + 1000), yo)
        x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in group_x])
        for kind, name in ((B.GEMV_AUTO, "auto"), (B.GEMV_MFMA_SPLIT, "mfma_split"), (B.GEMV_VALU, "valu")):
            G.say("grouped stack [%s] batch %d" % (name, batch))
            y_all = torch.full((yo,), float("nan"), dtype=torch.float16, device="cuda")
            B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), kind)
            torch.cuda.synchronize()
            got_all = y_all.cpu().view(torch.int16).numpy().view(np.uint16)
            at = 0
            for i, (L, layer) in enumerate(zip(Ls, layers)):
                got = got_all[at:at + batch * L.n_out]
                at += batch * L.n_out
                X = group_x[owner[i]]
                y1 = torch.full((batch, L.n_out), float("nan"), dtype=torch.float16, device="cuda")
                B.dbf_gemv(layer, G.f16_to_dev(X).data_ptr(), y1.data_ptr(), batch, G.stream_handle(), kind)
                torch.cuda.synchronize()
                assert np.array_equal(got, y1.cpu().view(torch.int16).numpy().view(np.uint16).reshape(-1)), (name, i)
                G.check(O.f16_bits_to_f64(got).reshape(batch, L.n_out), O.forward_from_packed(X, L, "dense"),
                        "grouped[%s] layer %d" % (name, i))
        assert B.dbf_stack_sync_timeouts(stack) == 0
        # groups must be consistent
        with pytest.raises(B.DbfError):
            B.dbf_stack_create_grouped(layers, [2, 4])        # q and gate do not share n_in
        with pytest.raises(B.DbfError):
            B.dbf_stack_create_grouped(layers, [3, 2])        # sizes do not cover the layers
        with pytest.raises(B.DbfError):
            B.dbf_stack_create_grouped(layers, [3, 0, 3])
    finally:
        stack.close()
        for l in layers:
            l.close()


# ---- batches of 2 and more: input quantised once per call ---------------------------------------


@pytest.mark.parametrize("mode", [1, 2, 3])
@pytest.mark.parametrize("shape,batch", [((700, 260, 390), 2), ((700, 260, 390), 7), ((1000, 50, 130), 3),
                                         ((3000, 200, 1500), 16), ((101, 77, 33), 9), ((4096, 512, 700), 4)])
def test_shared_quantised_input_equals_the_items_own_bit_for_bit(mode, shape, batch):
    """DBF_GEMV_AUTO at batch >= 2 quantises each stage input once per call and lets the items copy it into LDS
    (mode 1, here also with rows that need several LDS chunks) or read it from memory tile by tile (mode 2; mode 3:
    a row tile per wavefront -- here, with one row tile per work item, three of the four wavefronts idle).
    The quantiser uses the arithmetic of the items' own prologue and the integer sums are exact, so the result
    must equal, bit for bit, the kind in which every item quantises for itself (checked against the oracle
    here too).  Shapes with columns that are no multiple of 8 take the scalar input path."""
    n_in, n_out, k = shape
    seed = I.seed_for(1, 70 + batch)
    L = I.make_layer(n_in, n_out, k, seed)
    X = I.make_activations(batch, n_in, seed)
    ref = O.forward_from_packed(X, L, "dense")
    layer = G.pack(L)
    try:
        what = "shared-q mode %d n_in=%d n_out=%d k=%d batch=%d" % (mode, n_in, n_out, k, batch)
        G.say("start " + what)
        own = G.run_gemv(layer, X, B.GEMV_MFMA_SPLIT)
        B.dbf_tuning_set(B.TUNE_SHARED_Q, mode)
        B.dbf_tuning_set(B.TUNE_COL_PIECES, 0)      # (batch 2 would otherwise take the column-piece list)
        l2 = G.pack(L)                               # the piece list is decided when the plan is built
        try:
            shared = G.run_gemv(l2, X, B.GEMV_AUTO)
            again = G.run_gemv(l2, X, B.GEMV_AUTO)   # the per-layer buffers are reused from call to call
        finally:
            l2.close()
        G.check(shared, ref, what)
        assert np.array_equal(shared, own), what
        assert np.array_equal(again, own), what + " (second call)"
    finally:
        layer.close()


@pytest.mark.parametrize("span", [4, 5, 16])
@pytest.mark.parametrize("batch", [2, 7, 16])
def test_a_row_tile_per_wavefront_equals_per_layer_calls(batch, span):
    """Work items of `span` row tiles whose wavefronts take a row tile each (groups of four; the last group of an
    item, and of a layer, may be short) and read the quantised input from memory: bit for bit the per-layer
    two-launch result, on layers with 1 to 17 row tiles per stage and ragged columns."""
    shapes = [(520, 1030, 2100), (1000, 130, 77), (4100, 1300, 600), (96, 2176, 640)]
    Ls = [I.make_layer(n_in, n_out, k, I.seed_for(1, 190 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    plain = [G.pack(L) for L in Ls]
    B.dbf_tuning_set(B.TUNE_STACK_SPAN_B, span)
    B.dbf_tuning_set(B.TUNE_STACK_SPAN_A, span)
    B.dbf_tuning_set(B.TUNE_SHARED_Q, 3)
    B.dbf_tuning_set(B.TUNE_COL_PIECES, 0)
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        G.say("start rows-per-wavefront stack batch=%d span=%d" % (batch, span))
        Xs = [I.make_activations(batch, L.n_in, 400 + i) for i, L in enumerate(Ls)]
        x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
        for rep in range(2):   # (the second call finds the reduction buffers and counters as the first left them)
            y_all = torch.full((sum(batch * L.n_out for L in Ls),), float("nan"), dtype=torch.float16, device="cuda")
            B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), B.GEMV_AUTO)
            torch.cuda.synchronize()
            got = G.dev_to_f64(y_all)
            at = 0
            for L, layer, X in zip(Ls, plain, Xs):
                B.dbf_tuning_reset()
                want = G.run_gemv(layer, X, B.GEMV_MFMA_SPLIT)
                B.dbf_tuning_set(B.TUNE_SHARED_Q, 3)
                n = batch * L.n_out
                assert np.array_equal(got[at:at + n].reshape(batch, L.n_out), want), (L.n_in, L.n_out, L.k, rep)
                at += n
    finally:
        stack.close()
        for layer in layers + plain:
            layer.close()


@pytest.mark.parametrize("batch", [4, 16])
def test_stack_at_larger_batches_equals_per_layer_calls(batch):
    """A stack call at batch 4 and 16 (one quantiser launch per stage for all layers) against per-layer calls of
    the kind in which every item quantises for itself."""
    shapes = [(512, 384, 200), (1000, 130, 77), (512, 512, 256), (4096, 256, 300)]
    Ls = [I.make_layer(n_in, n_out, k, I.seed_for(1, 90 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        G.say("start stack batch=%d" % batch)
        Xs = [I.make_activations(batch, L.n_in, 300 + i) for i, L in enumerate(Ls)]
        x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
        y_all = torch.full((sum(batch * L.n_out for L in Ls),), float("nan"), dtype=torch.float16, device="cuda")
        B.dbf_stack_gemv(stack, x_all.data_ptr(), y_all.data_ptr(), batch, G.stream_handle(), B.GEMV_AUTO)
        torch.cuda.synchronize()
        got = G.dev_to_f64(y_all)
        at = 0
        for L, layer, X in zip(Ls, layers, Xs):
            want = G.run_gemv(layer, X, B.GEMV_MFMA_SPLIT)
            n = batch * L.n_out
            assert np.array_equal(got[at:at + n].reshape(batch, L.n_out), want), (L.n_in, L.n_out, L.k)
            at += n
    finally:
        stack.close()
        for layer in layers:
            layer.close()


@pytest.mark.parametrize("forced", [False, True])
def test_long_rows_plans_quantise_once_per_call_at_every_batch(forced):
    """A stack most of whose sign bytes are in layers with long stage inputs (one above 6144 values, the other above
    4096) quantises every stage input once per call at batch 1 and 2 as well (DBF_GEMV_AUTO; `forced`: the knob
    instead of the rule, on a stack the rule would leave alone).  The quantiser uses the arithmetic of the items'
    own prologue and the sums are exact integers, so every batch must give, bit for bit, the two-launch kind's
    result on a plan built without the rule; batch 1 is also checked against the oracle."""
    shapes = [(6400, 200, 4160), (4160, 130, 6272), (512, 512, 256)] if not forced else [(700, 260, 390), (1000, 50, 130)]
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 1700 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    B.dbf_tuning_set(B.TUNE_LONG_ROWS, 0)
    plain_layers = [G.pack(L) for L in Ls]
    plain = B.dbf_stack_create(plain_layers)
    B.dbf_tuning_set(B.TUNE_LONG_ROWS, 1 if forced else -1)
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        for batch in (1, 2, 1, 5, 16, 1):
            Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 1800 + 10 * batch + i)) for i, L in enumerate(Ls)]
            x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
            n_y = batch * sum(L.n_out for L in Ls)
            outs = []
            for st, kind in ((plain, B.GEMV_MFMA_SPLIT), (stack, B.GEMV_AUTO)):
                G.say("long rows forced=%s batch %d kind %d" % (forced, batch, kind))
                y = torch.full((n_y,), float("nan"), dtype=torch.float16, device="cuda")
                B.dbf_stack_gemv(st, x_all.data_ptr(), y.data_ptr(), batch, G.stream_handle(), kind)
                torch.cuda.synchronize()
                outs.append(y)
            assert np.array_equal(outs[0].cpu().view(torch.int16).numpy(), outs[1].cpu().view(torch.int16).numpy()), batch
            if batch == 1:
                got = G.dev_to_f64(outs[1])
                at = 0
                for L, X in zip(Ls, Xs):
                    ref = O.forward_from_packed(X, L, "dense")
                    G.check(got[at:at + L.n_out].reshape(1, L.n_out), ref, "long rows n_in=%d k=%d" % (L.n_in, L.k))
                    at += L.n_out
        assert B.dbf_stack_sync_timeouts(stack) == 0
    finally:
        stack.close()
        plain.close()
        for l in layers + plain_layers:
            l.close()


# ---- the bounded wait of the one-launch kernel ----------------------------------------------------


@pytest.mark.parametrize("batch,pieces", [(1, 0), (1, 3), (2, 0)])
def test_a_wait_that_gives_up_is_visible_in_y_and_leaves_the_counters_consistent(batch, pieces):
    """The give-up path of the device-side waits, driven from the host: with the bound set to zero a workgroup
    whose producer is not finished at its first look gives up at once.  Every kernel still exits normally.
    Required: every fp16 output is either the correct value (bit for bit that of the two-launch kind) or a
    quiet NaN, whole row tiles at a time; the sticky counter says how many workgroups gave up; and the NEXT call
    with the normal bound is fully correct, i.e. the counters were left consistent."""
    shapes = [(8192, 1024, 1024)] * 6      # a long B stage (8 x 1 MiB per layer), many A-stage workgroups
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 1200 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 1300 + i)) for i, L in enumerate(Ls)]
    if pieces:
        B.dbf_tuning_set(B.TUNE_COL_PIECES, pieces)
        B.dbf_tuning_set(B.TUNE_FUSED_MIN_B_ITEMS, 0)   # (only the default kind takes the piece list: make it take one launch)
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
        n_y = batch * sum(L.n_out for L in Ls)

        def call(kind):
            y = torch.full((n_y,), 1.0, dtype=torch.float16, device="cuda")
            B.dbf_stack_gemv(stack, x_all.data_ptr(), y.data_ptr(), batch, G.stream_handle(), kind)
            torch.cuda.synchronize()
            return y.cpu().view(torch.int16).numpy().view(np.uint16).copy()

        want = call(B.GEMV_MFMA_SPLIT)
        assert B.dbf_stack_sync_timeouts(stack) == 0
        fused = B.GEMV_AUTO if pieces else B.GEMV_MFMA
        assert np.array_equal(call(fused), want)                       # the path under test, normal bound
        B.dbf_tuning_set(B.TUNE_WAIT_LIMIT_US, 0)
        G.say("one launch with a zero wait bound, batch %d pieces %d" % (batch, pieces))
        got = call(fused)
        gave_up = B.dbf_stack_sync_timeouts(stack)
        flagged = (got & 0x7C00) == 0x7C00                              # exponent all ones: infinity or NaN
        G.say("  %d workgroups gave up, %d of %d outputs are flagged" % (gave_up, int(flagged.sum()), got.size))
        assert np.array_equal(got[~flagged], want[~flagged])
        assert (gave_up > 0) == bool(flagged.any())
        assert np.all(got[flagged] == 0x7E00)
        # NaNs come in whole row tiles of 128 outputs per batch row
        per_tile = flagged.reshape(len(Ls), batch, -1, 128)
        assert np.all(per_tile.all(axis=3) | ~per_tile.any(axis=3))
        assert gave_up > 0, "every producer had finished before any consumer looked: enlarge the B stage"
        B.dbf_tuning_set(B.TUNE_WAIT_LIMIT_US, 250000)
        for rep in range(2):
            assert np.array_equal(call(fused), want), rep
        assert B.dbf_stack_sync_timeouts(stack) == gave_up     # sticky, and nothing new
    finally:
        stack.close()
        for l in layers:
            l.close()


def test_one_launch_calls_may_switch_between_the_lists_of_a_plan():
    """The device-side counters of a plan count row tiles, not work items, so consecutive one-launch calls may use
    different cuts of the same layers (several row tiles per workgroup at batch 1, one at batch 16, column
    pieces under DBF_GEMV_AUTO) in any order; every call must equal the two-launch
    kind bit for bit."""
    shapes = [(700, 1030, 520), (4100, 300, 260), (512, 512, 256)]
    Ls = [I.make_layer(n_in, n_out, k, seed=I.seed_for(5, 1400 + i)) for i, (n_in, n_out, k) in enumerate(shapes)]
    B.dbf_tuning_set(B.TUNE_STACK_SPAN_B, 3)
    B.dbf_tuning_set(B.TUNE_STACK_SPAN_A, 2)
    B.dbf_tuning_set(B.TUNE_FUSED_MIN_B_ITEMS, 0)     # (the default kind, too, in one launch: a stack this short would take two)
    layers = [G.pack(L) for L in Ls]
    stack = B.dbf_stack_create(layers)
    try:
        want = {}
        sequence = [(1, B.GEMV_MFMA), (16, B.GEMV_MFMA), (1, B.GEMV_AUTO), (2, B.GEMV_MFMA), (3, B.GEMV_AUTO),
                    (16, B.GEMV_MFMA), (1, B.GEMV_MFMA), (4, B.GEMV_AUTO), (9, B.GEMV_MFMA), (1, B.GEMV_AUTO)]
        for step, (batch, kind) in enumerate(sequence):
            Xs = [I.make_activations(batch, L.n_in, I.seed_for(5, 1500 + i)) for i, L in enumerate(Ls)]
            x_all = torch.cat([G.f16_to_dev(X).reshape(-1) for X in Xs])
            n_y = batch * sum(L.n_out for L in Ls)
            outs = []
            for knd in (B.GEMV_MFMA_SPLIT, kind) if batch not in want else (kind,):
                y = torch.full((n_y,), float("nan"), dtype=torch.float16, device="cuda")
                B.dbf_stack_gemv(stack, x_all.data_ptr(), y.data_ptr(), batch, G.stream_handle(), knd)
                torch.cuda.synchronize()
                outs.append(y.cpu().view(torch.int16).numpy().copy())
            if batch not in want:
                want[batch] = outs[0]
            G.say("call %d: batch %d kind %d" % (step, batch, kind))
            assert np.array_equal(outs[-1], want[batch]), (step, batch, kind)
        assert B.dbf_stack_sync_timeouts(stack) == 0
    finally:
        stack.close()
        for l in layers:
            l.close()
