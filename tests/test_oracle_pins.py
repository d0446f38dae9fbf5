"""Pins for the CPU oracle: every check compares oracle/ against something the
paper or the mathematics fixes and that is computed here by other means
(scalar loops with math.fsum, closed forms, printed numbers), never against
the oracle's own matrix expressions.
"""
import itertools
import math

import numpy as np
import pytest

from oracle import dbf_oracle as O
from paper_2505_11076_amd import inputs as I
from conftest import read_golden


def _rand_layer(rng, n_out, n_in, k):
    A = rng.integers(0, 2, size=(n_out, k)) * 2 - 1
    B = rng.integers(0, 2, size=(k, n_in)) * 2 - 1
    a = rng.uniform(-2, 2, size=n_out)
    m = rng.uniform(-2, 2, size=k)
    b = rng.uniform(-2, 2, size=n_in)
    return a, A, m, B, b


def _brute_weight(a, A, m, B, b):
    """W'[i,l] = a_i b_l sum_j m_j A[i,j] B[j,l] by scalar loops (section 3)."""
    n_out, k = A.shape
    n_in = B.shape[1]
    W = [[0.0] * n_in for _ in range(n_out)]
    for i in range(n_out):
        for l in range(n_in):
            s = math.fsum(float(m[j]) * float(A[i, j]) * float(B[j, l]) for j in range(k))
            W[i][l] = float(a[i]) * float(b[l]) * s
    return W


def _brute_forward(X, W):
    """Y[t,i] = sum_l X[t,l] W[i,l]  (Y = X W^T) by scalar loops."""
    T = len(X)
    n_out = len(W)
    n_in = len(W[0])
    return [[math.fsum(float(X[t][l]) * W[i][l] for l in range(n_in)) for i in range(n_out)]
            for t in range(T)]


# --- the dense product itself --------------------------------------------------------------


@pytest.mark.parametrize("shape", [(3, 5, 4), (8, 8, 8), (7, 2, 5), (1, 6, 3), (5, 1, 2)])
def test_dense_weight_matches_sum_of_outer_products(shape):
    n_out, n_in, k = shape
    rng = np.random.default_rng(11 + n_out * 100 + n_in * 10 + k)
    a, A, m, B, b = _rand_layer(rng, n_out, n_in, k)
    W = np.array(_brute_weight(a, A, m, B, b))
    got = O.dense_weight(a, A, m, B, b)
    assert got.shape == (n_out, n_in)            # catches a transposed result
    np.testing.assert_allclose(got, W, rtol=1e-13, atol=1e-14)


def test_dense_weight_exhaustive_2x2x2():
    """All 256 sign patterns of a 2x2x2 factorisation against scalar loops."""
    a = np.array([0.75, -1.25])
    m = np.array([1.5, 0.3])
    b = np.array([-0.4, 2.0])
    for bits in itertools.product([-1, 1], repeat=8):
        A = np.array(bits[:4]).reshape(2, 2)
        B = np.array(bits[4:]).reshape(2, 2)
        W = np.array(_brute_weight(a, A, m, B, b))
        np.testing.assert_allclose(O.dense_weight(a, A, m, B, b), W, rtol=1e-14, atol=1e-15)


@pytest.mark.parametrize("shape", [(4, 6, 3, 2), (8, 8, 8, 3), (2, 9, 5, 1)])
def test_forward_matches_scalar_loops(shape):
    n_out, n_in, k, T = shape
    rng = np.random.default_rng(23 + sum(shape))
    a, A, m, B, b = _rand_layer(rng, n_out, n_in, k)
    X = rng.standard_normal((T, n_in))
    ref = np.array(_brute_forward(X.tolist(), _brute_weight(a, A, m, B, b)))
    for fn in (O.forward_dense, O.forward_staged):
        got = fn(X, a, A, m, B, b)
        assert got.shape == (T, n_out)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_rank_one_closed_form():
    """k = 1: Y[t,i] = a_i A[i,0] m_0 sum_l B[0,l] b_l X[t,l]."""
    rng = np.random.default_rng(5)
    n_out, n_in, T = 9, 13, 3
    a, A, m, B, b = _rand_layer(rng, n_out, n_in, 1)
    X = rng.standard_normal((T, n_in))
    for t in range(T):
        inner = math.fsum(float(B[0, l]) * b[l] * X[t, l] for l in range(n_in))
        for i in range(n_out):
            want = a[i] * A[i, 0] * m[0] * inner
            for fn in (O.forward_dense, O.forward_staged):
                got = fn(X, a, A, m, B, b)[t, i]
                assert abs(got - want) <= 1e-13 * max(1.0, abs(want))


def test_all_plus_one_closed_form():
    """A = B = +1: Y[t,i] = a_i (sum_j m_j) (b . X[t])."""
    rng = np.random.default_rng(6)
    n_out, n_in, k, T = 6, 10, 7, 2
    a, _, m, _, b = _rand_layer(rng, n_out, n_in, k)
    A = np.ones((n_out, k))
    B = np.ones((k, n_in))
    X = rng.standard_normal((T, n_in))
    msum = math.fsum(m)
    for fn in (O.forward_dense, O.forward_staged):
        Y = fn(X, a, A, m, B, b)
        for t in range(T):
            bx = math.fsum(b[l] * X[t, l] for l in range(n_in))
            for i in range(n_out):
                assert abs(Y[t, i] - a[i] * msum * bx) <= 1e-12 * abs(a[i] * msum * bx) + 1e-14


def test_single_entry_probe_recovers_one_weight():
    """X = e_l picks column l of W': Y[0,i] = a_i b_l sum_j m_j A[i,j] B[j,l].

    Asymmetric shapes and distinct scales make a swapped A/B, a swapped a/b or
    a transposed operand change the answer.
    """
    rng = np.random.default_rng(7)
    n_out, n_in, k = 4, 7, 5
    a, A, m, B, b = _rand_layer(rng, n_out, n_in, k)
    for l in range(n_in):
        X = np.zeros((1, n_in))
        X[0, l] = 1.0
        Y = O.forward_dense(X, a, A, m, B, b)
        for i in range(n_out):
            want = a[i] * b[l] * math.fsum(m[j] * A[i, j] * B[j, l] for j in range(k))
            assert abs(Y[0, i] - want) <= 1e-13 * max(1.0, abs(want))


def test_staged_equals_dense_at_config_sizes():
    """The two groupings of the scales are the same product (section 3)."""
    for cfg, T in ((I.CONFIG1, 8), (I.CONFIG2, 2)):
        L = I.make_layer(seed=I.seed_for(1), **cfg)
        X = I.make_activations(T, cfg["n_in"], I.seed_for(1))
        yd = O.forward_from_packed(X, L, "dense")
        ys = O.forward_from_packed(X, L, "staged")
        scale = np.max(np.abs(yd))
        assert np.max(np.abs(yd - ys)) <= 1e-12 * scale


# --- invariances of the middle index -----------------------------------------------------------


def test_invariances():
    rng = np.random.default_rng(8)
    n_out, n_in, k, T = 6, 9, 5, 3
    a, A, m, B, b = _rand_layer(rng, n_out, n_in, k)
    X = rng.standard_normal((T, n_in))
    Y = O.forward_dense(X, a, A, m, B, b)
    # permuting the middle index
    p = rng.permutation(k)
    np.testing.assert_allclose(O.forward_dense(X, a, A[:, p], m[p], B[p, :], b), Y, rtol=1e-12, atol=1e-13)
    # flipping column j of A together with row j of B
    A2, B2 = A.copy(), B.copy()
    A2[:, 2] *= -1
    B2[2, :] *= -1
    np.testing.assert_allclose(O.forward_dense(X, a, A2, m, B2, b), Y, rtol=1e-12, atol=1e-13)
    # flipping m_j together with column j of A
    A3, m3 = A.copy(), m.copy()
    A3[:, 1] *= -1
    m3[1] *= -1
    np.testing.assert_allclose(O.forward_dense(X, a, A3, m3, B, b), Y, rtol=1e-12, atol=1e-13)
    # flipping only one of them must change the result (the check has teeth)
    assert np.max(np.abs(O.forward_dense(X, a, A3, m, B, b) - Y)) > 1e-6
    # linearity in X
    X2 = rng.standard_normal((T, n_in))
    np.testing.assert_allclose(O.forward_dense(2.5 * X - X2, a, A, m, B, b),
                               2.5 * Y - O.forward_dense(X2, a, A, m, B, b), rtol=1e-11, atol=1e-12)


def test_variance_law_for_random_signs():
    """Var(y_i) = a_i^2 (sum_j m_j^2) (sum_l b_l^2 x_l^2) over i.i.d. fair signs."""
    L = I.make_layer(seed=I.seed_for(2), **I.CONFIG2)
    X = I.make_activations(1, 4096, I.seed_for(2))
    y = O.forward_from_packed(X, L, "staged")[0]
    a = O.f16_bits_to_f64(L.a)
    m = O.f16_bits_to_f64(L.m)
    b = O.f16_bits_to_f64(L.b)
    x = O.f16_bits_to_f64(X[0])
    pred = a * a * np.sum(m * m) * np.sum(b * b * x * x)
    ratio = np.mean(y * y / pred)
    assert 0.9 < ratio < 1.1


# --- interchange formats -----------------------------------------------------------------------------


@pytest.mark.parametrize("cols", [1, 31, 32, 33, 256, 2985, 5970])
def test_packing_round_trip(cols):
    rng = np.random.default_rng(cols)
    rows = 5
    S = I.random_signs(rng, rows, cols)
    words = O.pack_signs(S)
    assert words.dtype == np.uint32 and words.shape == (rows, (cols + 31) // 32)
    back = O.unpack_signs(words, rows, cols)
    assert np.array_equal(back, S.astype(np.float64))
    if cols % 32:
        assert np.all(words[:, -1] >> np.uint32(cols % 32) == 0)


def test_canonical_bit_positions_by_hand():
    """Element c is bit c%32 (LSB first) of word c//32; set bit = +1."""
    S = -np.ones((2, 40), dtype=np.int8)
    S[0, 0] = 1
    S[0, 33] = 1
    S[1, 31] = 1
    w = O.pack_signs(S)
    assert w.tolist() == [[1, 2], [0x80000000, 0]]
    one = O.unpack_signs(np.array([[0x5, 0x0]], dtype=np.uint32), 1, 34)
    assert one[0, :4].tolist() == [1.0, -1.0, 1.0, -1.0] and one[0, 33] == -1.0


def test_generator_words_match_generator_signs_format():
    """Words drawn directly have clean tails and decode to +-1 only."""
    rng = np.random.default_rng(3)
    w = I.random_sign_words(rng, 7, 45)
    assert np.all(w[:, -1] >> np.uint32(13) == 0)
    S = O.unpack_signs(w, 7, 45)
    assert set(np.unique(S).tolist()) <= {-1.0, 1.0}
    assert np.array_equal(O.pack_signs(S.astype(np.int8)), w)


def test_pack_rejects_non_signs():
    with pytest.raises(ValueError):
        O.pack_signs(np.array([[1, 0, -1]]))


def test_f16_decode_exact():
    pats = np.array([0x3C00, 0xBC00, 0x0001, 0x7BFF, 0x2000, 0x0000], dtype=np.uint16)
    want = [1.0, -1.0, 2.0 ** -24, 65504.0, 2.0 ** -7, 0.0]
    assert O.f16_bits_to_f64(pats).tolist() == want


# --- storage accounting against the numbers the paper prints -------------------------------------


def test_storage_numbers_from_the_paper():
    g = read_golden("paper_storage_numbers.txt")
    n = 4096
    assert O.middle_dim_for_bits(1.0, n, n) == int(g["square_1bit_middle_over_n"] * n)
    assert O.middle_dim_for_bits(2.0, n, n) == int(g["square_2bit_middle_over_n"] * n)
    k2 = O.middle_dim_for_bits(2.0, n, n)
    assert round(O.scale_vector_bits_per_weight(n, n, k2), 3) == g["scale_vectors_bpw_4096sq_2bit"]
    for (r, c) in ((4096, 4096), (4096, 11008), (11008, 4096), (4096, 14336), (8192, 8192)):
        assert O.step_bits_per_weight(r, c, 32) <= g["step32_bpw_upper_bound"]


def test_bits_per_weight_formula():
    assert O.bits_per_weight(512, 512, 256) == 1.0
    assert O.bits_per_weight(4096, 4096, 2048) == 1.0
    assert O.bits_per_weight(4096, 4096, 4096) == 2.0
    # 2985 * 15104 = 45 085 440 sign bits over 4096 * 11008 = 45 088 768 weights
    assert abs(O.bits_per_weight(4096, 11008, 2985) - 45085440 / 45088768) < 1e-15
    assert abs(O.bits_per_weight(11008, 4096, 5970) - 90170880 / 45088768) < 1e-15
    assert 0.9999 < O.bits_per_weight(4096, 11008, 2985) < 1.0
    # floor rounding reproduces the middle sizes of the workloads
    assert O.middle_dim_for_bits(1.0, 4096, 11008) == 2985
    assert O.middle_dim_for_bits(2.0, 4096, 11008) == 5970
    assert O.middle_dim_for_bits(1.5, 4096, 4096) == 3072
    assert O.middle_dim_for_bits(1.5, 11008, 4096) == 4477
    # bits actually stored: two sign matrices of n*k and k*m entries
    n, m, k = 24, 40, 7
    assert O.bits_per_weight(n, m, k) == (n * k + k * m) / (n * m)


def test_gated_error_measure():
    y = np.array([[1.0, -2.0, 0.0, 4.0]])
    rms = math.sqrt((1 + 4 + 0 + 16) / 4)
    yt = y + np.array([[0.0, 0.0, 0.01, 0.0]])
    assert abs(O.gated_relative_error(yt, y) - 0.01 / rms) < 1e-15
    yt = y + np.array([[0.0, 0.0, 0.0, 0.04]])
    assert abs(O.gated_relative_error(yt, y) - 0.01) < 1e-15


def test_forward_from_packed_against_hand_decoded_bits():
    """The packed entry point: decode words and fp16 patterns with Python
    integer/struct operations and evaluate by scalar loops."""
    import struct

    def h2f(u):
        return struct.unpack("<e", struct.pack("<H", int(u)))[0]

    L = I.make_layer(n_in=37, n_out=5, k=34, seed=99)
    X = I.make_activations(2, 37, 99)
    A = [[1.0 if (int(L.A_bits[i, j // 32]) >> (j % 32)) & 1 else -1.0 for j in range(34)] for i in range(5)]
    B = [[1.0 if (int(L.B_bits[j, l // 32]) >> (l % 32)) & 1 else -1.0 for l in range(37)] for j in range(34)]
    a = [h2f(v) for v in L.a]
    m = [h2f(v) for v in L.m]
    b = [h2f(v) for v in L.b]
    Xf = [[h2f(v) for v in row] for row in X]
    W = _brute_weight(np.array(a), np.array(A), np.array(m), np.array(B), np.array(b))
    ref = np.array(_brute_forward(Xf, W))
    for mode in ("dense", "staged"):
        got = O.forward_from_packed(X, L, mode)
        np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-18)


def test_sampled_rows_equal_the_dense_product_and_the_brute_force():
    """The sampled-rows entry point (used where decoding all of A at full size is too slow)
    must return exactly the chosen columns of the dense result, in the order asked for,
    repeated and unsorted indices included; a scalar-loop evaluation pins it independently."""
    import struct

    def h2f(u):
        return struct.unpack("<e", struct.pack("<H", int(u)))[0]

    L = I.make_layer(n_in=70, n_out=45, k=33, seed=123)
    X = I.make_activations(3, 70, 124)
    rows = [44, 0, 7, 7, 31, 12]
    got = O.forward_rows_from_packed(X, L, rows)
    full = O.forward_from_packed(X, L, "dense")
    assert got.shape == (3, len(rows))
    np.testing.assert_allclose(got, full[:, rows], rtol=1e-12, atol=1e-18)
    # one entry by hand: y[t, i] = a_i * sum_j A[i,j] m_j * sum_l B[j,l] b_l x[t,l]
    t, i = 2, 31
    acc = []
    for j in range(33):
        Aij = 1.0 if (int(L.A_bits[i, j // 32]) >> (j % 32)) & 1 else -1.0
        inner = math.fsum((1.0 if (int(L.B_bits[j, l // 32]) >> (l % 32)) & 1 else -1.0) * h2f(L.b[l]) * h2f(X[t, l])
                          for l in range(70))
        acc.append(Aij * h2f(L.m[j]) * inner)
    want = h2f(L.a[i]) * math.fsum(acc)
    assert got[t, rows.index(31)] == pytest.approx(want, rel=1e-12)
    with pytest.raises(ValueError):
        O.forward_rows_from_packed(X, L, [45])
    with pytest.raises(ValueError):
        O.forward_rows_from_packed(X, L, [-1])


# ---------------------------------------------------------------------------
# Middle-channel pruning (section 3.5)
# ---------------------------------------------------------------------------


@pytest.mark.parametrize("shape", [(7, 5, 9), (33, 40, 70), (64, 31, 129)])
def test_pruning_equals_zeroing_the_dropped_scales(shape):
    """W' = sum_j m_j A[:,j] B[j,:]: dropping channel j removes exactly the term that m_j = 0
    removes.  The pruned layer's dense weight must equal the original's with those scales zeroed
    (independent of how prune_middle re-encodes anything)."""
    n_in, n_out, k = shape
    L = I.make_layer(n_in, n_out, k, seed=4242 + k)
    rng = np.random.default_rng(99 + k)
    keep = np.sort(rng.choice(k, size=max(1, (2 * k) // 3), replace=False))
    A2, B2, m2, k2 = O.prune_middle(L.A_bits, L.B_bits, L.m, n_out, k, n_in, keep)
    assert k2 == keep.size
    a, m, b = O.f16_bits_to_f64(L.a), O.f16_bits_to_f64(L.m), O.f16_bits_to_f64(L.b)
    m_zeroed = np.zeros_like(m)
    m_zeroed[keep] = m[keep]
    W_ref = O.dense_weight(a, O.unpack_signs(L.A_bits, n_out, k), m_zeroed, O.unpack_signs(L.B_bits, k, n_in), b)
    W_new = O.dense_weight(a, O.unpack_signs(A2, n_out, k2), O.f16_bits_to_f64(m2), O.unpack_signs(B2, k2, n_in), b)
    assert np.max(np.abs(W_new - W_ref)) <= 1e-15 * max(1.0, np.max(np.abs(W_ref))) * k


def test_pruning_moves_every_entry_to_its_new_place():
    """Entry by entry, with the bit positions of the canonical format computed by hand: sign
    (i, j') of the new A is sign (i, keep[j']) of the old one, row j' of the new B is row keep[j']
    of the old B, and the tail bits of the last word of a row are zero."""
    n_in, n_out, k = 37, 29, 70
    L = I.make_layer(n_in, n_out, k, seed=777)
    keep = np.array([0, 3, 4, 31, 32, 33, 63, 64, 69])
    A2, B2, m2, k2 = O.prune_middle(L.A_bits, L.B_bits, L.m, n_out, k, n_in, keep)
    Aw = np.asarray(L.A_bits, dtype=np.uint32).reshape(n_out, -1)
    Bw = np.asarray(L.B_bits, dtype=np.uint32).reshape(k, -1)
    assert A2.shape == (n_out, 1) and B2.shape == (k2, 2) and k2 == 9
    for i in range(n_out):
        for jn, jo in enumerate(keep):
            assert (int(A2[i, jn // 32]) >> (jn % 32)) & 1 == (int(Aw[i, jo // 32]) >> (jo % 32)) & 1
        assert int(A2[i, 0]) >> 9 == 0
    for jn, jo in enumerate(keep):
        assert np.array_equal(B2[jn], Bw[jo])
    assert np.array_equal(m2, np.asarray(L.m, dtype=np.uint16)[keep])


def test_pruning_identity_and_argument_errors():
    n_in, n_out, k = 20, 10, 40
    L = I.make_layer(n_in, n_out, k, seed=31)
    A2, B2, m2, k2 = O.prune_middle(L.A_bits, L.B_bits, L.m, n_out, k, n_in, np.arange(k))
    assert k2 == k and np.array_equal(A2, np.asarray(L.A_bits).reshape(n_out, -1))
    assert np.array_equal(B2, np.asarray(L.B_bits).reshape(k, -1)) and np.array_equal(m2, L.m)
    for bad in ([], [3, 3], [5, 2], [-1, 2], [0, 40]):
        with pytest.raises(ValueError):
            O.prune_middle(L.A_bits, L.B_bits, L.m, n_out, k, n_in, bad)


# ---------------------------------------------------------------------------
# SVID projection (section 3.2)
# ---------------------------------------------------------------------------


def test_svid_converges_to_the_top_singular_triple_of_abs_z():
    """Power iteration on |Z| (all entries positive: a simple, positive top singular pair) must reach
    what a dense SVD gives: sigma_1 u_1 v_1^T, the best rank-one approximation of |Z|."""
    rng = np.random.default_rng(5)
    Z = rng.standard_normal((37, 23))
    S, a, m = O.svid(Z, iters=60)
    U, sv, Vt = np.linalg.svd(np.abs(Z))
    u1, v1 = np.abs(U[:, 0]), np.abs(Vt[0])          # the sign of a singular pair is free; positive here
    assert np.allclose(np.outer(a, m), sv[0] * np.outer(u1, v1), rtol=0, atol=1e-10 * sv[0])
    assert abs(np.linalg.norm(m) - 1.0) < 1e-14 and abs(np.linalg.norm(a) - sv[0]) < 1e-10 * sv[0]
    assert np.array_equal(S, np.where(Z >= 0, 1.0, -1.0))
    # and it is the best rank-one fit: no nearby rank-one matrix is closer to |Z|
    best = np.linalg.norm(np.abs(Z) - np.outer(a, m))
    for _ in range(20):
        a2 = a * (1 + 0.05 * rng.standard_normal(a.shape))
        m2 = m * (1 + 0.05 * rng.standard_normal(m.shape))
        assert np.linalg.norm(np.abs(Z) - np.outer(a2, m2)) >= best


def test_svid_is_exact_on_matrices_of_its_own_form():
    """If Z = p . S . q^T with p, q > 0, then |Z| = p q^T has rank one: one round already gives
    a m^T = p q^T, and SVID(Z) = Z (the projection keeps the members of its set)."""
    rng = np.random.default_rng(6)
    p, q = rng.uniform(0.5, 2.0, 19), rng.uniform(0.5, 2.0, 31)
    S0 = np.where(rng.random((19, 31)) < 0.5, 1.0, -1.0)
    Z = p[:, None] * S0 * q[None, :]
    for iters in (1, 2, 7):
        S, a, m = O.svid(Z, iters)
        assert np.array_equal(S, S0)
        assert np.allclose(np.outer(a, m), np.outer(p, q), rtol=1e-13, atol=0)
        assert np.allclose(a[:, None] * S * m[None, :], Z, rtol=1e-13, atol=0)


def test_svid_first_round_by_hand_and_the_sign_of_zero():
    """One round written out with scalar loops: v0 = 1/sqrt(cols); u = |Z| v0 normalised; v = |Z|^T u;
    sigma = |v|.  Zero entries get the sign +1."""
    Z = np.array([[1.0, -2.0, 0.0], [-3.0, 4.0, -0.0]])
    S, a, m = O.svid(Z, 1)
    assert np.array_equal(S, np.array([[1.0, -1.0, 1.0], [-1.0, 1.0, 1.0]]))
    v0 = 1.0 / math.sqrt(3.0)
    u = [(1.0 + 2.0 + 0.0) * v0, (3.0 + 4.0 + 0.0) * v0]
    nu = math.sqrt(u[0] ** 2 + u[1] ** 2)
    u = [u[0] / nu, u[1] / nu]
    v = [1.0 * u[0] + 3.0 * u[1], 2.0 * u[0] + 4.0 * u[1], 0.0]
    sigma = math.sqrt(sum(x * x for x in v))
    assert np.allclose(a, [sigma * u[0], sigma * u[1]], rtol=1e-15)
    assert np.allclose(m, [x / sigma for x in v], rtol=1e-15)
    with pytest.raises(ValueError):
        O.svid(Z, 0)


# ---------------------------------------------------------------------------
# ADMM update (section 3.2)
# ---------------------------------------------------------------------------


def _admm_case(p, q, r, seed):
    rng = np.random.default_rng(seed)
    B = rng.standard_normal((p, q)) / math.sqrt(p)
    W = rng.standard_normal((p, r))
    S = np.where(rng.random((q, r)) < 0.5, 1.0, -1.0)
    a, m = rng.uniform(0.2, 1.5, q), rng.uniform(0.2, 1.5, r)
    U = 0.3 * rng.standard_normal((q, r))
    return B, W, S, a, m, U


def test_admm_w_hat_satisfies_the_normal_equations_and_minimises_its_objective():
    """W_hat is the minimiser over X of f(X) = 1/2 ||B X - W||^2 + rho/2 ||X - A + U||^2 (the first line of
    the generic ADMM iteration with f the least-squares error and z = A), so the gradient
    B^T (B X - W) + rho (X - A + U) vanishes there and every other X does worse."""
    for (p, q, r, rho) in ((13, 7, 9, 1.0), (6, 11, 5, 0.25), (20, 20, 3, 4.0)):
        B, W, S, a, m, U = _admm_case(p, q, r, 40 + p)
        A = a[:, None] * S * m[None, :]
        W_hat = O.admm_step(B, W, rho, S, a, m, U, 3)[4]
        grad = B.T @ (B @ W_hat - W) + rho * (W_hat - A + U)
        assert np.max(np.abs(grad)) < 1e-11 * (1.0 + np.max(np.abs(W)))
        f = lambda X: 0.5 * np.sum((B @ X - W) ** 2) + 0.5 * rho * np.sum((X - A + U) ** 2)
        rng = np.random.default_rng(p)
        for _ in range(10):
            assert f(W_hat + 1e-3 * rng.standard_normal(W_hat.shape)) > f(W_hat)


def test_admm_w_hat_equals_an_augmented_least_squares_solve():
    """The same minimiser from a library routine that never forms B^T B: stack sqrt(rho) I under B and
    sqrt(rho) (A - U) under W and solve the tall least-squares problem."""
    B, W, S, a, m, U = _admm_case(17, 8, 6, 77)
    rho = 0.7
    A = a[:, None] * S * m[None, :]
    tall = np.vstack([B, math.sqrt(rho) * np.eye(8)])
    rhs = np.vstack([W, math.sqrt(rho) * (A - U)])
    X = np.linalg.lstsq(tall, rhs, rcond=None)[0]
    assert np.allclose(O.admm_step(B, W, rho, S, a, m, U, 2)[4], X, rtol=0, atol=1e-12)


def test_admm_fixed_point_when_w_is_exactly_factorisable():
    """If W = B A* with A* of the SVID form, then A = A*, U = 0 is a fixed point of the update:
    W_hat = (B^T B + rho I)^-1 (B^T B A* + rho A*) = A*, SVID(A*) = A*, U stays 0."""
    B, _, S, a, m, _ = _admm_case(15, 6, 10, 5)
    A_star = a[:, None] * S * m[None, :]
    S2, a2, m2, U2, W_hat = O.admm_step(B, B @ A_star, 1.0, S, a, m, np.zeros((6, 10)), 1)
    assert np.allclose(W_hat, A_star, rtol=0, atol=1e-12)
    assert np.array_equal(S2, S)
    assert np.allclose(np.outer(a2, m2), np.outer(a, m), rtol=1e-11, atol=0)
    assert np.max(np.abs(U2)) < 1e-11


def test_admm_scalar_closed_form_and_the_dual_update():
    """p = q = r = 1: W_hat = (b w + rho (A - u)) / (b^2 + rho); SVID of a scalar z is z itself
    (sign(z) * |z| * 1), so A' = W_hat + u and u' = u + W_hat - A' = 0.  Checked for both signs of z."""
    for (b, w, s, a, m, u, rho) in ((2.0, 3.0, 1.0, 0.5, 1.0, 0.25, 1.0), (1.5, -4.0, -1.0, 2.0, 1.0, -0.5, 2.0)):
        S2, a2, m2, U2, W_hat = O.admm_step([[b]], [[w]], rho, [[s]], [a], [m], [[u]], 2)
        want = (b * w + rho * (s * a * m - u)) / (b * b + rho)
        assert abs(W_hat[0, 0] - want) < 1e-15
        z = want + u
        assert S2[0, 0] == (1.0 if z >= 0 else -1.0)
        assert abs(a2[0] * m2[0] - abs(z)) < 1e-15 and abs(U2[0, 0]) < 1e-15


def test_admm_large_penalty_limit_and_conservation():
    """rho -> infinity pins X to A - U: W_hat -> A - U.  And for any rho the three outputs are tied by
    U' + A' = U + W_hat (the dual update), whatever SVID returns."""
    B, W, S, a, m, U = _admm_case(9, 5, 7, 3)
    A = a[:, None] * S * m[None, :]
    W_hat = O.admm_step(B, W, 1e12, S, a, m, U, 1)[4]
    assert np.allclose(W_hat, A - U, rtol=0, atol=1e-9)
    S2, a2, m2, U2, W_hat = O.admm_step(B, W, 1.0, S, a, m, U, 4)
    assert np.allclose(U2 + a2[:, None] * S2 * m2[None, :], U + W_hat, rtol=0, atol=1e-13)
    S3, a3, m3 = O.svid(W_hat + U, 4)
    assert np.array_equal(S2, S3) and np.array_equal(a2, a3) and np.array_equal(m2, m3)


def test_admm_precomputed_form_matches_and_rejects_bad_shapes():
    B, W, S, a, m, U = _admm_case(12, 6, 8, 11)
    rho = 1.0
    Minv = np.linalg.inv(B.T @ B + rho * np.eye(6))
    full = O.admm_step(B, W, rho, S, a, m, U, 3)
    pre = O.admm_step_from(Minv, B.T @ W, rho, S, a, m, U, 3)
    for x, y in zip(full, pre):
        assert np.array_equal(x, y)
    # the precomputed form applies its first argument from the left as it stands (no transpose): with a
    # non-symmetric matrix in its place, W_hat solves M2^-1 X = rhs, which a library solve checks
    M2 = Minv + np.triu(np.ones((6, 6)), 1) * 0.01
    A = a[:, None] * S * m[None, :]
    rhs = B.T @ W + rho * (A - U)
    W_hat2 = O.admm_step_from(M2, B.T @ W, rho, S, a, m, U, 1)[4]
    assert np.allclose(np.linalg.solve(M2, W_hat2), rhs, rtol=0, atol=1e-11)
    assert not np.allclose(np.linalg.solve(M2.T, W_hat2), rhs, rtol=0, atol=1e-4)
    # and the full update solves (B^T B + rho I) W_hat = rhs
    assert np.allclose(np.linalg.solve(B.T @ B + rho * np.eye(6), rhs), full[4], rtol=0, atol=1e-12)
    with pytest.raises(ValueError):
        O.admm_step_from(Minv[:5], B.T @ W, rho, S, a, m, U, 1)
    with pytest.raises(ValueError):
        O.admm_step(B, W[:5], rho, S, a, m, U, 1)
    with pytest.raises(ValueError):
        O.admm_step(B, W, 0.0, S, a, m, U, 1)


def test_admm_constants_against_library_solves_and_the_fixed_factor_entry_by_entry():
    """Minv from the Cholesky route must be the inverse a general solver finds (and symmetric, and a two-sided
    inverse); C is a plain product; feeding both to the precomputed form gives the full update.  The dense
    fixed factor is checked entry by entry with scalar loops on an asymmetric shape (catches a transposed S, b
    and m2 swapped)."""
    B, W, S, a, m, U = _admm_case(14, 9, 5, 31)
    for rho in (1.0, 0.05, 7.0):
        Minv, C = O.admm_constants(B, W, rho)
        G = B.T @ B + rho * np.eye(9)
        assert np.allclose(Minv, np.linalg.solve(G, np.eye(9)), rtol=0, atol=1e-12 * np.max(np.abs(Minv)) * np.linalg.cond(G))
        assert np.allclose(Minv @ G, np.eye(9), atol=1e-12) and np.allclose(G @ Minv, np.eye(9), atol=1e-12)
        assert np.array_equal(Minv, Minv.T) or np.allclose(Minv, Minv.T, rtol=0, atol=1e-15)
        assert np.allclose(C, np.array([[sum(B[l, j] * W[l, o] for l in range(14)) for o in range(5)] for j in range(9)]),
                           rtol=1e-13, atol=1e-13)
        full = O.admm_step(B, W, rho, S, a, m, U, 2)
        pre = O.admm_step_from(Minv, C, rho, S, a, m, U, 2)
        assert np.array_equal(full[0], pre[0])
        for x, y in zip(full[1:], pre[1:]):
            assert np.allclose(x, y, rtol=0, atol=1e-11)
    rng = np.random.default_rng(8)
    q, p = 4, 7
    Sg = np.where(rng.random((q, p)) < 0.5, 1.0, -1.0)
    b, m2 = rng.uniform(0.5, 2.0, p), rng.uniform(0.5, 2.0, q)
    Bd = O.fixed_factor_dense(Sg, b, m2)
    assert Bd.shape == (p, q)
    for l in range(p):
        for j in range(q):
            assert Bd[l, j] == b[l] * Sg[j, l] * m2[j]
    with pytest.raises(ValueError):
        O.fixed_factor_dense(Sg, m2, b)
    with pytest.raises(ValueError):
        O.admm_constants(B, W[:3], 1.0)


def test_admm_iterations_approach_a_factorisable_target():
    """Behaviour over several updates: with W = B A* (A* of the SVID form) and a start far from A*, repeated
    updates bring the projected iterate A = a . S . m^T closer to a least-squares fit: the residual ||B A - W||
    after 30 updates is a thousandth of the start's (here the iteration recovers an exact fit).  (ADMM on this non-convex set has no guarantee, but a wrong
    sign in the dual update or in the right-hand side makes the residual grow instead; seeds fixed.)"""
    rng = np.random.default_rng(21)
    p, q, r = 40, 12, 16
    B = rng.standard_normal((p, q)) / math.sqrt(p)
    S_star = np.where(rng.random((q, r)) < 0.5, 1.0, -1.0)
    A_star = rng.uniform(0.5, 1.5, q)[:, None] * S_star * rng.uniform(0.5, 1.5, r)[None, :]
    W = B @ A_star
    S = np.where(rng.random((q, r)) < 0.5, 1.0, -1.0)
    a, m, U = np.full(q, 0.1), np.full(r, 0.1), np.zeros((q, r))
    res0 = np.linalg.norm(B @ (a[:, None] * S * m[None, :]) - W)
    for _ in range(30):
        S, a, m, U, _ = O.admm_step(B, W, 1.0, S, a, m, U, 3)
    res = np.linalg.norm(B @ (a[:, None] * S * m[None, :]) - W)
    assert res < 1e-3 * res0, (res0, res)
    # and a corrupted dual update (U - W_hat + A' instead of U + W_hat - A') does not get there
    S2 = np.where(np.random.default_rng(22).random((q, r)) < 0.5, 1.0, -1.0)
    a2, m2, U2 = np.full(q, 0.1), np.full(r, 0.1), np.zeros((q, r))
    for _ in range(30):
        S2n, a2n, m2n, U2n, W_hat = O.admm_step(B, W, 1.0, S2, a2, m2, U2, 3)
        U2 = U2 - W_hat + a2n[:, None] * S2n * m2n[None, :]
        S2, a2, m2 = S2n, a2n, m2n
    res_bad = np.linalg.norm(B @ (a2[:, None] * S2 * m2[None, :]) - W)
    assert res < res_bad
