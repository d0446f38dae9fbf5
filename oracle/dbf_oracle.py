"""CPU oracle for the Double Binary Factorization (DBF) layer forward.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP
path is checked against.  Only tests/, __graft_entry__.smoke() and bench.py's
cpu_baseline leg may import it; the product path never does.  It shares no
code with the HIP path and imports nothing from it.

What it computes (paper, section 3, "Double binary factorization"):

    W' = (a . A . m^T)(B . b^T)          -- the factorised weight, n_out x n_in
    Y  = X W'^T                          -- the layer output, batch x n_out

with A (n_out x k) and B (k x n_in) sign matrices, a, m, b vectors.  The
method reaches exactly this dense product (it only re-associates it), so the
oracle is the definition written out in IEEE fp64: decode the signs, form W'
densely, multiply.  `forward_staged` evaluates the paper's forward-pass
expression left to right instead; both must agree to rounding.

Parity pins (tests/test_oracle_pins.py): k=1 rank-one closed form, brute-force
sum of outer products on tiny shapes (exhaustive for <= 2x2x2), all-ones
closed form, pure-Python fsum re-evaluation, invariances of the middle index,
variance law for random signs, packing round trip, the bits-per-weight
numbers the paper prints; the sampled-rows variant against the dense one; pruning of middle
channels against zeroing their scales and against a per-entry loop; the SVID projection
against the singular value decomposition it converges to, exact rank-one inputs and its
fixed point; the ADMM update against the normal equations of its least-squares step, an augmented
least-squares solve by a library routine, its fixed point at an exactly factorisable W and the scalar
closed form; its constant matrices against library solves and the entry-by-entry definition of the fixed
factor.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------------------
# Decoding of the interchange formats
# ---------------------------------------------------------------------------


def f16_bits_to_f64(u16) -> np.ndarray:
    """IEEE binary16 bit patterns (uint16) -> float64, exactly."""
    u16 = np.ascontiguousarray(u16, dtype=np.uint16)
    return u16.view(np.float16).astype(np.float64)


def unpack_signs(words, rows: int, cols: int) -> np.ndarray:
    """Canonical packed words -> float64 matrix of +-1.

    Element c of row r is bit (c mod 32), least significant first, of word
    (c div 32) of that row; a set bit is +1, a clear bit is -1.
    """
    words = np.asarray(words, dtype=np.uint32).reshape(rows, -1)
    need = (cols + 31) // 32
    if words.shape[1] != need:
        raise ValueError("expected %d words per row, got %d" % (need, words.shape[1]))
    # bytes of a little-endian word in memory order are bits 0-7, 8-15, 16-23, 24-31, and within a byte
    # "little" bit order lists the least significant bit first: position c of the unpacked row is bit c mod 32
    # of word c div 32
    as_bytes = np.ascontiguousarray(words.astype("<u4")).view(np.uint8).reshape(rows, 4 * need)
    bits = np.unpackbits(as_bytes, axis=1, bitorder="little")[:, :cols]
    return np.where(bits == 1, 1.0, -1.0)


def pack_signs(S) -> np.ndarray:
    """Matrix of +-1 -> canonical packed words (inverse of unpack_signs)."""
    S = np.asarray(S)
    if S.ndim != 2:
        raise ValueError("sign matrix must be 2-D")
    if not np.all((S == 1) | (S == -1)):
        raise ValueError("entries must be -1 or +1")
    rows, cols = S.shape
    words = np.zeros((rows, (cols + 31) // 32), dtype=np.uint32)
    for c in range(cols):
        plus = (S[:, c] == 1).astype(np.uint32)
        words[:, c // 32] |= plus << np.uint32(c % 32)
    return words


# ---------------------------------------------------------------------------
# The forward product
# ---------------------------------------------------------------------------


def dense_weight(a, A, m, B, b) -> np.ndarray:
    """W' = diag(a) A diag(m) B diag(b) in fp64 (section 3, factorisation)."""
    a = np.asarray(a, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    n_out, k = A.shape
    k2, n_in = B.shape
    if k != k2 or a.shape != (n_out,) or m.shape != (k,) or b.shape != (n_in,):
        raise ValueError("shape mismatch")
    left = a[:, None] * A * m[None, :]      # a . A . m^T
    right = B * b[None, :]                  # B . b^T
    return left @ right


def forward_dense(X, a, A, m, B, b) -> np.ndarray:
    """Y = X W'^T with W' formed densely (section 3, forward pass)."""
    X = np.asarray(X, dtype=np.float64)
    W = dense_weight(a, A, m, B, b)
    return X @ W.T


def forward_staged(X, a, A, m, B, b) -> np.ndarray:
    """((((X . b^T) B^T) . m^T) A^T) . a^T, left to right, fp64."""
    X = np.asarray(X, dtype=np.float64)
    a = np.asarray(a, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    B = np.asarray(B, dtype=np.float64)
    u = X * b[None, :]
    t = u @ B.T
    t = t * m[None, :]
    v = t @ A.T
    return v * a[None, :]


def forward_from_packed(X_f16_bits, layer, mode: str = "dense") -> np.ndarray:
    """Decode a packed layer (canonical words + fp16 bit patterns) and run it.

    `layer` needs attributes n_in, n_out, k, A_bits, B_bits, a, m, b.
    X_f16_bits is (batch, n_in) uint16.  Returns float64 (batch, n_out).
    """
    A = unpack_signs(layer.A_bits, layer.n_out, layer.k)
    B = unpack_signs(layer.B_bits, layer.k, layer.n_in)
    a = f16_bits_to_f64(layer.a)
    m = f16_bits_to_f64(layer.m)
    b = f16_bits_to_f64(layer.b)
    X = f16_bits_to_f64(X_f16_bits).reshape(-1, layer.n_in)
    if mode == "dense":
        return forward_dense(X, a, A, m, B, b)
    if mode == "staged":
        return forward_staged(X, a, A, m, B, b)
    raise ValueError("mode must be 'dense' or 'staged'")


def forward_rows_from_packed(X_f16_bits, layer, rows) -> np.ndarray:
    """Selected output columns Y[:, rows] of a packed layer, staged order, fp64.

    For full-size layers where decoding all of A is the slow part: the middle
    activations need every row of B, but output i only needs row i of A
    (section 3, forward pass: y_i = a_i * sum_j A[i,j] m_j t_j).
    Returns float64 (batch, len(rows)).
    """
    rows = np.asarray(rows, dtype=np.int64)
    if rows.ndim != 1 or np.any(rows < 0) or np.any(rows >= layer.n_out):
        raise ValueError("rows must be a 1-D list of output indices")
    words_A = np.asarray(layer.A_bits, dtype=np.uint32).reshape(layer.n_out, -1)
    A_sel = unpack_signs(words_A[rows], len(rows), layer.k)
    B = unpack_signs(layer.B_bits, layer.k, layer.n_in)
    a = f16_bits_to_f64(layer.a)[rows]
    m = f16_bits_to_f64(layer.m)
    b = f16_bits_to_f64(layer.b)
    X = f16_bits_to_f64(X_f16_bits).reshape(-1, layer.n_in)
    return forward_staged(X, a, A_sel, m, B, b)


# ---------------------------------------------------------------------------
# Middle-channel pruning (section 3.5, "Nonuniform layer compression ratios")
# ---------------------------------------------------------------------------


def prune_middle(A_words, B_words, m_f16_bits, n_out: int, k: int, n_in: int, keep):
    """Keeps the middle channels listed in `keep` (strictly increasing indices < k), in order.

    The paper treats the middle dimension as channels and keeps those with the highest scores
    (section 3.5); how the scores are obtained needs gradients and is not part of this.  The
    structural step written out: decode the signs, take columns `keep` of A, rows `keep` of B and
    entries `keep` of m, encode again.  Returns (A_words', B_words', m_bits', k').
    """
    keep = np.asarray(keep, dtype=np.int64)
    if keep.ndim != 1 or keep.size < 1 or np.any(keep < 0) or np.any(keep >= k) or np.any(np.diff(keep) <= 0):
        raise ValueError("keep must be a non-empty strictly increasing list of middle indices")
    A = unpack_signs(A_words, n_out, k)
    B = unpack_signs(B_words, k, n_in)
    m = np.ascontiguousarray(m_f16_bits, dtype=np.uint16).reshape(-1)
    return pack_signs(A[:, keep]), pack_signs(B[keep, :]), m[keep].copy(), int(keep.size)


# ---------------------------------------------------------------------------
# SVID projection (section 3.2, "Computing Double Binary Factorization")
# ---------------------------------------------------------------------------


def svid(Z, iters: int):
    """SVID(Z) = a . Sign(Z) . m^T with a m^T the rank-1 decomposition of |Z| by power iteration.

    The paper's steps, in its order: Z_pm1 = Sign(Z); rank-1 decomposition of |Z| "using power
    iteration"; SVID(Z) = a . Z_pm1 . m^T.  What the paper leaves open, and the reading taken:
      * Sign(0) = +1 (a sign matrix has entries from {-1, +1} only);
      * the iteration starts from the constant unit vector v = 1/sqrt(cols) and runs `iters` rounds of
        u <- |Z| v / ||.||,  v <- |Z|^T u,  sigma <- ||v||,  v <- v / sigma;
      * the singular value goes to the left factor: a = sigma u, m = v (only the product a m^T matters).
    Returns (S, a, m): S float64 matrix of +-1, a (rows,), m (cols,), all fp64.
    """
    Z = np.asarray(Z, dtype=np.float64)
    if Z.ndim != 2 or iters < 1:
        raise ValueError("Z must be a matrix and iters >= 1")
    S = np.where(Z >= 0.0, 1.0, -1.0)
    M = np.abs(Z)
    rows, cols = M.shape
    v = np.full(cols, 1.0 / np.sqrt(cols))
    u = np.zeros(rows)
    sigma = 0.0
    for _ in range(iters):
        u = M @ v
        nu = np.sqrt(np.sum(u * u))
        u = u / nu if nu > 0.0 else u
        v = M.T @ u
        sigma = np.sqrt(np.sum(v * v))
        v = v / sigma if sigma > 0.0 else v
    return S, sigma * u, v


# ---------------------------------------------------------------------------
# One ADMM update (section 3.2, the three-line ADMM update after the SVID definition)
# ---------------------------------------------------------------------------


def admm_step_from(Minv, C, rho: float, S, a, m, U, svid_iters: int):
    """The ADMM update with its two constant matrices already formed:
    Minv = (B^T B + rho I)^-1 and C = B^T W do not change while B and W are fixed, so an implementation
    forms them once per outer iteration and repeats only what is written here.

        A     = a . S . m^T                       (the current iterate, in SVID form)
        W_hat = Minv (C + rho (A - U))            (as printed: the inverse times the right-hand side)
        Z     = W_hat + U
        (S', a', m') = SVID(Z);   A' = a' . S' . m'^T
        U'    = U + W_hat - A'
    Returns (S', a', m', U', W_hat), all fp64.
    """
    Minv = np.asarray(Minv, dtype=np.float64)
    C = np.asarray(C, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    a = np.asarray(a, dtype=np.float64)
    m = np.asarray(m, dtype=np.float64)
    U = np.asarray(U, dtype=np.float64)
    q, r = C.shape
    if Minv.shape != (q, q) or S.shape != (q, r) or U.shape != (q, r) or a.shape != (q,) or m.shape != (r,):
        raise ValueError("shape mismatch")
    A = a[:, None] * S * m[None, :]
    W_hat = Minv @ (C + rho * (A - U))
    S2, a2, m2 = svid(W_hat + U, svid_iters)
    A2 = a2[:, None] * S2 * m2[None, :]
    return S2, a2, m2, U + W_hat - A2, W_hat


def admm_constants(B, W, rho: float):
    """The two matrices of the update that stay constant while B and W are fixed (section 3.2):
    Minv = (B^T B + rho I)^-1 and C = B^T W.  The paper does not say how it solves the system; B^T B + rho I
    is symmetric positive definite, and the textbook route is taken: Cholesky factorisation G = L L^T, then
    G^-1 = L^-T L^-1.  Returns (Minv, C), fp64."""
    B = np.asarray(B, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    if B.ndim != 2 or W.ndim != 2 or B.shape[0] != W.shape[0] or rho <= 0.0:
        raise ValueError("B (p x q), W (p x r), rho > 0")
    q = B.shape[1]
    G = B.T @ B + rho * np.eye(q)
    L = np.linalg.cholesky(G)
    Linv = np.linalg.inv(L)
    return Linv.T @ Linv, B.T @ W


def fixed_factor_dense(S, b, m2) -> np.ndarray:
    """The fixed factor of the least-squares form as a dense matrix: B = diag(b) S^T diag(m2) (p x q) for a sign
    matrix S (q x p) with scale vectors b (p) and m2 (q) -- the transposed right factor m2 . B_pm1 . b^T of the
    paper's alternating minimisation (section 3.2)."""
    S = np.asarray(S, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    m2 = np.asarray(m2, dtype=np.float64)
    if S.ndim != 2 or b.shape != (S.shape[1],) or m2.shape != (S.shape[0],):
        raise ValueError("S (q x p), b (p), m2 (q)")
    return b[:, None] * S.T * m2[None, :]


def admm_step(B, W, rho: float, S, a, m, U, svid_iters: int):
    """One ADMM update as the paper prints it, for the least-squares form min_X ||B X - W|| with X
    constrained to the SVID form:

        W_hat = (B^T B + rho I)^-1 (B^T W + rho (A - U)),  A' = SVID(W_hat + U),  U' = U + W_hat - A'.

    B is (p x q), W (p x r), the iterate A = a . S . m^T and the scaled dual U are (q x r).  (The
    subproblem of the alternating minimisation, min_A ||A B - W||, has this form after transposition.)
    Returns (S', a', m', U', W_hat), all fp64.
    """
    B = np.asarray(B, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    if B.ndim != 2 or W.ndim != 2 or B.shape[0] != W.shape[0] or rho <= 0.0:
        raise ValueError("B (p x q), W (p x r), rho > 0")
    q = B.shape[1]
    G = B.T @ B + rho * np.eye(q)
    return admm_step_from(np.linalg.inv(G), B.T @ W, rho, S, a, m, U, svid_iters)


# ---------------------------------------------------------------------------
# Storage accounting (section 3, "Middle dimension size" / "Storage size")
# ---------------------------------------------------------------------------


def bits_per_weight(n: int, m: int, k: int) -> float:
    """Sign bits stored per original weight: k (n + m) / (n m)."""
    return k * (n + m) / (n * m)


def middle_dim_for_bits(bits: float, n: int, m: int) -> int:
    """k = bits * n m / (n + m), rounded down to an integer."""
    return int(np.floor(bits * n * m / (n + m)))


def scale_vector_bits_per_weight(n: int, m: int, k: int) -> float:
    """Cost of the three fp16 vectors (sizes n, k, m) per original weight."""
    return 16.0 * (n + k + m) / (n * m)


def step_bits_per_weight(n: int, m: int, step: int = 32) -> float:
    """Change in bits/weight when the middle size moves by `step`."""
    return step * (n + m) / (n * m)


# ---------------------------------------------------------------------------
# Error measure used by the parity gate
# ---------------------------------------------------------------------------


def gated_relative_error(y_test, y_ref) -> float:
    """max_i |y_test - y_ref| / max(|y_ref|, rms(y_ref)), per output row.

    A pure element-wise relative error is meaningless where random-sign sums
    cancel to almost zero, so each element is measured against the larger of
    its own magnitude and the row's rms.
    """
    y_test = np.asarray(y_test, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    if y_ref.ndim == 1:
        y_ref = y_ref[None, :]
        y_test = y_test[None, :]
    rms = np.sqrt(np.mean(y_ref * y_ref, axis=1, keepdims=True))
    denom = np.maximum(np.abs(y_ref), rms)
    denom = np.where(denom == 0.0, 1.0, denom)
    return float(np.max(np.abs(y_test - y_ref) / denom)) if y_ref.size else 0.0
