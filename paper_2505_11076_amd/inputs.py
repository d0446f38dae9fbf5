"""Seeded synthetic inputs for Double Binary Factorization (DBF) layers.

This module only draws random numbers and arranges them in the canonical
interchange formats.  It holds none of the method's arithmetic (no products,
no rescales), so the CPU oracle's tests and the HIP path's tests can both feed
from it without sharing any code that computes a result.

Operands of one layer (paper, section 3, "Double binary factorization" and
"Middle dimension size"): sign matrices A (n_out x k) and B (k x n_in) with
entries in {-1,+1}, fp16 vectors a (n_out), m (k), b (n_in), fp16 input X
(batch x n_in).

Canonical bit format (the paper fixes none; this is the interchange format of
this library): row-major, the reduction dimension runs fastest, element c of a
row is bit (c & 31), LSB first, of 32-bit word (c >> 5); bit 1 means +1, bit 0
means -1; the unused high bits of a row's last word are zero.

Recipe (stands in for the compressed Llama layers the paper times): signs are
i.i.d. +-1 with p = 1/2, the three scale vectors are fp16(0.02 * U[0.5, 1.5)),
activations are fp16(N(0, 1)).  Seed = 1000 * config + index.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


def seed_for(config: int, index: int = 0) -> int:
    return 1000 * int(config) + int(index)


def words_per_row(cols: int) -> int:
    return (int(cols) + 31) // 32


def random_sign_words(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """rows x ceil(cols/32) uint32 words of i.i.d. fair bits, tail bits cleared."""
    w = words_per_row(cols)
    words = rng.integers(0, 1 << 32, size=(rows, w), dtype=np.uint64).astype(np.uint32)
    tail = cols & 31
    if tail:
        words[:, -1] &= np.uint32((1 << tail) - 1)
    return words


def random_signs(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """rows x cols int8 matrix of i.i.d. +-1."""
    return (rng.integers(0, 2, size=(rows, cols), dtype=np.int8) * 2 - 1).astype(np.int8)


def random_scale_fp16(rng: np.random.Generator, n: int) -> np.ndarray:
    """fp16(0.02 * U[0.5, 1.5)) returned as fp16 bit patterns (uint16)."""
    v = (0.02 * rng.uniform(0.5, 1.5, size=n)).astype(np.float16)
    return v.view(np.uint16).copy()


def random_activations_fp16(rng: np.random.Generator, batch: int, n_in: int) -> np.ndarray:
    """fp16(N(0,1)) of shape (batch, n_in) as fp16 bit patterns (uint16)."""
    v = rng.standard_normal(size=(batch, n_in)).astype(np.float16)
    return v.view(np.uint16).copy()


@dataclass
class LayerInputs:
    n_in: int
    n_out: int
    k: int
    A_bits: np.ndarray  # uint32 [n_out, ceil(k/32)]   canonical words
    B_bits: np.ndarray  # uint32 [k, ceil(n_in/32)]    canonical words
    a: np.ndarray       # uint16 [n_out]  fp16 bit patterns
    m: np.ndarray       # uint16 [k]
    b: np.ndarray       # uint16 [n_in]


def make_layer(n_in: int, n_out: int, k: int, seed: int) -> LayerInputs:
    rng = np.random.default_rng(seed)
    A_bits = random_sign_words(rng, n_out, k)
    B_bits = random_sign_words(rng, k, n_in)
    a = random_scale_fp16(rng, n_out)
    m = random_scale_fp16(rng, k)
    b = random_scale_fp16(rng, n_in)
    return LayerInputs(n_in, n_out, k, A_bits, B_bits, a, m, b)


def make_activations(batch: int, n_in: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed + 500)
    return random_activations_fp16(rng, batch, n_in)


# ---------------------------------------------------------------------------
# The five workload families (shapes only; sizes follow Llama-2-7B).
# ---------------------------------------------------------------------------

CONFIG1 = dict(n_in=512, n_out=512, k=256)                       # ~1 bit/weight, smoke size
CONFIG2 = dict(n_in=4096, n_out=4096, k=2048)                    # attention projection, 1.0 bpw
CONFIG3 = [                                                      # MLP shapes, ~1 and ~2 bpw
    dict(n_in=4096, n_out=11008, k=2985),
    dict(n_in=4096, n_out=11008, k=5970),
    dict(n_in=11008, n_out=4096, k=2985),
    dict(n_in=11008, n_out=4096, k=5970),
]
CONFIG4 = [                                                      # prefill shapes, T = 2048
    dict(n_in=4096, n_out=4096, k=4096, T=2048),
    dict(n_in=11008, n_out=4096, k=5970, T=2048),
]


def make_svid_matrix(rows: int, cols: int, seed: int) -> np.ndarray:
    """Input of the SVID projection: an unconstrained fp32 matrix as the ADMM iteration produces them
    (sum of a least-squares solution and a dual variable): i.i.d. N(0, 1), with a sprinkling of exact
    +0.0 and -0.0 entries so that the sign of zero is exercised."""
    rng = np.random.default_rng(seed + 700)
    Z = rng.standard_normal((rows, cols)).astype(np.float32)
    n_zero = max(2, (rows * cols) // 997)
    idx = rng.choice(rows * cols, size=n_zero, replace=False)
    flat = Z.reshape(-1)
    flat[idx[: n_zero // 2]] = 0.0
    flat[idx[n_zero // 2:]] = -0.0
    return Z


# Second workload: the layer sizes of the paper's matrix-vector timing table (Table 4: Llama-3
# shapes, printed as rows x columns of W = n_out x n_in) plus the grouped-query k/v projection
# 4096 -> 1024, each at the table's four sizes in bits per weight.  The middle sizes are written out
# (they follow the storage formula of section 3, "Middle dimension size"; a CPU test checks them
# against the oracle's statement of it -- this module holds none of the method's arithmetic).
TABLE4_SHAPES = [                                                # (n_out, n_in)
    (4096, 4096), (4096, 14336), (8192, 8192), (8192, 28672), (1024, 4096),
]
TABLE4_BITS = [1.0, 1.5, 2.0, 2.3]
TABLE4_K = {                                                     # (n_out, n_in) -> k at the four sizes
    (4096, 4096): [2048, 3072, 4096, 4710],
    (4096, 14336): [3185, 4778, 6371, 7327],
    (8192, 8192): [4096, 6144, 8192, 9420],
    (8192, 28672): [6371, 9557, 12743, 14654],
    (1024, 4096): [819, 1228, 1638, 1884],
}
CONFIG4_PRUNED_K = {(4096, 4096): 3072, (4096, 11008): 4477}     # (n_out, n_in) -> k at 1.5 bits per weight


def table4_k(bits: float, n_out: int, n_in: int) -> int:
    return TABLE4_K[(n_out, n_in)][TABLE4_BITS.index(bits)]


def table4_configs() -> list[dict]:
    return [dict(n_in=n_in, n_out=n_out, k=table4_k(bits, n_out, n_in), bits=bits)
            for (n_out, n_in) in TABLE4_SHAPES for bits in TABLE4_BITS]


def llama2_7b_stack_shapes(n_blocks: int = 32) -> list[dict]:
    """Linear layers of a Llama-2-7B-shaped decoder at 1.5 bits per weight.

    Per block: q, k, v, o (4096 -> 4096), gate, up (4096 -> 11008),
    down (11008 -> 4096).  The middle size is floor(1.5 * n*m / (n+m)):
    3072 for the square layers and 4477 for the MLP layers.
    """
    out = []
    for _ in range(n_blocks):
        for _ in range(4):
            out.append(dict(n_in=4096, n_out=4096, k=3072))
        for _ in range(2):
            out.append(dict(n_in=4096, n_out=11008, k=4477))
        out.append(dict(n_in=11008, n_out=4096, k=4477))
    return out


def make_admm_problem(p: int, q: int, r: int, seed: int):
    """Operands of one ADMM update of the factorisation (section 3.2) in the least-squares form
    min_X ||B X - W||: the fixed factor B (p x q, i.i.d. N(0, 1/p): rows of comparable norm, as after the
    paper's row normalisation), the target W (p x r, N(0, 1)), the current iterate in SVID form (signs S
    (q x r, +-1 as int8), a (q), m (r), positive) and the scaled dual variable U (q x r, N(0, 0.3^2)).
    fp32 throughout, as an fp32 implementation of the compression would hold them."""
    rng = np.random.default_rng(seed + 900)
    B = (rng.standard_normal((p, q)) / np.sqrt(p)).astype(np.float32)
    W = rng.standard_normal((p, r)).astype(np.float32)
    S = np.where(rng.random((q, r)) < 0.5, 1, -1).astype(np.int8)
    a = rng.uniform(0.2, 1.5, q).astype(np.float32)
    m = rng.uniform(0.2, 1.5, r).astype(np.float32)
    U = (0.3 * rng.standard_normal((q, r))).astype(np.float32)
    return B, W, S, a, m, U


def make_admm_packed_problem(p: int, q: int, r: int, seed: int):
    """The same update with the fixed factor in its packed form (section 3.2: the factor that stays fixed in an
    alternating step is itself a sign matrix with two scale vectors): signs S_B (q x p, +-1 as int8), the scales
    m2 (q, U[0.5, 1.5)) and b (p, U[0.5, 1.5) / sqrt(p), so that the columns of the dense factor have norms of order
    one and B^T B + rho I a condition number of a few units), plus W, the iterate and the dual as in
    make_admm_problem.  Returns (S_B, m2, b, W, S, a, m, U), fp32 / int8."""
    rng = np.random.default_rng(seed + 950)
    S_B = np.where(rng.random((q, p)) < 0.5, 1, -1).astype(np.int8)
    m2 = rng.uniform(0.5, 1.5, q).astype(np.float32)
    b = (rng.uniform(0.5, 1.5, p) / np.sqrt(p)).astype(np.float32)
    W = rng.standard_normal((p, r)).astype(np.float32)
    S = np.where(rng.random((q, r)) < 0.5, 1, -1).astype(np.int8)
    a = rng.uniform(0.2, 1.5, q).astype(np.float32)
    m = rng.uniform(0.2, 1.5, r).astype(np.float32)
    U = (0.3 * rng.standard_normal((q, r))).astype(np.float32)
    return S_B, m2, b, W, S, a, m, U
