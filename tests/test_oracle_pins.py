"""Pins for the CPU oracle (oracle/): it is checked against things other than itself --
a hand-worked example, exact rational brute force on tiny matrices, closed forms
(identity, diagonal, permutation, all-ones, 5-point Laplacian), exact integer
arithmetic, SciPy's CSR product, and algebraic invariants.  Each pin is chosen so that a
plausible mistake (dropped term, wrong sign or index, transposed operand, off-by-one in
row_ptr) fails at least one of them.
"""
from fractions import Fraction

import numpy as np
import pytest
import scipy.sparse as sp

import inputs
import oracle
from conftest import load_golden

U64 = 2.0 ** -53
U32 = 2.0 ** -24


def random_csr(rng, nrows, ncols, max_len, dtype=np.float64, dup=False, empty_frac=0.2):
    lens = rng.integers(0, max_len + 1, size=nrows)
    lens[rng.random(nrows) < empty_frac] = 0
    row_ptr = np.zeros(nrows + 1, dtype=np.int32)
    np.cumsum(lens, out=row_ptr[1:])
    nnz = int(row_ptr[-1])
    if dup:
        col = rng.integers(0, ncols, size=nnz).astype(np.int32)      # unsorted, duplicates allowed
    else:
        col = np.empty(nnz, dtype=np.int32)
        for i in range(nrows):
            k = lens[i]
            col[row_ptr[i]:row_ptr[i + 1]] = rng.permutation(ncols)[:k] if k <= ncols else rng.integers(0, ncols, k)
    val = rng.uniform(-1, 1, size=nnz).astype(dtype)
    return row_ptr, col, val


# ---- the hand-worked example ------------------------------------------------------------

def test_golden_hand_worked_example():
    g = load_golden("tiny_spmv.txt")
    rp = np.array(g["row_ptr"], dtype=np.int32)
    ci = np.array(g["col_idx"], dtype=np.int32)
    for dt in (np.float64, np.float32):
        v = np.array(g["values"], dtype=dt)
        x = np.array(g["x"], dtype=dt)
        want = np.array(g["y"], dtype=np.float64)
        assert np.array_equal(oracle.spmv(rp, ci, v, x).astype(np.float64), want)
        assert np.array_equal(oracle.spmv_wide(rp, ci, v, x), want)
        assert np.array_equal(oracle.abs_bound(rp, ci, v, x), np.array([5.0, 0.0, 8.5, 17.0]))


# ---- exact brute force on tiny matrices -------------------------------------------------

@pytest.mark.parametrize("shape", [(1, 1), (1, 9), (9, 1), (7, 13), (13, 7), (32, 32), (64, 40)])
@pytest.mark.parametrize("dup", [False, True])
def test_dense_brute_force_exact_rational(shape, dup):
    nrows, ncols = shape
    rng = np.random.default_rng(1000 * nrows + ncols + dup)
    for dt, u in ((np.float64, U64), (np.float32, U32)):
        rp, ci, v = random_csr(rng, nrows, ncols, min(ncols, 12) if not dup else 12, dtype=dt, dup=dup)
        x = rng.uniform(-1, 1, size=ncols).astype(dt)
        exact = oracle.dense_exact(nrows, ncols, rp, ci, v, x)
        # the absolute-value bound, again by brute force
        bnd = oracle.dense_exact(nrows, ncols, rp, ci, np.abs(v), np.abs(x))
        if dup:   # |a1 + a2| <= |a1| + |a2|: recompute the bound per stored entry
            bnd = [sum((abs(Fraction(float(v[k]))) * abs(Fraction(float(x[ci[k]])))
                        for k in range(rp[i], rp[i + 1])), Fraction(0)) for i in range(nrows)]
        y = oracle.spmv(rp, ci, v, x)
        yw = oracle.spmv_wide(rp, ci, v, x)
        ab = oracle.abs_bound(rp, ci, v, x)
        for i in range(nrows):
            n_i = int(rp[i + 1] - rp[i])
            b = bnd[i]
            # sequential summation error bound: n_i * u * sum|a||x| (first order, generous factor 1.01)
            assert abs(Fraction(float(y[i])) - exact[i]) <= Fraction(1.01 * n_i * u) * b
            # wide accumulation: one final rounding to double, plus negligible inner error
            assert abs(Fraction(float(yw[i])) - exact[i]) <= Fraction(2 * U64) * b
            assert abs(Fraction(float(ab[i])) - b) <= Fraction(2 * U64) * b
            if n_i == 0:
                assert y[i] == 0 and yw[i] == 0 and ab[i] == 0 and not np.signbit(y[i])


def test_rectangular_catches_transposed_operand():
    # 2 x 3 matrix whose transpose product is different in shape and value
    rp = np.array([0, 2, 3], dtype=np.int32)
    ci = np.array([0, 2, 1], dtype=np.int32)
    v = np.array([1.0, 10.0, 100.0])
    x = np.array([1.0, 2.0, 3.0])
    assert np.array_equal(oracle.spmv(rp, ci, v, x), [31.0, 200.0])


# ---- closed forms -----------------------------------------------------------------------

@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_identity_diagonal_permutation_are_bit_exact(dt):
    rng = np.random.default_rng(7)
    n = 1000
    x = rng.uniform(-1, 1, n).astype(dt)
    rp = np.arange(n + 1, dtype=np.int32)
    ident = np.arange(n, dtype=np.int32)
    assert np.array_equal(oracle.spmv(rp, ident, np.ones(n, dt), x), x)
    d = rng.uniform(-1, 1, n).astype(dt)
    assert np.array_equal(oracle.spmv(rp, ident, d, x), d * x)             # one rounded product per row
    perm = rng.permutation(n).astype(np.int32)
    assert np.array_equal(oracle.spmv(rp, perm, np.ones(n, dt), x), x[perm])
    assert np.array_equal(oracle.spmv_wide(rp, perm, np.ones(n, dt), x), x[perm].astype(np.float64))


def test_all_ones_gives_row_lengths():
    m = inputs.SMALL["C3"]()
    ones = np.ones(m.nnz)
    y = oracle.spmv(m.row_ptr, m.col_idx, ones, np.ones(m.ncols))
    assert np.array_equal(y, np.diff(m.row_ptr).astype(np.float64))
    y32 = oracle.spmv(m.row_ptr, m.col_idx, ones.astype(np.float32), np.ones(m.ncols, np.float32))
    assert np.array_equal(y32, np.diff(m.row_ptr).astype(np.float32))


def test_unperturbed_laplacian_closed_forms():
    g = 37
    m = inputs.laplace2d(g=g, integer=True)          # integer mode: exactly 4 / -1
    assert set(np.unique(m.values)) == {-1.0, 4.0}
    i, j = np.divmod(np.arange(g * g), g)
    # x = 1: each missing neighbour leaves +1
    missing = (i == 0).astype(int) + (i == g - 1) + (j == 0) + (j == g - 1)
    y = oracle.spmv(m.row_ptr, m.col_idx, m.values, np.ones(g * g))
    assert np.array_equal(y, missing.astype(np.float64))
    # x linear in (i, j): the discrete Laplacian vanishes on interior rows
    x = (3.0 * i - 5.0 * j + 11.0)
    y = oracle.spmv(m.row_ptr, m.col_idx, m.values, x)
    interior = missing == 0
    assert np.all(y[interior] == 0)
    # boundary rows: 4x - (present neighbours) evaluated with integers
    xi = (3 * i - 5 * j + 11).astype(np.int64)
    want = 4 * xi
    want[i > 0] -= xi[np.flatnonzero(i > 0) - g]
    want[i < g - 1] -= xi[np.flatnonzero(i < g - 1) + g]
    want[j > 0] -= xi[np.flatnonzero(j > 0) - 1]
    want[j < g - 1] -= xi[np.flatnonzero(j < g - 1) + 1]
    assert np.array_equal(y, want.astype(np.float64))


# ---- exact integer arithmetic -----------------------------------------------------------

@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_integer_valued_matrices_match_int64_arithmetic(name, dt):
    m = inputs.SMALL[name](integer=True)
    x = inputs.vector(m.ncols, integer=True)
    prod = m.values.astype(np.int64) * x.astype(np.int64)[m.col_idx]
    csum = np.concatenate([[0], np.cumsum(prod)])
    want = csum[m.row_ptr[1:]] - csum[m.row_ptr[:-1]]              # int64 row sums, exact
    assert np.abs(prod).max() * np.diff(m.row_ptr).max() < 2 ** 24    # representable in fp32 too
    v = m.values.astype(dt)
    for fn in (oracle.spmv, oracle.spmv_wide):
        y = fn(m.row_ptr, m.col_idx, v, x.astype(dt))
        assert np.array_equal(y.astype(np.float64), want.astype(np.float64)), fn.__name__
        y8 = fn(m.row_ptr, m.col_idx, v, x.astype(dt), threads=8)
        assert np.array_equal(y8, y)
    ab = oracle.abs_bound(m.row_ptr, m.col_idx, v, x.astype(dt))
    acs = np.concatenate([[0], np.cumsum(np.abs(prod))])
    assert np.array_equal(ab, (acs[m.row_ptr[1:]] - acs[m.row_ptr[:-1]]).astype(np.float64))


# ---- an independent library routine -----------------------------------------------------

@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_scipy_csr_product(name):
    m = inputs.SMALL[name]()
    x = inputs.vector(m.ncols)
    A = sp.csr_matrix((m.values, m.col_idx, m.row_ptr), shape=(m.nrows, m.ncols))
    y_lib = A @ x
    bnd = abs(A) @ np.abs(x)
    lens = np.diff(m.row_ptr)
    y = oracle.spmv(m.row_ptr, m.col_idx, m.values, x)
    yw = oracle.spmv_wide(m.row_ptr, m.col_idx, m.values, x)
    ab = oracle.abs_bound(m.row_ptr, m.col_idx, m.values, x)
    # both sides carry at most n_i*u*bound of rounding each
    assert np.all(np.abs(y - y_lib) <= 2.02 * lens * U64 * bnd)
    assert np.all(np.abs(yw - y_lib) <= 1.01 * (lens + 2) * U64 * bnd)
    assert np.all(np.abs(ab - bnd) <= 1.01 * (lens + 2) * U64 * bnd)
    ok, worst = oracle.check(y_lib, m.row_ptr, m.col_idx, m.values, x)
    assert ok and worst < 1.0
    # fp32: SciPy in float64 on the rounded inputs is the exact-product reference
    v32, x32 = m.values.astype(np.float32), x.astype(np.float32)
    A32 = sp.csr_matrix((v32.astype(np.float64), m.col_idx, m.row_ptr), shape=A.shape)
    y_lib32 = A32 @ x32.astype(np.float64)
    bnd32 = abs(A32) @ np.abs(x32.astype(np.float64))
    yw32 = oracle.spmv_wide(m.row_ptr, m.col_idx, v32, x32)
    assert yw32.dtype == np.float64
    assert np.all(np.abs(yw32 - y_lib32) <= 2.02 * lens * U64 * bnd32)
    y32 = oracle.spmv(m.row_ptr, m.col_idx, v32, x32)
    assert y32.dtype == np.float32
    assert np.all(np.abs(y32 - y_lib32) <= 1.01 * (lens + 1) * U32 * bnd32)


# ---- algebraic invariants ---------------------------------------------------------------

def test_scaling_by_two_is_bit_exact():
    m = inputs.SMALL["C5"]()
    x = inputs.vector(m.ncols)
    y = oracle.spmv(m.row_ptr, m.col_idx, m.values, x)
    assert np.array_equal(oracle.spmv(m.row_ptr, m.col_idx, m.values, 2 * x), 2 * y)
    assert np.array_equal(oracle.spmv(m.row_ptr, m.col_idx, -m.values, x), -y)


def test_split_and_adjoint_identities():
    m = inputs.SMALL["C3"]()
    x = inputs.vector(m.ncols)
    rng = np.random.default_rng(3)
    mask = rng.random(m.nnz) < 0.5
    y = oracle.spmv_wide(m.row_ptr, m.col_idx, m.values, x)
    y1 = oracle.spmv_wide(m.row_ptr, m.col_idx, np.where(mask, m.values, 0.0), x)
    y2 = oracle.spmv_wide(m.row_ptr, m.col_idx, np.where(mask, 0.0, m.values), x)
    bnd = oracle.abs_bound(m.row_ptr, m.col_idx, m.values, x)
    assert np.all(np.abs(y - (y1 + y2)) <= 4 * U64 * bnd)
    # z^T (A x) == (A^T z)^T x with A^T built by SciPy
    z = rng.uniform(-1, 1, m.nrows)
    At = sp.csr_matrix((m.values, m.col_idx, m.row_ptr), shape=(m.nrows, m.ncols)).T.tocsr()
    w = oracle.spmv_wide(At.indptr.astype(np.int32), At.indices.astype(np.int32), At.data, z)
    lhs, rhs = float(z @ y), float(w @ x)
    scale = float(np.abs(z) @ bnd)
    assert abs(lhs - rhs) <= 1e-13 * scale


def test_check_rejects_planted_mistakes():
    """A mistake planted in a copy of the oracle's result must be caught by the tolerance test."""
    m = inputs.SMALL["C1"]()
    x = inputs.vector(m.ncols)
    y = oracle.spmv(m.row_ptr, m.col_idx, m.values, x)
    assert oracle.check(y, m.row_ptr, m.col_idx, m.values, x)[0]
    # drop the last term of one row
    bad = y.copy()
    k = m.row_ptr[124] - 1
    bad[123] -= m.values[k] * x[m.col_idx[k]]
    assert not oracle.check(bad, m.row_ptr, m.col_idx, m.values, x)[0]
    # shift rows by one (off-by-one in row_ptr)
    assert not oracle.check(np.roll(y, 1), m.row_ptr, m.col_idx, m.values, x)[0]
    # a relative perturbation of 1e-11 on one entry
    bad = y.copy()
    bad[5] += 1e-11 * oracle.abs_bound(m.row_ptr, m.col_idx, m.values, x)[5]
    assert not oracle.check(bad, m.row_ptr, m.col_idx, m.values, x)[0]
    # NaN is never accepted
    bad = y.copy()
    bad[0] = np.nan
    assert not oracle.check(bad, m.row_ptr, m.col_idx, m.values, x)[0]


def test_oracle_rejects_bad_csr():
    with pytest.raises(ValueError):
        oracle.spmv([0, 2], [0, 5], [1.0, 1.0], [1.0, 1.0])
    with pytest.raises(ValueError):
        oracle.spmv([0, 3], [0, 1], [1.0, 1.0], [1.0, 1.0])
