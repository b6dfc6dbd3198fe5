"""Structure of the seeded synthetic inputs: the recipe each family promises holds, and the
output is a pure function of the seed (independent of the thread count)."""
import os
import subprocess
import sys

import numpy as np
import pytest

import inputs


def rows(m):
    return [m.col_idx[m.row_ptr[i]:m.row_ptr[i + 1]] for i in range(m.nrows)]


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_csr_is_well_formed_sorted_distinct(name):
    m = inputs.SMALL[name]()
    assert m.row_ptr.dtype == np.int32 and m.col_idx.dtype == np.int32 and m.values.dtype == np.float64
    assert m.row_ptr[0] == 0 and np.all(np.diff(m.row_ptr) >= 0) and m.row_ptr[-1] == m.col_idx.size
    assert m.col_idx.min() >= 0 and m.col_idx.max() < m.ncols
    # ascending strictly inside each row: differences are > 0 except across row starts
    d = np.diff(m.col_idx.astype(np.int64))
    starts = m.row_ptr[1:-1]
    starts = starts[(starts > 0) & (starts < m.nnz)]
    interior = np.ones(m.nnz - 1, dtype=bool)
    interior[starts - 1] = False
    assert np.all(d[interior] > 0)
    assert np.all(np.abs(m.values) <= 4.01)


def test_uniform_has_fixed_row_length():
    m = inputs.uniform(n=5000, k=10)
    assert np.all(np.diff(m.row_ptr) == 10)
    assert abs(m.col_idx.mean() / 5000 - 0.5) < 0.01
    assert np.all(np.abs(m.values) <= 1) and abs(m.values.mean()) < 0.02


def test_laplace_structure_and_perturbation():
    g = 50
    m = inputs.laplace2d(g=g)
    assert m.nnz == 5 * g * g - 4 * g
    r = np.repeat(np.arange(m.nrows), np.diff(m.row_ptr))
    off = m.col_idx - r
    assert set(np.unique(off)) == {-g, -1, 0, 1, g}
    diag = off == 0
    assert np.all(np.abs(m.values[diag] - 4.0) <= 0.01) and np.all(np.abs(m.values[~diag] + 1.0) <= 0.01)
    assert m.values[diag].std() > 0.004          # perturbed, not constant


def test_powerlaw_row_lengths():
    m = inputs.powerlaw(n=400_000, cap=100_000)
    L = np.diff(m.row_ptr)
    assert L.min() == 1 and L.max() <= 100_000
    assert 12.0 < L.mean() < 20.0
    assert L.var() > 100                          # "irregular" by the paper's rule (Section I, Problem 2)
    assert 0.25 < np.mean(L == 1) < 0.40
    # tail exponent: P(L > 4t) / P(L > t) ~ 4^-1.1
    t = 50
    ratio = np.mean(L > 4 * t) / np.mean(L > t)
    assert 0.15 < ratio < 0.30


def test_fem3_blocks():
    nb, w = 3000, 200
    m = inputs.fem3(nb=nb, window=w)
    L = np.diff(m.row_ptr)
    assert np.all(L % 3 == 0) and L.min() >= 27 and L.max() <= 81
    assert np.all(L[0::3] == L[1::3]) and np.all(L[0::3] == L[2::3])
    for br in (0, 1, 1234, nb - 1):
        c0, c1, c2 = (m.col_idx[m.row_ptr[3 * br + t]:m.row_ptr[3 * br + t + 1]] for t in range(3))
        assert np.array_equal(c0, c1) and np.array_equal(c0, c2)
        bc = c0[0::3] // 3
        assert np.array_equal(c0.reshape(-1, 3), 3 * bc[:, None] + np.arange(3))
        assert br in bc and np.all(np.abs(bc - br) <= w) and np.all(np.diff(bc) > 0)
    assert 9 * 3 * nb <= m.nnz // 3 <= 27 * 3 * nb


def test_hybrid_heavy_rows():
    m = inputs.hybrid(n=200_000, n_heavy=11, heavy_len=30_000)
    L = np.diff(m.row_ptr)
    heavy = m.meta["heavy_rows"]
    assert heavy.size == 11 and np.all(np.diff(heavy) > 0)
    assert np.array_equal(np.flatnonzero(L > 8), heavy) and np.all(L[heavy] == 30_000)
    light = np.delete(L, heavy)
    assert light.min() == 2 and light.max() == 8 and abs(light.mean() - 5.0) < 0.05


def test_vector_and_integer_mode():
    x = inputs.vector(100_000)
    assert np.all(np.abs(x) <= 1) and abs(x.mean()) < 0.01 and abs(x.std() - 3 ** -0.5) < 0.01
    xi = inputs.vector(100_000, integer=True)
    assert set(np.unique(xi)) == {-3.0, -2.0, -1.0, 1.0, 2.0, 3.0}
    m = inputs.SMALL["C3"](integer=True)
    assert set(np.unique(m.values)) <= {-3.0, -2.0, -1.0, 1.0, 2.0, 3.0}


def test_output_does_not_depend_on_thread_count():
    code = ("import inputs, hashlib, numpy as np;"
            "m = inputs.SMALL['C3'](); x = inputs.vector(1000);"
            "print(hashlib.sha1(m.row_ptr.tobytes() + m.col_idx.tobytes() + m.values.tobytes() + x.tobytes()).hexdigest())")
    out = []
    for nt in ("1", "5"):
        env = dict(os.environ, OMP_NUM_THREADS=nt)
        out.append(subprocess.check_output([sys.executable, "-c", code], env=env,
                                           cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__)))))
    assert out[0] == out[1]
