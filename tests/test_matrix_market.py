"""spmv_mm_read against an independent reader (scipy.io.mmread) on files written here, the error
paths, and the command line in host-only mode.  No GPU."""
import json
import os
import subprocess
import sys

import numpy as np
import pytest
import scipy.io
import scipy.sparse as sp

import paper_2212_10432_amd as lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def write_mm(path, field, sym, nrows, ncols, entries, comments=("% written by the test",)):
    with open(path, "w") as f:
        f.write(f"%%MatrixMarket matrix coordinate {field} {sym}\n")
        for c in comments:
            f.write(c + "\n")
        f.write(f"{nrows} {ncols} {len(entries)}\n")
        for e in entries:
            f.write(" ".join(str(t) for t in e) + "\n")


def random_entries(rng, nrows, ncols, n, field, lower=False, strict=False):
    seen, out = set(), []
    while len(out) < n:
        i, j = int(rng.integers(1, nrows + 1)), int(rng.integers(1, ncols + 1))
        if lower and j > i:
            i, j = j, i
        if strict and i == j:
            continue
        if (i, j) in seen:
            continue
        seen.add((i, j))
        if field == "pattern":
            out.append((i, j))
        elif field == "integer":
            out.append((i, j, int(rng.integers(-9, 10))))
        else:
            out.append((i, j, repr(float(rng.normal()))))
    return out


def as_csr(nrows, ncols, rp, ci, va):
    A = sp.csr_matrix((va, ci, rp), shape=(nrows, ncols))
    A.sum_duplicates()
    A.sort_indices()
    return A


@pytest.mark.parametrize("field,sym", [("real", "general"), ("integer", "general"), ("pattern", "general"),
                                       ("real", "symmetric"), ("pattern", "symmetric"), ("real", "skew-symmetric")])
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_reader_matches_scipy(tmp_path, field, sym, dt):
    rng = np.random.default_rng(5)
    nrows, ncols = (40, 40) if sym != "general" else (37, 53)
    ents = random_entries(rng, nrows, ncols, 300, field, lower=sym != "general", strict=sym == "skew-symmetric")
    path = str(tmp_path / "m.mtx")
    write_mm(path, field, sym, nrows, ncols, ents, comments=("% a comment", "%", ""))
    n, m, rp, ci, va = lib.spmv_mm_read(path, dt)
    assert (n, m) == (nrows, ncols) and rp.dtype == np.int32 and ci.dtype == np.int32 and va.dtype == dt
    assert rp[0] == 0 and rp[-1] == ci.size == va.size and np.all(np.diff(rp) >= 0)
    for r in range(n):
        assert np.all(np.diff(ci[rp[r]:rp[r + 1]]) > 0)      # ascending, no repeats in this file
    want = scipy.io.mmread(path).tocsr().astype(dt)
    want.sort_indices()
    got = as_csr(n, m, rp, ci, va)
    assert np.array_equal(got.indptr, want.indptr) and np.array_equal(got.indices, want.indices)
    assert np.array_equal(got.data, want.data)


def test_repeated_positions_are_kept_in_file_order(tmp_path):
    path = str(tmp_path / "d.mtx")
    write_mm(path, "real", "general", 3, 3, [(2, 2, 1.5), (1, 3, 2.0), (2, 2, -4.0), (2, 1, 7.0), (2, 2, 0.25)])
    n, m, rp, ci, va = lib.spmv_mm_read(path)
    assert list(rp) == [0, 1, 5, 5] and list(ci) == [2, 0, 1, 1, 1] and list(va) == [2.0, 7.0, 1.5, -4.0, 0.25]


def test_empty_matrix_and_crlf(tmp_path):
    path = str(tmp_path / "e.mtx")
    with open(path, "wb") as f:
        f.write(b"%%MatrixMarket matrix coordinate real general\r\n% c\r\n4 5 0\r\n")
    n, m, rp, ci, va = lib.spmv_mm_read(path)
    assert (n, m) == (4, 5) and list(rp) == [0] * 5 and ci.size == 0 and va.size == 0
    with open(path, "wb") as f:
        f.write(b"%%MatrixMarket MATRIX Coordinate Real General\r\n2 2 2\r\n1 1 1e0\r\n2 1 -2.5E+1\r\n")
    n, m, rp, ci, va = lib.spmv_mm_read(path)
    assert list(rp) == [0, 1, 2] and list(ci) == [0, 0] and list(va) == [1.0, -25.0]


@pytest.mark.parametrize("text,status", [
    ("", lib.SPMV_ERR_INVALID_ARG),
    ("hello\n1 1 0\n", lib.SPMV_ERR_INVALID_ARG),
    ("%%MatrixMarket matrix array real general\n2 2\n1\n2\n3\n4\n", lib.SPMV_ERR_UNSUPPORTED),
    ("%%MatrixMarket matrix coordinate complex general\n1 1 1\n1 1 1 0\n", lib.SPMV_ERR_UNSUPPORTED),
    ("%%MatrixMarket matrix coordinate complex hermitian\n1 1 1\n1 1 1 0\n", lib.SPMV_ERR_UNSUPPORTED),
    ("%%MatrixMarket matrix coordinate real general\n2 2\n", lib.SPMV_ERR_INVALID_ARG),
    ("%%MatrixMarket matrix coordinate real general\n2 2 2\n1 1 1.0\n", lib.SPMV_ERR_INVALID_ARG),
    ("%%MatrixMarket matrix coordinate real general\n2 2 1\n3 1 1.0\n", lib.SPMV_ERR_BAD_CSR),
    ("%%MatrixMarket matrix coordinate real general\n2 2 1\n1 0 1.0\n", lib.SPMV_ERR_BAD_CSR),
    ("%%MatrixMarket matrix coordinate real general\n2 2 1\n1 1\n", lib.SPMV_ERR_INVALID_ARG),
    ("%%MatrixMarket matrix coordinate real symmetric\n2 3 1\n1 1 1.0\n", lib.SPMV_ERR_INVALID_ARG),
    ("%%MatrixMarket matrix coordinate real skew-symmetric\n2 2 1\n1 1 1.0\n", lib.SPMV_ERR_INVALID_ARG),
    # a truncated line must not borrow its missing numbers from the line after it
    ("%%MatrixMarket matrix coordinate real general\n3 3 2\n1\n2 3 5.0\n", lib.SPMV_ERR_INVALID_ARG),
    ("%%MatrixMarket matrix coordinate real general\n3 3 2\n1 2\n3 3 5.0\n", lib.SPMV_ERR_INVALID_ARG),
    ("%%MatrixMarket matrix coordinate real general\n3 3\n2\n1 1 1.0\n2 2 1.0\n", lib.SPMV_ERR_INVALID_ARG),
    ("%%MatrixMarket matrix coordinate pattern general\n3 3 2\n1\n2 3\n", lib.SPMV_ERR_INVALID_ARG),
    # an entry count the file cannot possibly hold
    ("%%MatrixMarket matrix coordinate real general\n3 3 2000000000\n1 1 1.0\n", lib.SPMV_ERR_INVALID_ARG),
])
def test_malformed_files_are_refused(tmp_path, text, status):
    path = str(tmp_path / "bad.mtx")
    with open(path, "w") as f:
        f.write(text)
    with pytest.raises(lib.SpmvError) as e:
        lib.spmv_mm_read(path)
    assert e.value.status == status and e.value.message


def test_missing_file(tmp_path):
    with pytest.raises(lib.SpmvError) as e:
        lib.spmv_mm_read(str(tmp_path / "nope.mtx"))
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG


def test_command_line_host_only(tmp_path):
    rng = np.random.default_rng(9)
    path = str(tmp_path / "c.mtx")
    write_mm(path, "real", "general", 300, 300, random_entries(rng, 300, 300, 2000, "real"))
    out = subprocess.run([sys.executable, "-m", "paper_2212_10432_amd", path, "--host-only", "--plan", "light=sell,sigma=64", "--json"],
                         cwd=ROOT, capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    d = json.loads(out.stdout)
    assert d["nrows"] == 300 and d["nnz"] == 2000 and d["spec"].startswith("light=sell,sigma=64")
    assert "BMW_PAD" in d["operators"]


def test_large_file_parsed_in_pieces(tmp_path):
    """A file of several megabytes (many pieces for the threaded parser), comments and blank lines between the
    entries, repeated positions, CRLF ends: same matrix as scipy reads; a malformed line is reported with its
    entry number; what follows the announced entries is not looked at."""
    rng = np.random.default_rng(9)
    nrows, ncols, n = 3000, 2500, 250_000
    i = rng.integers(1, nrows + 1, n); j = rng.integers(1, ncols + 1, n); v = rng.integers(-99, 100, n)
    lines = [f"{a} {b} {c}.5" for a, b, c in zip(i, j, v)]
    body = []
    for k, l in enumerate(lines):
        body.append(l)
        if k % 5000 == 17:
            body += ["% a comment in the middle", ""]
    path = str(tmp_path / "big.mtx")
    with open(path, "w", newline="") as f:
        f.write("%%MatrixMarket matrix coordinate real general\r\n")
        f.write(f"{nrows} {ncols} {n}\r\n")
        f.write("\r\n".join(body) + "\r\n")
        f.write("this line comes after the last announced entry and is never parsed\r\n")
    assert os.path.getsize(path) > 3_000_000
    nr, nc, rp, ci, va = lib.spmv_mm_read(path, np.float64)
    want = sp.coo_matrix((v + np.where(v >= 0, 0.5, -0.5), (i - 1, j - 1)), shape=(nrows, ncols)).tocsr()
    want.sort_indices()
    got = as_csr(nr, nc, rp, ci, va)
    assert np.array_equal(got.indptr, want.indptr) and np.array_equal(got.indices, want.indices)
    assert np.allclose(got.data, want.data, rtol=0, atol=0)
    for r in range(0, nr, 97):                      # columns ascend inside a row, repeats allowed
        assert np.all(np.diff(ci[rp[r]:rp[r + 1]]) >= 0)
    # the same file with entry 200001 broken
    bad = list(lines)
    bad[200_000] = "12 x 1.0"
    with open(path, "w") as f:
        f.write("%%MatrixMarket matrix coordinate real general\n")
        f.write(f"{nrows} {ncols} {n}\n")
        f.write("\n".join(bad) + "\n")
    with pytest.raises(lib.SpmvError) as e:
        lib.spmv_mm_read(path, np.float64)
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG and "200001" in str(e.value)
