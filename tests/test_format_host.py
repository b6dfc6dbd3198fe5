"""Host format builder (C++, through the C ABI in host-only mode) against the NumPy reference
builders of oracle/format_ref.py: every format array bit for bit, the round trip
decode(arrays) == input matrix, and the closed forms the synthetic families imply.
No GPU is touched: the plans are built with host_only, which keeps the arrays in host memory."""
import numpy as np
import pytest
import scipy.sparse as sp

import inputs
import paper_2212_10432_amd as lib
from oracle import format_ref as ref

TINY = {
    "C1": lambda **kw: inputs.uniform(n=1000, k=10, **kw),
    "C2": lambda **kw: inputs.laplace2d(g=37, **kw),
    "C3": lambda **kw: inputs.powerlaw(n=5003, cap=3000, **kw),
    "C4": lambda **kw: inputs.fem3(nb=701, window=60, **kw),
    "C5": lambda **kw: inputs.hybrid(n=20011, n_heavy=5, heavy_len=5000, **kw),
}

SPECS = {
    "C1": ["light=wbm", "light=csrv,lpr=256", "light=xl,w=128,rb=256,chunk=512", "light=coo", "light=xnb,k=8,r=4", "light=nnzb,r=4", "light=xs,k=8,sigma=256", "light=csrv", "light=csrv,lpr=4,sigma=128", "light=sell", "light=sell,sigma=256", "light=sell,sigma=-1",
           "light=bin,smax=4,sigma=128"],
    "C2": ["dia=1,dia_fill=0.999,light=wbm", "dia=1,dia_fill=0.999,light=xl,w=64,rb=64", "light=xl,w=256,rb=128", "dia=1,dia_fill=0.999,light=coo", "dia=1,dia_fill=0.999,light=xnb,k=8,r=4", "light=xnb,k=24,r=16", "dia=1,dia_fill=0.999,light=nnzb,r=4", "light=nnzb,r=16", "dia=1,dia_fill=0.999,light=xs,k=8,sigma=64", "dia=1,light=sell", "light=sell,sigma=64", "light=csrv,lpr=2", "dia=1,dia_fill=0.999,light=csrv,lpr=1"],
    "C3": ["light=wbm", "heavy=1024,tile=2048,light=wbm", "light=bin,smax=16,sigma=512,chunk=256,wg=1", "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=0,wg=1", "light=csrv,lpr=256,chunk=512", "light=xl,w=512,rb=1024", "heavy=1024,tile=2048,light=xl,w=1024,rb=512,chunk=2048", "light=xl", "light=xnb,k=16,r=8", "heavy=1024,tile=2048,light=xnb,k=8,r=16", "light=nnzb,r=8", "light=nnzb,r=16", "heavy=1024,tile=2048,light=nnzb,r=4", "light=xs,k=16,sigma=512", "heavy=1024,tile=2048,light=xs,k=8,sigma=0", "light=csrv,chunk=512", "light=bin,smax=16,sigma=512,chunk=256",
           "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=512", "heavy=600,tile=1024,light=csrv,lpr=8",
           "heavy=256,tile=512,light=sell,sigma=128", "heavy=1024,tile=2048,hd=1,light=xl,w=1024,rb=512", "heavy=256,tile=512,hd=1,light=sell,sigma=128",
           "heavy=256,tile=512,piece=16,light=sell,sigma=128", "heavy=1024,tile=2048,hd=1,piece=32,light=xl,w=1024,rb=512", "heavy=64,tile=4096,piece=4,light=csrv"],
    "C4": ["light=bsell,block=3,sigma=256", "light=bsell,block=3,sigma=0,remap=1", "light=bsell,block=3,sigma=2048,xwin=1,remap=1", "light=sell,sigma=512",
           "light=csrv,lpr=16"],
    "C5": ["heavy=64,tile=2048,light=wbm", "light=bin,smax=16,sigma=256,chunk=1024,wg=1", "heavy=64,tile=2048,light=xl,w=2048,rb=4096,chunk=4096", "light=xl,w=4096,rb=16384", "heavy=64,tile=2048,light=coo", "heavy=64,tile=2048,light=xnb,k=32,r=4", "heavy=64,tile=2048,light=nnzb,r=8", "heavy=64,tile=2048,light=xs,k=16,sigma=1024", "heavy=64,tile=2048,light=sell,sigma=1024", "light=bin,smax=16,sigma=256,chunk=1024",
           "heavy=1000,tile=4096,light=csrv,lpr=2", "heavy=64,tile=2048,hd=1,light=xl", "heavy=64,tile=8192,hd=1,light=csrv",
           "heavy=64,tile=8192,hd=1,piece=64,light=csrv", "heavy=64,tile=2048,piece=8,light=xl,w=2048,rb=4096", "heavy=64,tile=16384,hd=1,light=csrv"],
}


def host_plan(m, spec, values=None):
    v = m.values if values is None else values
    return lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, v, force_plan=spec, host_only=True)


def as_scipy(nrows, ncols, r, c, v):
    A = sp.coo_matrix((v, (r, c)), shape=(nrows, ncols)).tocsr()
    A.sum_duplicates()
    A.eliminate_zeros()
    A.sort_indices()
    return A


def same_matrix(A, B):
    return (A.shape == B.shape and np.array_equal(A.indptr, B.indptr) and np.array_equal(A.indices, B.indices)
            and np.array_equal(A.data, B.data))


CASES = [(name, spec) for name in SPECS for spec in SPECS[name]]


@pytest.mark.parametrize("name,spec", CASES)
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_arrays_match_reference_and_decode_to_input(name, spec, dt):
    m = TINY[name]()
    vals = m.values.astype(dt)
    P = host_plan(m, spec, vals)
    got = P.arrays()
    want = ref.ref_plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, spec)
    assert sorted(got) == sorted(want)
    for k in want:
        assert got[k].dtype == want[k].dtype, k
        assert np.array_equal(got[k], want[k]), k
    p = ref.parse_spec(spec)
    A_in = as_scipy(m.nrows, m.ncols, np.repeat(np.arange(m.nrows), np.diff(m.row_ptr)), m.col_idx, vals)
    for arrays in (got, want):
        r, c, v = ref.decode(arrays, m.nrows, m.ncols, block=p["block"], tile=p["tile"], xl_w=p["w"], xl_rb=p["rb"])
        assert r.size == 0 or (r.min() >= 0 and r.max() < m.nrows and c.min() >= 0 and c.max() < m.ncols)
        assert same_matrix(as_scipy(m.nrows, m.ncols, r, c, v), A_in)
    d = P.describe()
    assert sum(part["nnz"] for part in d["parts"]) == m.nnz
    b_plan, b_csr = P.bytes()
    v = vals.itemsize
    assert b_csr == m.nnz * (v + 4) + 4 * (m.nrows + 1) + v * m.ncols + v * m.nrows
    P.destroy()


def test_structural_invariants():
    m = TINY["C3"]()
    spec = "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=512"
    P = host_plan(m, spec)
    a = P.arrays()
    lens = np.diff(m.row_ptr)
    # origin rows of all row-owning parts + heavy rows partition the row set
    owned = np.concatenate([a["bin0.sell.origin_rows"], a["bin1.csrv8.seg_row"],
                            np.unique(np.where(a["bin2.csrv64.seg_row"] < 0, ~a["bin2.csrv64.seg_row"], a["bin2.csrv64.seg_row"])),
                            a["heavy.rows"]])
    assert np.array_equal(np.sort(owned), np.arange(m.nrows))
    # offsets are non-decreasing and end at the totals
    for k in ("bin0.sell.slice_ptr", "bin1.csrv8.seg_ptr", "bin2.csrv64.seg_ptr", "heavy.unit_ptr"):
        assert a[k][0] == 0 and np.all(np.diff(a[k]) >= 0)
    assert a["bin0.sell.slice_ptr"][-1] == a["bin0.sell.cols"].size
    assert a["heavy.unit_ptr"][-1] == a["heavy.vals"].size >= lens[a["heavy.rows"]].sum()
    assert np.count_nonzero(a["heavy.vals"]) == lens[a["heavy.rows"]].sum()
    # SORT_BMTB: in every stripe the lanes hold each heavy row exactly once
    nh = a["heavy.rows"].size
    lr = a["heavy.lane_row"].reshape(-1, 64 * (-(-nh // 64)))
    for row in lr:
        assert np.array_equal(np.sort(row[row != 0xFFFF]), np.arange(nh))
    assert np.all(lens[a["heavy.rows"]] > 1024)
    # padding = sum over slices of (slice width - row length)
    order = a["bin0.sell.origin_rows"]
    pad = 0
    for s in range(len(a["bin0.sell.slice_ptr"]) - 1):
        L = lens[order[s * 64:(s + 1) * 64]]
        pad += 64 * L.max() - L.sum()
    assert a["bin0.sell.cols"].size - lens[order].sum() == pad
    # rows reduced through atomics are exactly the zeroed rows
    sr = a["bin2.csrv64.seg_row"]
    atomic_rows = np.unique(~sr[sr < 0])
    assert np.array_equal(a["zero.rows"], atomic_rows)
    assert np.all(lens[atomic_rows] > 512)
    # stable descending sort inside each window of 256 rows
    for b in range(0, order.size, 256):
        w = order[b:b + 256]
        assert np.all(np.diff(lens[w]) <= 0)
        for L in np.unique(lens[w]):
            assert np.all(np.diff(w[lens[w] == L]) > 0)
    P.destroy()


def test_closed_form_uniform_rows_need_no_padding_and_no_permutation():
    m = TINY["C1"]()
    for spec in ("light=sell,sigma=-1", "light=sell,sigma=256"):
        a = host_plan(m, spec).arrays()
        assert np.array_equal(a["sell.origin_rows"], np.arange(m.nrows))        # stable sort = identity
        assert a["sell.cols"].size == 64 * 10 * (-(-m.nrows // 64))
    a = host_plan(m, "light=sell").arrays()
    assert "sell.origin_rows" not in a                                           # row = 64*slice + lane
    assert np.array_equal(a["sell.slice_ptr"], 640 * np.arange(-(-m.nrows // 64) + 1))


def test_closed_form_wavefront_bitmaps_of_uniform_rows():
    """Every row of C1 has 10 entries: entry g of the stream starts a row exactly when g % 10 == 0, a
    tile of 512 entries is preceded by ceil(512 i / 10) row starts, and the stream is the CSR itself."""
    m = TINY["C1"]()
    a = host_plan(m, "light=wbm").arrays()
    total = m.nnz
    g = np.arange(a["wbm.cols"].size)
    bits = ((a["wbm.mask"][g // 64] >> (g % 64).astype(np.uint64)) & np.uint64(1)).astype(bool)
    assert np.array_equal(bits, (g % 10 == 0) & (g < total))
    ntiles = -(-total // 512)
    assert np.array_equal(a["wbm.tile_row"], np.minimum(-(-(512 * np.arange(ntiles + 1)) // 10), m.nrows))
    assert np.array_equal(a["wbm.cols"][:total], m.col_idx) and np.array_equal(a["wbm.vals"][:total], m.values)
    assert not a["wbm.vals"][total:].any() and np.array_equal(a["wbm.rows"], np.arange(m.nrows))
    # rows cut by a tile border reduce through atomics: 512 i / 10 is whole only when i % 5 == 0
    borders = sorted({(min(total, 512 * i) - 1) // 10 for i in range(1, ntiles + 1)} | {(512 * i) // 10 for i in range(1, ntiles) if (512 * i) % 10})
    assert np.array_equal(a["zero.rows"], [r for r in borders if r < m.nrows])


def _both(m, spec, vals=None):
    """The library's arrays and the reference builder's, for pins that must hold for each of them."""
    v = m.values if vals is None else vals
    P = host_plan(m, spec, v)
    a = P.arrays()
    P.destroy()
    return a, ref.ref_plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, v, spec)


def test_closed_form_csr_segments_of_uniform_rows():
    """Rows of exactly 10 entries: sorted (stably) they keep their order, segment i is row i at 10 i.  Rows of
    exactly 200 entries cut into segments of at most 64: four segments at 200 i + {0, 64, 128, 192}, marked
    as segments that add through atomics (~row), and every row is zeroed first."""
    m = TINY["C1"]()
    n = m.nrows
    for a in _both(m, "light=csrv,lpr=4,sigma=128"):
        assert np.array_equal(a["csrv.seg_ptr"], 10 * np.arange(n + 1))
        assert np.array_equal(a["csrv.seg_row"], np.arange(n))
        assert np.array_equal(a["csrv.cols"], m.col_idx) and np.array_equal(a["csrv.vals"], m.values)
    m = inputs.uniform(n=300, k=200)       # rows of exactly 200 entries, cut into segments of at most 64
    n = m.nrows
    for a in _both(m, "light=csrv,lpr=64,chunk=64"):
        want = (200 * np.arange(n)[:, None] + np.array([0, 64, 128, 192])[None, :]).reshape(-1)
        assert np.array_equal(a["csrv.seg_ptr"], np.append(want, 200 * n))
        assert np.array_equal(a["csrv.seg_row"], ~np.repeat(np.arange(n), 4))
        assert np.array_equal(a["zero.rows"], np.arange(n))


def test_closed_form_nnz_balanced_tiles_of_uniform_rows():
    """Rows of exactly 10 entries, R = 8 entries per lane: entry g of the stream belongs to lane (g % 512) // 8
    of tile g // 512 and is stored at 512 (g // 512) + 64 (g % 8) + (g % 512) // 8; it starts a row exactly
    when g % 10 == 0; ceil(512 i / 10) rows start before tile i."""
    m = TINY["C1"]()
    total, R = m.nnz, 8
    g = np.arange(total)
    dst = 512 * (g // 512) + 64 * (g % 8) + (g % 512) // 8
    for a in _both(m, "light=nnzb,r=8"):
        assert a["nnzb.cols"].size == 512 * -(-total // 512)
        assert np.array_equal(a["nnzb.cols"][dst], m.col_idx) and np.array_equal(a["nnzb.vals"][dst], m.values)
        assert np.count_nonzero(a["nnzb.vals"]) == np.count_nonzero(m.values)
        bit = (a["nnzb.bits"][64 * (g // 512) + (g % 512) // 8] >> (g % 8)) & 1
        assert np.array_equal(bit.astype(bool), g % 10 == 0)
        assert int(np.unpackbits(a["nnzb.bits"].view(np.uint8)).sum()) == m.nrows       # nothing set in the padding
        ntiles = -(-total // 512)
        assert np.array_equal(a["nnzb.tile_row"], np.minimum(-(-(512 * np.arange(ntiles + 1)) // 10), m.nrows))
        assert np.array_equal(a["nnzb.rows"], np.arange(m.nrows))


def test_hand_worked_two_pass_layout():
    """A 128 x 128 matrix with the diagonal (i, i) = 1 + i and the anti-diagonal (i, 127 - i) = -(1 + i), windows of
    64 columns, blocks of 64 rows, fp64 (vectors of 2 entries).  Every (window, block) run has 64 entries, so
    nothing is padded.  Memory order: window 0 = [run(0,0): the diagonal of rows 0..63 | run(0,1): the
    anti-diagonal of rows 64..127], window 1 = [run(1,0): the anti-diagonal of rows 0..63 | run(1,1): the
    diagonal of rows 64..127]."""
    n = 128
    i = np.arange(n)
    lo, hi = np.minimum(i, 127 - i), np.maximum(i, 127 - i)
    ci = np.stack([lo, hi], axis=1).reshape(-1).astype(np.int32)
    on_diag = np.stack([lo == i, hi == i], axis=1).reshape(-1)
    va = np.where(on_diag, 1.0, -1.0) * (1 + np.repeat(i, 2))
    rp = (2 * np.arange(n + 1)).astype(np.int32)
    spec = "light=xl,w=64,rb=64"
    P = lib.Plan(n, n, rp, ci, va, force_plan=spec, host_only=True)
    got = P.arrays()
    P.destroy()
    first, second = i[:64], i[64:]
    vals = np.concatenate([1.0 + first, -(1.0 + second), -(1.0 + first), 1.0 + second])
    lcol = np.concatenate([first, 127 - second, 63 - first, second - 64]).astype(np.uint16)
    code = lambda e: (e // 2) * 8 + 7                          # a full group: first vector, 8 vectors
    glist = np.array([code(e) for e in (0, 16, 32, 48, 128, 144, 160, 176, 64, 80, 96, 112, 192, 208, 224, 240)], dtype=np.int32)
    items = np.zeros((8, 3), dtype=np.int32)                   # window 0 on XCD 0, window 1 on XCD 1, six fillers
    items[0], items[1] = (0, 0, 128), (1, 128, 256)
    for a in (got, ref.ref_plan(n, n, rp, ci, va, spec)):
        assert np.array_equal(a["xl.vals"], vals)
        assert np.array_equal(a["xl.lcol"], lcol)
        assert np.array_equal(a["xl.gptr"], [0, 8, 16])
        assert np.array_equal(a["xl.glist"], glist)
        assert np.array_equal(a["xl.lrow"], np.tile(np.arange(64, dtype=np.uint16), 4))
        assert np.array_equal(a["xl.items"].reshape(-1, 3), items)
        assert "xl.rows" not in a                               # the part owns every row in order


def _one_entry_per_row_and_stripe():
    """64 rows x 1024 columns; row i has one entry in each of the 16 stripes of 64 columns: (i, 64 j + i) =
    1000 j + i + 1."""
    i, j = np.meshgrid(np.arange(64), np.arange(16), indexing="ij")
    ci = (64 * j + i).reshape(-1).astype(np.int32)
    va = (1000.0 * j + i + 1).reshape(-1)
    rp = (16 * np.arange(65)).astype(np.int32)
    return rp, ci, va


def test_hand_worked_xcd_striped_sell():
    """16 stripes on 8 XCDs: XCD k owns stripes k and k + 8, so the units (one slice of 64 rows, one entry
    wide, per stripe) follow each other as stripes 0, 8, 1, 9, ...; lane l of unit u owns slot 64 u + l, and
    row i lists its 16 slots in stripe order."""
    rp, ci, va = _one_entry_per_row_and_stripe()
    spec = "light=xs,k=16,sigma=0"
    P = lib.Plan(64, 1024, rp, ci, va, force_plan=spec, host_only=True)
    got = P.arrays()
    P.destroy()
    stripe_of_unit = np.array([u // 2 + 8 * (u % 2) for u in range(16)])
    unit_of_stripe = np.argsort(stripe_of_unit)
    lane = np.arange(64)
    for a in (got, ref.ref_plan(64, 1024, rp, ci, va, spec)):
        assert np.array_equal(a["xs.unit_ptr"], 64 * np.arange(17))
        assert np.array_equal(a["xs.xbase"], 2 * np.arange(9))
        assert np.array_equal(a["xs.cols"].reshape(16, 64), 64 * stripe_of_unit[:, None] + lane[None, :])
        assert np.array_equal(a["xs.vals"].reshape(16, 64), 1000.0 * stripe_of_unit[:, None] + lane[None, :] + 1)
        assert np.array_equal(a["xs.pptr"], 16 * np.arange(65))
        assert np.array_equal(a["xs.pslot"].reshape(64, 16), 64 * unit_of_stripe[None, :] + lane[:, None])
        assert "xs.rows" not in a


def test_hand_worked_xcd_striped_nnz_balanced_tiles():
    """The same matrix with tiles of 64 lanes x 4 entries: a stripe's 64 one-entry segments fill a quarter of
    its tile (lanes 0..15, all four bits set), the rest is padding at the stripe's first column; tiles
    follow each other as stripes 0, 8, 1, 9, ...; segment 64 t + i is row i of tile t's stripe."""
    rp, ci, va = _one_entry_per_row_and_stripe()
    spec = "light=xnb,k=16,r=4"
    P = lib.Plan(64, 1024, rp, ci, va, force_plan=spec, host_only=True)
    got = P.arrays()
    P.destroy()
    stripe_of_tile = np.array([t // 2 + 8 * (t % 2) for t in range(16)])
    tile_of_stripe = np.argsort(stripe_of_tile)
    pos = np.arange(256)                                            # position in a stripe's stream
    at = 64 * (pos % 4) + pos // 4                                  # where the tile stores it
    for a in (got, ref.ref_plan(64, 1024, rp, ci, va, spec)):
        cols, vals = a["xnb.cols"].reshape(16, 256), a["xnb.vals"].reshape(16, 256)
        for t, s_ in enumerate(stripe_of_tile):
            assert np.array_equal(cols[t][at], np.where(pos < 64, 64 * s_ + pos, 64 * s_))
            assert np.array_equal(vals[t][at], np.where(pos < 64, 1000.0 * s_ + pos + 1, 0.0))
        assert np.array_equal(a["xnb.bits"].reshape(16, 64), np.tile(np.where(np.arange(64) < 16, 15, 0), (16, 1)))
        assert np.array_equal(a["xnb.tile_row"], 64 * np.arange(17))
        assert np.array_equal(a["xnb.xbase"], 2 * np.arange(9))
        assert np.array_equal(a["xnb.seg_row"], np.tile(np.arange(64), 16))
        assert np.array_equal(a["xnb.bbase"], np.concatenate([64 * tile_of_stripe, 64 * tile_of_stripe + 64]))
        assert np.array_equal(a["xnb.open_slots"], 64 * np.arange(1, 17) - 1)


def test_closed_form_laplacian_diagonals():
    g = 37
    m = TINY["C2"]()
    P = host_plan(m, "dia=1,light=sell")
    a = P.arrays()
    assert np.array_equal(a["dia.offsets"], [-g, -1, 0, 1, g])
    assert set(a) == {"dia.offsets", "dia.vals"}                                 # nothing left over
    n = g * g
    ld = a["dia.vals"].size // 5
    dv = a["dia.vals"].reshape(5, ld)[:, :n]
    # explicit zeros in valid slots: the +-1 diagonals skip the grid's row ends (2*(g-1) slots);
    # the slots outside the matrix are zero too: 2*g + 2 of them
    inside_zero = sum(int(np.sum(dv[d, max(0, -o):min(n, n - o)] == 0)) for d, o in enumerate([-g, -1, 0, 1, g]))
    assert inside_zero == 2 * (g - 1)
    assert int(np.sum(dv == 0)) == 2 * (g - 1) + 2 * g + 2 == 5 * n - m.nnz
    P.destroy()


def test_closed_form_fem_blocks_are_full():
    m = TINY["C4"]()
    P = host_plan(m, "light=bsell,block=3,sigma=256")
    a, d = P.arrays(), P.describe()
    nblocks = m.nnz // 9
    assert d["census"]["block_fill"]["3"] == pytest.approx(1.0)
    order = a["bsell.origin_brows"]
    nblk = np.diff(m.row_ptr)[0::3] // 3
    pad_blocks = a["bsell.bcols"].size - nblocks
    want_pad = sum(64 * nblk[order[s:s + 64]].max() - nblk[order[s:s + 64]].sum() for s in range(0, order.size, 64))
    assert pad_blocks == want_pad
    assert int(np.count_nonzero(a["bsell.vals"])) == m.nnz
    P.destroy()


def test_closed_form_hybrid_heavy_split_selects_the_generated_rows():
    m = TINY["C5"]()
    for thr in (9, 64, 4999):
        a = host_plan(m, f"heavy={thr},tile=2048,light=sell,sigma=1024").arrays()
        assert np.array_equal(a["heavy.rows"], m.meta["heavy_rows"])
        assert np.count_nonzero(a["heavy.vals"]) == 5 * 5000
        assert "zero.rows" not in a          # heavy rows are summed from scratch, not through atomics


def test_closed_form_pieces_of_full_rows_need_no_padding():
    """Heavy rows of equal length cut into pieces that divide it: every lane is full, and the count of
    units per stripe follows from the counts alone.  20 rows of 4096 entries in one stripe make 20480
    pieces of 4, more than a stripe's 8192 lanes, so the piece length doubles to 16 (5120 lanes)."""
    nh, L, nlight = 20, 4096, 300
    lens = np.concatenate([np.full(nh, L), np.full(nlight, 2)])
    rp = np.zeros(lens.size + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    ci = np.concatenate([np.tile(np.arange(L), nh), np.tile([1, 7], nlight)]).astype(np.int32)
    va = np.arange(1, rp[-1] + 1, dtype=np.float32)
    for piece, eff in ((4, 16), (64, 64), (4096, 4096)):
        spec = f"heavy=64,tile=8192,piece={piece},light=csrv"
        P = lib.Plan(lens.size, L, rp, ci, va, force_plan=spec, host_only=True)
        a = P.arrays()
        lanes = nh * L // eff
        units = -(-lanes // 64)
        assert np.array_equal(a["heavy.sunits"], [0, units])
        assert a["heavy.vals"].size == units * 64 * eff and np.count_nonzero(a["heavy.vals"]) == nh * L
        assert np.array_equal(np.diff(a["heavy.unit_ptr"]), np.full(units, 64 * eff))
        assert np.array_equal(a["heavy.lane_row"][:lanes], np.repeat(np.arange(nh), L // eff))   # stable order: row by row
        want = ref.ref_plan(lens.size, L, rp, ci, va, spec)
        for k in want:
            assert np.array_equal(a[k], want[k]), k
        P.destroy()


def test_heavy_rows_of_a_two_pass_leaf_have_no_reduce_launch_of_their_own():
    """`heavy=..,light=xl`: the heavy launch runs first and the two-pass reduce launch adds its partial sums
    (hptr: heavy rows per row block, hloc: their local rows); with another light design the heavy part keeps
    its own reduce launch."""
    m = TINY["C5"]()
    P = host_plan(m, "heavy=64,tile=2048,light=xl,w=2048,rb=4096")
    assert [q["name"] for q in P.describe()["parts"]] == ["heavy", "xl", "xl.reduce"]
    a = P.arrays()
    hr = a["heavy.rows"]
    assert np.array_equal(hr, m.meta["heavy_rows"])
    assert np.array_equal(a["xl.hloc"], hr % 4096)                       # the part owns every row: position = row
    assert np.array_equal(np.diff(a["xl.hptr"]), np.bincount(hr // 4096, minlength=-(-m.nrows // 4096)))
    P.destroy()
    P = host_plan(m, "heavy=64,tile=2048,light=sell,sigma=1024")
    assert [q["name"] for q in P.describe()["parts"]] == ["sell", "heavy", "heavy.reduce"]
    assert "xl.hptr" not in P.arrays()
    P.destroy()


def test_two_pass_items_keep_a_window_on_one_xcd():
    """Item i of the multiply launch runs on XCD i mod 8: every window's pieces share one residue and follow
    each other there; the pieces of a window tile its entries; fillers are empty and only at the ends."""
    m = TINY["C3"]()
    for spec in ("light=xl,w=256,rb=1024,chunk=64", "light=xl,w=512,rb=512,chunk=4096"):
        P = host_plan(m, spec)
        it = P.arrays()["xl.items"].reshape(-1, 3)
        assert it.shape[0] % 8 == 0
        real = it[:, 2] > it[:, 1]
        assert np.all(it[~real] == 0)
        seen = {}
        for k in range(8):
            lane = it[k::8]
            r = real[k::8]
            assert not np.any(r[np.argmin(r):]) or np.all(r)       # fillers only after the last real item
            lane = lane[r]
            w = lane[:, 0]
            change = np.flatnonzero(np.diff(w)) + 1
            for seg in np.split(np.arange(len(w)), change):
                assert int(w[seg[0]]) not in seen                   # a window appears in one place only
                seen[int(w[seg[0]])] = k
                assert np.array_equal(lane[seg[1:], 1], lane[seg[:-1], 2])   # pieces are adjacent
        counts = [int(real[k::8].sum()) for k in range(8)]
        per_window = np.bincount(it[real, 0])
        assert max(counts) - min(counts) <= per_window.max()        # dealt to the shortest sequence
        assert int((it[real, 2] - it[real, 1]).sum()) == P.arrays()["xl.vals"].size
        P.destroy()


@pytest.mark.parametrize("extra_rows,extra_cols", [(1, 1), (2, 0), (0, 2), (1, 2)])
@pytest.mark.parametrize("spec", ["light=bsell,block=3,sigma=256", "light=bsell,block=3,sigma=2048,xwin=1,remap=1"])
def test_blocks_with_a_ragged_edge(spec, extra_rows, extra_cols):
    """Dimensions that are not multiples of the block edge: whole blocks go to the blocked part, the last
    rows and columns to a CSR part that accumulates; the arrays match the reference and decode to the input."""
    m = TINY["C4"]()
    rng = np.random.default_rng(3)
    A = sp.csr_matrix((m.values, m.col_idx, m.row_ptr), shape=(m.nrows, m.ncols))
    if extra_cols:
        A = sp.hstack([A, sp.random(m.nrows, extra_cols, density=0.3, random_state=1, data_rvs=lambda k: rng.integers(1, 9, k).astype(float))])
    if extra_rows:
        A = sp.vstack([A, sp.random(extra_rows, A.shape[1], density=0.02, random_state=2, data_rvs=lambda k: rng.integers(1, 9, k).astype(float))])
    A = A.tocsr(); A.sort_indices()
    nr, nc = A.shape
    rp, ci, va = A.indptr.astype(np.int32), A.indices.astype(np.int32), A.data.astype(np.float64)
    P = lib.Plan(nr, nc, rp, ci, va, force_plan=spec, host_only=True)
    got = P.arrays()
    names = [q["name"] for q in P.describe()["parts"]]
    P.destroy()
    assert names == ["bsell"] + (["zero"] if extra_rows else []) + ["csrv"]
    want = ref.ref_plan(nr, nc, rp, ci, va, spec)
    assert sorted(got) == sorted(want)
    for k in want:
        assert np.array_equal(got[k], want[k]), k
    if extra_rows:
        assert np.array_equal(got["zero.rows"], np.arange(nr - extra_rows, nr))
    r, c, v = ref.decode(got, nr, nc, block=3)
    assert same_matrix(as_scipy(nr, nc, r, c, v), as_scipy(nr, nc, np.repeat(np.arange(nr), np.diff(rp)), ci, va))


def test_duplicates_and_unsorted_columns_are_accepted():
    rng = np.random.default_rng(5)
    nrows, ncols = 300, 300
    lens = rng.integers(0, 12, nrows)
    rp = np.zeros(nrows + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    r = np.repeat(np.arange(nrows), lens)
    ci = np.clip(r + rng.integers(-3, 4, rp[-1]), 0, ncols - 1).astype(np.int32)   # banded, duplicates, unsorted
    va = rng.integers(-3, 4, rp[-1]).astype(np.float64)
    A_in = as_scipy(nrows, ncols, r, ci, va)
    for spec in ("light=csrv", "light=sell,sigma=64", "dia=1,light=sell", "light=bsell,block=3", "light=bsell,block=2,sigma=32,xwin=1",
                 "heavy=8,tile=64,light=sell"):
        P = lib.Plan(nrows, ncols, rp, ci, va, force_plan=spec, host_only=True)
        assert P.describe()["census"]["cols_sorted"] is False
        p = ref.parse_spec(spec)
        rr, cc, vv = ref.decode(P.arrays(), nrows, ncols, block=p["block"], tile=p["tile"])
        assert same_matrix(as_scipy(nrows, ncols, rr, cc, vv), A_in), spec
        P.destroy()


def test_empty_and_degenerate_matrices():
    z = np.zeros(0)
    for nrows, ncols in ((0, 0), (5, 7), (1, 1)):
        rp = np.zeros(nrows + 1, np.int32)
        for spec in ("light=csrv", "light=sell", "light=bin", "heavy=4,light=sell"):
            P = lib.Plan(nrows, ncols, rp, np.zeros(0, np.int32), z, force_plan=spec, host_only=True)
            assert P.describe()["nnz"] == 0
            P.destroy()
    # search without timing picks a deterministic candidate
    m = TINY["C3"]()
    specs = {lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, search_budget_ms=-1, host_only=True).describe()["spec"]
             for _ in range(2)}
    assert len(specs) == 1


def test_errors():
    m = TINY["C1"]()
    E = lib.SpmvError
    with pytest.raises(E) as e:
        lib.Plan(m.nrows, m.ncols, m.row_ptr[::-1].copy(), m.col_idx, m.values, host_only=True, force_plan="light=csrv")
    assert e.value.status == lib.SPMV_ERR_BAD_CSR
    bad = m.col_idx.copy(); bad[17] = m.ncols
    with pytest.raises(E) as e:
        lib.Plan(m.nrows, m.ncols, m.row_ptr, bad, m.values, host_only=True, force_plan="light=csrv")
    assert e.value.status == lib.SPMV_ERR_BAD_CSR
    with pytest.raises(E) as e:
        lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan="light=csrv", nnz=m.nnz - 1)
    assert e.value.status == lib.SPMV_ERR_BAD_CSR
    for spec in ("light=nope", "lpr=3", "tile=100", "sigma=-2", "block=5", "foo=1", "light", "heavy=4,light=bsell", "piece=16,light=csrv", "heavy=64,piece=6,light=csrv"):
        with pytest.raises(E) as e:
            lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan=spec)
        assert e.value.status == lib.SPMV_ERR_INVALID_ARG, spec
    with pytest.raises(E) as e:      # smaller than one block
        lib.Plan(2, 2, np.array([0, 1, 2], np.int32), np.array([0, 1], np.int32), np.ones(2), host_only=True, force_plan="light=bsell,block=3")
    assert e.value.status == lib.SPMV_ERR_UNSUPPORTED
    with pytest.raises(E) as e:      # no populated diagonal in a random matrix
        lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan="dia=1,light=sell")
    assert e.value.status == lib.SPMV_ERR_UNSUPPORTED
    with pytest.raises(E) as e:      # a search that times candidates needs a device
        lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True)
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG
    with pytest.raises(E) as e:
        lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values.astype(np.float16), host_only=True, force_plan="light=csrv")
    assert e.value.status == lib.SPMV_ERR_UNSUPPORTED
    P = host_plan(m, "light=csrv")
    with pytest.raises(E) as e:      # a host-only plan cannot run
        lib.spmv_run(P.handle, 0x1000, 0x2000, 0)
    assert e.value.status == lib.SPMV_ERR_UNSUPPORTED
    P.destroy()
    lib.spmv_plan_destroy(None)      # NULL is OK


def test_random_matrices_random_plans_decode_to_input():
    """Random shapes under random legal specs, built by the C++ builder in host memory: the arrays
    equal the reference builder's and decode back to the input matrix."""
    rng = np.random.default_rng(7)
    lights = ["csrv,lpr=4,chunk=64", "sell,sigma=64", "bin,smax=4,sigma=64,chunk=128", "nnzb,r=4", "xs,k=8,sigma=128",
              "xnb,k=16,r=8", "xl,w=64,rb=128,chunk=100", "xl,w=512,rb=64", "coo"]
    for case in range(25):
        nrows, ncols = int(rng.integers(1, 700)), int(rng.integers(1, 700))
        lens = rng.integers(0, int(rng.choice([3, 12, 40])), nrows)
        lens[rng.random(nrows) < 0.3] = 0
        for _ in range(int(rng.integers(0, 3))):
            lens[int(rng.integers(0, nrows))] = int(rng.integers(50, 900))
        rp = np.zeros(nrows + 1, np.int32)
        np.cumsum(lens, out=rp[1:])
        r = np.repeat(np.arange(nrows), lens)
        # ascending columns inside a row (the reference builders assume it), repeats allowed
        ci = np.sort(rng.integers(0, ncols, rp[-1]) + r * ncols).astype(np.int64) - r * ncols
        ci = ci.astype(np.int32)
        va = rng.integers(1, 9, rp[-1]).astype(np.float64)
        A_in = as_scipy(nrows, ncols, r, ci, va)
        head = (f"heavy={int(rng.choice([8, 30]))},tile={int(rng.choice([64, 256]))}," + ("hd=1," if rng.random() < 0.5 else "")
                + (f"piece={int(rng.choice([4, 8, 16]))}," if rng.random() < 0.5 else "")) if rng.random() < 0.6 else ""
        spec = head + "light=" + str(rng.choice(lights))
        try:
            P = lib.Plan(nrows, ncols, rp, ci, va, force_plan=spec, host_only=True)
        except lib.SpmvError as e:
            assert e.status == lib.SPMV_ERR_UNSUPPORTED, (spec, e)
            continue
        got = P.arrays()
        want = ref.ref_plan(nrows, ncols, rp, ci, va, spec)
        assert sorted(got) == sorted(want), (case, spec)
        for k in want:
            assert got[k].dtype == want[k].dtype and np.array_equal(got[k], want[k]), (case, spec, k)
        p = ref.parse_spec(spec)
        rr, cc, vv = ref.decode(got, nrows, ncols, block=p["block"], tile=p["tile"], xl_w=p["w"], xl_rb=p["rb"])
        assert same_matrix(as_scipy(nrows, ncols, rr, cc, vv), A_in), (case, spec)
        P.destroy()


# ---- plan trees (the paper's Operator Graph with branches, Section IV-B) ------------------------
TREES = {
    "C1": ["cols(4){light=sell,sigma=256}", "bin2(3){light=sell}{light=csrv,lpr=4}"],
    "C3": ["rows(8:64:1024){light=sell,sigma=128}{light=csrv,lpr=8}{light=csrv,lpr=64}{heavy=1024,tile=512,light=csrv}",
           "rows(16:256){light=xl,w=512,rb=1024}{light=nnzb,r=8}{heavy=256,tile=1024,hd=1,light=csrv}",
           "bin2(6){light=sell}{light=wbm}", "cut(2:64){light=sell,sigma=0}", "cut(4:1){light=csrv,lpr=16}",
           "rows(64){cols(2){light=sell}{light=xl,w=256,rb=512}}{light=csrv,lpr=64,chunk=512}",
           "cols(3){rows(32){light=xl,w=256,rb=256}{light=csrv,lpr=16}}",
           "rows(100){light=xs,k=8,sigma=256}{light=xnb,k=8,r=4}",
           "rows(64:512){light=xl,w=1024,rb=512}{heavy=64,tile=512,light=csrv}{heavy=512,tile=2048,light=csrv}"],
    "C5": ["cut(8:100){light=sell,sigma=0}", "rows(8){light=xl,w=2048,rb=4096}{heavy=8,tile=2048,hd=1,light=csrv}",
           "rows(4:8){light=sell}{light=coo}{cols(2){heavy=8,tile=1024,light=csrv}}"],
}
TREE_CASES = [(n, s) for n in TREES for s in TREES[n]]


@pytest.mark.parametrize("name,spec", TREE_CASES)
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_plan_trees_match_reference_and_decode_to_input(name, spec, dt):
    m = TINY[name]()
    vals = m.values.astype(dt)
    P = host_plan(m, spec, vals)
    got = P.arrays()
    leaves = {}
    want = ref.ref_plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, spec, leaves)
    assert sorted(got) == sorted(want)
    for k in got:
        assert got[k].dtype == want[k].dtype and np.array_equal(got[k], want[k]), k
    r, c, v = ref.decode(got, m.nrows, m.ncols, leaves=leaves)
    assert same_matrix(as_scipy(m.nrows, m.ncols, r, c, v), as_scipy(m.nrows, m.ncols, np.repeat(np.arange(m.nrows), np.diff(m.row_ptr)), m.col_idx, vals))
    d = P.describe()
    assert sum(part["nnz"] for part in d["parts"]) == m.nnz
    P2 = host_plan(m, d["spec"], vals)                       # the printed tree parses back to itself
    assert P2.describe()["spec"] == d["spec"] and P2.describe()["operators"] == d["operators"]
    P.destroy(); P2.destroy()


def test_row_classes_of_a_tree_partition_the_rows():
    """ROW_DIV by length class: child i owns exactly the rows with c_i < length <= c_(i+1); the
    HYB-like cut of the hybrid family (lengths 2..8 against 5000) is found by the ratio rule."""
    m = TINY["C3"]()
    lens = np.diff(m.row_ptr)
    a = host_plan(m, "rows(8:64){light=csrv,lpr=1,sigma=1}{light=csrv,lpr=8,sigma=1}{light=csrv,lpr=64,sigma=1}").arrays()
    for i, (lo, hi) in enumerate([(-1, 8), (8, 64), (64, 10 ** 9)]):
        rows = np.sort(a[f"r{i}.csrv.seg_row"])
        assert np.array_equal(rows, np.flatnonzero((lens > lo) & (lens <= hi)))
    m5 = TINY["C5"]()
    a5 = host_plan(m5, "cut(8:1){light=csrv,lpr=1,sigma=1}").arrays()
    assert np.array_equal(np.sort(a5["p0.csrv.seg_row"]), m5.meta["heavy_rows"])       # the five rows of 5000
    assert a5["p1.csrv.seg_row"].size == m5.nrows - 5
    a2 = host_plan(m, "bin2(4){light=csrv,lpr=1,sigma=1}{light=csrv,lpr=1,sigma=1}").arrays()
    for b in range(5):
        if f"b{b}.csrv.seg_row" in a2:
            L = lens[a2[f"b{b}.csrv.seg_row"]]
            assert np.all(L < 2) if b == 0 else (np.all(L >= 2 ** b) and (b == 4 or np.all(L < 2 ** (b + 1))))


@pytest.mark.parametrize("spec", ["rows(8){light=sell}", "rows(8:4){light=sell}", "rows(){light=sell}", "bin2(4){light=sell}",
                                  "cut(1:5){light=sell}", "cols(1){light=sell}", "cols(3){light=sell}{light=sell}",
                                  "rows(8){dia=1,light=sell}{light=sell}", "rows(8){light=bsell}{light=sell}", "rows(8){light=sell}{light=sell",
                                  "rows(8{light=sell}{light=sell}", "light=sell}", "rows(8)light=sell"])
def test_malformed_trees_are_refused(spec):
    m = TINY["C1"]()
    if spec == "rows(8){light=sell}":
        host_plan(m, spec).destroy()          # one design for every class is legal
        return
    with pytest.raises(lib.SpmvError) as e:
        host_plan(m, spec)
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG
