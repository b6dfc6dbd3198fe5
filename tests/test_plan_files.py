"""Plan files: a plan written with spmv_plan_save and read back with spmv_plan_load is the same plan
(spec, launch list, every format array bit for bit), without the matrix; damaged files are refused.
Host-only plans make this checkable without a GPU."""
import numpy as np
import pytest

import inputs
import paper_2212_10432_amd as lib

CASES = [
    ("C1", "light=csrv,lpr=4,sigma=128"), ("C1", "light=xl,w=1024,rb=2048,chunk=4096"),
    ("C2", "dia=1,dia_fill=0.999,light=sell"), ("C2", "dia=1,drows=2,light=sell"),
    ("C3", "heavy=1024,tile=2048,hd=1,light=xl"), ("C3", "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=512"),
    ("C3", "light=nnzb,r=8"), ("C4", "light=bsell,block=3,sigma=2048,xwin=1,remap=1"),
    ("C5", "heavy=64,tile=2048,light=xnb,k=32,r=4"), ("C5", "heavy=64,tile=2048,light=xs,k=16,sigma=1024"),
]


@pytest.mark.parametrize("name,spec", CASES)
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_round_trip_is_the_same_plan(tmp_path, name, spec, dt):
    m = inputs.SMALL[name]()
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values.astype(dt), force_plan=spec, host_only=True)
    path = str(tmp_path / "plan.bin")
    P.save(path)
    Q = lib.Plan.load(path, host_only=True)
    assert (Q.nrows, Q.ncols, Q.value_dtype) == (m.nrows, m.ncols, np.dtype(dt))
    a, b = P.arrays(), Q.arrays()
    assert list(a) == list(b)
    for k in a:
        assert a[k].dtype == b[k].dtype and np.array_equal(a[k], b[k]), k
    da, db = P.describe(), Q.describe()
    assert da == db
    assert P.bytes() == Q.bytes() and P.launch_names() == Q.launch_names()
    P.destroy(); Q.destroy()


def test_damaged_files_are_refused(tmp_path):
    m = inputs.SMALL["C3"]()
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan="heavy=1024,tile=2048,light=xl", host_only=True)
    path = str(tmp_path / "plan.bin")
    P.save(path)
    P.destroy()
    good = open(path, "rb").read()
    cases = {
        "empty": b"", "short": good[:10], "truncated": good[: len(good) // 2], "longer": good + b"\0",
        "magic": b"X" + good[1:], "flipped": good[:4000] + bytes([good[4000] ^ 1]) + good[4001:],
        "size": good[:8] + (2 ** 50).to_bytes(8, "little") + good[16:], "text": b"%%MatrixMarket matrix coordinate real general\n",
    }
    for what, data in cases.items():
        bad = str(tmp_path / f"{what}.bin")
        open(bad, "wb").write(data)
        with pytest.raises(lib.SpmvError) as e:
            lib.spmv_plan_load(bad, host_only=True)
        assert e.value.status == lib.SPMV_ERR_INVALID_ARG, what
    with pytest.raises(lib.SpmvError) as e:
        lib.spmv_plan_load(str(tmp_path / "missing.bin"), host_only=True)
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG
    Q = lib.Plan.load(path, host_only=True)       # the undamaged file still loads
    Q.destroy()


def test_save_to_an_unwritable_path(tmp_path):
    m = inputs.SMALL["C1"]()
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan="light=sell", host_only=True)
    with pytest.raises(lib.SpmvError) as e:
        P.save(str(tmp_path / "no_such_dir" / "plan.bin"))
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG
    P.destroy()
