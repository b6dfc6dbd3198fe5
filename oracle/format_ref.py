"""TEST ORACLE -- not part of the product.  Reference format builders and decoders in NumPy.

The library's host builder (C++) turns CSR into operator-composed layouts.  This module restates
each layout from its definition, independently and slowly, so that the library's index arrays can
be compared bit for bit, and decodes any plan's arrays back to (row, col, value) triples so that
"the layout still holds exactly the input matrix" can be checked for every plan.

Operators follow Table II of the paper; the readings of what it leaves open are:
  SORT / SORT_SUB  stable, decreasing row length; windows of sigma rows from the part's first row
  *_PAD            pad every row of a 64-row slice to the slice's longest row with value 0 and the
                   column of the row's last real entry (an empty row takes the first column of the
                   slice's first row, 0 if that is empty too)
  BIN              three bins: length <= smax, <= 128, > 128
  ROW_DIV (heavy)  rows longer than the threshold
  COL_DIV (heavy)  stripes of `tile` columns; SORT_BMTB inside a stripe: heavy rows by decreasing
                   entries in that stripe (stable); slices of 64 rows padded with (value 0, column 0)
Diagonal extraction, heavy-row split and dense blocks are the strategies Section VII-F names as
missing from the paper; they are built from their textbook definitions.

Parity pins: tests/test_format_host.py checks these builders against closed forms (C1: stable sort
is the identity and padding is zero; C2: five diagonals at {-g,-1,0,1,g} with 4g explicit zeros;
C4: 3x3 fill is 100 %; C5: the heavy split selects exactly the generator's heavy rows; uniform rows:
CSR segments, nnz-balanced tiles and wavefront bitmaps at their closed-form places), against layouts
written out by hand (two-pass part: a 128 x 128 diagonal + anti-diagonal matrix; XCD-striped SELL and
XCD-striped tiles: 64 rows with one entry in each of 16 stripes; heavy pieces: 20 full rows), and checks
that decode(reference arrays) reproduces the input matrix for every plan.
"""
from __future__ import annotations

import numpy as np

WAVE = 64


def parse_spec(spec: str) -> dict:
    d = dict(dia=0, dia_fill=0.5, heavy=0, tile=8192, light="csrv", lpr=0, chunk=0,
             sigma=0, block=3, smax=16, remap=0, xwin=0, k=8, r=8, w=0, rb=16384, hd=0, piece=0)
    for tok in spec.split(","):
        if not tok:
            continue
        k, v = tok.split("=")
        d[k] = v if k == "light" else (float(v) if k == "dia_fill" else int(float(v)))
    return d


def parse_tree(spec: str) -> dict:
    """Plan tree: a flat spec is a leaf; rows(c1:..:cn){..}.., bin2(k){..}{..}, cut(rho:min){..} and
    cols(k){..}.. divide the rows or columns of their sub-matrix among their children."""
    t = spec.strip()
    for word in ("rows", "bin2", "cut", "cols"):
        if t.startswith(word + "("):
            close = t.index(")")
            cuts = [int(v) for v in t[len(word) + 1:close].split(":")]
            kids, pos = [], close + 1
            while pos < len(t):
                assert t[pos] == "{", t
                level, q = 0, pos
                while True:
                    level += t[q] == "{"
                    level -= t[q] == "}"
                    if level == 0:
                        break
                    q += 1
                kids.append(parse_tree(t[pos + 1:q]))
                pos = q + 1
            return dict(node=word, cuts=cuts, kids=kids)
    d = parse_spec(t)
    d["node"] = "leaf"
    return d


def _sort_rows(rows, lens, sigma):
    rows = np.asarray(rows, dtype=np.int32)
    if sigma == 0 or rows.size < 2:
        return rows
    win = rows.size if sigma < 0 else sigma
    out = []
    for b in range(0, rows.size, win):
        w = rows[b:b + win]
        out.append(w[np.argsort(-lens[w], kind="stable")])
    return np.concatenate(out)


def _row_entries(rp, r):
    return slice(int(rp[r]), int(rp[r + 1]))


def ref_sell(rp, ci, va, rows, sigma, nrows_total, name):
    lens = np.diff(rp).astype(np.int64)
    rows = np.asarray(rows, dtype=np.int32)
    if rows.size == 0:
        return {}
    ident = sigma == 0 and rows.size == nrows_total and np.array_equal(rows, np.arange(nrows_total))
    order = _sort_rows(rows, lens, sigma)
    n = order.size
    nsl = -(-n // WAVE)
    slice_ptr = np.zeros(nsl + 1, dtype=np.int64)
    for s in range(nsl):
        slice_ptr[s + 1] = slice_ptr[s] + WAVE * lens[order[s * WAVE:(s + 1) * WAVE]].max()
    cols = np.zeros(slice_ptr[-1], dtype=np.int32)
    vals = np.zeros(slice_ptr[-1], dtype=va.dtype)
    for s in range(nsl):
        base, w = slice_ptr[s], (slice_ptr[s + 1] - slice_ptr[s]) // WAVE
        e0 = _row_entries(rp, order[s * WAVE])
        fallback = ci[e0.start] if e0.stop > e0.start else 0
        for lane in range(WAVE):
            i = s * WAVE + lane
            pos = base + lane + WAVE * np.arange(w)
            if i < n:
                e = _row_entries(rp, order[i])
                L = e.stop - e.start
                cols[pos[:L]] = ci[e]
                vals[pos[:L]] = va[e]
                cols[pos[L:]] = ci[e.stop - 1] if L else fallback
            else:
                cols[pos] = fallback
    out = {name + ".slice_ptr": slice_ptr, name + ".cols": cols, name + ".vals": vals}
    if not ident:
        out[name + ".origin_rows"] = order
    return out


def ref_csrv(rp, ci, va, rows, lpr, chunk, sigma, acc, nrows_total, name, zero_rows):
    lens = np.diff(rp).astype(np.int64)
    rows = np.asarray(rows, dtype=np.int32)
    if rows.size == 0:
        return {}
    split = chunk > 0 and lens[rows].max() > chunk
    ident = (not split) and sigma == 0 and rows.size == nrows_total and np.array_equal(rows, np.arange(nrows_total))
    if ident:
        return {name + ".seg_ptr": np.asarray(rp, dtype=np.int32), name + ".cols": ci, name + ".vals": va}
    order = _sort_rows(rows, lens, sigma)
    seg_ptr, seg_row, cols, vals, pos = [], [], [], [], 0
    for r in order:
        e = _row_entries(rp, r)
        L = e.stop - e.start
        if split and L > chunk:
            if not acc:
                zero_rows.append(int(r))
            for o in range(0, L, chunk):
                seg_ptr.append(pos + o)
                seg_row.append(~int(r))
        else:
            seg_ptr.append(pos)
            seg_row.append(int(r))
        cols.append(ci[e])
        vals.append(va[e])
        pos += L
    seg_ptr.append(pos)
    return {name + ".seg_ptr": np.array(seg_ptr, dtype=np.int32), name + ".seg_row": np.array(seg_row, dtype=np.int32),
            name + ".cols": np.concatenate(cols).astype(np.int32), name + ".vals": np.concatenate(vals).astype(va.dtype)}


def diag_census(nrows, ncols, rp, ci, fill=0.5):
    """Offsets whose population (entries / rows where the offset stays inside the matrix) >= fill."""
    r = np.repeat(np.arange(nrows, dtype=np.int64), np.diff(rp))
    off, cnt = np.unique(ci.astype(np.int64) - r, return_counts=True)
    keep = []
    for o, c in zip(off, cnt):
        valid = min(nrows, ncols - o) - max(0, -o)
        if valid > 0 and c >= fill * valid and 2 * c >= valid:
            keep.append(int(o))
    return np.array(keep, dtype=np.int32)


def ref_dia(nrows, ncols, rp, ci, va, offs):
    ld = -(-nrows // WAVE) * WAVE
    r = np.repeat(np.arange(nrows, dtype=np.int64), np.diff(rp))
    off = ci.astype(np.int64) - r
    on = np.isin(off, offs)
    dv = np.zeros((len(offs), ld), dtype=va.dtype)
    d_idx = np.searchsorted(offs, off[on])
    np.add.at(dv, (d_idx, r[on]), va[on])
    rem_rp = np.zeros(nrows + 1, dtype=np.int32)
    np.cumsum(np.bincount(r[~on], minlength=nrows), out=rem_rp[1:])
    return {"dia.offsets": np.asarray(offs, dtype=np.int32), "dia.vals": dv.reshape(-1)}, (rem_rp, ci[~on], va[~on])


def _block_value_pos(B, itemsize, q):
    """Position, inside the 64*B*B-value record of one block, of value q = B*ri + ci of each lane:
    the first NV*V values of a lane are packed in vectors of V = 16/itemsize (vector p of lane l at
    V*(64*p + l)), the rest follow one per lane.  Returns (offset, lane stride)."""
    BB, V = B * B, 16 // itemsize
    NV = BB // V
    if q < NV * V:
        return (q // V) * WAVE * V + (q % V), V
    return NV * V * WAVE + (q - NV * V) * WAVE, 1


def ref_bsell(nrows, ncols, rp, ci, va, B, sigma, xwin=0):
    nb = nrows // B
    bcl = []
    for br in range(nb):
        e = slice(int(rp[br * B]), int(rp[(br + 1) * B]))
        bcl.append(np.unique(ci[e] // B))
    nblk = np.array([len(b) for b in bcl], dtype=np.int64)
    order = _sort_rows(np.arange(nb, dtype=np.int32), nblk, sigma)
    nsl = -(-nb // WAVE)
    slice_ptr = np.zeros(nsl + 1, dtype=np.int64)
    for s in range(nsl):
        slice_ptr[s + 1] = slice_ptr[s] + WAVE * nblk[order[s * WAVE:(s + 1) * WAVE]].max()
    bcols = np.zeros(slice_ptr[-1], dtype=np.int32)
    vals = np.zeros(slice_ptr[-1] * B * B, dtype=va.dtype)
    for s in range(nsl):
        base, w = slice_ptr[s], (slice_ptr[s + 1] - slice_ptr[s]) // WAVE
        first = bcl[order[s * WAVE]]
        fallback = first[0] if len(first) else 0
        for lane in range(WAVE):
            i = s * WAVE + lane
            if i >= nb:
                bcols[base + lane + WAVE * np.arange(w)] = fallback
                continue
            br = order[i]
            bc = bcl[br]
            L = len(bc)
            bcols[base + lane + WAVE * np.arange(L)] = bc
            bcols[base + lane + WAVE * np.arange(L, w)] = bc[-1] if L else fallback
            for ri in range(B):
                e = _row_entries(rp, br * B + ri)
                j = np.searchsorted(bc, ci[e] // B)
                for jj, cc, vv in zip(j, ci[e], va[e]):
                    off, stride = _block_value_pos(B, va.dtype.itemsize, ri * B + int(cc) % B)
                    vals[(base + jj * WAVE) * B * B + off + stride * lane] += vv
    out = {"bsell.slice_ptr": slice_ptr, "bsell.bcols": bcols, "bsell.vals": vals}
    if sigma != 0:
        out["bsell.origin_brows"] = order
    if xwin:
        G = 32                                   # slices per workgroup
        win = []
        for g in range(-(-nsl // G)):
            seg = bcols[slice_ptr[g * G]:slice_ptr[min(nsl, (g + 1) * G)]]
            lo, hi = (int(seg.min()), int(seg.max())) if seg.size else (0, -1)
            win += [lo * B, (hi - lo + 1) * B]
        out["bsell.xwin"] = np.array(win, dtype=np.int32)
        # index compression: the block column as a 16-bit offset from the group's first block column
        local = np.zeros(bcols.size, dtype=np.uint16)
        for g in range(-(-nsl // G)):
            b0, b1 = slice_ptr[g * G], slice_ptr[min(nsl, (g + 1) * G)]
            local[b0:b1] = bcols[b0:b1] - win[2 * g] // B
        del out["bsell.bcols"]
        out["bsell.bcols16"] = local
    return out


def _count_pieces(rowseg, P, delta):
    """Number of pieces when every segment is cut greedily into runs of stored length <= P."""
    total = 0
    for lc, _ in rowseg:
        if lc.size == 0:
            continue
        if delta:
            gap = np.diff(lc)
            cost = np.concatenate([[1], 1 + np.where(gap > 255, (gap - 1) // 255, 0)])
        else:
            cost = np.ones(lc.size, dtype=np.int64)
        stored = 0
        for k, c in enumerate(cost):
            if k == 0 or stored + c > P:
                total += 1
                stored = 1           # the first entry of a run stores no bridges
            else:
                stored += c
    return total


def ref_stripe(ncols, rp, ci, va, hrows, tile, delta=0, piece=0):
    """Heavy rows cut into column stripes; inside a stripe the rows are ordered by decreasing number
    of entries in that stripe (stable), sliced by 64 and padded per slice (value 0, local column 0).

    delta=1: 8-bit column differences.  A lane with local columns c_0 <= c_1 <= ... is stored as the
    byte sequence d_0 = 0, d_k = c_k - c_(k-1), where a gap g > 255 is first bridged by
    (g - 1) // 255 entries (255, value 0).  Lanes are ordered by the stored length (entries +
    bridges), a slice is padded with (0, 0) to its longest lane rounded up to a multiple of 4.
    lane_meta = c_0 << 16 | heavy row (0xFFFF: none).  dcols packs entries 4q..4q+3 of a lane into
    one little-endian 32-bit word at unit_ptr[u] / 4 + 64 q + lane.

    piece=P>0: a (row, stripe) segment is cut into runs of at most P stored entries (a run takes entries
    while its stored length, bridges included, stays within P; the run after it starts with an absolute
    column, so the bridges of the gap between them are not stored), every run a lane of its own (rows
    without entries in the stripe take none); P doubles for a stripe until it has at most 8192 lanes.
    sunits[s] = first unit of stripe s."""
    nh = len(hrows)
    if nh == 0:
        return {}
    ns = -(-ncols // tile)
    unit_ptr, sunits = [0], [0]
    lane_row, lane_meta = [], []
    lcols, vals = [], []

    def encode(lc, vv):
        if not delta:
            return lc.astype(np.uint16), vv, 0
        d, v2 = [], []
        for k in range(lc.size):
            gap = int(lc[k] - lc[k - 1]) if k else 0
            while gap > 255:
                d.append(255); v2.append(0.0); gap -= 255
            d.append(gap); v2.append(vv[k])
        return np.array(d, dtype=np.uint8), np.array(v2, dtype=va.dtype), int(lc[0]) if lc.size else 0

    for s in range(ns):
        rowseg = []
        for r in hrows:
            e = _row_entries(rp, r)
            c = ci[e]
            m = (c >= s * tile) & (c < (s + 1) * tile)
            rowseg.append(((c[m] - s * tile).astype(np.int64), va[e][m]))
        lanes = []                                # (heavy row, stored columns, stored values, first column)
        if piece <= 0:
            for h, (lc, vv) in enumerate(rowseg):
                lanes.append((h,) + encode(lc, vv))
        else:
            P = piece
            while _count_pieces(rowseg, P, delta) > 8192:
                P *= 2
            for h, (lc, vv) in enumerate(rowseg):
                o = 0
                while o < lc.size:       # a piece takes entries while its stored length stays within P
                    n = 1
                    while o + n < lc.size and len(encode(lc[o:o + n + 1], vv[o:o + n + 1])[0]) <= P:
                        n += 1
                    lanes.append((h,) + encode(lc[o:o + n], vv[o:o + n]))
                    o += n
        key = np.array([len(l[1]) for l in lanes], dtype=np.int64)
        order = np.argsort(-key, kind="stable")
        nu = -(-len(lanes) // WAVE)
        sunits.append(sunits[-1] + nu)
        for g in range(nu):
            members = order[g * WAVE:(g + 1) * WAVE]
            w = int(key[members[0]])
            if delta:
                w = -(-w // 4) * 4
            lc = np.zeros((w, WAVE), dtype=np.uint8 if delta else np.uint16)
            vv = np.zeros((w, WAVE), dtype=va.dtype)
            lr = np.full(WAVE, 0xFFFF, dtype=np.uint16)
            lm = np.full(WAVE, 0xFFFF, dtype=np.uint32)
            for lane, i in enumerate(members):
                h, cc, v2, c0 = lanes[i]
                lc[:len(cc), lane] = cc
                vv[:len(cc), lane] = v2
                lr[lane] = h
                lm[lane] = (c0 << 16) | h
            if delta:   # (w, 64) -> words: [w/4][lane][4]
                lc = lc.reshape(w // 4, 4, WAVE).transpose(0, 2, 1)
            lcols.append(lc.reshape(-1))
            vals.append(vv.reshape(-1))
            lane_row.append(lr)
            lane_meta.append(lm)
            unit_ptr.append(unit_ptr[-1] + w * WAVE)
    cat = lambda xs, dt: np.concatenate(xs).astype(dt) if xs else np.zeros(0, dtype=dt)
    out = {"heavy.unit_ptr": np.array(unit_ptr, dtype=np.int32),
           "heavy.vals": cat(vals, va.dtype), "heavy.rows": np.asarray(hrows, dtype=np.int32)}
    if delta:
        out["heavy.dcols"] = np.ascontiguousarray(cat(lcols, np.uint8)).view("<u4")
        out["heavy.lane_meta"] = cat(lane_meta, np.uint32)
    else:
        out["heavy.lcols"] = cat(lcols, np.uint16)
        out["heavy.lane_row"] = cat(lane_row, np.uint16)
    if piece > 0:
        out["heavy.sunits"] = np.array(sunits, dtype=np.int32)
    return out


def ref_xs(ncols, rp, ci, va, rows, K, sigma, nrows_total):
    """XCD-striped SELL: K column stripes of W = ceil(ncols/K) (rounded up to 64) columns; stripe s
    belongs to XCD s mod 8.  Per stripe and per window of sigma part positions, the rows with entries
    in the stripe are sorted by that count (stable, decreasing), sliced by 64 and padded.  Units are
    ordered XCD by XCD, then stripe, then window.  Lane l of unit u owns scratch slot 64*u + l; pslot
    lists the slots of each row in stripe order, pptr delimits them."""
    rows = np.asarray(rows, dtype=np.int32)
    n = rows.size
    if n == 0:
        return {}
    ident = n == nrows_total and np.array_equal(rows, np.arange(nrows_total))
    W = -(-ncols // K)
    W = max(WAVE, -(-W // WAVE) * WAVE)
    win = n if sigma <= 0 else sigma
    seg = np.zeros((n, K), dtype=np.int64)
    for i, r in enumerate(rows):
        e = _row_entries(rp, r)
        np.add.at(seg[i], ci[e] // W, 1)
    pptr = np.zeros(n + 1, dtype=np.int32)
    np.cumsum((seg > 0).sum(axis=1), out=pptr[1:])
    unit_ptr, cols, vals, xbase = [0], [], [], []
    pslot = np.full(int(pptr[-1]), -1, dtype=np.int32)
    for k in range(8):
        xbase.append(len(unit_ptr) - 1)
        for s in range(k, K, 8):
            for w0 in range(0, n, win):
                part = np.array([i for i in range(w0, min(n, w0 + win)) if seg[i, s] > 0], dtype=np.int64)
                part = part[np.argsort(-seg[part, s], kind="stable")] if part.size else part
                for q in range(0, part.size, WAVE):
                    members = part[q:q + WAVE]
                    w = int(seg[members[0], s])
                    cc = np.zeros((w, WAVE), dtype=np.int32)
                    vv = np.zeros((w, WAVE), dtype=va.dtype)
                    fallback = None
                    u = len(unit_ptr) - 1
                    for lane, i in enumerate(members):
                        e = _row_entries(rp, rows[i])
                        c, v = ci[e], va[e]
                        m = (c // W) == s
                        L = int(m.sum())
                        cc[:L, lane] = c[m]
                        vv[:L, lane] = v[m]
                        cc[L:, lane] = c[m][-1]
                        if lane == 0:
                            fallback = c[m][0]
                        pslot[pptr[i] + int((seg[i, :s] > 0).sum())] = u * WAVE + lane
                    cc[:, len(members):] = fallback
                    cols.append(cc.reshape(-1)); vals.append(vv.reshape(-1))
                    unit_ptr.append(unit_ptr[-1] + w * WAVE)
    xbase.append(len(unit_ptr) - 1)
    cat = lambda parts, dt: np.concatenate(parts).astype(dt) if parts else np.zeros(0, dtype=dt)
    out = {"xs.unit_ptr": np.array(unit_ptr, dtype=np.int64), "xs.cols": cat(cols, np.int32), "xs.vals": cat(vals, va.dtype),
           "xs.pslot": pslot, "xs.xbase": np.array(xbase, dtype=np.int64), "xs.pptr": pptr}
    if not ident:
        out["xs.rows"] = rows
    return out


def ref_nnzb(rp, ci, va, rows, R, acc, zero_rows):
    """nnz-balanced tiles: the entries of the part's non-empty rows form one stream; lane l of tile i
    holds the R consecutive entries from 64*R*i + R*l, stored at 64*R*i + 64*t + l (t < R); bit t of
    bits[64*i + l] marks an entry that starts a row; tile_row[i] counts the row starts before tile i.
    Rows open at a tile border, and empty rows, are zeroed by an earlier launch."""
    lens = np.diff(rp).astype(np.int64)
    keep = [int(r) for r in rows if lens[r] > 0]
    if not acc:
        zero_rows += [int(r) for r in rows if lens[r] == 0]
    if not keep:
        return {}
    stream_c = np.concatenate([ci[_row_entries(rp, r)] for r in keep])
    stream_v = np.concatenate([va[_row_entries(rp, r)] for r in keep])
    starts = np.concatenate([[0], np.cumsum(lens[keep])])[:-1]
    total = stream_c.size
    tsz = WAVE * R
    ntiles = -(-total // tsz)
    g = np.arange(ntiles * tsz)
    dst = (g // tsz) * tsz + ((g % tsz) % R) * WAVE + (g % tsz) // R
    cols = np.zeros(ntiles * tsz, dtype=np.int32)
    vals = np.zeros(ntiles * tsz, dtype=va.dtype)
    cols[dst[:total]] = stream_c
    vals[dst[:total]] = stream_v
    bits = np.zeros(ntiles * WAVE, dtype=np.uint8 if R <= 8 else np.uint16)
    for st in starts:
        bits[(st // tsz) * WAVE + (st % tsz) // R] |= 1 << ((st % tsz) % R)
    tile_row = np.zeros(ntiles + 1, dtype=np.int32)
    np.cumsum(np.bincount(starts // tsz, minlength=ntiles), out=tile_row[1:])
    if not acc:
        owner = np.repeat(np.arange(len(keep)), lens[keep])          # stream position -> row index
        for t in range(ntiles):
            zero_rows.append(keep[owner[min(total, (t + 1) * tsz) - 1]])
            if starts[owner[t * tsz]] != t * tsz:
                zero_rows.append(keep[owner[t * tsz]])
    return {"nnzb.cols": cols, "nnzb.vals": vals, "nnzb.bits": bits, "nnzb.tile_row": tile_row,
            "nnzb.rows": np.array(keep, dtype=np.int32)}


def ref_wbm(rp, ci, va, rows, acc, zero_rows, steps=8):
    """One entry per lane, one row-start bitmap per wavefront step: the entries of the part's non-empty
    rows form one stream, stored as it is and padded with (value 0, column 0) to a whole tile of
    64*steps entries; bit g % 64 of mask[g // 64] marks an entry that starts a row; tile_row[i] counts
    the row starts before tile i.  Rows open at a tile border, and empty rows, are zeroed first."""
    lens = np.diff(rp).astype(np.int64)
    keep = [int(r) for r in rows if lens[r] > 0]
    if not acc:
        zero_rows += [int(r) for r in rows if lens[r] == 0]
    if not keep:
        return {}
    stream_c = np.concatenate([ci[_row_entries(rp, r)] for r in keep])
    stream_v = np.concatenate([va[_row_entries(rp, r)] for r in keep])
    starts = np.concatenate([[0], np.cumsum(lens[keep])])[:-1]
    total = stream_c.size
    tsz = WAVE * steps
    ntiles = -(-total // tsz)
    cols = np.zeros(ntiles * tsz, dtype=np.int32)
    vals = np.zeros(ntiles * tsz, dtype=va.dtype)
    cols[:total] = stream_c
    vals[:total] = stream_v
    mask = np.zeros(ntiles * steps, dtype=np.uint64)
    for st in starts:
        mask[st // WAVE] |= np.uint64(1) << np.uint64(st % WAVE)
    tile_row = np.zeros(ntiles + 1, dtype=np.int32)
    np.cumsum(np.bincount(starts // tsz, minlength=ntiles), out=tile_row[1:])
    if not acc:
        owner = np.repeat(np.arange(len(keep)), lens[keep])
        for t in range(ntiles):
            zero_rows.append(keep[owner[min(total, (t + 1) * tsz) - 1]])
            if starts[owner[t * tsz]] != t * tsz:
                zero_rows.append(keep[owner[t * tsz]])
    return {"wbm.cols": cols, "wbm.vals": vals, "wbm.mask": mask, "wbm.tile_row": tile_row,
            "wbm.rows": np.array(keep, dtype=np.int32)}


def ref_xnb(ncols, rp, ci, va, rows, K, R, nrows_total):
    """XCD-striped nnz-balanced tiles.  K stripes of W = ceil(ncols/K) (rounded up to 64) columns, XCD k
    owning stripes k, k+8, ...; the streams are laid out XCD by XCD.  Inside a stripe the (row, stripe)
    segments follow each other in part order; the stream is padded to whole tiles of 64*R entries with
    (value 0, first column of the stripe) and stored transposed per tile.  Segments are numbered in
    stream order.  seg_row[q]: part position of segment q's row modulo 1024; bbase[b*K + s]: number of
    the first segment of stripe s at or after part position 1024*b (row nblk: end of the stripe)."""
    rows = np.asarray(rows, dtype=np.int32)
    n = rows.size
    if n == 0:
        return {}
    ident = n == nrows_total and np.array_equal(rows, np.arange(nrows_total))
    W = -(-ncols // K)
    W = max(WAVE, -(-W // WAVE) * WAVE)
    tsz = WAVE * R
    BLK = 1024
    nblk = -(-n // BLK)
    bbase = np.zeros((nblk + 1) * K, dtype=np.int32)
    seg_row = []
    cols, vals, marks, xbase = [], [], [], []
    ntiles = nsegs = 0
    for k in range(8):
        xbase.append(ntiles)
        for s in range(k, K, 8):
            sc, sv, sm = [], [], []
            q = nsegs
            for i, r in enumerate(rows):
                if i % BLK == 0:
                    bbase[(i // BLK) * K + s] = q
                e = _row_entries(rp, r)
                m = (ci[e] // W) == s
                L = int(m.sum())
                if L:
                    sc.append(ci[e][m]); sv.append(va[e][m])
                    sm.append(np.concatenate([[1], np.zeros(L - 1, dtype=np.int64)]))
                    seg_row.append(i % BLK)
                    q += 1
            bbase[nblk * K + s] = q
            nsegs = q
            if not sc:
                continue
            sc, sv, sm = np.concatenate(sc), np.concatenate(sv), np.concatenate(sm)
            pad = -sc.size % tsz
            cols.append(np.concatenate([sc, np.full(pad, min(s * W, ncols - 1), dtype=np.int32)]))
            vals.append(np.concatenate([sv, np.zeros(pad, dtype=va.dtype)]))
            marks.append(np.concatenate([sm, np.zeros(pad, dtype=np.int64)]))
            ntiles += (sc.size + pad) // tsz
    xbase.append(ntiles)
    if ntiles:
        cols, vals, marks = np.concatenate(cols), np.concatenate(vals), np.concatenate(marks)
    else:
        cols, vals, marks = np.zeros(0, np.int32), np.zeros(0, va.dtype), np.zeros(0, np.int64)
    g = np.arange(ntiles * tsz)
    dst = (g // tsz) * tsz + ((g % tsz) % R) * WAVE + (g % tsz) // R
    tc = np.zeros(ntiles * tsz, dtype=np.int32); tv = np.zeros(ntiles * tsz, dtype=va.dtype)
    tc[dst] = cols; tv[dst] = vals
    bits = np.zeros(ntiles * WAVE, dtype=np.uint8 if R <= 8 else np.uint16)
    pos = np.flatnonzero(marks)
    np.bitwise_or.at(bits, (pos // tsz) * WAVE + (pos % tsz) // R, (1 << ((pos % tsz) % R)).astype(bits.dtype))
    tile_row = np.zeros(ntiles + 1, dtype=np.int32)
    np.cumsum(np.bincount(pos // tsz, minlength=ntiles), out=tile_row[1:])
    out = {"xnb.cols": tc, "xnb.vals": tv.astype(va.dtype), "xnb.bits": bits, "xnb.tile_row": tile_row,
           "xnb.xbase": np.array(xbase, dtype=np.int64), "xnb.seg_row": np.array(seg_row, dtype=np.uint16),
           "xnb.bbase": bbase}
    opens = set()
    for t in range(ntiles):
        if not marks[t * tsz]:
            opens.add(int(tile_row[t]) - 1)
        opens.add(int(tile_row[t + 1]) - 1)
    if opens:
        out["xnb.open_slots"] = np.array(sorted(opens), dtype=np.int32)
    if not ident:
        out["xnb.rows"] = rows
    return out


def ref_xl(ncols, rp, ci, va, rows, W, RB, chunk, nrows_total, skip=()):
    """Two passes with x windows in LDS.  Windows of W columns (0: 64 KiB worth of values), blocks of
    RB part positions.  Entry (part position i, column c) is in run (s, b) = (c // W, i // RB); runs
    are stored window by window, block by block inside a window, by part position and row order
    inside a run; a run is padded to a whole 16-byte vector (N = 2 doubles / 4 floats), a window to 16
    entries, with (value 0, local column 0).
    items: (window, first entry, end entry) pieces of a window's entries, m = ceil(len / chunk)
    pieces of ceil16(ceil(len / m)) entries; chunk 0 means 128 KiB of values.  Item i runs on XCD i mod 8: a window's
    items all go, one after the other, to the XCD that has the fewest items so far (lowest on a tie), the
    eight sequences are interleaved and the shorter ones filled with empty items (0, 0, 0).
    glist: for block b the groups of runs (0, b), (1, b), ...: a run cut into groups of up to 16
    entries, a list entry being 8 * (first entry // N) + (entries in the group // N - 1); gptr: the
    list's offsets per block.  lrow is stored in list order, 16 slots per group: lrow[16 p + t] is the
    local row of entry N * (glist[p] >> 3) + t (0 in unused slots and for padding).
    Rows listed in `skip` stay in the part but contribute no entries (rows of other parts kept so that
    the part's rows are one contiguous range and no row map is stored)."""
    rows = np.asarray(rows, dtype=np.int32)
    n = rows.size
    if n == 0:
        return {}
    ident = n == nrows_total and np.array_equal(rows, np.arange(nrows_total))
    if W == 0:
        W = 65536 // va.dtype.itemsize
    G, N = 16, 16 // va.dtype.itemsize
    S = max(1, -(-ncols // W))
    B = -(-n // RB)
    lens = (rp[rows + 1] - rp[rows]).astype(np.int64)
    lens[np.isin(rows, np.asarray(skip, dtype=np.int64))] = 0               # rows kept in the part without their entries
    pos_of_entry = np.repeat(np.arange(n, dtype=np.int64), lens)           # part position i
    src = np.concatenate([np.arange(rp[r], rp[r] + L, dtype=np.int64) for r, L in zip(rows, lens)]) if lens.sum() else np.zeros(0, np.int64)
    c = ci[src].astype(np.int64)
    run = (c // W) * B + pos_of_entry // RB
    order = np.argsort(run, kind="stable")                                   # keeps (i, row order) inside a run
    cnt = np.bincount(run, minlength=S * B).astype(np.int64).reshape(S, B)
    ceil_to = lambda v, q: -(-v // q) * q
    padded = ceil_to(cnt, N)                                                 # a run holds whole 16-byte vectors
    wstart = np.concatenate([[0], np.cumsum(ceil_to(padded.sum(axis=1), G))])   # a window starts on a multiple of 16
    tot = int(wstart[-1])
    rbeg = wstart[:-1, None] + np.cumsum(padded, axis=1) - padded            # (S, B): first entry of run (s, b)
    vals = np.zeros(tot, dtype=va.dtype)
    lcol = np.zeros(tot, dtype=np.uint16)
    lrow_by_entry = np.zeros(tot, dtype=np.uint16)
    run_sorted = run[order]
    first = np.concatenate([[0], np.cumsum(cnt.reshape(-1))])[run_sorted]  # rank of the run's first entry among the real entries
    dst = rbeg.reshape(-1)[run_sorted] + (np.arange(order.size) - first)
    vals[dst] = va[src[order]]
    lcol[dst] = (c[order] % W).astype(np.uint16)
    lrow_by_entry[dst] = (pos_of_entry[order] % RB).astype(np.uint16)
    chunk = ceil_to(chunk, G) if chunk > 0 else 131072 // va.dtype.itemsize
    per_xcd = [[] for _ in range(8)]              # items whose number is k mod 8 run on XCD k
    for s_ in range(S):
        b0, e0 = int(wstart[s_]), int(wstart[s_ + 1])
        if e0 == b0:
            continue
        m = -(-(e0 - b0) // chunk)
        per = ceil_to(-(-(e0 - b0) // m), G)
        k = min(range(8), key=lambda q: (len(per_xcd[q]), q))   # the XCD with the fewest items so far
        for cpos in range(b0, e0, per):
            per_xcd[k].append([s_, cpos, min(e0, cpos + per)])
    items = []
    for j in range(max(len(q) for q in per_xcd)):
        for q in per_xcd:
            items += q[j] if j < len(q) else [0, 0, 0]
    gptr = np.zeros(B + 1, dtype=np.int32)
    glist, lrow = [], []
    for b in range(B):
        ng = 0
        for s_ in range(S):
            g0, L = int(rbeg[s_, b]), int(padded[s_, b])
            for off in range(0, L, G):
                ln = min(G, L - off)
                glist.append(((g0 + off) // N) * 8 + (ln // N - 1))
                slot = np.zeros(G, dtype=np.uint16)
                slot[:ln] = lrow_by_entry[g0 + off:g0 + off + ln]
                lrow.append(slot)
                ng += 1
        gptr[b + 1] = gptr[b] + ng
    glist = np.array(glist, dtype=np.int32)
    lrow = np.concatenate(lrow) if lrow else np.zeros(0, np.uint16)
    out = {"xl.vals": vals, "xl.lcol": lcol, "xl.gptr": gptr, "xl.glist": glist, "xl.lrow": lrow}
    if items:
        out["xl.items"] = np.array(items, dtype=np.int32)
    else:
        del out["xl.vals"], out["xl.lcol"]
    if not ident:
        out["xl.rows"] = rows
    return out


def _ref_leaf(nrows, ncols, rp, ci, va, p, rows, whole, acc, span) -> dict:
    """The arrays of one leaf (a flat design) over the rows `rows` (ascending) of the matrix."""
    out = {}
    if p["dia"]:
        assert whole and not acc
        offs = diag_census(nrows, ncols, rp, ci, p["dia_fill"])
        arrays, (rp, ci, va) = ref_dia(nrows, ncols, rp, ci, va, offs)
        out.update(arrays)
        acc = True
        if ci.size == 0:
            return out
    lens = np.diff(rp).astype(np.int64)
    if p["light"] == "bsell":
        assert whole and not acc
        B = p["block"]
        nrB, ncB = nrows // B * B, ncols // B * B
        if nrB == nrows and ncB == ncols:
            out.update(ref_bsell(nrows, ncols, rp, ci, va, B, p["sigma"], p["xwin"]))
            return out
        # ragged edge: whole blocks go to the blocked part, the last rows and columns to a CSR part that
        # accumulates; the rows past the last whole block row are zeroed first
        r_of = np.repeat(np.arange(nrows), np.diff(rp))
        inside = (r_of < nrB) & (ci < ncB)
        rp_m = np.concatenate([[0], np.cumsum(np.bincount(r_of[inside], minlength=nrows)[:nrB])]).astype(np.int32)
        out.update(ref_bsell(nrB, ncB, rp_m, ci[inside], va[inside], B, p["sigma"], p["xwin"]))
        rp_r = np.concatenate([[0], np.cumsum(np.bincount(r_of[~inside], minlength=nrows))]).astype(np.int32)
        with_entries = np.flatnonzero(np.diff(rp_r) > 0).astype(np.int32)
        if with_entries.size:
            out.update(ref_csrv(rp_r, ci[~inside], va[~inside], with_entries, 0, 0, 0, True, nrows, "csrv", []))
        if nrB < nrows:
            out["zero.rows"] = np.arange(nrB, nrows, dtype=np.int32)
        return out
    rows = np.asarray(rows, dtype=np.int32)
    is_heavy = (lens[rows] > p["heavy"]) if p["heavy"] > 0 else np.zeros(rows.size, dtype=bool)
    heavy = rows[is_heavy]
    is_light = ~is_heavy
    if acc:
        is_light &= lens[rows] > 0
    light = rows[is_light]
    zero_rows = []      # rows reduced through atomics (segments of a cut row); heavy rows have their own reduce launch
    if p["light"] == "csrv":
        lpr = p["lpr"]
        out.update(ref_csrv(rp, ci, va, light, lpr, p["chunk"], p["sigma"], acc, nrows, "csrv", zero_rows))
    elif p["light"] == "sell":
        out.update(ref_sell(rp, ci, va, light, p["sigma"], nrows, "sell"))
    elif p["light"] == "coo":
        if light.size:
            out["coo.rows"] = np.repeat(light, lens[light]).astype(np.int32)
            out["coo.cols"] = np.concatenate([ci[_row_entries(rp, r)] for r in light]).astype(np.int32)
            out["coo.vals"] = np.concatenate([va[_row_entries(rp, r)] for r in light]).astype(va.dtype)
            if not acc:
                zero_rows += [int(r) for r in light]
    elif p["light"] == "nnzb":
        out.update(ref_nnzb(rp, ci, va, light, p["r"], acc, zero_rows))
    elif p["light"] == "wbm":
        out.update(ref_wbm(rp, ci, va, light, acc, zero_rows))
    elif p["light"] == "xnb":
        out.update(ref_xnb(ncols, rp, ci, va, light, p["k"], p["r"], nrows))
    elif p["light"] == "xl":
        # the part may own rows it has no entries for: this leaf's heavy rows, or (span) the rows of the
        # sibling leaves that run after it; their own launches overwrite those y elements later
        owner = span if span is not None else (rows if heavy.size else None)
        if not acc and owner is not None:
            owner = np.asarray(owner, dtype=np.int32)
            out.update(ref_xl(ncols, rp, ci, va, owner, p["w"], p["rb"], p["chunk"], nrows, skip=np.setdiff1d(owner, light)))
            if heavy.size:
                # this part's reduce launch also adds the heavy part's partial sums: per block of RB part
                # positions the range of heavy rows in it (hptr) and their local rows (hloc)
                pos = np.searchsorted(owner, heavy)
                assert np.array_equal(owner[pos], heavy)
                nblocks = -(-owner.size // p["rb"])
                hptr = np.concatenate([[0], np.cumsum(np.bincount(pos // p["rb"], minlength=nblocks))]).astype(np.int32)
                out["xl.hptr"] = hptr
                out["xl.hloc"] = (pos % p["rb"]).astype(np.uint16)
        else:
            out.update(ref_xl(ncols, rp, ci, va, light, p["w"], p["rb"], p["chunk"], nrows))
    elif p["light"] == "xs":
        out.update(ref_xs(ncols, rp, ci, va, light, p["k"], p["sigma"], nrows))
    elif p["light"] == "bin":
        L = lens[light]
        out.update(ref_sell(rp, ci, va, light[L <= p["smax"]], p["sigma"], nrows, "bin0.sell"))
        out.update(ref_csrv(rp, ci, va, light[(L > p["smax"]) & (L <= 128)], 8, 0, p["sigma"], acc, nrows, "bin1.csrv8", zero_rows))
        out.update(ref_csrv(rp, ci, va, light[L > max(128, p["smax"])], 256 if p.get("wg") else 64, p["chunk"], 0, acc, nrows,
                            "bin2.csrwg" if p.get("wg") else "bin2.csrv64", zero_rows))
    else:
        raise ValueError(p["light"])
    out.update(ref_stripe(ncols, rp, ci, va, heavy, p["tile"], p["hd"], p.get("piece", 0)))
    if zero_rows:
        out["zero.rows"] = np.array(sorted(set(zero_rows)), dtype=np.int32)
    return out


def _column_stripe(rp, ci, va, rows, c0, c1):
    """The rows `rows` restricted to columns [c0, c1); other rows empty; same row numbering."""
    nrows = rp.size - 1
    keep = np.zeros(ci.size, dtype=bool)
    for r in rows:
        e = _row_entries(rp, r)
        keep[e] = (ci[e] >= c0) & (ci[e] < c1)
    owner = np.repeat(np.arange(nrows), np.diff(rp))
    cnt = np.bincount(owner[keep], minlength=nrows)
    rp2 = np.zeros(nrows + 1, dtype=rp.dtype)
    np.cumsum(cnt, out=rp2[1:])
    return rp2, ci[keep], va[keep]


def _ref_node(nrows, ncols, rp, ci, va, node, rows, whole, acc, span, prefix, out, leaves):
    if node["node"] == "leaf":
        arrays = _ref_leaf(nrows, ncols, rp, ci, va, node, rows, whole, acc, span)
        out.update({prefix + k: v for k, v in arrays.items()})
        leaves[prefix] = node
        return
    kids, cuts = node["kids"], node["cuts"]
    kid = lambda i: kids[0] if len(kids) == 1 else kids[i]
    lens = np.diff(rp).astype(np.int64)
    rows = np.asarray(rows, dtype=np.int32)

    def run_classes(classes, design, tag):
        first = True
        for i, cls in enumerate(classes):
            if len(cls) == 0:
                continue
            k = kid(design[i])
            can_span = (first and not acc and span is None and k["node"] == "leaf" and k["light"] == "xl"
                        and not k["heavy"] and len(cls) < rows.size)
            _ref_node(nrows, ncols, rp, ci, va, k, np.asarray(cls, dtype=np.int32), False, acc,
                      rows if can_span else None, f"{prefix}{tag}{i}.", out, leaves)
            first = False

    if node["node"] == "rows":
        c = np.searchsorted(np.asarray(cuts), lens[rows], side="left")       # cuts[c-1] < L <= cuts[c]
        run_classes([rows[c == i] for i in range(len(cuts) + 1)], list(range(len(cuts) + 1)), "r")
    elif node["node"] == "bin2":
        k2 = cuts[0]
        L = lens[rows]
        b = np.where(L < 2, 0, np.minimum(k2, np.floor(np.log2(np.maximum(L, 1))).astype(np.int64)))
        run_classes([rows[b == i] for i in range(k2 + 1)], [0] * k2 + [1], "b")
    elif node["node"] == "cut":
        rho, minrows = cuts
        order = rows[np.argsort(-lens[rows], kind="stable")]
        classes = [[]]
        for i, r in enumerate(order):
            classes[-1].append(int(r))
            if (i + 1 < order.size and len(classes[-1]) >= minrows and lens[r] > 0
                    and lens[r] >= rho * lens[order[i + 1]]):
                classes.append([])
        run_classes([sorted(c) for c in classes], [0] * len(classes), "p")
    elif node["node"] == "cols":
        K = cuts[0]
        W = -(-ncols // K)
        for j in range(K):
            rp2, ci2, va2 = _column_stripe(rp, ci, va, rows, j * W, min(ncols, (j + 1) * W))
            _ref_node(nrows, ncols, rp2, ci2, va2, kid(j), rows, False, acc or j > 0, None, f"{prefix}c{j}.", out, leaves)
    else:
        raise ValueError(node["node"])


def ref_plan(nrows, ncols, rp, ci, va, spec: str, leaves=None) -> dict:
    """All format arrays of the plan `spec` for a CSR matrix with ascending columns in each row.
    `leaves` (a dict, optional) receives {name prefix: leaf parameters} for decode()."""
    out = {}
    _ref_node(nrows, ncols, rp, ci, va, parse_tree(spec), np.arange(nrows, dtype=np.int32), True, False, None, "",
              out, leaves if leaves is not None else {})
    return out


# ---- decoding: plan arrays -> (row, col, value) triples --------------------------------------

def _unit_stripes(a, nunits, nh):
    """Stripe of every unit of a heavy part: from sunits when the part has one, else ceil(nh/64) units a stripe."""
    if "sunits" in a:
        su = np.asarray(a["sunits"], dtype=np.int64)
        return np.repeat(np.arange(su.size - 1), np.diff(su))
    return np.arange(nunits) // max(1, -(-nh // WAVE))


_PART_NAMES = ("bin0.sell", "bin1.csrv8", "bin2.csrv64", "bin2.csrwg", "zero", "coo", "xl", "xnb", "nnzb", "wbm", "xs", "dia",
               "bsell", "sell", "csrv", "heavy")


def decode(arrays: dict, nrows: int, ncols: int, block: int = 3, tile: int = 8192, xl_w: int = 0, xl_rb: int = 16384,
           leaves: dict | None = None):
    """Every stored entry of every part as COO triples (padding included: it carries value 0).
    The part kind is recognised from the array names; `leaves` ({name prefix: leaf parameters}, from
    ref_plan) supplies block / tile / w / rb per leaf of a plan tree, the keyword arguments otherwise."""
    R, C, V = [], [], []
    prefixes = sorted({k.rsplit(".", 1)[0] for k in arrays})
    for full in prefixes:
        a = {k.rsplit(".", 1)[1]: v for k, v in arrays.items() if k.rsplit(".", 1)[0] == full}
        pre = next(n for n in _PART_NAMES if full == n or full.endswith("." + n))
        path = full[:len(full) - len(pre)]
        if leaves is not None:
            lp = leaves[path]
            block, tile, xl_w, xl_rb = lp["block"], lp["tile"], lp["w"], lp["rb"]
        if pre == "zero":
            continue
        if pre == "coo":
            R.append(a["rows"].astype(np.int64)); C.append(a["cols"]); V.append(a["vals"])
            continue
        if pre == "xl":
            if "vals" not in a:
                continue
            vv, lc, lr, it, gp, gl = a["vals"], a["lcol"], a["lrow"], a["items"], a["gptr"], a["glist"]
            W_ = xl_w if xl_w else 65536 // vv.dtype.itemsize
            N_ = 16 // vv.dtype.itemsize
            win = np.full(vv.size, -1, dtype=np.int64)        # entry -> window, from the items
            for s_, b0, e0 in it.reshape(-1, 3):
                win[b0:e0] = s_
            assert np.all(win >= 0)
            blk_of_group = np.repeat(np.arange(gp.size - 1), np.diff(gp))
            posn = np.full(vv.size, -1, dtype=np.int64)        # entry -> part position, from the group list
            for p_, code in enumerate(gl):
                g0, ln = (int(code) >> 3) * N_, ((int(code) & 7) + 1) * N_
                assert np.all(posn[g0:g0 + ln] == -1) and not np.any(lr[16 * p_ + ln:16 * p_ + 16])
                posn[g0:g0 + ln] = blk_of_group[p_] * xl_rb + lr[16 * p_:16 * p_ + ln].astype(np.int64)
            assert not np.any(vv[posn < 0])                    # what no group lists is padding
            rws = np.asarray(a["rows"]) if "rows" in a else np.arange(nrows)
            listed = posn >= 0
            assert not np.any(vv[listed & (posn >= rws.size)])
            keep = listed & (posn < rws.size)
            R.append(rws[posn[keep]].astype(np.int64)); C.append(win[keep] * W_ + lc[keep].astype(np.int64)); V.append(vv[keep])
            continue
        if pre == "xnb":
            cc, vv, bb, sr, bbs = a["cols"], a["vals"], a["bits"], a["seg_row"], a["bbase"]
            if cc.size == 0:
                continue
            R_ = cc.size // bb.size
            tsz = WAVE * R_
            nseg = int(a["tile_row"][-1])
            nrows_part = len(a["rows"]) if "rows" in a else nrows
            nblk = -(-nrows_part // 1024)
            K_ = bbs.size // (nblk + 1)
            seg_row = np.full(nseg, -1, dtype=np.int64)     # segment number -> part position
            for blk in range(nblk):
                for s_ in range(K_):
                    q0, q1 = int(bbs[blk * K_ + s_]), int(bbs[(blk + 1) * K_ + s_])
                    seg_row[q0:q1] = blk * 1024 + sr[q0:q1].astype(np.int64)
            assert np.all(seg_row >= 0)
            rws = a.get("rows", np.arange(nrows_part))
            g = np.arange(cc.size)
            src = (g // tsz) * tsz + ((g % tsz) % R_) * WAVE + (g % tsz) // R_
            mark = ((bb[(g // tsz) * WAVE + (g % tsz) // R_].astype(np.int64) >> ((g % tsz) % R_)) & 1).astype(np.int64)
            segidx = np.cumsum(mark) - 1
            R.append(np.asarray(rws)[seg_row[segidx]].astype(np.int64)); C.append(cc[src]); V.append(vv[src])
            continue
        if pre == "wbm":
            cc, vv, mk, rws = a["cols"], a["vals"], a["mask"], a["rows"]
            g = np.arange(cc.size)
            mark = ((mk[g // WAVE] >> (g % WAVE).astype(np.uint64)) & np.uint64(1)).astype(np.int64)
            rowidx = np.cumsum(mark) - 1
            R.append(rws[rowidx].astype(np.int64)); C.append(cc); V.append(vv)
            continue
        if pre == "nnzb":
            cc, vv, bb, rws = a["cols"], a["vals"], a["bits"], a["rows"]
            R_ = cc.size // bb.size
            tsz = WAVE * R_
            g = np.arange(cc.size)
            src = (g // tsz) * tsz + ((g % tsz) % R_) * WAVE + (g % tsz) // R_      # stream order -> storage
            mark = ((bb[(g // tsz) * WAVE + (g % tsz) // R_].astype(np.int64) >> ((g % tsz) % R_)) & 1).astype(np.int64)
            rowidx = np.cumsum(mark) - 1
            R.append(rws[rowidx].astype(np.int64)); C.append(cc[src]); V.append(vv[src])
            continue
        if pre == "xs":
            up, cc, vv, ps, pp = a["unit_ptr"], a["cols"], a["vals"], a["pslot"], a["pptr"]
            rws = a.get("rows", np.arange(len(pp) - 1))
            owner = np.full((len(up) - 1) * WAVE, -1, dtype=np.int64)      # slot -> part position
            owner[ps] = np.repeat(np.arange(len(pp) - 1), np.diff(pp))
            assert np.unique(ps).size == ps.size
            for u in range(len(up) - 1):
                base, w = int(up[u]), int(up[u + 1] - up[u]) // WAVE
                for lane in range(WAVE):
                    pos = base + lane + WAVE * np.arange(w)
                    i = owner[u * WAVE + lane]
                    if i < 0:
                        assert not np.any(vv[pos])
                        continue
                    R.append(np.full(w, int(rws[i]), dtype=np.int64)); C.append(cc[pos]); V.append(vv[pos])
            continue
        if pre == "dia":
            offs, dv = a["offsets"], a["vals"]
            ld = dv.size // max(len(offs), 1)
            for d, off in enumerate(offs):
                r = np.arange(nrows, dtype=np.int64)
                c = r + int(off)
                ok = (c >= 0) & (c < ncols)
                R.append(r[ok]); C.append(c[ok]); V.append(dv[d * ld:d * ld + nrows][ok])
        elif pre == "bsell":
            sp, vv = a["slice_ptr"], a["vals"]
            if "bcols16" in a:       # offsets from the first block column of the group of 32 slices
                lo = np.asarray(a["xwin"])[0::2] // block
                first = np.repeat(lo, np.diff(sp[np.minimum(np.arange(lo.size + 1) * 32, len(sp) - 1)]))
                bc = a["bcols16"].astype(np.int64) + first
            else:
                bc = a["bcols"]
            nb = nrows // block
            order = a.get("origin_brows", np.arange(nb, dtype=np.int32))
            BB = block * block
            for s in range(len(sp) - 1):
                base, w = int(sp[s]), int(sp[s + 1] - sp[s]) // WAVE
                for lane in range(WAVE):
                    i = s * WAVE + lane
                    if i >= nb:
                        continue
                    br = int(order[i])
                    for j in range(w):
                        b = int(bc[base + j * WAVE + lane])
                        for q in range(BB):
                            off, stride = _block_value_pos(block, vv.dtype.itemsize, q)
                            R.append([br * block + q // block]); C.append([b * block + q % block])
                            V.append([vv[(base + j * WAVE) * BB + off + stride * lane]])
        elif "slice_ptr" in a:   # SELL
            sp, cc, vv = a["slice_ptr"], a["cols"], a["vals"]
            nsl = len(sp) - 1
            order = a.get("origin_rows")
            for s in range(nsl):
                base, w = int(sp[s]), int(sp[s + 1] - sp[s]) // WAVE
                for lane in range(WAVE):
                    i = s * WAVE + lane
                    if order is None:
                        if i >= nrows:
                            continue
                        r = i
                    else:
                        if i >= len(order):
                            continue
                        r = int(order[i])
                    pos = base + lane + WAVE * np.arange(w)
                    R.append(np.full(w, r, dtype=np.int64)); C.append(cc[pos]); V.append(vv[pos])
        elif "dcols" in a:       # heavy stripes, 8-bit column differences
            up, dw, vv, hr, lm = a["unit_ptr"], a["dcols"], a["vals"], a["rows"], a["lane_meta"]
            db = np.ascontiguousarray(dw.astype("<u4")).view(np.uint8)       # byte 4*word + (entry % 4)
            stripe_of = _unit_stripes(a, len(up) - 1, len(hr))
            for u in range(len(up) - 1):
                s = int(stripe_of[u])
                base, w = int(up[u]), int(up[u + 1] - up[u]) // WAVE
                j = np.arange(w)
                for lane in range(WAVE):
                    h, c0 = int(lm[u * WAVE + lane]) & 0xFFFF, int(lm[u * WAVE + lane]) >> 16
                    pos = base + lane + WAVE * j
                    d = db[base + (j // 4) * 4 * WAVE + lane * 4 + j % 4].astype(np.int64)
                    if h == 0xFFFF:
                        assert not np.any(vv[pos]) and not np.any(d)
                        continue
                    R.append(np.full(w, int(hr[h]), dtype=np.int64)); C.append(c0 + np.cumsum(d) + s * tile); V.append(vv[pos])
        elif "lcols" in a:       # heavy stripes
            up, lc, vv, hr, lr = a["unit_ptr"], a["lcols"], a["vals"], a["rows"], a["lane_row"]
            stripe_of = _unit_stripes(a, len(up) - 1, len(hr))
            for u in range(len(up) - 1):
                s = int(stripe_of[u])
                base, w = int(up[u]), int(up[u + 1] - up[u]) // WAVE
                for lane in range(WAVE):
                    h = int(lr[u * WAVE + lane])
                    pos = base + lane + WAVE * np.arange(w)
                    if h == 0xFFFF:
                        assert not np.any(vv[pos])
                        continue
                    R.append(np.full(w, int(hr[h]), dtype=np.int64)); C.append(lc[pos].astype(np.int64) + s * tile); V.append(vv[pos])
        else:                    # CSR segments
            sp, cc, vv = a["seg_ptr"], a["cols"], a["vals"]
            sr = a.get("seg_row")
            for g in range(len(sp) - 1):
                r = g if sr is None else int(sr[g])
                if r < 0:
                    r = ~r
                e = slice(int(sp[g]), int(sp[g + 1]))
                R.append(np.full(e.stop - e.start, r, dtype=np.int64)); C.append(cc[e]); V.append(vv[e])
    if not R:
        return np.zeros(0, np.int64), np.zeros(0, np.int64), np.zeros(0)
    return (np.concatenate([np.asarray(x, dtype=np.int64) for x in R]),
            np.concatenate([np.asarray(x, dtype=np.int64) for x in C]),
            np.concatenate([np.asarray(x) for x in V]))
