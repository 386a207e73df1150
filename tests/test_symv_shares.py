"""Host logic of the balanced SYMV/HEMV kernel: the table of shares that the planner hands to the
kernels (Section 6.2: equal contiguous shares of a work line).  The table is checked against a
piece-by-piece enumeration of the stored triangle written out here: every piece belongs to exactly one
share, in order, no share is empty, the shares are as long as the partition allows, and the owners
of a chunk's first and last piece are the ones named.  No GPU is involved."""
import itertools

import pytest

from paper_1410_1726_amd import binding as kmv

TILE_ROWS = {"s": 256, "d": 128, "c": 128, "z": 64}
C = 16


def enumerate_pieces(prec, uplo, n, shift, ct, kt, fixed, edge=0):
    """[(chunk, piece in chunk, weight)] in line order, from the definition: piece (k, p) exists when some
    stored element (i, j), j in panel p, has its row slot i + shift in chunk k; its weight counts the groups
    of kt row tiles of the chunk that hold such an element, times kt, plus `fixed`.  The tiles rarely divide into
    whole chunks: the short chunk is the FIRST one for lower storage (the chunk grid starts `coff` tiles before
    tile 0) and the last one for upper storage - where the triangle is narrow."""
    tr = TILE_ROWS[prec]
    ntiles = -(-(n + shift) // tr)
    coff = (ct - ntiles % ct) % ct if uplo == "L" else 0
    coff -= coff % kt                    # a multiple of the unit's tiles: only the matrix's last chunk ends inside a unit
    nchunks = -(-(ntiles + coff) // ct)
    npanels = -(-n // C)
    out = []
    for k in range(nchunks):
        tbeg, tend = max(k * ct - coff, 0), min((k + 1) * ct - coff, ntiles)
        j = 0
        for p in range(npanels):
            c0, c1 = p * C, min(p * C + C, n) - 1           # columns of the panel
            groups = edges = 0
            for g in range(-(-(tend - tbeg) // kt)):
                t0, t1 = tbeg + g * kt, min(tbeg + g * kt + kt, tend)
                r0, r1 = max(t0 * tr - shift, 0), min(t1 * tr - shift, n) - 1      # rows of the group
                if r1 < r0:
                    continue
                # lower: some row >= some column of the panel; upper: some row <= some column
                stored = (r1 >= c0) if uplo == "L" else (r0 <= c1)
                groups += stored
                first_tile_cut = (k == 0 and g == 0 and shift > 0)
                last_tile_cut = (tend == ntiles and g == (tend - 1 - tbeg) // kt and ntiles * tr - shift > n)
                edges += stored and (first_tile_cut or last_tile_cut)
            if groups:
                out.append((k, j, groups * kt + fixed + edges * edge))
                j += 1
    return out, nchunks


CASES = [(prec, uplo, n, shift, ct, kt, slots, fixed, edge)
         for prec in "sdcz" for uplo in "LU"
         for n, shift in ((2049, 0), (2600, 5), (4099, 0), (5000, 15), (8192, 1), (12289, 7))
         for ct, kt in ((4, 1), (8, 1), (8, 2), (4, 2), (12, 1), (16, 1))
         for slots, fixed, edge in ((768, 1, 2), (512, 3, 0), (100, 0, 1))]


@pytest.mark.parametrize("prec,uplo,n,shift,ct,kt,slots,fixed,edge", CASES[::7] + CASES[3::11])
def test_shares_tile_the_pieces(prec, uplo, n, shift, ct, kt, slots, fixed, edge):
    if shift >= TILE_ROWS[prec]:
        shift = TILE_ROWS[prec] - 1
    pieces, nchunks = enumerate_pieces(prec, uplo, n, shift, ct, kt, fixed, edge)
    got = kmv.symv_shares(prec, uplo, n, shift, ct, kt, slots, fixed, edge)
    assert got is not None
    workers, work, start, first, last = got
    assert work == sum(w for _, _, w in pieces)
    assert 1 <= workers <= slots
    assert start[0] == (0, 0) and start[workers] == (nchunks, 0)
    # positions of the pieces on the line, and the share each start entry points at
    index = {(k, j): i for i, (k, j, _) in enumerate(pieces)}
    index[(nchunks, 0)] = len(pieces)
    begin = [0]
    for _, _, w in pieces:
        begin.append(begin[-1] + w)
    bounds = [index[e] for e in start]
    assert bounds == sorted(bounds) and len(set(bounds)) == len(bounds), "a share is empty or out of order"
    q, r = divmod(work, workers)
    for y in range(workers):
        s_y = y * q + min(y, r)                               # starting point of Section 6.2
        i = bounds[y]
        assert begin[i] >= s_y and (i == 0 or begin[i - 1] < s_y), "share does not start at the first piece at or after s(y)"
    # owners of every chunk's first and last piece
    owner = {}
    for y in range(workers):
        for i in range(bounds[y], bounds[y + 1]):
            owner[i] = y
    for k in range(nchunks):
        mine = [i for i, (kk, _, _) in enumerate(pieces) if kk == k]
        assert first[k] == owner[mine[0]] and last[k] == owner[mine[-1]]


def test_shares_argument_checks():
    assert kmv.symv_shares("d", "X", 4096, 0, 8, 1, 768, 1) is None
    assert kmv.symv_shares("q", "L", 4096, 0, 8, 1, 768, 1) is None
    assert kmv.symv_shares("d", "L", 0, 0, 8, 1, 768, 1) is None
    assert kmv.symv_shares("d", "L", 4096, 128, 8, 1, 768, 1) is None      # shift beyond a tile
    assert kmv.symv_shares("d", "L", 4096, 0, 5, 1, 768, 1) is None
    assert kmv.symv_shares("z", "L", 1 << 20, 0, 4, 1, 768, 1) is None     # more chunks than the tables hold
    y, work, start, first, last = kmv.symv_shares("d", "L", 4096, 0, 4, 1, 100000, 1)
    assert y <= 800


def test_shares_weigh_stored_tiles_only():
    """a diagonal piece is lighter than a full one: with no fixed part the line is exactly the number of
    (row tile, panel) cells that hold stored elements"""
    for prec, uplo in itertools.product("sdz", "LU"):
        n, tr = 6000, TILE_ROWS[prec]
        cells = 0
        for t in range(-(-n // tr)):
            for p in range(-(-n // C)):
                r0, r1 = t * tr, min(t * tr + tr, n) - 1
                c0, c1 = p * C, min(p * C + C, n) - 1
                cells += (r1 >= c0) if uplo == "L" else (r0 <= c1)
        assert kmv.symv_shares(prec, uplo, n, 0, 8, 1, 768, 0)[1] == cells
