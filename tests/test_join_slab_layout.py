"""Host-side enumeration of the workgroup join's slab layout (the local join of Sec. 3.1; k_join in
csrc/knng_build.hip): which thread stores which 16-byte piece of which member row of a slab, for
every member-slot count, slab width, row length and member count the kernel is instantiated or
launched with.

This is a mirror of the kernel's index arithmetic (slab_map, issue_slab and the store of step A), kept
here because a mistake in it does not show as a wrong number but as a write over the arrays that
follow the slab in LDS (member ids among them) and then as a gather from a corrupted row number.
The statements checked are the ones the kernel relies on:
  * every piece of every member row below nTot is stored exactly once, at its own place;
  * nothing is stored outside the NCOLS rows of the slab, and nothing beyond a row's LD words;
  * a stored row at or beyond nTot only ever holds a loaded copy of the last member (full-width slabs);
  * every row number read from the member array lies below nTot, and every 16-byte piece loaded from
    a row lies inside the row.
"""
import itertools

import pytest


def _slab_map(d, k0, DS, tid):
    ln = min(d - k0, DS)
    len16 = (ln + 15) & ~15
    q4 = len16 >> 2
    qshift = 2
    while (1 << qshift) < q4:
        qshift += 1
    return dict(len16=len16, q4=q4, qshift=qshift, RP=256 >> qshift, c4=tid & ((1 << qshift) - 1),
                rsub=tid >> qshift, col_ok=(tid & ((1 << qshift) - 1)) < q4)


def _check(S16, DS, d, nTot):
    NCOLS, LD = 32 * S16, DS + 4
    NL = NCOLS * (DS // 4) // 256
    for k0 in range(0, d, DS):
        written = {}
        for tid in range(256):
            sm = _slab_map(d, k0, DS, tid)
            # issue_slab: rows read from the member array, pieces read from the rows
            t = k0 + 4 * sm["c4"]
            t = t if t < d else d - 4                      # VEC: d % 4 == 0
            if nTot > 0:
                assert 0 <= t <= d - 4
                for i in range(NL):
                    row = sm["rsub"] + i * sm["RP"]
                    rid_index = row if row < nTot else nTot - 1
                    assert 0 <= rid_index < nTot
            if not sm["col_ok"]:
                continue
            full = sm["len16"] == DS
            for i in range(NL):
                if not (i * sm["RP"] < nTot):              # the group was not loaded
                    continue
                row = sm["rsub"] + i * sm["RP"]
                if full or row < nTot:
                    col = 4 * sm["c4"]
                    assert row < NCOLS, (S16, DS, d, nTot, k0, tid, i, row)
                    assert col + 4 <= LD
                    assert (row, col) not in written
                    written[(row, col)] = (tid, i)
        ln16 = (min(d - k0, DS) + 15) & ~15
        for row in range(nTot):
            for col in range(0, ln16, 4):
                assert (row, col) in written, (S16, DS, d, nTot, k0, row, col)
        for (row, col) in written:
            assert col < ln16
            if row >= nTot:
                assert ln16 == DS                          # only full-width slabs store a group's spare rows


@pytest.mark.parametrize("S16,DS", [(3, 64), (4, 64), (8, 32)])
def test_every_piece_is_stored_once_and_nothing_outside_the_slab(S16, DS):
    NCOLS = 32 * S16
    ds = sorted(set([4, 8, 12, 16, 20, 28, 32, 36, 48, 60, 64, 68, 96, 100, 124, 128, 132, 192, 200, 256, 960]))
    tots = sorted(set([0, 1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 63, 64, 65, 95, 96, 97, 127, 128, 129, 255, 256]))
    for d, nTot in itertools.product(ds, tots):
        if nTot <= NCOLS:
            _check(S16, DS, d, nTot)


def test_the_predicate_that_was_once_missing_matters():
    """Without the per-row test on a narrower last slab (rows per group no divisor of the slot count)
    a store lands beyond the slab's rows: 96 slots, rows of 12 words (one k-step of 16), 64 rows per group."""
    S16, DS, d, nTot = 3, 64, 12, 70
    NCOLS, NL = 32 * S16, 32 * S16 * (DS // 4) // 256
    beyond = 0
    for tid in range(256):
        sm = _slab_map(d, 0, DS, tid)
        if not sm["col_ok"]:
            continue
        for i in range(NL):
            if i * sm["RP"] < nTot and sm["rsub"] + i * sm["RP"] >= NCOLS:
                beyond += 1                                # what an unconditional store would have written
    assert beyond > 0
    _check(S16, DS, d, nTot)                               # with the predicate: inside
