"""Index-only emulation, on the CPU, of the copy kernels' addressing: which 16-byte units does
each lane of each wavefront touch, for the gather / scatter kernel (16 KiB pieces of manifest
entries) and for the slice kernels of the host swap (64 KiB windows of a staging slice that cut
chunks at arbitrary places)?  Every unit must lie inside the piece it belongs to, inside the
padded chunk, and -- for the slice kernels -- inside the ring that holds the slice; together the
units must cover every staged byte exactly once.

This is the check that once found a copy running 1 024 bytes past the ring: the per-lane
unrolled loop bounded its units by the chunk length only, and a chunk that straddles the end of a
slice was copied beyond the window.  The emulation can replay that rule (bound_by_piece=False)
and must then see the overrun, which shows that it is sharp enough to notice.

The constants are read from the sources; the index arithmetic is restated here."""
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2202_07848_amd", "csrc")


def constant(path, name):
    text = open(os.path.join(CSRC, path)).read()
    m = re.search(r"constexpr\s+\w+\s+%s\s*=\s*([^;]+);" % name, text)
    assert m, name
    return int(eval(m.group(1), {"__builtins__": {}}, {}))


LANES, UNIT = 64, 16
MOVE_UNROLL = constant("stream_copy.h", "MOVE_UNROLL")
COPY_PIECE_LOG2 = constant("ckpt_internal.h", "COPY_PIECE_LOG2")
WINDOW = constant("transport.hip", "WINDOW")


def pad16(x):
    return (x + 15) & ~15


def move_piece_units(lo, hi, length, bound_by_piece=True):
    """Offsets (inside the chunk) of the 16-byte units one wavefront touches when it copies
    bytes [lo, hi) of a chunk of `length` bytes: lane l starts at lo + 16 l and takes MOVE_UNROLL
    units 1 KiB apart per trip, trips 16 KiB apart; a unit is touched if it starts below the
    chunk's length and (the rule under test) below the end of the piece."""
    out = []
    base = lo + UNIT * np.arange(LANES, dtype=np.int64)
    span = LANES * UNIT * MOVE_UNROLL
    while (base < hi).any():
        o = (base[base < hi][:, None] + LANES * UNIT * np.arange(MOVE_UNROLL)[None, :]).ravel()
        keep = o < length
        if bound_by_piece:
            keep &= o < hi
        out.append(o[keep])
        base = base + span
    return np.concatenate(out) if out else np.zeros(0, np.int64)


def ragged_manifest(chunk, seed, nentries=60):
    """(len, stage_off) of a manifest as the compaction writes it: mostly full chunks, some
    short last chunks of every residue mod 16."""
    rng = np.random.default_rng(seed)
    lens = np.where(rng.random(nentries) < 0.6, chunk,
                    rng.integers(1, chunk + 1, size=nentries)).astype(np.int64)
    lens[:16] = np.minimum(chunk, chunk // 2 + np.arange(16) + 1)       # every residue
    padded = (lens + 15) // 16 * 16
    off = np.concatenate([[0], np.cumsum(padded)[:-1]])
    return lens, off, int(padded.sum())


@pytest.mark.parametrize("chunk", [256, 4096, 65536, 1 << 20])
def test_gather_pieces_stay_inside_their_piece_and_cover_each_chunk_once(chunk):
    piece_log2 = min(chunk.bit_length() - 1, COPY_PIECE_LOG2)
    lens, off, staged = ragged_manifest(chunk, chunk, nentries=40 if chunk > 65536 else 60)
    for length in lens.tolist():
        padded = pad16(length)
        seen = np.zeros(padded // UNIT, dtype=np.int32)
        for piece in range(chunk >> piece_log2):
            lo = piece << piece_log2
            hi = min(lo + (1 << piece_log2), padded)
            if lo >= hi:
                continue
            units = move_piece_units(lo, hi, length)
            assert units.size and units.min() >= lo and units.max() + UNIT <= hi
            np.add.at(seen, units // UNIT, 1)
        assert (seen == 1).all()


def slice_walk(lens, off, staged, slice_bytes, bound_by_piece=True):
    """All (ring offset) units the gather slice kernel writes, per slice, and the worst distance
    by which a unit ends past its slice."""
    worst, hits = 0, np.zeros(staged // UNIT, dtype=np.int32)
    for b0 in range(0, staged, slice_bytes):
        b1 = min(staged, b0 + slice_bytes)
        for w_lo in range(b0, b1, WINDOW):
            w_hi = min(w_lo + WINDOW, b1)
            e = int(np.searchsorted(off, w_lo, side="right")) - 1
            pos = w_lo
            while e < lens.size and pos < w_hi:
                length, so = int(lens[e]), int(off[e])
                seg_hi = min(so + pad16(length), w_hi)
                # (a unit that straddles `length` is written whole: its pad bytes are zeros)
                units = move_piece_units(pos - so, seg_hi - so, length, bound_by_piece)
                ring = so - b0 + units
                if ring.size:
                    worst = max(worst, int(ring.max()) + UNIT - (b1 - b0))
                    assert ring.min() >= 0
                    inside = units[(units + so < b1)]
                    np.add.at(hits, (so + inside) // UNIT, 1)
                pos = seg_hi
                e += 1
    return worst, hits


@pytest.mark.parametrize("chunk,slice_bytes", [(4096, 65536), (65536, 65536), (1 << 20, 65536),
                                              (1 << 20, 3 * 65536), (256, 2 * 65536)])
def test_slice_windows_never_leave_the_ring_and_cover_staging_once(chunk, slice_bytes):
    lens, off, staged = ragged_manifest(chunk, 7 + chunk, nentries=24 if chunk > 65536 else 200)
    worst, hits = slice_walk(lens, off, staged, slice_bytes)
    assert worst <= 0, f"{worst} bytes written past the end of a slice"
    assert (hits == 1).all()


def test_the_emulation_sees_the_overrun_of_the_length_only_bound():
    # 1 MiB chunks through 64 KiB slices, units bounded by the chunk length only: a chunk that
    # continues behind the slice makes the unrolled loop run on past the ring
    lens, off, staged = ragged_manifest(1 << 20, 3, nentries=20)
    worst, _ = slice_walk(lens, off, staged, 65536, bound_by_piece=False)
    assert worst >= 1024
