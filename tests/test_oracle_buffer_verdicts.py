"""Pins of the oracle's per-buffer verdicts (the paper compares whole buffers, sec. 5.2.1; here a
buffer differs when any of its chunks does).  Expected values come from byte comparison of the
buffers themselves and from NumPy reductions over hand-made masks, never from the oracle."""
import numpy as np
import pytest

import oracle

SIZES = [5000, 256, 0, 1300, 77, 4096, 0, 513]
CHUNK = 256


def owners(sizes, chunk):
    return np.concatenate([np.full((n + chunk - 1) // chunk, i, dtype=np.int64)
                           for i, n in enumerate(sizes)])


@pytest.mark.parametrize("seed", [1, 2, 3, 4, 5])
def test_random_masks_against_a_numpy_reduction(seed):
    rng = np.random.default_rng(seed)
    own = owners(SIZES, CHUNK)
    mask = (rng.random(own.size) < [0.02, 0.1, 0.5, 0.0, 1.0][seed - 1]).astype(np.uint8)
    mask[mask != 0] = rng.integers(1, 256, size=int(mask.sum()), dtype=np.uint8)   # any non-zero value marks
    dirty, counts = oracle.buffer_verdicts(SIZES, CHUNK, mask)
    want = np.zeros(len(SIZES), np.uint8)
    np.maximum.at(want, own, (mask != 0).astype(np.uint8))
    assert np.array_equal(dirty, want)
    assert counts == {"buffers": int(want.sum()),
                      "bytes": int(sum(n for n, d in zip(SIZES, want) if d))}


def test_verdict_equals_byte_inequality_of_the_buffers():
    """Through the whole path: buffers rewritten at single bytes (first byte, last byte, ragged
    tail), mask from the diff; a buffer's verdict must equal 'its bytes differ'."""
    rng = np.random.default_rng(9)
    ref = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in SIZES]
    new = [b.copy() for b in ref]
    new[0][4999] ^= 1
    new[3][0] ^= 1
    new[7][512] ^= 1
    mask, _ = oracle.diff(new, CHUNK, oracle.fingerprint(new, CHUNK), oracle.fingerprint(ref, CHUNK))
    dirty, counts = oracle.buffer_verdicts(SIZES, CHUNK, mask)
    assert dirty.tolist() == [int(not np.array_equal(a, b)) for a, b in zip(ref, new)]
    assert counts == {"buffers": 3, "bytes": 5000 + 1300 + 513}


def test_each_single_chunk_marks_exactly_its_buffer():
    own = owners(SIZES, CHUNK)
    for k in range(own.size):
        mask = np.zeros(own.size, np.uint8)
        mask[k] = 1
        dirty, counts = oracle.buffer_verdicts(SIZES, CHUNK, mask)
        assert np.flatnonzero(dirty).tolist() == [int(own[k])]
        assert counts == {"buffers": 1, "bytes": SIZES[own[k]]}


def test_empty_list_and_only_empty_buffers():
    dirty, counts = oracle.buffer_verdicts([], CHUNK, np.zeros(0, np.uint8))
    assert dirty.size == 0 and counts == {"buffers": 0, "bytes": 0}
    dirty, counts = oracle.buffer_verdicts([0, 0], CHUNK, np.zeros(0, np.uint8))
    assert dirty.tolist() == [0, 0] and counts == {"buffers": 0, "bytes": 0}


def test_mask_andnot_truth_table_and_random():
    a = np.array([0, 0, 1, 1, 7, 0, 255, 3], np.uint8)
    b = np.array([0, 1, 0, 1, 0, 9, 255, 0], np.uint8)
    assert oracle.mask_andnot(a, b).tolist() == [0, 0, 1, 0, 1, 0, 0, 1]
    rng = np.random.default_rng(3)
    a = rng.integers(0, 3, size=5000, dtype=np.uint8)
    b = rng.integers(0, 3, size=5000, dtype=np.uint8)
    assert np.array_equal(oracle.mask_andnot(a, b), ((a != 0) & (b == 0)).astype(np.uint8))
    assert oracle.mask_andnot(np.zeros(0, np.uint8), np.zeros(0, np.uint8)).size == 0


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_marks_from_buffers_is_a_numpy_repeat_and_inverts_the_verdicts(seed):
    rng = np.random.default_rng(seed)
    flags = rng.integers(0, 2, size=len(SIZES), dtype=np.uint8) * rng.integers(1, 256, size=len(SIZES), dtype=np.uint8)
    marks = oracle.marks_from_buffers(SIZES, CHUNK, flags)
    counts = [(n + CHUNK - 1) // CHUNK for n in SIZES]
    assert np.array_equal(marks, np.repeat((flags != 0).astype(np.uint8), counts))
    # verdicts of those marks give the flags back, for buffers that have chunks at all
    dirty, _ = oracle.buffer_verdicts(SIZES, CHUNK, marks)
    assert dirty.tolist() == [int(f != 0 and n > 0) for f, n in zip(flags, SIZES)]


def test_marks_from_buffers_predict_the_diff_when_whole_buffers_differ():
    """The use: buffers 1 and 5 are per-replica state; flagged, their chunks are exactly what
    the comparison of two replicas marks."""
    rng = np.random.default_rng(4)
    ref = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in SIZES]
    new = [b.copy() for b in ref]
    for i in (1, 5):
        new[i][:] = rng.integers(0, 256, size=new[i].size, dtype=np.uint8)
    mask, _ = oracle.diff(new, CHUNK, oracle.fingerprint(new, CHUNK), oracle.fingerprint(ref, CHUNK))
    flags = np.zeros(len(SIZES), np.uint8)
    flags[[1, 5]] = 1
    assert np.array_equal(oracle.marks_from_buffers(SIZES, CHUNK, flags), mask)
    assert oracle.marks_from_buffers([], CHUNK, np.zeros(0, np.uint8)).size == 0
