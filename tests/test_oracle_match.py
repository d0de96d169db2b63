"""Pins of the oracle's content-addressed match (paper sec. 5.2.1: a checksum
is looked up by content, a hit at another address is a device-to-device move):
brute-force comparison of every (snapshot, reference) checksum pair in NumPy,
hand-built cases, and a full reconstruction of the snapshot from staging,
reference and duplicates."""
import numpy as np
import pytest

import oracle


def brute_src(dig, ref):
    """The definition, pair by pair."""
    out = np.empty(dig.size, dtype=np.int64)
    for k in range(dig.size):
        if k < ref.size and ref[k] == dig[k]:
            out[k] = k
            continue
        hits = np.flatnonzero(ref == dig[k])
        if hits.size:
            out[k] = hits[0]
            continue
        earlier = np.flatnonzero(dig[:k] == dig[k])
        out[k] = -2 - earlier[0] if earlier.size else -1
    return out


def make_case(rng, chunk, nref_bufs=9, zero_chunks=True):
    """Reference buffers, and a snapshot whose chunks are a mix of: unchanged, moved
    (same bytes elsewhere), new, duplicated new, all-zero."""
    sizes = [int(rng.integers(1, 9)) * chunk + int(rng.choice([0, 0, 17, chunk // 2]))
             for _ in range(nref_bufs)]
    ref = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]
    snap = [b.copy() for b in ref]
    # move: swap two buffers' leading chunks, copy a reference chunk somewhere else
    snap[0][:chunk], snap[3][:chunk] = ref[3][:chunk].copy(), ref[0][:chunk].copy()
    snap[5][:chunk] = ref[7][:chunk]
    # new content, and a duplicate of it later on
    fresh = rng.integers(0, 256, size=chunk, dtype=np.uint8)
    snap[1][:chunk] = fresh
    snap[6][:chunk] = fresh
    snap[8][:chunk] = fresh
    if zero_chunks:
        snap[2][:chunk] = 0
        snap[4][:chunk] = 0
    # extra buffer appended: geometry differs from the reference
    snap.append(np.concatenate([ref[2][:chunk], rng.integers(0, 256, size=100, dtype=np.uint8)]))
    return ref, snap


@pytest.mark.parametrize("chunk", [256, 1024])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_match_equals_pairwise_definition(chunk, seed):
    rng = np.random.default_rng(seed)
    ref, snap = make_case(rng, chunk)
    rdig, sdig = oracle.fingerprint(ref, chunk), oracle.fingerprint(snap, chunk)
    src, mask, cnt = oracle.match(snap, chunk, sdig, rdig)
    want = brute_src(sdig, rdig)
    assert np.array_equal(src, want)
    assert np.array_equal(mask, (want == -1).astype(np.uint8))
    assert cnt["nsame"] == int((want == np.arange(want.size)).sum())
    assert cnt["nmoved"] == int(((want >= 0) & (want != np.arange(want.size))).sum())
    assert cnt["ndup"] == int((want <= -2).sum())
    assert cnt["nnew"] == int((want == -1).sum())
    lens = oracle.chunk_lens(snap, chunk).astype(np.int64)
    assert cnt["staged_bytes"] == int(((lens + 15) // 16 * 16)[want == -1].sum())
    assert cnt["nmoved"] >= 3 and cnt["ndup"] >= 2 and cnt["nnew"] >= 2


def test_match_hand_case():
    chunk = 256
    a, b, c, z = (np.full(chunk, v, dtype=np.uint8) for v in (1, 2, 3, 0))
    ref = [np.concatenate([a, b]), np.concatenate([c])]
    snap = [np.concatenate([b, a, z]), np.concatenate([c, z, np.full(10, 9, np.uint8)])]
    rdig, sdig = oracle.fingerprint(ref, chunk), oracle.fingerprint(snap, chunk)
    src, mask, cnt = oracle.match(snap, chunk, sdig, rdig)
    # snapshot chunks: b a z | c z tail ; reference chunks: a b | c
    assert src.tolist() == [1, 0, -1, 2, -2 - 2, -1]
    assert mask.tolist() == [0, 0, 1, 0, 0, 1]
    assert cnt == {"nsame": 0, "nmoved": 3, "ndup": 1, "nnew": 2, "staged_bytes": 256 + 16,
                   "table_full": 0}


def test_match_prefers_same_position_and_lowest_reference_position():
    chunk = 256
    a = np.full(chunk, 7, dtype=np.uint8)
    ref = [np.concatenate([a, a, a])]
    snap = [np.concatenate([a, a, a, a])]
    d = oracle.fingerprint(ref, chunk)
    s = oracle.fingerprint(snap, chunk)
    src, mask, cnt = oracle.match(snap, chunk, s, d)
    assert src.tolist() == [0, 1, 2, 0] and mask.sum() == 0
    assert cnt["nsame"] == 3 and cnt["nmoved"] == 1


def test_match_with_empty_reference_marks_first_occurrences():
    chunk = 256
    a, b = np.full(chunk, 1, np.uint8), np.full(chunk, 2, np.uint8)
    snap = [np.concatenate([a, b, a, a, b])]
    s = oracle.fingerprint(snap, chunk)
    src, mask, cnt = oracle.match(snap, chunk, s, np.zeros(0, dtype=np.uint64))
    assert src.tolist() == [-1, -1, -2, -2, -3]
    assert mask.tolist() == [1, 1, 0, 0, 0]


@pytest.mark.parametrize("seed", [4, 5])
def test_snapshot_is_rebuilt_from_staging_reference_and_duplicates(seed):
    chunk = 512
    rng = np.random.default_rng(seed)
    ref, snap = make_case(rng, chunk)
    rdig, sdig = oracle.fingerprint(ref, chunk), oracle.fingerprint(snap, chunk)
    src, mask, cnt = oracle.match(snap, chunk, sdig, rdig)
    staging, man, c2 = oracle.compact(snap, chunk, mask, sdig)
    assert c2["ndirty"] == cnt["nnew"] and c2["staged_bytes"] == cnt["staged_bytes"]
    arenas = [np.full(b.size + 64, 0xEE, np.uint8) for b in snap]
    dst = [a[32:32 + b.size] for a, b in zip(arenas, snap)]
    for d in dst:
        d[:] = 0x5C
    assert oracle.restore(dst, chunk, staging, man) == 0
    assert oracle.apply_matches(dst, ref, chunk, src) == 0
    for a, d, s in zip(arenas, dst, snap):
        assert np.array_equal(d, s)
        assert np.all(a[:32] == 0xEE) and np.all(a[32 + s.size:] == 0xEE)


def test_apply_matches_skips_impossible_sources():
    chunk = 256
    ref = [np.arange(512, dtype=np.uint8) % 251]
    dst = [np.zeros(600, dtype=np.uint8)]
    src = np.array([5, 1, -2 - 2], dtype=np.int64)   # no ref chunk 5; fine; dup of itself-or-later
    assert oracle.apply_matches(dst, ref, chunk, src) == 2
    assert np.array_equal(dst[0][256:512], ref[0][256:512]) and dst[0][:256].sum() == 0
    # length mismatch: the 88-byte last chunk cannot come from a 256-byte reference chunk
    src = np.array([0, 1, 0], dtype=np.int64)
    assert oracle.apply_matches(dst, ref, chunk, src) == 1
