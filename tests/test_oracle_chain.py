"""Pins of the oracle's chain restore (paper sec. 4.6: later snapshots of one process hold only
what changed since the one before, so a restore applies a chain of them, oldest first).

None of the expected values comes from the oracle: the links (staging + manifest) are sliced out
of the states with NumPy here, and the expected destination is composed per chunk from the state
of the latest link that holds the chunk."""
import numpy as np
import pytest

import oracle

SIZES = [5000, 256, 0, 1300, 77, 4096]
CHUNK = 256


def pieces(sizes, chunk):
    return [(i, o, min(chunk, n - o)) for i, n in enumerate(sizes) for o in range(0, n, chunk)]


def link_of(state, chunk, chosen):
    """Staging and manifest of the chunks `chosen` (ascending chunk ids) of `state`, built by
    slicing: each chunk padded with zeros to a multiple of 16, entries in ascending order."""
    pcs = pieces([b.size for b in state], chunk)
    parts, man, soff = [], np.zeros(len(chosen), dtype=oracle.ENTRY_DTYPE), 0
    for e, k in enumerate(chosen):
        i, o, n = pcs[k]
        parts.append(state[i][o:o + n])
        parts.append(np.zeros((-n) % 16, np.uint8))
        man[e] = (i, n, o, soff, 0xD16E57 + k)
        soff += n + (-n) % 16
    staging = np.concatenate(parts) if parts else np.zeros(0, np.uint8)
    return staging, man


def random_chain(seed, nlinks, sizes=SIZES, chunk=CHUNK):
    rng = np.random.default_rng(seed)
    n = len(pieces(sizes, chunk))
    states = [[rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes] for _ in range(nlinks)]
    chosen = [np.sort(rng.choice(n, size=int(rng.integers(0, n + 1)), replace=False))
              for _ in range(nlinks)]
    return states, chosen


def composed(start, states, chosen, chunk):
    """Per chunk: the bytes of the latest link that holds it, else what was there."""
    out = [b.copy() for b in start]
    pcs = pieces([b.size for b in start], chunk)
    for k, (i, o, n) in enumerate(pcs):
        holders = [l for l, c in enumerate(chosen) if k in set(c.tolist())]
        if holders:
            out[i][o:o + n] = states[holders[-1]][i][o:o + n]
    return out


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
@pytest.mark.parametrize("nlinks", [1, 2, 5])
def test_chain_equals_latest_holder_per_chunk(seed, nlinks):
    states, chosen = random_chain(seed, nlinks)
    links = [link_of(s, CHUNK, c) for s, c in zip(states, chosen)]
    start = [np.full(n, 0xA5, np.uint8) for n in SIZES]
    arenas = [np.full(n + 64, 0xEE, np.uint8) for n in SIZES]
    dst = [a[32:32 + n] for a, n in zip(arenas, SIZES)]
    for d, s in zip(dst, start):
        d[:] = s
    stats = oracle.restore_chain(dst, CHUNK, links)
    want = composed(start, states, chosen, CHUNK)
    for a, d, w in zip(arenas, dst, want):
        assert np.array_equal(d, w)
        assert np.all(a[:32] == 0xEE) and np.all(a[32 + d.size:] == 0xEE)
    union = set().union(*[set(c.tolist()) for c in chosen])
    assert stats == {"written": len(union), "superseded": sum(c.size for c in chosen) - len(union),
                     "rejected": 0}


def test_order_of_the_links_decides():
    states, _ = random_chain(7, 2)
    n = len(pieces(SIZES, CHUNK))
    both = [np.arange(n), np.arange(n)]
    links = [link_of(s, CHUNK, c) for s, c in zip(states, both)]
    dst = [np.zeros(s, np.uint8) for s in SIZES]
    oracle.restore_chain(dst, CHUNK, links)
    assert all(np.array_equal(d, s) for d, s in zip(dst, states[1]))
    oracle.restore_chain(dst, CHUNK, links[::-1])
    assert all(np.array_equal(d, s) for d, s in zip(dst, states[0]))


def test_empty_chain_and_empty_links_touch_nothing():
    dst = [np.full(s, 0x3C, np.uint8) for s in SIZES]
    assert oracle.restore_chain(dst, CHUNK, []) == {"written": 0, "superseded": 0, "rejected": 0}
    empty = (np.zeros(0, np.uint8), np.zeros(0, oracle.ENTRY_DTYPE))
    assert oracle.restore_chain(dst, CHUNK, [empty, empty])["written"] == 0
    assert all(np.all(d == 0x3C) for d in dst)


def test_entries_that_are_not_whole_chunks_of_the_destination_are_skipped():
    """A shortened chunk, an offset inside a chunk, a last chunk given the full length, a buffer
    outside the list, bytes past the end of staging, an odd staging offset: each is skipped and
    counted, and the entries around it are applied."""
    rng = np.random.default_rng(11)
    state = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in SIZES]
    n = len(pieces(SIZES, CHUNK))
    staging, man = link_of(state, CHUNK, np.arange(n))
    pcs = pieces(SIZES, CHUNK)
    last_of_0 = max(k for k, p in enumerate(pcs) if p[0] == 0)      # 5000 = 19 * 256 + 136
    bad = man.copy()
    bad["len"][1] = 240                       # not the whole chunk
    bad["buf_off"][2] += 16                   # inside a chunk
    bad["len"][last_of_0] = CHUNK             # runs past the buffer
    bad["buf"][4] = len(SIZES)                # no such buffer
    bad["stage_off"][n - 1] = staging.size - 16          # would read past staging
    bad["stage_off"][6] += 8                  # not a multiple of 16
    broken = {1, 2, last_of_0, 4, n - 1, 6}
    dst = [np.full(s, 0x77, np.uint8) for s in SIZES]
    stats = oracle.restore_chain(dst, CHUNK, [(staging, bad)])
    assert stats == {"written": n - len(broken), "superseded": 0, "rejected": len(broken)}
    for k, (i, o, ln) in enumerate(pcs):
        got = dst[i][o:o + ln]
        assert np.all(got == 0x77) if k in broken else np.array_equal(got, state[i][o:o + ln])


def test_a_rejected_entry_of_a_later_link_leaves_the_earlier_bytes():
    states, _ = random_chain(13, 2)
    n = len(pieces(SIZES, CHUNK))
    links = [link_of(s, CHUNK, np.arange(n)) for s in states]
    links[1][1]["buf"][3] = 99
    dst = [np.zeros(s, np.uint8) for s in SIZES]
    stats = oracle.restore_chain(dst, CHUNK, links)
    assert stats == {"written": n, "superseded": n - 1, "rejected": 1}
    for k, (i, o, ln) in enumerate(pieces(SIZES, CHUNK)):
        assert np.array_equal(dst[i][o:o + ln], states[0 if k == 3 else 1][i][o:o + ln])


def test_each_link_is_bounded_by_its_own_staging():
    """Link 1's staging is shorter than link 0's: an entry of link 1 that points past its own
    staging, but inside link 0's size, is skipped."""
    states, _ = random_chain(17, 2)
    n = len(pieces(SIZES, CHUNK))
    first = link_of(states[0], CHUNK, np.arange(n))
    staging, man = link_of(states[1], CHUNK, np.arange(4))
    man["stage_off"][3] = staging.size          # multiple of 16, first byte past the end
    assert staging.size + CHUNK <= first[0].size
    dst = [np.zeros(s, np.uint8) for s in SIZES]
    stats = oracle.restore_chain(dst, CHUNK, [first, (staging, man)])
    assert stats == {"written": n, "superseded": 3, "rejected": 1}
    for k, (i, o, ln) in enumerate(pieces(SIZES, CHUNK)):
        assert np.array_equal(dst[i][o:o + ln], states[1 if k < 3 else 0][i][o:o + ln])


def test_full_snapshot_then_deltas_from_the_oracle_path_restore_the_latest_state():
    """The chain the path itself produces: a first snapshot without reference, then deltas
    against the digests of the one before; applied as one chain it gives the last state."""
    rng = np.random.default_rng(5)
    states = [[rng.integers(0, 256, size=s, dtype=np.uint8) for s in SIZES]]
    for step in range(4):
        nxt = [b.copy() for b in states[-1]]
        for _ in range(3 + step):
            i = int(rng.choice([q for q, b in enumerate(nxt) if b.size]))
            off = int(rng.integers(0, nxt[i].size))
            nxt[i][off:off + int(rng.integers(1, 600))] ^= 0x5A
        states.append(nxt)
    links, prev = [], None
    for st in states:
        dig = oracle.fingerprint(st, CHUNK)
        mask, _ = oracle.diff(st, CHUNK, dig, prev)
        staging, man, _ = oracle.compact(st, CHUNK, mask, dig)
        links.append((staging, man))
        prev = dig
    for upto in range(1, len(states) + 1):
        dst = [np.zeros(s, np.uint8) for s in SIZES]
        stats = oracle.restore_chain(dst, CHUNK, links[:upto])
        assert all(np.array_equal(d, s) for d, s in zip(dst, states[upto - 1]))
        assert stats["rejected"] == 0 and stats["written"] == len(pieces(SIZES, CHUNK))


# ---- folding a chain into one link -----------------------------------------------------------

def composed_link(sizes, states, chosen, chunk):
    """What the merged link must be, built by slicing: chunks in ascending id, each from the
    state of the latest link that holds it; digests are the ones link_of gave that link."""
    pcs = pieces(sizes, chunk)
    parts, rows, soff = [], [], 0
    for k, (i, o, n) in enumerate(pcs):
        holders = [l for l, c in enumerate(chosen) if k in set(c.tolist())]
        if not holders:
            continue
        parts += [states[holders[-1]][i][o:o + n], np.zeros((-n) % 16, np.uint8)]
        rows.append((i, n, o, soff, 0xD16E57 + k))
        soff += n + (-n) % 16
    man = np.array(rows, dtype=oracle.ENTRY_DTYPE) if rows else np.zeros(0, oracle.ENTRY_DTYPE)
    return (np.concatenate(parts) if parts else np.zeros(0, np.uint8)), man


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
@pytest.mark.parametrize("nlinks", [1, 2, 5])
def test_merged_link_is_the_latest_holder_of_every_chunk_in_ascending_order(seed, nlinks):
    states, chosen = random_chain(seed, nlinks)
    # digests differ per link so that a merged entry shows which link it came from
    links = []
    for l, (s, c) in enumerate(zip(states, chosen)):
        staging, man = link_of(s, CHUNK, c)
        man["digest"] += np.uint64(l << 32)
        links.append((staging, man))
    staging, man, counts, stats = oracle.merge_chain(SIZES, CHUNK, links)
    want_staging, want_man = composed_link(SIZES, states, chosen, CHUNK)
    pcs = pieces(SIZES, CHUNK)
    for row in want_man:                      # the digest of the holder: its link's offset added
        k = pcs.index((int(row["buf"]), int(row["buf_off"]), int(row["len"])))
        row["digest"] += np.uint64(max(l for l, c in enumerate(chosen) if k in set(c.tolist())) << 32)
    assert np.array_equal(staging, want_staging)
    assert man.tolist() == want_man.tolist()
    union = set().union(*[set(c.tolist()) for c in chosen])
    assert counts == {"ndirty": len(union), "staged_bytes": want_staging.size, "overflow": 0}
    assert stats == {"written": len(union), "superseded": sum(c.size for c in chosen) - len(union),
                     "rejected": 0}
    # offsets: exclusive prefix sum of the padded lengths, strictly increasing
    pad = (man["len"].astype(np.uint64) + 15) // 16 * 16
    assert np.array_equal(man["stage_off"], np.concatenate([[0], np.cumsum(pad)[:-1]]).astype(np.uint64))


@pytest.mark.parametrize("seed", [5, 6])
def test_merged_link_restores_to_what_the_chain_restores_to(seed):
    """Applied to the same destination, the one merged link and the whole chain give the same
    bytes (the destination is compared with the NumPy composition, not with the other call)."""
    states, chosen = random_chain(seed, 4)
    links = [link_of(s, CHUNK, c) for s, c in zip(states, chosen)]
    staging, man, _, _ = oracle.merge_chain(SIZES, CHUNK, links)
    start = [np.full(n, 0x42, np.uint8) for n in SIZES]
    want = composed(start, states, chosen, CHUNK)
    dst = [b.copy() for b in start]
    assert oracle.restore(dst, CHUNK, staging, man) == 0
    assert all(np.array_equal(d, w) for d, w in zip(dst, want))


def test_merge_skips_what_the_chain_restore_skips_and_keeps_the_earlier_holder():
    states, _ = random_chain(13, 2)
    n = len(pieces(SIZES, CHUNK))
    links = [link_of(s, CHUNK, np.arange(n)) for s in states]
    links[1][1]["buf"][3] = 99                # no such buffer
    links[1][1]["len"][5] -= 16               # not the whole chunk
    links[1][1]["stage_off"][7] = links[1][0].size       # past its staging
    staging, man, counts, stats = oracle.merge_chain(SIZES, CHUNK, links)
    assert stats == {"written": n, "superseded": n - 3, "rejected": 3} and counts["ndirty"] == n
    dst = [np.zeros(s, np.uint8) for s in SIZES]
    assert oracle.restore(dst, CHUNK, staging, man) == 0
    for k, (i, o, ln) in enumerate(pieces(SIZES, CHUNK)):
        assert np.array_equal(dst[i][o:o + ln], states[0 if k in (3, 5, 7) else 1][i][o:o + ln])


def test_merge_capacities_follow_the_compaction_rule():
    """Entry e is written only if e < manifest_cap, its bytes only if they also end inside
    staging_cap; every chunk not fully staged counts as overflow; the need is always reported."""
    states, chosen = random_chain(3, 3)
    links = [link_of(s, CHUNK, c) for s, c in zip(states, chosen)]
    full_staging, full_man, full_counts, _ = oracle.merge_chain(SIZES, CHUNK, links)
    m = full_man.size
    assert m > 6
    for mcap, scap in ((m - 2, full_staging.size), (m, int(full_man["stage_off"][4]) + 100),
                       (3, int(full_man["stage_off"][5])), (0, 0)):
        staging, man, counts, _ = oracle.merge_chain(SIZES, CHUNK, links, scap, mcap, fill=0xA5)
        fit_e = min(m, mcap)
        pad = (full_man["len"].astype(np.int64) + 15) // 16 * 16
        fit_b = int(np.sum((full_man["stage_off"].astype(np.int64) + pad <= scap)[:fit_e]))
        assert counts == {"ndirty": m, "staged_bytes": full_counts["staged_bytes"], "overflow": m - fit_b}
        assert man[:fit_e].tolist() == full_man[:fit_e].tolist()
        end = int(full_man["stage_off"][fit_b - 1] + pad[fit_b - 1]) if fit_b else 0
        assert np.array_equal(staging[:end], full_staging[:end]) and np.all(staging[end:] == 0xA5)


def test_merge_of_nothing_is_empty():
    staging, man, counts, stats = oracle.merge_chain(SIZES, CHUNK, [])
    assert staging.size == 0 and man.size == 0
    assert counts == {"ndirty": 0, "staged_bytes": 0, "overflow": 0}
    assert stats == {"written": 0, "superseded": 0, "rejected": 0}


# ---- a restore restricted to some chunks --------------------------------------------------------

@pytest.mark.parametrize("seed", [1, 2, 3])
def test_restricted_chain_writes_only_marked_chunks(seed):
    """With `only`, an unmarked chunk keeps its bytes whatever the links hold; a marked one gets
    the bytes of its latest holder; the counts are those of the chain cut down to marked chunks."""
    rng = np.random.default_rng(100 + seed)
    states, chosen = random_chain(seed, 4)
    links = [link_of(s, CHUNK, c) for s, c in zip(states, chosen)]
    n = len(pieces(SIZES, CHUNK))
    only = (rng.random(n) < 0.5).astype(np.uint8)
    only[only != 0] = rng.integers(1, 256, size=int(only.sum()), dtype=np.uint8)
    start = [np.full(s, 0xA5, np.uint8) for s in SIZES]
    dst = [b.copy() for b in start]
    stats = oracle.restore_chain(dst, CHUNK, links, only)
    kept = [np.array([k for k in c.tolist() if only[k]], dtype=np.int64) for c in chosen]
    want = composed(start, states, kept, CHUNK)
    assert all(np.array_equal(d, w) for d, w in zip(dst, want))
    union = set().union(*[set(c.tolist()) for c in kept])
    assert stats == {"written": len(union), "superseded": sum(c.size for c in kept) - len(union),
                     "rejected": 0}


def test_restriction_to_nothing_and_to_everything():
    states, chosen = random_chain(8, 3)
    links = [link_of(s, CHUNK, c) for s, c in zip(states, chosen)]
    n = len(pieces(SIZES, CHUNK))
    dst = [np.full(s, 0x3C, np.uint8) for s in SIZES]
    assert oracle.restore_chain(dst, CHUNK, links, np.zeros(n, np.uint8)) == \
        {"written": 0, "superseded": 0, "rejected": 0}
    assert all(np.all(d == 0x3C) for d in dst)
    a = [np.full(s, 0x3C, np.uint8) for s in SIZES]
    b = [np.full(s, 0x3C, np.uint8) for s in SIZES]
    assert oracle.restore_chain(a, CHUNK, links, np.ones(n, np.uint8)) == oracle.restore_chain(b, CHUNK, links)
    assert all(np.array_equal(x, y) for x, y in zip(a, composed(b, states, chosen, CHUNK)))


def test_a_switch_between_ranks_that_changed_different_chunks():
    """What the restriction is for (sec. 5.2.1): the device holds rank A, rank B comes in.  Both
    are kept as deltas against a base of which a full copy exists.  B may equal the base where A
    does not, so B's delta alone would leave A's bytes behind; the chain [full base, B's delta]
    restricted to the chunks whose checksums differ between A and B gives B exactly, and reads the
    base only where B does not hold the chunk itself."""
    rng = np.random.default_rng(21)
    base = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in SIZES]
    a, b = [x.copy() for x in base], [x.copy() for x in base]
    a[0][300:900] ^= 0x11          # A alone changes chunks 1..3 of buffer 0
    b[0][2060:2100] ^= 0x22        # B alone changes chunk 8
    a[3][0:50] ^= 0x33             # both change chunk 0 of buffer 3, differently
    b[3][0:50] ^= 0x44
    a[5][1000:1100] ^= 0x55        # both change a chunk of buffer 5 to the same bytes
    b[5][1000:1100] ^= 0x55
    dig = {name: oracle.fingerprint(st, CHUNK) for name, st in (("base", base), ("a", a), ("b", b))}
    full_mask, _ = oracle.diff(base, CHUNK, dig["base"], None)
    base_link = oracle.compact(base, CHUNK, full_mask, dig["base"])[:2]
    b_mask, _ = oracle.diff(b, CHUNK, dig["b"], dig["base"])
    b_link = oracle.compact(b, CHUNK, b_mask, dig["b"])[:2]
    incoming, _ = oracle.diff(b, CHUNK, dig["b"], dig["a"])       # where the resident rank differs
    dst = [x.copy() for x in a]
    stats = oracle.restore_chain(dst, CHUNK, [base_link, b_link], incoming)
    assert all(np.array_equal(d, x) for d, x in zip(dst, b))
    assert stats["written"] == int(incoming.sum()) == 3 + 1 + 1    # not the chunk both set alike
    wrong = [x.copy() for x in a]                                  # B's delta alone is not enough
    oracle.restore(wrong, CHUNK, *b_link)
    assert not all(np.array_equal(d, x) for d, x in zip(wrong, b))
