"""The oracle's independent pins as one function, runnable against any build of
ckpt_oracle.c:  python tests/oracle_pins.py [path/to/lib.so]  exits 0 when every
pin holds, 1 when one fails.  (A planted mistake may also corrupt memory and
crash the process; the mutation test runs this file as a child for that reason.)"""
import ctypes
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import oracle  # noqa: E402
import xxhash  # noqa: E402
from test_oracle_xxh64 import VECTORS  # noqa: E402


def pattern_bufs(sizes, seed):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]


def pins_hold() -> bool:
    """All independent pins, evaluated against whatever library `oracle` currently wraps."""
    try:
        for _, data, want in VECTORS:
            assert oracle.xxh64(data) == want
        sizes = [0, 1, 17, 255, 256, 257, 1000, 4097, 31]
        chunk = 256
        bufs = pattern_bufs(sizes, 1)
        pieces = [(i, o, b[o:o + chunk]) for i, b in enumerate(bufs) for o in range(0, b.size, chunk)]
        assert oracle.nchunks(bufs, chunk) == len(pieces)
        for threads in (1, 3):
            dig = oracle.fingerprint(bufs, chunk, threads)
            assert dig.tolist() == [xxhash.xxh64_intdigest(p[2].tobytes(), 0) for p in pieces]
        other = [b.copy() for b in bufs]
        other[4][0] ^= 1
        other[6][999] ^= 1
        other[7][4096] ^= 1
        odig = oracle.fingerprint(other, chunk)
        mask, cnt = oracle.diff(other, chunk, odig, dig)
        brute = [int(not np.array_equal(d, other[i][o:o + chunk])) for i, o, d in pieces]
        assert mask.tolist() == brute and cnt["ndirty"] == 3
        allm, _ = oracle.diff(bufs, chunk, dig, None)
        assert allm.all()
        sel = allm.copy()
        sel[[1, 2, 5, 11]] = 0           # a partial mask: entry index != chunk index
        staging, man, cnt = oracle.compact(bufs, chunk, sel, dig)
        want, entries, soff = [], [], 0
        for k, (i, o, d) in enumerate(pieces):
            if not sel[k]:
                continue
            pad = (-d.size) % 16
            want.append(np.concatenate([d, np.zeros(pad, np.uint8)]))
            entries.append((i, d.size, o, soff, int(dig[k])))
            soff += d.size + pad
        assert cnt["staged_bytes"] == soff and np.array_equal(staging, np.concatenate(want))
        assert [(int(e["buf"]), int(e["len"]), int(e["buf_off"]), int(e["stage_off"]),
                 int(e["digest"])) for e in man] == entries
        staging, man, cnt = oracle.compact(bufs, chunk, allm, dig)
        arenas = [np.full(b.size + 64, 0xEE, np.uint8) for b in bufs]
        dst = [a[32:32 + b.size] for a, b in zip(arenas, bufs)]
        assert oracle.restore(dst, chunk, staging, man) == 0
        for a, d, b in zip(arenas, dst, bufs):
            assert np.array_equal(d, b) and np.all(a[:32] == 0xEE) and np.all(a[32 + b.size:] == 0xEE)
        owner_pins()
        widened_pins()
        chain_pins()
        verdict_pins()
        return True
    except AssertionError:
        return False


def widened_pins():
    """The pins of the content-addressed match, of the moves it drives and of the squashing
    validation, as their own test files state them (called here so that the mutation test can
    run them against a deliberately broken build)."""
    import test_oracle_match as tm
    import test_validate_mutations as tv
    for chunk in (256, 1024):
        for seed in (1, 2, 3):
            tm.test_match_equals_pairwise_definition(chunk, seed)
    tm.test_match_hand_case()
    tm.test_match_prefers_same_position_and_lowest_reference_position()
    tm.test_match_with_empty_reference_marks_first_occurrences()
    for seed in (4, 5):
        tm.test_snapshot_is_rebuilt_from_staging_reference_and_duplicates(seed)
    tm.test_apply_matches_skips_impossible_sources()
    for kind in tv.KINDS:
        tv.test_oracle_verdict_matches_construction(kind)
    tv.test_oracle_no_mutation_at_all_and_empty()


def chain_pins():
    """The pins of the chain restore, as tests/test_oracle_chain.py states them."""
    import test_oracle_chain as tc
    for seed in (1, 2, 3, 4):
        for nlinks in (1, 2, 5):
            tc.test_chain_equals_latest_holder_per_chunk(seed, nlinks)
    tc.test_order_of_the_links_decides()
    tc.test_empty_chain_and_empty_links_touch_nothing()
    tc.test_entries_that_are_not_whole_chunks_of_the_destination_are_skipped()
    tc.test_a_rejected_entry_of_a_later_link_leaves_the_earlier_bytes()
    tc.test_each_link_is_bounded_by_its_own_staging()
    tc.test_full_snapshot_then_deltas_from_the_oracle_path_restore_the_latest_state()
    for seed in (1, 2, 3, 4):
        for nlinks in (1, 2, 5):
            tc.test_merged_link_is_the_latest_holder_of_every_chunk_in_ascending_order(seed, nlinks)
    for seed in (5, 6):
        tc.test_merged_link_restores_to_what_the_chain_restores_to(seed)
    tc.test_merge_skips_what_the_chain_restore_skips_and_keeps_the_earlier_holder()
    tc.test_merge_capacities_follow_the_compaction_rule()
    tc.test_merge_of_nothing_is_empty()
    for seed in (1, 2, 3):
        tc.test_restricted_chain_writes_only_marked_chunks(seed)
    tc.test_restriction_to_nothing_and_to_everything()
    tc.test_a_switch_between_ranks_that_changed_different_chunks()


def verdict_pins():
    """The pins of the per-buffer verdicts, as tests/test_oracle_buffer_verdicts.py states them."""
    import test_oracle_buffer_verdicts as tb
    for seed in (1, 2, 3, 4, 5):
        tb.test_random_masks_against_a_numpy_reduction(seed)
    tb.test_verdict_equals_byte_inequality_of_the_buffers()
    tb.test_each_single_chunk_marks_exactly_its_buffer()
    tb.test_empty_list_and_only_empty_buffers()
    tb.test_mask_andnot_truth_table_and_random()
    for seed in (1, 2, 3):
        tb.test_marks_from_buffers_is_a_numpy_repeat_and_inverts_the_verdicts(seed)
    tb.test_marks_from_buffers_predict_the_diff_when_whole_buffers_differ()


def worker_states(world, seed, sizes=(5000, 256, 0, 1300, 77), chunk=256):
    """States of `world` workers: a common base, then per worker a few private rewrites, some of
    them shared by two workers (so groups of every size between 1 and world appear)."""
    rng = np.random.default_rng(seed)
    base = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]
    states = [[b.copy() for b in base] for _ in range(world)]
    for r in range(world):
        for _ in range(4):
            i = int(rng.choice([q for q, b in enumerate(base) if b.size]))
            off = int(rng.integers(0, base[i].size))
            patch = rng.integers(0, 256, size=min(300, base[i].size - off), dtype=np.uint8)
            for q in {r, int(rng.integers(0, world))}:        # sometimes one more worker gets it
                states[q][i][off:off + patch.size] = patch
    return states, chunk


def owner_pins():
    """Cross-worker upload ownership against what its purpose fixes, by brute force:
    (1) at every chunk position every distinct content is uploaded by exactly one of the workers
    that hold it; (2) a store filled from the uploads alone restores every worker's state;
    (3) content all workers share is spread evenly (rank r takes positions k = r mod world);
    (4) all-different content: every worker uploads everything; (5) a world of one likewise."""
    for world, seed in ((1, 5), (2, 6), (3, 7), (5, 8)):
        states, chunk = worker_states(world, seed)
        digs = np.stack([oracle.fingerprint(st, chunk) for st in states])
        n = digs.shape[1]
        lens = oracle.chunk_lens(states[0], chunk)
        masks, store = [], {}
        for r in range(world):
            mask, cnt = oracle.upload_owners(states[r], chunk, digs, r)
            masks.append(mask)
            assert cnt["ndirty"] == int(mask.sum())
            assert cnt["staged_bytes"] == int(((lens[mask == 1] + 15) // 16 * 16).sum())
            staging, man, _ = oracle.compact(states[r], chunk, mask, digs[r])
            for e in man:                                      # the upload: keyed by place and checksum
                key = (int(e["buf"]), int(e["buf_off"]), int(e["digest"]))
                assert key not in store, "content uploaded twice"
                store[key] = staging[int(e["stage_off"]):int(e["stage_off"]) + int(e["len"])]
        masks = np.stack(masks)
        sizes_seen = set()
        for k in range(n):
            for value in set(digs[:, k].tolist()):
                holders = [r for r in range(world) if int(digs[r, k]) == value]
                sizes_seen.add(len(holders))
                assert sum(int(masks[r, k]) for r in holders) == 1
        assert world < 3 or {1, 2, world} <= sizes_seen         # the input really has mixed groups
        for r in range(world):                                  # download: rebuild from the store
            pos = 0
            for i, b in enumerate(states[r]):
                for off in range(0, b.size, chunk):
                    got = store[(i, off, int(digs[r, pos]))]
                    assert np.array_equal(got, b[off:off + chunk])
                    pos += 1
    states, chunk = worker_states(1, 9)
    same = np.stack([oracle.fingerprint(states[0], chunk)] * 4)
    for r in range(4):
        mask, _ = oracle.upload_owners(states[0], chunk, same, r)
        assert np.array_equal(np.flatnonzero(mask), np.arange(r, same.shape[1], 4))
    apart = same + np.arange(4, dtype=np.uint64)[:, None]
    for r in range(4):
        mask, cnt = oracle.upload_owners(states[0], chunk, apart, r)
        assert mask.all() and cnt["ndirty"] == same.shape[1]




def use_library(path):
    good = oracle._load()
    other = ctypes.CDLL(path)
    for fn in ("ora_xxh64", "ora_nchunks", "ora_chunk_lens", "ora_fingerprint", "ora_diff",
               "ora_compact", "ora_restore", "ora_restore_chain", "ora_merge_chain",
               "ora_buffer_verdicts", "ora_mask_andnot", "ora_marks_from_buffers",
               "ora_upload_owners", "ora_match", "ora_apply_matches", "ora_validate_mutations"):
        getattr(other, fn).restype = getattr(good, fn).restype
        getattr(other, fn).argtypes = getattr(good, fn).argtypes
    oracle._lib = other


if __name__ == "__main__":
    if len(sys.argv) > 1:
        use_library(sys.argv[1])
    sys.exit(0 if pins_hold() else 1)
