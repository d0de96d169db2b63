"""GPU parity of the content-addressed match and of the moves it implies
(paper sec. 5.2.1) against the oracle: src, mask and counts bit-exact, and the
snapshot rebuilt from staging + reference + duplicates byte for byte."""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_07848_amd import binding as ck
from gpu_util import DeviceBuffers, counts_dict, run_compact, run_fingerprint, u64
from test_oracle_match import make_case

pytestmark = pytest.mark.gpu


def run_match(plan, dig, ref, n_ref):
    n = plan.nchunks
    ws = torch.empty(ck.match_workspace_bytes(n_ref, n), dtype=torch.uint8, device="cuda")
    ws.fill_(0x3C)                                     # the call must initialise its tables itself
    src = torch.full((max(1, n),), 12345, dtype=torch.int64, device="cuda")
    mask = torch.full((max(1, n),), 0x77, dtype=torch.uint8, device="cuda")
    counts = torch.full((6,), -1, dtype=torch.int64, device="cuda")
    ck.match(plan, dig, ref, ws, src, mask, counts, n_ref=n_ref)
    torch.cuda.synchronize()
    c = counts.cpu().numpy().view(np.uint64)
    return src, mask, {f: int(v) for f, v in zip(ck.MATCH_COUNT_FIELDS, c)}


@pytest.mark.parametrize("chunk", [256, 4096])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_match_and_rebuild(chunk, seed):
    rng = np.random.default_rng(seed)
    ref, snap = make_case(rng, chunk)
    d_ref, d_snap = DeviceBuffers(ref, chunk), DeviceBuffers(snap, chunk)
    rdig, sdig = run_fingerprint(d_ref.plan), run_fingerprint(d_snap.plan)
    n, n_ref = d_snap.plan.nchunks, d_ref.plan.nchunks
    o_rdig, o_sdig = oracle.fingerprint(ref, chunk), oracle.fingerprint(snap, chunk)
    assert np.array_equal(u64(sdig, n), o_sdig) and np.array_equal(u64(rdig, n_ref), o_rdig)

    want_src, want_mask, want_cnt = oracle.match(snap, chunk, o_sdig, o_rdig)
    src, mask, cnt = run_match(d_snap.plan, sdig, rdig, n_ref)
    assert np.array_equal(src[:n].cpu().numpy(), want_src)
    assert np.array_equal(mask[:n].cpu().numpy(), want_mask)
    assert cnt == want_cnt and cnt["nmoved"] >= 3 and cnt["ndup"] >= 2

    # stage the new chunks only, then rebuild the snapshot in a garbage-filled destination
    want_st, want_man, _ = oracle.compact(snap, chunk, want_mask, o_sdig)
    staging, manifest, _ = run_compact(d_snap.plan, mask, sdig, want_st.size, want_man.size)
    assert np.array_equal(staging.cpu().numpy()[:want_st.size], want_st)
    garbage = [np.full(b.size, 0x5C, dtype=np.uint8) for b in snap]
    dst = DeviceBuffers(garbage, chunk)
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ck.restore(dst.plan, staging, want_st.size, manifest, want_man.size)
    ck.apply_matches(dst.plan, d_ref.plan, src, rejected)
    torch.cuda.synchronize()
    assert int(rejected.item()) == 0
    want_dst = [g.copy() for g in garbage]
    assert oracle.restore(want_dst, chunk, want_st, want_man) == 0
    assert oracle.apply_matches(want_dst, ref, chunk, want_src) == 0
    got, img = dst.host()
    for g, w, s in zip(got, want_dst, snap):
        assert np.array_equal(g, w) and np.array_equal(g, s)
    assert dst.canaries_intact(img) and d_ref.canaries_intact() and d_snap.canaries_intact()


@pytest.mark.parametrize("n,n_ref,domain", [(5000, 5000, 40), (3000, 7000, 1 << 62), (4097, 0, 9),
                                            (1, 1, 2), (20000, 20000, 3000)])
def test_match_on_synthetic_digests(n, n_ref, domain):
    """Digest arrays chosen freely (the lookup never reads chunk bytes): tiny key
    domains force long probe chains and many duplicates; the all-ones digest,
    which doubles as the empty-slot marker inside the tables, must still work."""
    rng = np.random.default_rng(n + n_ref)
    chunk = 256
    host = [np.zeros(n * chunk - 100, dtype=np.uint8)]        # n chunks, the last one short
    dev = DeviceBuffers(host, chunk)
    assert dev.plan.nchunks == n
    dig = rng.integers(0, domain, size=n, dtype=np.uint64)
    ref = rng.integers(0, domain, size=n_ref, dtype=np.uint64)
    ones = np.uint64(0xFFFFFFFFFFFFFFFF)
    dig[rng.integers(0, n, size=max(1, n // 50))] = ones
    if n_ref:
        ref[rng.integers(0, n_ref, size=max(1, n_ref // 70))] = ones
        same = rng.integers(0, min(n, n_ref), size=min(n, n_ref) // 3)
        dig[same] = ref[same]                                 # plenty of same-place hits
    want_src, want_mask, want_cnt = oracle.match(host, chunk, dig, ref)
    d_dig = torch.from_numpy(dig.view(np.int64)).cuda()
    d_ref = torch.from_numpy(ref.view(np.int64)).cuda() if n_ref else None
    src, mask, cnt = run_match(dev.plan, d_dig, d_ref, n_ref)
    assert np.array_equal(src[:n].cpu().numpy(), want_src)
    assert np.array_equal(mask[:n].cpu().numpy(), want_mask)
    assert cnt == want_cnt


def test_match_without_reference_keeps_first_occurrences_only():
    chunk = 256
    a, b = np.full(chunk, 1, np.uint8), np.full(chunk, 2, np.uint8)
    snap = [np.concatenate([a, b, a, a, b]), np.zeros(0, np.uint8), np.concatenate([b, a[:40]])]
    dev = DeviceBuffers(snap, chunk)
    dig = run_fingerprint(dev.plan)
    src, mask, cnt = run_match(dev.plan, dig, None, 0)
    assert src[:7].cpu().numpy().tolist() == [-1, -1, -2, -2, -3, -3, -1]
    assert cnt["nnew"] == 3 and cnt["ndup"] == 4 and cnt["staged_bytes"] == 256 + 256 + 48


def test_apply_matches_rejects_impossible_sources_and_checks_arguments():
    chunk = 256
    ref = [(np.arange(512) % 251).astype(np.uint8)]
    d_ref = DeviceBuffers(ref, chunk)
    dst_host = [np.zeros(600, dtype=np.uint8)]
    dst = DeviceBuffers(dst_host, chunk)
    src = np.array([5, 1, -2 - 2], dtype=np.int64)
    want = [b.copy() for b in dst_host]
    want_rej = oracle.apply_matches(want, ref, chunk, src)
    rejected = torch.zeros(1, dtype=torch.int64, device="cuda")
    ck.apply_matches(dst.plan, d_ref.plan, torch.from_numpy(src).cuda(), rejected)
    torch.cuda.synchronize()
    assert int(rejected.item()) == want_rej == 2
    got, img = dst.host()
    assert np.array_equal(got[0], want[0]) and dst.canaries_intact(img)
    other = DeviceBuffers(ref, 512)
    with pytest.raises(ck.CkptError) as e:
        ck.apply_matches(dst.plan, other.plan, torch.from_numpy(src).cuda())
    assert e.value.status == -3
    small = torch.empty(64, dtype=torch.uint8, device="cuda")
    dig = run_fingerprint(dst.plan)
    with pytest.raises(ck.CkptError) as e:
        ck.match(dst.plan, dig, dig, small, torch.zeros(3, dtype=torch.int64, device="cuda"),
                 torch.zeros(3, dtype=torch.uint8, device="cuda"),
                 torch.zeros(6, dtype=torch.int64, device="cuda"))
    assert e.value.status == -5


def permuted_case(rng, chunk):
    """Same geometry for reference and snapshot; the snapshot's chunks are the reference's
    after a permutation with 2-cycles and 3-cycles, plus new, duplicated and unchanged chunks."""
    sizes = [6 * chunk, 3 * chunk + 100, 5 * chunk, 2 * chunk + 100, 4 * chunk]
    ref = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]
    snap = [b.copy() for b in ref]

    def ch(bufs, b, j):
        return bufs[b][j * chunk:(j + 1) * chunk]

    # 2-cycle, 3-cycle, a chain into a chunk that becomes new, the two equal-length tails swapped
    snap[0][0:chunk], snap[2][0:chunk] = ch(ref, 2, 0).copy(), ch(ref, 0, 0).copy()
    snap[0][chunk:2 * chunk] = ch(ref, 2, 1)
    snap[2][chunk:2 * chunk] = ch(ref, 4, 1)
    snap[4][chunk:2 * chunk] = ch(ref, 0, 1)
    snap[4][2 * chunk:3 * chunk] = ch(ref, 4, 3)
    fresh = rng.integers(0, 256, size=chunk, dtype=np.uint8)
    snap[4][3 * chunk:4 * chunk] = fresh
    snap[0][5 * chunk:6 * chunk] = fresh
    snap[1][3 * chunk:], snap[3][2 * chunk:] = ref[3][2 * chunk:].copy(), ref[1][3 * chunk:].copy()
    return ref, snap


@pytest.mark.parametrize("chunk", [256, 65536])
def test_moves_inside_one_memory_image(chunk):
    rng = np.random.default_rng(chunk)
    ref, snap = permuted_case(rng, chunk)
    d_snap = DeviceBuffers(snap, chunk)
    image = DeviceBuffers(ref, chunk)                 # holds the reference; becomes the snapshot
    n = image.plan.nchunks
    rdig, sdig = run_fingerprint(image.plan), run_fingerprint(d_snap.plan)
    o_rdig, o_sdig = oracle.fingerprint(ref, chunk), oracle.fingerprint(snap, chunk)
    want_src, want_mask, want_cnt = oracle.match(snap, chunk, o_sdig, o_rdig)
    src, mask, cnt = run_match(d_snap.plan, sdig, rdig, n)
    assert np.array_equal(src[:n].cpu().numpy(), want_src) and cnt == want_cnt
    assert cnt["nmoved"] >= 8 and cnt["ndup"] == 1 and cnt["nnew"] == 1
    want_st, want_man, _ = oracle.compact(snap, chunk, want_mask, o_sdig)
    staging, manifest, _ = run_compact(d_snap.plan, mask, sdig, want_st.size, want_man.size)

    moved = (want_src >= 0) & (want_src != np.arange(n))
    lens = oracle.chunk_lens(snap, chunk).astype(np.int64)
    need = int(((lens + 15) // 16 * 16)[moved].sum())
    temp = torch.full((need + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    ws = torch.empty(ck.moves_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")

    # too little room: nothing at all may move
    ck.apply_moves_inplace(image.plan, src, temp, ws, counts, rejected, temp_cap=need - 16)
    torch.cuda.synchronize()
    c = counts_dict(counts)
    assert c["ndirty"] == int(moved.sum()) and c["staged_bytes"] == need and c["overflow"] > 0
    got, _ = image.host()
    assert all(np.array_equal(g, r) for g, r in zip(got, ref))

    ck.apply_moves_inplace(image.plan, src, temp, ws, counts, rejected, temp_cap=need)
    ck.restore(image.plan, staging, want_st.size, manifest, want_man.size)
    ck.apply_matches(image.plan, None, src)
    torch.cuda.synchronize()
    assert counts_dict(counts) == {"ndirty": int(moved.sum()), "staged_bytes": need, "overflow": 0}
    assert int(rejected.item()) == 0
    assert bool((temp[need:] == 0xA5).all())
    # the oracle rebuilds out of place: sources are read from an untouched copy of the reference
    want = [b.copy() for b in ref]
    assert oracle.restore(want, chunk, want_st, want_man) == 0
    assert oracle.apply_matches(want, ref, chunk, want_src) == 0
    got, img = image.host()
    for g, w, s in zip(got, want, snap):
        assert np.array_equal(g, w) and np.array_equal(g, s)
    assert image.canaries_intact(img)



def random_permuted_case(seed):
    """A memory image whose full chunks are shuffled by a random permutation (any cycle
    structure), with a few chunks replaced by new content, some of it repeated."""
    rng = np.random.default_rng(500 + seed)
    chunk = int(rng.choice([256, 1024, 4096]))
    sizes = [int(rng.integers(1, 12)) * chunk + int(rng.choice([0, 0, 1, 40, chunk // 2]))
             for _ in range(int(rng.integers(2, 9)))]
    ref = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]
    snap = [b.copy() for b in ref]
    slots = [(i, j * chunk) for i, n in enumerate(sizes) for j in range(n // chunk)]
    perm = rng.permutation(len(slots))
    moved = rng.random(len(slots)) < 0.7
    for t, s in enumerate(perm):
        if moved[t]:
            (di, do), (si, so) = slots[t], slots[int(s)]
            snap[di][do:do + chunk] = ref[si][so:so + chunk]
    fresh = rng.integers(0, 256, size=chunk, dtype=np.uint8)
    for t in rng.choice(len(slots), size=min(3, len(slots)), replace=False):
        di, do = slots[int(t)]
        snap[di][do:do + chunk] = fresh if rng.random() < 0.7 else \
            rng.integers(0, 256, size=chunk, dtype=np.uint8)
    return chunk, ref, snap


@pytest.mark.parametrize("seed", range(12))
def test_random_permutation_inside_one_memory_image(seed):
    chunk, ref, snap = random_permuted_case(seed)
    d_snap = DeviceBuffers(snap, chunk)
    image = DeviceBuffers(ref, chunk)
    n = image.plan.nchunks
    rdig, sdig = run_fingerprint(image.plan), run_fingerprint(d_snap.plan)
    o_rdig, o_sdig = oracle.fingerprint(ref, chunk), oracle.fingerprint(snap, chunk)
    want_src, want_mask, want_cnt = oracle.match(snap, chunk, o_sdig, o_rdig)
    src, mask, cnt = run_match(d_snap.plan, sdig, rdig, n)
    assert np.array_equal(src[:n].cpu().numpy(), want_src) and cnt == want_cnt
    assert np.array_equal(mask[:n].cpu().numpy(), want_mask)
    want_st, want_man, _ = oracle.compact(snap, chunk, want_mask, o_sdig)
    staging, manifest, _ = run_compact(d_snap.plan, mask, sdig, want_st.size, want_man.size)
    moved = (want_src >= 0) & (want_src != np.arange(n))
    lens = oracle.chunk_lens(snap, chunk).astype(np.int64)
    need = int(((lens + 15) // 16 * 16)[moved].sum())
    temp = torch.full((need + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    ws = torch.empty(ck.moves_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ck.apply_moves_inplace(image.plan, src, temp, ws, counts, rejected, temp_cap=need)
    ck.restore(image.plan, staging, want_st.size, manifest, want_man.size)
    ck.apply_matches(image.plan, None, src)
    torch.cuda.synchronize()
    assert counts_dict(counts) == {"ndirty": int(moved.sum()), "staged_bytes": need, "overflow": 0}
    assert int(rejected.item()) == 0
    assert bool((temp[need:] == 0xA5).all())
    got, img = image.host()
    assert all(np.array_equal(g, s) for g, s in zip(got, snap))
    assert image.canaries_intact(img)


def test_inplace_move_with_an_impossible_source_leaves_its_destination_alone():
    """A move whose source is no chunk of the plan, or a chunk of another length, is rejected in
    both phases: its temporary slot is never filled and its destination keeps its bytes (it used
    to receive whatever the slot held); the other moves of the same call are carried out."""
    chunk = 1024
    rng = np.random.default_rng(77)
    ref = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in (5 * chunk, 3 * chunk + 100)]
    image = DeviceBuffers(ref, chunk)
    n = image.plan.nchunks                                    # 5 + 4 chunks, chunk 8 is short
    src = np.arange(n, dtype=np.int64)
    src[0], src[1] = 1, 0                                     # a good swap
    src[2] = n + 5                                            # no such chunk
    src[3] = 8                                                # the short chunk: another length
    src[6] = 4                                                # a good move
    moved = (src >= 0) & (src != np.arange(n))
    need = int(moved.sum()) * chunk
    temp = torch.full((need + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    ws = torch.empty(ck.moves_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ck.apply_moves_inplace(image.plan, torch.from_numpy(src).cuda(), temp, ws, counts, rejected,
                           temp_cap=need)
    torch.cuda.synchronize()
    assert int(rejected.item()) == 2
    want = [b.copy() for b in ref]
    want[0][0:chunk], want[0][chunk:2 * chunk] = ref[0][chunk:2 * chunk], ref[0][0:chunk]
    want[1][chunk:2 * chunk] = ref[0][4 * chunk:5 * chunk]    # chunk 6 = buffer 1, second chunk
    got, img = image.host()
    for g, w in zip(got, want):                              # chunks 2 and 3 still hold the reference
        assert np.array_equal(g, w)
    assert image.canaries_intact(img)
