"""ckpt_restore_chain on the GPU against the oracle's chain restore (paper sec. 4.6: a restore
applies a chain of incremental snapshots, oldest first).  Destination bytes, canaries around the
buffers and the three statistics are compared; the links reach both sides as the same bytes."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


def evolve(rng, state, nwrites, span):
    new = [b.copy() for b in state]
    for _ in range(nwrites):
        i = int(rng.choice([k for k, b in enumerate(new) if b.size]))
        off = int(rng.integers(0, new[i].size))
        new[i][off:off + int(rng.integers(1, span))] ^= 0x6B
    return new


def oracle_links(states, chunk, first_is_full=True):
    """One (staging, manifest) per state from the oracle's own path: state 0 whole (or against
    nothing at all when not first_is_full), every later one against the digests before it."""
    links, prev = [], None
    for st in states:
        dig = oracle.fingerprint(st, chunk)
        mask, _ = oracle.diff(st, chunk, dig, prev)
        staging, man, _ = oracle.compact(st, chunk, mask, dig)
        links.append((staging, man))
        prev = dig
    return links if first_is_full else links[1:]


def upload(links, slack=64):
    """Links as device tensors in the shape the binding takes; staging gets `slack` more bytes
    than staging_bytes says, so a read past the stated size would not fault but would be wrong."""
    import torch
    out = []
    for staging, man in links:
        s = torch.from_numpy(np.concatenate([staging, np.full(slack, 0x99, np.uint8)])).cuda()
        m = torch.from_numpy(np.concatenate([man.view(np.uint8).reshape(-1),
                                             np.zeros(32, np.uint8)])).cuda()
        out.append((s, int(staging.size), m, int(man.size), None))
    return out


def run_chain(dst, dev_links, with_stats=True, only=None):
    import torch
    from paper_2202_07848_amd import binding as ck
    ws = torch.full((ck.restore_chain_workspace_bytes(dst.plan.nchunks) + 16,), 0xEE,
                    dtype=torch.uint8, device="cuda")
    stats = torch.full((3,), -7, dtype=torch.int64, device="cuda") if with_stats else None
    d_only = None if only is None else torch.from_numpy(
        np.concatenate([only, np.full(16, 0xFF, np.uint8)])).cuda()
    ck.restore_chain(dst.plan, dev_links, ws, stats, only=d_only)
    torch.cuda.synchronize()
    if stats is None:
        return None
    v = stats.cpu().numpy().view(np.uint64)
    return {"written": int(v[0]), "superseded": int(v[1]), "rejected": int(v[2])}


def check(sizes, chunk, links, start_byte=0x5A, only=None):
    from gpu_util import DeviceBuffers
    start = [np.full(n, start_byte, np.uint8) for n in sizes]
    want = [b.copy() for b in start]
    want_stats = oracle.restore_chain(want, chunk, links, only)
    dst = DeviceBuffers(start, chunk)
    got_stats = run_chain(dst, upload(links), only=only)
    got, img = dst.host()
    for i, (g, w) in enumerate(zip(got, want)):
        assert np.array_equal(g, w), f"buffer {i} differs"
    assert dst.canaries_intact(img)
    assert got_stats == want_stats
    return want_stats


@pytest.mark.parametrize("chunk,sizes,span", [
    (256, [5000, 256, 0, 1300, 77, 4096, 16, 100000], 700),
    (4096, [40000, 4096, 123457, 0, 8192, 70001, 1, 4095, 4097], 3000),
    (65536, [1 << 20, 65536, 200001, 0, 65535, 65537, 3 << 16, 48], 50000),     # 4 pieces per chunk
    (1 << 20, [(3 << 20) + 4321, 1 << 20, 77777, (2 << 20) - 16], 300000),      # 64 pieces per chunk
])
@pytest.mark.parametrize("nlinks", [1, 2, 5])
def test_chain_from_the_snapshot_path(chunk, sizes, span, nlinks):
    rng = np.random.default_rng(chunk % 1000 + nlinks)
    states = [[rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]]
    for s in range(nlinks - 1):
        states.append(evolve(rng, states[-1], 3 + 2 * s, span))
    stats = check(sizes, chunk, oracle_links(states, chunk))
    assert stats["rejected"] == 0 and stats["written"] == oracle.nchunks(states[0], chunk)
    if nlinks > 1:
        stats = check(sizes, chunk, oracle_links(states, chunk, first_is_full=False))
        assert 0 < stats["written"] < oracle.nchunks(states[0], chunk)


def sliced_link(state, chunk, chosen):
    """A link holding exactly the chunks `chosen`, in the given order (may repeat)."""
    pcs = [(i, o, min(chunk, b.size - o)) for i, b in enumerate(state) for o in range(0, b.size, chunk)]
    parts, man, soff = [], np.zeros(len(chosen), dtype=oracle.ENTRY_DTYPE), 0
    for e, k in enumerate(chosen):
        i, o, n = pcs[k]
        parts += [state[i][o:o + n], np.zeros((-n) % 16, np.uint8)]
        man[e] = (i, n, o, soff, k)
        soff += n + (-n) % 16
    return (np.concatenate(parts) if parts else np.zeros(0, np.uint8)), man


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_subsets_in_sixteen_links(seed):
    """The longest chain one call takes; every link holds a random subset, so most chunks have
    several holders and some have none."""
    from paper_2202_07848_amd import binding as ck
    sizes, chunk = [9000, 512, 0, 2600, 150, 8192, 33000], 512
    rng = np.random.default_rng(seed)
    n = sum((s + chunk - 1) // chunk for s in sizes)
    links = []
    for _ in range(ck.CHAIN_MAX):
        state = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
        chosen = np.sort(rng.choice(n, size=int(rng.integers(0, n // 3)), replace=False))
        links.append(sliced_link(state, chunk, chosen.tolist()))
    stats = check(sizes, chunk, links)
    assert stats["superseded"] > 0 and stats["written"] < n


@pytest.mark.parametrize("seed", [1, 2, 3])
@pytest.mark.parametrize("density", [0.0, 0.1, 0.6, 1.0])
def test_restore_restricted_to_marked_chunks(seed, density):
    """d_only: unmarked chunks keep their bytes and their entries are counted nowhere; bad
    entries are still counted."""
    sizes, chunk = [9000, 512, 0, 2600, 150, 8192, 33000], 512
    rng = np.random.default_rng(50 + seed)
    n = sum((s + chunk - 1) // chunk for s in sizes)
    links = []
    for _ in range(5):
        state = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
        chosen = np.sort(rng.choice(n, size=int(rng.integers(1, n)), replace=False))
        links.append(sliced_link(state, chunk, chosen.tolist()))
    links[2][1]["buf"][0] = 77                 # one entry that fits nowhere
    only = (rng.random(n) < density).astype(np.uint8)
    only[only != 0] = rng.integers(1, 256, size=int(only.sum()), dtype=np.uint8)
    stats = check(sizes, chunk, links, only=only)
    assert stats["rejected"] == 1 and stats["written"] <= int((only != 0).sum())


def test_a_chunk_held_twice_by_one_link_and_unsorted_entries():
    """Manifests this library never writes: entries in descending order and the same chunk twice
    in one link with different bytes.  The later entry's bytes must stay, as in a one-by-one
    restore."""
    sizes, chunk = [3000, 1024, 700], 256
    rng = np.random.default_rng(4)
    a = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    b = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    n = sum((s + chunk - 1) // chunk for s in sizes)
    sa, ma = sliced_link(a, chunk, list(range(n))[::-1])
    sb, mb = sliced_link(b, chunk, [3, 5, 3, 11, 5, 18])
    # after b's entries the same link holds chunks 3 and 5 once more, with state a's bytes
    again = ma[[n - 1 - 3, n - 1 - 5]].copy()
    again["stage_off"] += sb.size
    twice = (np.concatenate([sb, sa]), np.concatenate([mb, again]))
    stats = check(sizes, chunk, [(sa, ma), (sb, mb), twice])
    assert stats["rejected"] == 0 and stats["written"] == n


def test_entries_that_are_not_whole_chunks_are_skipped_like_the_oracle_does():
    sizes, chunk = [5000, 256, 0, 1300, 77, 4096], 256
    rng = np.random.default_rng(11)
    s0 = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    s1 = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    n = sum((s + chunk - 1) // chunk for s in sizes)
    first = sliced_link(s0, chunk, list(range(0, n, 2)))
    staging, man = sliced_link(s1, chunk, list(range(n)))
    man["len"][1] = 240                       # not the whole chunk
    man["buf_off"][2] += 16                   # inside a chunk
    man["len"][19] = chunk                    # last chunk of buffer 0 (136 bytes) given full length
    man["buf"][4] = len(sizes)                # no such buffer
    man["stage_off"][n - 1] = staging.size - 16          # would read past staging
    man["stage_off"][6] += 8                  # not a multiple of 16
    man["buf"][8] = 2                         # the empty buffer
    man["buf_off"][10] = 1 << 40              # far outside
    stats = check(sizes, chunk, [first, (staging, man)])
    assert stats["rejected"] == 8


def test_each_link_is_bounded_by_its_own_staging_size():
    sizes, chunk = [5000, 256, 1300], 256
    rng = np.random.default_rng(17)
    s0 = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    s1 = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    n = sum((s + chunk - 1) // chunk for s in sizes)
    first = sliced_link(s0, chunk, list(range(n)))
    staging, man = sliced_link(s1, chunk, [0, 1, 2, 3])
    man["stage_off"][3] = staging.size
    stats = check(sizes, chunk, [first, (staging, man)])
    assert stats == {"written": n, "superseded": 3, "rejected": 1}


def test_entry_count_read_from_device_counts_and_no_stats():
    """d_counts->ndirty below the capacity cuts the link short; above it the capacity holds.
    Without a stats pointer the bytes are the same."""
    import torch
    from gpu_util import DeviceBuffers
    sizes, chunk = [5000, 256, 1300, 4096], 256
    rng = np.random.default_rng(23)
    s0 = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    s1 = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    n = sum((s + chunk - 1) // chunk for s in sizes)
    l0, l1 = sliced_link(s0, chunk, list(range(n))), sliced_link(s1, chunk, list(range(0, n, 3)))
    for ndirty0, ndirty1 in ((7, 2), (n + 50, 0), (0, 5)):
        dev = upload([l0, l1])
        counts = [torch.tensor([nd, 0, 0], dtype=torch.int64, device="cuda") for nd in (ndirty0, ndirty1)]
        dev = [d[:4] + (c,) for d, c in zip(dev, counts)]
        want = [np.full(s, 0x11, np.uint8) for s in sizes]
        cut = [(l0[0], l0[1][:min(ndirty0, n)]), (l1[0], l1[1][:min(ndirty1, l1[1].size)])]
        want_stats = oracle.restore_chain(want, chunk, cut)
        for with_stats in (True, False):
            dst = DeviceBuffers([np.full(s, 0x11, np.uint8) for s in sizes], chunk)
            got_stats = run_chain(dst, dev, with_stats)
            got, img = dst.host()
            assert all(np.array_equal(g, w) for g, w in zip(got, want)) and dst.canaries_intact(img)
            assert got_stats == (want_stats if with_stats else None)


def test_empty_chain_empty_links_and_empty_plan():
    import torch
    from gpu_util import DeviceBuffers
    from paper_2202_07848_amd import binding as ck
    sizes, chunk = [5000, 256], 256
    dst = DeviceBuffers([np.full(s, 0x3C, np.uint8) for s in sizes], chunk)
    assert run_chain(dst, []) == {"written": 0, "superseded": 0, "rejected": 0}
    empty = (None, 0, None, 0, None)
    assert run_chain(dst, [empty, empty]) == {"written": 0, "superseded": 0, "rejected": 0}
    got, img = dst.host()
    assert all(np.all(g == 0x3C) for g in got) and dst.canaries_intact(img)
    nothing = ck.Plan([], chunk)
    ws = torch.zeros(64, dtype=torch.uint8, device="cuda")
    stats = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    st, man = sliced_link([np.arange(256, dtype=np.uint8)], chunk, [0])
    ck.restore_chain(nothing, upload([(st, man)]), ws, stats)
    torch.cuda.synchronize()
    assert stats.tolist() == [0, 0, 1]


def test_same_result_as_restores_one_by_one_on_the_device():
    """The definition, taken on the GPU itself: ckpt_restore per link in order."""
    import torch
    from gpu_util import DeviceBuffers
    from paper_2202_07848_amd import binding as ck
    sizes, chunk = [300000, 65536, 0, 99999, 70000], 4096
    rng = np.random.default_rng(31)
    states = [[rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]]
    for s in range(5):
        states.append(evolve(rng, states[-1], 6 + s, 20000))
    dev = upload(oracle_links(states, chunk))
    one, two = (DeviceBuffers([np.zeros(n, np.uint8) for n in sizes], chunk) for _ in range(2))
    for staging, nbytes, man, cap, _ in dev:
        ck.restore(one.plan, staging, nbytes, man, cap)
    stats = run_chain(two, dev)
    assert torch.equal(one.arena, two.arena)
    got, _ = two.host()
    assert all(np.array_equal(g, s) for g, s in zip(got, states[-1]))
    assert stats["written"] == two.plan.nchunks and stats["superseded"] > 0


def test_argument_checks():
    import torch
    from gpu_util import DeviceBuffers
    from paper_2202_07848_amd import binding as ck
    dst = DeviceBuffers([np.zeros(1000, np.uint8)], 256)
    ws = torch.zeros(ck.restore_chain_workspace_bytes(dst.plan.nchunks) + 16, dtype=torch.uint8,
                     device="cuda")
    st, man = sliced_link([np.zeros(1000, np.uint8)], 256, [0, 1])
    link = upload([(st, man)])[0]
    with pytest.raises(ck.CkptError) as e:
        ck.restore_chain(dst.plan, [link] * (ck.CHAIN_MAX + 1), ws)
    assert e.value.status == -1
    with pytest.raises(ck.CkptError) as e:
        ck.restore_chain(dst.plan, [link], ws[:8])
    assert e.value.status == -5                           # workspace too small
    with pytest.raises(ck.CkptError) as e:
        ck.restore_chain(dst.plan, [link], ws[8:])
    assert e.value.status == -2                           # workspace not 16-byte aligned
    with pytest.raises(ck.CkptError) as e:
        ck.restore_chain(dst.plan, [(link[0][16:][8:], 16, link[2], 2, None)], ws)
    assert e.value.status == -2                           # staging not 16-byte aligned
    with pytest.raises(ck.CkptError) as e:
        ck.restore_chain(dst.plan, [(link[0], link[1], None, 2, None)], ws)
    assert e.value.status == -1                           # entries promised, no manifest
    with pytest.raises(ck.CkptError) as e:
        ck.restore_chain(dst.plan, [(link[0], link[1], link[2], 1 << 40, None)], ws)
    assert e.value.status == -1


def test_chain_restore_replays_from_a_hip_graph_with_changing_entry_counts():
    """The call only enqueues kernels and reads the entry counts on the device, so it can be
    captured; between replays the links' counts and the destination change through eager work,
    and every replay must give what the oracle gives for those counts."""
    import torch
    from gpu_util import DeviceBuffers
    from paper_2202_07848_amd import binding as ck
    sizes, chunk = [50000, 4096, 0, 12345, 70001], 4096
    rng = np.random.default_rng(41)
    states = [[rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes] for _ in range(3)]
    n = sum((s + chunk - 1) // chunk for s in sizes)
    chosen = [list(range(n)), list(range(0, n, 2)), list(range(1, n, 3))]
    links = [sliced_link(s, chunk, c) for s, c in zip(states, chosen)]
    counts = [torch.tensor([len(c), 0, 0], dtype=torch.int64, device="cuda") for c in chosen]
    dev = [d[:4] + (c,) for d, c in zip(upload(links), counts)]
    dst = DeviceBuffers([np.zeros(s, np.uint8) for s in sizes], chunk)
    ws = torch.zeros(ck.restore_chain_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    stats = torch.zeros(3, dtype=torch.int64, device="cuda")

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        ck.restore_chain(dst.plan, dev, ws, stats, stream=side)      # eager warm-up
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ck.restore_chain(dst.plan, dev, ws, stats, stream=side)
    torch.cuda.synchronize()

    for replay, cut in enumerate([(n, len(chosen[1]), len(chosen[2])), (5, 0, 3), (n, 2, 0),
                                  (0, 0, 0), (n, len(chosen[1]), len(chosen[2]))]):
        for c, k in zip(counts, cut):
            c[0] = k
        dst.arena.copy_(DeviceBuffers([np.full(s, replay, np.uint8) for s in sizes], chunk).arena)
        ws.fill_(0xEE)
        stats.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = [np.full(s, replay, np.uint8) for s in sizes]
        want_stats = oracle.restore_chain(want, chunk, [(l[0], l[1][:k]) for l, k in zip(links, cut)])
        got, img = dst.host()
        assert all(np.array_equal(g, w) for g, w in zip(got, want)), replay
        assert dst.canaries_intact(img), replay
        v = stats.cpu().numpy().view(np.uint64)
        assert {"written": int(v[0]), "superseded": int(v[1]), "rejected": int(v[2])} == want_stats


# ---- folding a chain into one link -----------------------------------------------------------

def run_merge(plan, dev_links, staging_cap, manifest_cap, fill=0xA5, slack=256):
    import torch
    from paper_2202_07848_amd import binding as ck
    staging = torch.full((staging_cap + slack,), fill, dtype=torch.uint8, device="cuda")
    manifest = torch.full((manifest_cap * 32 + slack,), fill, dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    stats = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    ws = torch.full((ck.merge_chain_workspace_bytes(plan.nchunks) + 16,), 0xEE, dtype=torch.uint8,
                    device="cuda")
    ck.merge_chain(plan, dev_links, staging, manifest, counts, ws, stats, staging_cap=staging_cap,
                   manifest_cap=manifest_cap)
    torch.cuda.synchronize()
    c = counts.cpu().numpy().view(np.uint64)
    v = stats.cpu().numpy().view(np.uint64)
    return (staging.cpu().numpy(), manifest.cpu().numpy(),
            {"ndirty": int(c[0]), "staged_bytes": int(c[1]), "overflow": int(c[2])},
            {"written": int(v[0]), "superseded": int(v[1]), "rejected": int(v[2])})


def check_merge(sizes, chunk, links, caps=None, fill=0xA5):
    """GPU merge against the oracle's: staging and manifest byte for byte including the untouched
    fill behind what was written and the slack behind the capacities, counts and stats."""
    from gpu_util import DeviceBuffers
    if caps is None:
        o_st, o_man, o_counts, o_stats = oracle.merge_chain(sizes, chunk, links, fill=fill)
        caps = (o_st.size, o_man.size)
    else:
        o_st, o_man, o_counts, o_stats = oracle.merge_chain(sizes, chunk, links, caps[0], caps[1],
                                                            fill=fill)
    geometry = DeviceBuffers([np.full(n, 0x31, np.uint8) for n in sizes], chunk)
    before = geometry.arena.clone()
    st, man, counts, stats = run_merge(geometry.plan, upload(links), caps[0], caps[1], fill)
    assert counts == o_counts and stats == o_stats
    assert np.array_equal(st[:caps[0]], o_st) and np.all(st[caps[0]:] == fill)
    assert np.array_equal(man[:caps[1] * 32], o_man.view(np.uint8).reshape(-1))
    assert np.all(man[caps[1] * 32:] == fill)
    import torch
    assert torch.equal(before, geometry.arena)            # the plan's buffers are not touched
    return o_st, o_man, o_counts, o_stats


@pytest.mark.parametrize("chunk,sizes,span", [
    (256, [5000, 256, 0, 1300, 77, 4096, 16, 100000], 700),
    (4096, [40000, 4096, 123457, 0, 8192, 70001, 1, 4095, 4097], 3000),
    (65536, [1 << 20, 65536, 200001, 0, 65535, 65537, 3 << 16, 48], 50000),
    (1 << 20, [(3 << 20) + 4321, 1 << 20, 77777, (2 << 20) - 16], 300000),
])
@pytest.mark.parametrize("nlinks", [1, 3, 5])
def test_merge_of_chains_from_the_snapshot_path(chunk, sizes, span, nlinks):
    rng = np.random.default_rng(chunk % 1000 + 7 * nlinks)
    states = [[rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]]
    for s in range(nlinks):
        states.append(evolve(rng, states[-1], 3 + 2 * s, span))
    links = oracle_links(states, chunk, first_is_full=False)      # deltas only
    st, man, counts, stats = check_merge(sizes, chunk, links)
    assert stats["rejected"] == 0 and 0 < counts["ndirty"] < oracle.nchunks(states[0], chunk)
    # the merged link, applied to the first state, gives the last one
    dst = [b.copy() for b in states[0]]
    assert oracle.restore(dst, chunk, st, man) == 0
    assert all(np.array_equal(d, s) for d, s in zip(dst, states[-1]))


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_merge_of_random_subsets_in_sixteen_links(seed):
    from paper_2202_07848_amd import binding as ck
    sizes, chunk = [9000, 512, 0, 2600, 150, 8192, 33000], 512
    rng = np.random.default_rng(seed)
    n = sum((s + chunk - 1) // chunk for s in sizes)
    links = []
    for _ in range(ck.CHAIN_MAX):
        state = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
        chosen = np.sort(rng.choice(n, size=int(rng.integers(0, n // 3)), replace=False))
        links.append(sliced_link(state, chunk, chosen.tolist()))
    _, _, counts, stats = check_merge(sizes, chunk, links)
    assert stats["superseded"] > 0 and counts["ndirty"] == stats["written"] < n


def test_merge_with_bad_entries_unsorted_manifests_and_a_chunk_held_twice():
    sizes, chunk = [5000, 256, 0, 1300, 77, 4096], 256
    rng = np.random.default_rng(11)
    a = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    b = [rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes]
    n = sum((s + chunk - 1) // chunk for s in sizes)
    sa, ma = sliced_link(a, chunk, list(range(0, n, 2))[::-1])           # descending
    sb, mb = sliced_link(b, chunk, [3, 5, 3, 11, 5, 18, 7, 9, 21])
    mb["len"][6] = 240                        # chunk 7: not the whole chunk
    mb["buf_off"][7] += 16                    # chunk 9: inside a chunk
    mb["buf"][8] = len(sizes)                 # no such buffer
    again = ma[[0, 1]].copy()                 # two more holders inside link b, with a's bytes
    again["stage_off"] += sb.size
    twice = (np.concatenate([sb, sa]), np.concatenate([mb, again]))
    _, _, _, stats = check_merge(sizes, chunk, [(sa, ma), twice])
    assert stats["rejected"] == 3


def test_merge_capacities():
    sizes, chunk = [5000, 256, 1300, 4096, 77], 256
    rng = np.random.default_rng(29)
    states = [[rng.integers(0, 256, size=s, dtype=np.uint8) for s in sizes] for _ in range(3)]
    n = sum((s + chunk - 1) // chunk for s in sizes)
    links = [sliced_link(s, chunk, sorted(rng.choice(n, size=n // 2, replace=False).tolist()))
             for s in states]
    st, man, counts, _ = check_merge(sizes, chunk, links)
    m = man.size
    for caps in ((st.size, m - 2), (int(man["stage_off"][4]) + 100, m), (int(man["stage_off"][5]), 3),
                 (st.size - 16, m), (0, 0), (st.size + 4096, m + 9)):
        _, _, c, _ = check_merge(sizes, chunk, links, caps)
        assert c["ndirty"] == m and c["staged_bytes"] == counts["staged_bytes"]


def test_merge_of_nothing_and_argument_checks():
    import torch
    from gpu_util import DeviceBuffers
    from paper_2202_07848_amd import binding as ck
    sizes, chunk = [5000, 256], 256
    _, _, counts, stats = check_merge(sizes, chunk, [])
    assert counts == {"ndirty": 0, "staged_bytes": 0, "overflow": 0}
    empty = (np.zeros(0, np.uint8), np.zeros(0, oracle.ENTRY_DTYPE))
    check_merge(sizes, chunk, [empty, empty])
    geometry = DeviceBuffers([np.zeros(n, np.uint8) for n in sizes], chunk)
    link = upload([sliced_link([np.zeros(n, np.uint8) for n in sizes], chunk, [0, 1])])[0]
    ws = torch.zeros(ck.merge_chain_workspace_bytes(geometry.plan.nchunks) + 16, dtype=torch.uint8,
                     device="cuda")
    out = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    man = torch.zeros(4 * 32, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    for args, status in (((geometry.plan, [link], out, man, None, ws), -1),
                         ((geometry.plan, [link] * 17, out, man, counts, ws), -1),
                         ((geometry.plan, [link], out, man, counts, ws[:64]), -5),
                         ((geometry.plan, [link], out[8:], man, counts, ws), -2),
                         ((geometry.plan, [link], out, man, counts, ws[8:]), -2)):
        with pytest.raises(ck.CkptError) as e:
            ck.merge_chain(*args)
        assert e.value.status == status


def test_merged_link_through_the_device_restore_equals_the_chain_restore():
    """merge then ckpt_restore == ckpt_restore_chain, on the device, and both equal the last
    state of the chain."""
    import torch
    from gpu_util import DeviceBuffers
    from paper_2202_07848_amd import binding as ck
    sizes, chunk = [300000, 65536, 0, 99999, 70000], 4096
    rng = np.random.default_rng(37)
    states = [[rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]]
    for s in range(5):
        states.append(evolve(rng, states[-1], 6 + s, 20000))
    dev = upload(oracle_links(states, chunk, first_is_full=False))
    one, two = (DeviceBuffers(states[0], chunk) for _ in range(2))
    n = one.plan.nchunks
    staging = torch.zeros(n * chunk, dtype=torch.uint8, device="cuda")
    manifest = torch.zeros(n * 32, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    ws = torch.zeros(ck.merge_chain_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    ck.merge_chain(one.plan, dev, staging, manifest, counts, ws)
    ck.restore_counted(one.plan, staging, staging.numel(), manifest, n, counts)
    run_chain(two, dev)
    assert torch.equal(one.arena, two.arena)
    got, _ = one.host()
    assert all(np.array_equal(g, s) for g, s in zip(got, states[-1]))


def test_links_and_merged_link_in_pinned_host_memory():
    """The links of a chain live where checkpoints live: outside the device.  With their staging
    areas in pinned host memory the kernels read the bytes over the host link themselves; the
    merged link may be written to pinned host memory too."""
    import torch
    from gpu_util import DeviceBuffers
    from paper_2202_07848_amd import binding as ck
    sizes, chunk = [300000, 65536, 0, 99999, 70000], 4096
    rng = np.random.default_rng(43)
    states = [[rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]]
    for s in range(3):
        states.append(evolve(rng, states[-1], 6 + s, 20000))
    links = oracle_links(states, chunk, first_is_full=False)
    dev = []
    for staging, man in links:
        host = torch.empty(max(16, staging.size), dtype=torch.uint8, pin_memory=True)
        host[:staging.size] = torch.from_numpy(staging)
        m = torch.from_numpy(man.view(np.uint8).reshape(-1).copy()).cuda()
        dev.append((host, int(staging.size), m, int(man.size), None))
    dst = DeviceBuffers(states[0], chunk)
    want = [b.copy() for b in states[0]]
    want_stats = oracle.restore_chain(want, chunk, links)
    assert run_chain(dst, dev) == want_stats
    got, img = dst.host()
    assert all(np.array_equal(g, s) for g, s in zip(got, states[-1])) and dst.canaries_intact(img)

    o_st, o_man, o_counts, _ = oracle.merge_chain(sizes, chunk, links)
    out = torch.full((o_st.size + 64,), 0xA5, dtype=torch.uint8).pin_memory()
    manifest = torch.zeros(o_man.size * 32, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    ws = torch.zeros(ck.merge_chain_workspace_bytes(dst.plan.nchunks), dtype=torch.uint8, device="cuda")
    ck.merge_chain(dst.plan, dev, out, manifest, counts, ws, staging_cap=o_st.size)
    torch.cuda.synchronize()
    assert np.array_equal(out.numpy()[:o_st.size], o_st) and np.all(out.numpy()[o_st.size:] == 0xA5)
    assert np.array_equal(ck.manifest_to_numpy(manifest, o_man.size), o_man)
    assert [int(x) for x in counts.cpu().numpy().view(np.uint64)] == [o_counts["ndirty"],
                                                                      o_counts["staged_bytes"], 0]
