"""Context switches between four time-sliced ranks that share one device-memory image
(paper sec. 5.1, 5.2.1, 6), on a reduced 1.3 B x4 configuration: every switch swaps the
outgoing rank's delta out to pinned host memory and the incoming rank's delta in, with no
host read in between.  The oracle plays the same rotation on host arrays (checksum, compare,
compact, restore); after every switch -- and after a whole rotation enqueued without any
synchronisation -- the device image, the swapped-out bytes, the manifests and the counts must
equal the oracle's."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DeviceBuffers
from paper_2202_07848_amd import binding as ck
from paper_2202_07848_amd import workloads as wl
from paper_2202_07848_amd.switching import TimeSlicedRanks

pytestmark = pytest.mark.gpu

NRANKS = 4


class OracleRanks:
    """The rotation on the host, step by step with the oracle's functions."""

    def __init__(self, w, base, first_state):
        self.chunk = w.chunk
        self.image = [b.copy() for b in first_state]
        self.ref = oracle.fingerprint(base, w.chunk, 8)
        self.staging = [None] * NRANKS
        self.manifest = [None] * NRANKS
        self.counts = [None] * NRANKS

    def delta_of(self, state):
        dig = oracle.fingerprint(state, self.chunk, 8)
        mask, _ = oracle.diff(state, self.chunk, dig, self.ref)
        return oracle.compact(state, self.chunk, mask, dig)

    def switch(self, outgoing, incoming):
        self.staging[outgoing], self.manifest[outgoing], self.counts[outgoing] = \
            self.delta_of(self.image)
        assert oracle.restore(self.image, self.chunk, self.staging[incoming],
                              self.manifest[incoming]) == 0


def run_a_mini_batch(w, rng, o, dev):
    """The resident rank changes some of its own (per-rank) state: fresh bytes in a few chunks
    of gradient and activation buffers, the same bytes on the host and on the device."""
    own = [i for i, b in enumerate(w.bufs) if not b.shared and b.nbytes >= 64]
    for i in rng.choice(own, size=6, replace=False).tolist():
        n = w.bufs[i].nbytes
        lo = int(rng.integers(0, n - 32))
        hi = min(n, lo + int(rng.integers(1, 3 * w.chunk)))
        fresh = rng.integers(0, 256, size=hi - lo, dtype=np.uint8)
        o.image[i][lo:hi] = fresh
        dev.arena[dev.offs[i] + lo:dev.offs[i] + hi] = torch.from_numpy(fresh).cuda()


def check_rank_area(sw, o, r):
    c = sw.counts[r].cpu().numpy().view(np.uint64)
    want = o.counts[r]
    assert (int(c[0]), int(c[1]), int(c[2])) == (want["ndirty"], want["staged_bytes"], 0)
    assert np.array_equal(sw.host[r].numpy()[:want["staged_bytes"]], o.staging[r])
    assert np.array_equal(ck.manifest_to_numpy(sw.manifest[r], want["ndirty"]), o.manifest[r])


@pytest.mark.parametrize("exchange", [True, False], ids=["exchange_pass", "out_then_in"])
@pytest.mark.parametrize("sync_every_switch", [True, False], ids=["checked_each_switch", "eager"])
def test_round_robin_of_four_ranks_matches_the_oracle(sync_every_switch, exchange):
    w = wl.config(4, 8)
    base = wl.numpy_replica(w, 0)
    ranks = [wl.numpy_replica(w, r) for r in range(1, NRANKS + 1)]
    dev = DeviceBuffers(ranks[0], w.chunk)                  # rank 0 is resident first
    o = OracleRanks(w, base, ranks[0])
    n = dev.plan.nchunks
    ref = torch.from_numpy(o.ref.view(np.int64)).cuda()
    cap_bytes, cap_entries = w.distinct_bytes + 16 * n, w.distinct_chunks
    sw = TimeSlicedRanks(dev.plan, ref, NRANKS, cap_bytes, cap_entries)

    # the other ranks' deltas reach their host areas the way they would in a running job:
    # each was resident once and was swapped out (here from a scratch copy of its state)
    for r in range(1, NRANKS):
        tmp = DeviceBuffers(ranks[r], w.chunk)
        one = TimeSlicedRanks(tmp.plan, ref, 1, cap_bytes, cap_entries)
        one.swap_out(0)
        torch.cuda.synchronize()
        sw.host[r].copy_(one.host[0])
        sw.manifest[r].copy_(one.manifest[0])
        sw.counts[r].copy_(one.counts[0])
        sw.mask[r].copy_(one.mask[0])
        o.staging[r], o.manifest[r], o.counts[r] = o.delta_of(ranks[r])
        check_rank_area(sw, o, r)

    rng = np.random.default_rng(4)
    side = torch.cuda.Stream()
    first_kernel_ran = torch.zeros(1, dtype=torch.int64, device="cuda")
    resident = 0
    for step in range(2 * NRANKS):                          # two full rotations
        run_a_mini_batch(w, rng, o, dev)
        nxt = (resident + 1) % NRANKS
        sw.switch(resident, nxt, exchange=exchange)
        o.switch(resident, nxt)
        # the incoming rank's first kernel, dispatched at once on another stream behind an event
        done = torch.cuda.Event()
        done.record()
        with torch.cuda.stream(side):
            side.wait_event(done)
            first_kernel_ran.add_(1)
        if sync_every_switch:
            torch.cuda.synchronize()
            assert int(sw.rejected.item()) == 0
            assert int(sw.serial.item()) == 0          # the deltas line up: one exchange pass
            check_rank_area(sw, o, resident)
            got, img = dev.host()
            assert all(np.array_equal(g, want) for g, want in zip(got, o.image)), step
            assert dev.canaries_intact(img)
        resident = nxt
    torch.cuda.synchronize()
    assert int(first_kernel_ran.item()) == 2 * NRANKS and int(sw.rejected.item()) == 0
    assert resident == 0
    got, img = dev.host()
    assert all(np.array_equal(g, want) for g, want in zip(got, o.image))
    assert dev.canaries_intact(img)
    for r in range(NRANKS):
        check_rank_area(sw, o, r)
    assert sw.same_dirty_set()
    # what is resident is rank 0 as it was when it was swapped out last, not the base
    assert not all(np.array_equal(g, b) for g, b in zip(got, base))


def test_exchange_falls_back_to_out_then_in_when_the_deltas_do_not_line_up():
    """A rank that also changed a chunk of shared state has one entry more than the rank that
    comes in: ckpt_exchange notices on the device and does swap-out, then swap-in; the result is
    what the oracle's compact followed by restore gives (that the incoming rank then sees the
    changed shared chunk is the caller's business, and the oracle's rotation sees it too)."""
    w = wl.config(4, 12)
    base = wl.numpy_replica(w, 0)
    ranks = [wl.numpy_replica(w, r) for r in (1, 2)]
    dev = DeviceBuffers(ranks[0], w.chunk)
    o = OracleRanks(w, base, ranks[0])
    n = dev.plan.nchunks
    ref = torch.from_numpy(o.ref.view(np.int64)).cuda()
    cap_bytes, cap_entries = w.nbytes + 16 * n, n
    sw = TimeSlicedRanks(dev.plan, ref, 2, cap_bytes, cap_entries)
    tmp = DeviceBuffers(ranks[1], w.chunk)
    one = TimeSlicedRanks(tmp.plan, ref, 1, cap_bytes, cap_entries)
    one.swap_out(0)
    torch.cuda.synchronize()
    for name in ("host", "manifest", "counts", "mask"):
        getattr(sw, name)[1].copy_(getattr(one, name)[0])
    o.staging[1], o.manifest[1], o.counts[1] = o.delta_of(ranks[1])
    # the resident rank touches a shared buffer (an early one, so every later entry shifts)
    shared = next(i for i, b in enumerate(w.bufs) if b.shared and b.nbytes >= w.chunk)
    o.image[shared][5] ^= 0x40
    dev.arena[dev.offs[shared] + 5] ^= 0x40
    for exchange in (True, False):
        sw.switch(0, 1, exchange=exchange)
        o.switch(0, 1)
        torch.cuda.synchronize()
        assert int(sw.rejected.item()) == 0
        if exchange:
            assert int(sw.serial.item()) > 0
        check_rank_area(sw, o, 0)
        got, img = dev.host()
        assert all(np.array_equal(g, want) for g, want in zip(got, o.image))
        assert dev.canaries_intact(img)
        sw.switch(1, 0, exchange=exchange)                 # and back, again with one entry more
        o.switch(1, 0)
        torch.cuda.synchronize()
        check_rank_area(sw, o, 1)
        got, img = dev.host()
        assert all(np.array_equal(g, want) for g, want in zip(got, o.image))


def test_switches_replay_from_hip_graphs():
    """A switch enqueues kernels only, so it can be captured once per (outgoing, incoming) pair
    and replayed: two ranks ping-pong through two graphs, with mutations of the resident rank and
    eager synchronisations between replays; every replay is checked against the oracle."""
    w = wl.config(4, 12)
    base = wl.numpy_replica(w, 0)
    ranks = [wl.numpy_replica(w, r) for r in (1, 2)]
    dev = DeviceBuffers(ranks[0], w.chunk)
    o = OracleRanks(w, base, ranks[0])
    n = dev.plan.nchunks
    ref = torch.from_numpy(o.ref.view(np.int64)).cuda()
    cap_bytes, cap_entries = w.distinct_bytes + 16 * n, w.distinct_chunks
    sw = TimeSlicedRanks(dev.plan, ref, 2, cap_bytes, cap_entries)
    tmp = DeviceBuffers(ranks[1], w.chunk)
    one = TimeSlicedRanks(tmp.plan, ref, 1, cap_bytes, cap_entries)
    one.swap_out(0)
    torch.cuda.synchronize()
    for name in ("host", "manifest", "counts", "mask"):
        getattr(sw, name)[1].copy_(getattr(one, name)[0])
    o.staging[1], o.manifest[1], o.counts[1] = o.delta_of(ranks[1])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graphs = {}
    with torch.cuda.stream(side):
        # an eager round trip on the capture stream first (and its twin on the host)
        for a, b in ((0, 1), (1, 0)):
            sw.switch(a, b, stream=side)
            o.switch(a, b)
        side.synchronize()
        for a, b in ((0, 1), (1, 0)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                sw.switch(a, b, stream=side)
            graphs[(a, b)] = g
    torch.cuda.synchronize()
    got, _ = dev.host()
    assert all(np.array_equal(x, y) for x, y in zip(got, o.image))

    rng = np.random.default_rng(9)
    resident = 0
    for step in range(6):
        run_a_mini_batch(w, rng, o, dev)
        nxt = 1 - resident
        graphs[(resident, nxt)].replay()
        o.switch(resident, nxt)
        torch.cuda.synchronize()
        assert int(sw.rejected.item()) == 0 and int(sw.serial.item()) == 0
        check_rank_area(sw, o, resident)
        got, img = dev.host()
        assert all(np.array_equal(x, y) for x, y in zip(got, o.image)), step
        assert dev.canaries_intact(img)
        resident = nxt


def test_manifest_alone_equals_the_manifest_of_compact():
    """ckpt_manifest writes what ckpt_compact writes as metadata -- entries, counts, overflow
    under capacity limits -- and moves no chunk bytes."""
    rng = np.random.default_rng(31)
    sizes = [70001, 0, 4096, 300000, 17, 65536 + 40]
    snap = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]
    chunk = 1024
    dev = DeviceBuffers(snap, chunk)
    n = dev.plan.nchunks
    o_dig = oracle.fingerprint(snap, chunk)
    mask_h = (rng.random(n) < 0.4).astype(np.uint8)
    mask, dig = torch.from_numpy(mask_h).cuda(), torch.from_numpy(o_dig.view(np.int64)).cuda()
    full_st, full_man, _ = oracle.compact(snap, chunk, mask_h, o_dig)
    for st_cap, man_cap in ((full_st.size, full_man.size), (full_st.size // 2, full_man.size),
                            (full_st.size, 3), (0, 0)):
        o_st, o_man, o_cnt = oracle.compact(snap, chunk, mask_h, o_dig, staging_cap=st_cap,
                                            manifest_cap=man_cap)
        manifest = torch.full((man_cap * 32 + 64,), 0xA5, dtype=torch.uint8, device="cuda")
        counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
        ck.manifest(dev.plan, mask, dig, manifest, counts, st_cap, man_cap)
        torch.cuda.synchronize()
        c = counts.cpu().numpy().view(np.uint64)
        assert {"ndirty": int(c[0]), "staged_bytes": int(c[1]), "overflow": int(c[2])} == o_cnt
        raw = manifest.cpu().numpy()
        assert np.array_equal(raw[:32 * man_cap].view(oracle.ENTRY_DTYPE), o_man)
        assert np.all(raw[32 * man_cap:] == 0xA5)
        got, img = dev.host()
        assert all(np.array_equal(a, b) for a, b in zip(got, snap)) and dev.canaries_intact(img)


def test_exchange_skips_entries_that_do_not_fit_and_checks_its_arguments():
    """An entry whose bytes do not fit a staging area is left alone in both directions and
    counted; the others are exchanged.  Host-side argument errors are synchronous."""
    rng = np.random.default_rng(41)
    chunk = 4096
    a = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in (5 * chunk, 2 * chunk + 100)]
    b = [rng.integers(0, 256, size=x.size, dtype=np.uint8) for x in a]
    dev = DeviceBuffers(a, chunk)                      # rank A resident
    n = dev.plan.nchunks
    dig_a, dig_b = oracle.fingerprint(a, chunk), oracle.fingerprint(b, chunk)
    ones = np.ones(n, np.uint8)
    st_a, man_a, cnt_a = oracle.compact(a, chunk, ones, dig_a)
    st_b, man_b, cnt_b = oracle.compact(b, chunk, ones, dig_b)
    need = st_a.size
    short = need - 4096 - 112                          # the last two entries no longer fit
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x).view(np.uint8).reshape(-1)).cuda()
    man_out, man_in = t(man_a), t(man_b)
    counts = torch.tensor([n, need, 0], dtype=torch.int64, device="cuda")
    out = torch.full((need + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    inn = torch.cat([t(st_b), torch.zeros(64, dtype=torch.uint8, device="cuda")])
    serial = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ck.exchange(dev.plan, man_out, counts, out, short, man_in, counts, inn, need, n, serial,
                rejected)
    torch.cuda.synchronize()
    assert int(serial.item()) == 0
    fits = (man_a["stage_off"].astype(np.int64) + (man_a["len"].astype(np.int64) + 15) // 16 * 16
            <= short)
    assert int(rejected.item()) == int((~fits).sum()) == 2
    got, img = dev.host()
    want = [x.copy() for x in a]
    assert oracle.restore(want, chunk, st_b, man_b[fits]) == 0
    assert all(np.array_equal(g, w) for g, w in zip(got, want)) and dev.canaries_intact(img)
    host_out = out.cpu().numpy()
    kept = int(man_a["stage_off"][fits][-1] + (int(man_a["len"][fits][-1]) + 15) // 16 * 16)
    assert np.array_equal(host_out[:kept], st_a[:kept]) and np.all(host_out[kept:] == 0xA5)
    # argument errors
    for bad in (dict(counts_out=None), dict(staging_out=None), dict(manifest_in=None)):
        args = dict(manifest_out=man_out, counts_out=counts, staging_out=out, manifest_in=man_in,
                    counts_in=counts, staging_in=inn)
        args.update(bad)
        with pytest.raises(ck.CkptError) as e:
            ck.exchange(dev.plan, args["manifest_out"], args["counts_out"], args["staging_out"],
                        need, args["manifest_in"], args["counts_in"], args["staging_in"], need, n)
        assert e.value.status == -1
    with pytest.raises(ck.CkptError) as e:
        ck.exchange(dev.plan, man_out, counts, out[8:], need, man_in, counts, inn, need, n)
    assert e.value.status == -2


def chunk_differences(w, a, b):
    """Number of chunks in which two states differ, by comparing their bytes."""
    count = 0
    for x, y in zip(a, b):
        for o in range(0, x.size, w.chunk):
            count += not np.array_equal(x[o:o + w.chunk], y[o:o + w.chunk])
    return count


@pytest.mark.parametrize("exchange", [False, True], ids=["by_checksums", "exchange_then_repair"])
def test_exact_switch_between_ranks_that_changed_different_chunks(exchange):
    """Ranks that differ from the base in different chunks: one changes shared state on its own,
    one has a per-rank buffer that equals the base, and every mini-batch rewrites a few chunks
    anywhere.  `switch_exact` must leave exactly the incoming rank's state on the device after
    every switch, having written exactly the chunks in which the two ranks differ; the oracle's
    restricted chain restore, replayed on the host, must agree."""
    w = wl.config(4, 8)
    base = wl.numpy_replica(w, 0)
    state = [wl.numpy_replica(w, r) for r in range(1, NRANKS + 1)]
    shared = [i for i, b in enumerate(w.bufs) if b.shared and b.nbytes >= 4 * w.chunk]
    own = [i for i, b in enumerate(w.bufs) if not b.shared and b.nbytes >= 64]
    state[1][shared[0]][w.chunk:w.chunk + 100] ^= 0x5A           # rank 1 changes shared state alone
    state[2][own[0]][:] = base[own[0]]                            # rank 2 equals the base there
    state[3][shared[1]][5:50] ^= 0x21
    state[3][own[1]][:] = base[own[1]]

    dev = DeviceBuffers(base, w.chunk)                            # the base is resident first
    n = dev.plan.nchunks
    o_ref = oracle.fingerprint(base, w.chunk, 8)
    ref = torch.from_numpy(o_ref.view(np.int64)).cuda()
    cap_bytes, cap_entries = 2 * w.distinct_bytes + 16 * n, n
    sw = TimeSlicedRanks(dev.plan, ref, NRANKS, cap_bytes, cap_entries, exact=True)
    sw.capture_base(max_slice_bytes=w.nbytes // 3)                # the base copy in several slices
    full_mask, _ = oracle.diff(base, w.chunk, o_ref, None)
    base_link = oracle.compact(base, w.chunk, full_mask, o_ref)[:2]
    assert len(sw.base_links) >= 3 and sw.base_bytes == base_link[0].size
    assert np.array_equal(np.concatenate([l[0].numpy()[:l[1]] for l in sw.base_links]), base_link[0])

    def put(r):                                                   # the rank's state onto the device
        for i, b in enumerate(state[r]):
            dev.arena[dev.offs[i]:dev.offs[i] + b.size] = torch.from_numpy(b).cuda()

    swapped = [None] * NRANKS                                     # each rank's state at its last swap-out
    for r in range(NRANKS):                                       # every rank has been resident once
        put(r)
        sw.swap_out(r)
        torch.cuda.synchronize()
        swapped[r] = [b.copy() for b in state[r]]
    resident = NRANKS - 1

    rng = np.random.default_rng(12)
    everywhere = [i for i, b in enumerate(w.bufs) if b.nbytes >= 64]
    for step in range(2 * NRANKS + 1):
        # a mini-batch of the resident rank: fresh bytes in a few chunks of ANY buffer
        for i in rng.choice(everywhere, size=5, replace=False).tolist():
            nb = w.bufs[i].nbytes
            lo = int(rng.integers(0, nb - 32))
            hi = min(nb, lo + int(rng.integers(1, 2 * w.chunk)))
            fresh = rng.integers(0, 256, size=hi - lo, dtype=np.uint8)
            state[resident][i][lo:hi] = fresh
            dev.arena[dev.offs[i] + lo:dev.offs[i] + hi] = torch.from_numpy(fresh).cuda()
        nxt = (resident + 2) % NRANKS if step % 3 == 2 else (resident + 1) % NRANKS
        sw.switch_exact(resident, nxt, exchange=exchange)
        torch.cuda.synchronize()
        swapped[resident] = [b.copy() for b in state[resident]]
        got, img = dev.host()
        assert all(np.array_equal(g, s) for g, s in zip(got, state[nxt])), step
        assert dev.canaries_intact(img) and int(sw.rejected.item()) == 0
        stats = [int(x) for x in sw.chain_stats.cpu().numpy().view(np.uint64)]

        # the same switch replayed on the host with the oracle
        dig_out = oracle.fingerprint(state[resident], w.chunk, 8)
        dig_in = oracle.fingerprint(swapped[nxt], w.chunk, 8)
        m_out, _ = oracle.diff(state[resident], w.chunk, dig_out, o_ref)
        m_in, _ = oracle.diff(swapped[nxt], w.chunk, dig_in, o_ref)
        delta = oracle.compact(swapped[nxt], w.chunk, m_in, dig_in)[:2]
        host_image = [b.copy() for b in state[resident]]
        if exchange:
            # the incoming delta whole, then the base's bytes where only the outgoing rank differs
            assert oracle.restore(host_image, w.chunk, *delta) == 0
            only = oracle.mask_andnot(m_out, m_in)
            o_stats = oracle.restore_chain(host_image, w.chunk, [base_link], only)
            assert stats[0] == int(only.sum())
        else:
            only, _ = oracle.diff(swapped[nxt], w.chunk, dig_in, dig_out)
            o_stats = oracle.restore_chain(host_image, w.chunk, [base_link, delta], only)
            assert stats[0] == chunk_differences(w, state[resident], state[nxt])
        assert all(np.array_equal(h, s) for h, s in zip(host_image, state[nxt]))
        assert [o_stats["written"], o_stats["superseded"], o_stats["rejected"]] == stats
        assert np.array_equal(sw.incoming[:n].cpu().numpy(), only)
        resident = nxt


@pytest.mark.parametrize("exchange", [False, True], ids=["by_checksums", "exchange_then_repair"])
def test_exact_switches_replay_from_hip_graphs(exchange):
    """switch_exact enqueues kernels only (the chain restore takes its links as kernel
    arguments and reads counts and the restriction on the device), so it replays from a graph:
    two ranks ping-pong through two graphs while the resident rank rewrites chunks anywhere,
    shared state included; after every replay the image is the incoming rank's state."""
    w = wl.config(4, 12)
    base = wl.numpy_replica(w, 0)
    state = [wl.numpy_replica(w, r) for r in (1, 2)]
    dev = DeviceBuffers(base, w.chunk)
    n = dev.plan.nchunks
    ref = torch.from_numpy(oracle.fingerprint(base, w.chunk, 8).view(np.int64)).cuda()
    sw = TimeSlicedRanks(dev.plan, ref, 2, 2 * w.distinct_bytes + 16 * n, n, exact=True)
    sw.capture_base(max_slice_bytes=w.nbytes // 2)

    def put(r):
        for i, b in enumerate(state[r]):
            dev.arena[dev.offs[i]:dev.offs[i] + b.size] = torch.from_numpy(b).cuda()

    for r in (0, 1):
        put(r)
        sw.swap_out(r)
        torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graphs = {}
    with torch.cuda.stream(side):
        for a, b in ((1, 0), (0, 1)):                   # eager round trip on the capture stream
            sw.switch_exact(a, b, stream=side, exchange=exchange)
        side.synchronize()
        for a, b in ((1, 0), (0, 1)):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                sw.switch_exact(a, b, stream=side, exchange=exchange)
            graphs[(a, b)] = g
    torch.cuda.synchronize()
    got, _ = dev.host()
    assert all(np.array_equal(x, y) for x, y in zip(got, state[1]))

    rng = np.random.default_rng(19)
    everywhere = [i for i, b in enumerate(w.bufs) if b.nbytes >= 64]
    resident = 1
    for step in range(6):
        for i in rng.choice(everywhere, size=4, replace=False).tolist():
            nb = w.bufs[i].nbytes
            lo = int(rng.integers(0, nb - 32))
            hi = min(nb, lo + int(rng.integers(1, 2 * w.chunk)))
            fresh = rng.integers(0, 256, size=hi - lo, dtype=np.uint8)
            state[resident][i][lo:hi] = fresh
            dev.arena[dev.offs[i] + lo:dev.offs[i] + hi] = torch.from_numpy(fresh).cuda()
        nxt = 1 - resident
        graphs[(resident, nxt)].replay()
        torch.cuda.synchronize()
        got, img = dev.host()
        assert all(np.array_equal(x, y) for x, y in zip(got, state[nxt])), step
        assert dev.canaries_intact(img)
        stats = [int(x) for x in sw.chain_stats.cpu().numpy().view(np.uint64)]
        assert stats[2] == 0 and int(sw.rejected.item()) == 0
        if not exchange:
            assert stats[0] == chunk_differences(w, state[resident], state[nxt])
        resident = nxt
