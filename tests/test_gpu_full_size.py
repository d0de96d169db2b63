"""GPU parity at the full sizes of the five configurations, in the launch
configurations bench.py times (same workload builders, same plans, same calls):
the three calls fingerprint / diff / compact, and the fused ckpt_snapshot whose
hint is the mask of a previous snapshot of the same state.

Every output is compared with the oracle, element by element, at full size:
each replica is streamed to the host in batches of whole buffers of at most
4 GiB; per batch the oracle fingerprints the reference's and the snapshot's
bytes (16 threads), diffs them, compacts the batch and restores it, and the
batch's slice of the GPU's results must equal the oracle's:
  * every digest of the reference and of the snapshot;
  * every mask byte;
  * every manifest entry (the oracle's batch-local buffer index and staging
    offset shifted by the batch's first buffer and by the staging bytes of the
    batches before it, so the offsets are pinned as one running prefix sum);
  * every staged byte, through those offsets;
  * the counts, against the sum over the batches.
Restore: the oracle restores the batch's delta into the host copy of the
reference, which must then equal the snapshot's bytes; on the device the same
delta goes into the reference replica's buffers, which must then equal the
snapshot replica's buffers byte for byte (device compare over every buffer).
Each test prints how many chunks it compared, which is N of the configuration
for every replica and path.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_07848_amd import binding as ck
from paper_2202_07848_amd import workloads as wl

pytestmark = pytest.mark.gpu

BATCH_BYTES = 4 << 30
THREADS = 16
PATHS = ("three_calls", "fused")


class Rep:
    def __init__(self, w, arena, offs):
        self.w, self.arena, self.offs = w, arena, offs
        base = arena.data_ptr()
        self.plan = ck.Plan([(base + int(o), b.nbytes) for o, b in zip(offs, w.bufs)], w.chunk)


class HostWindow:
    """Device bytes -> host through pinned slabs, 1 GiB per copy."""

    SLAB = 1 << 30

    def __init__(self, *slot_bytes):
        self.bufs = [torch.empty(n, dtype=torch.uint8, pin_memory=True) for n in slot_bytes]

    def fetch(self, slot, dev_tensor):
        n = dev_tensor.numel()
        dst = self.bufs[slot]
        assert n <= dst.numel()
        for lo in range(0, n, self.SLAB):
            hi = min(n, lo + self.SLAB)
            dst[lo:hi].copy_(dev_tensor[lo:hi])
        return dst.numpy()[:n]


def batches(w):
    """Consecutive buffers in list order, at most BATCH_BYTES each (a single larger buffer
    would be a batch of its own; none of the configurations has one).  Yields
    (first buffer, end buffer, first chunk id, end chunk id)."""
    b0 = k0 = 0
    size = k = 0
    for i, spec in enumerate(w.bufs):
        if size and size + spec.nbytes > BATCH_BYTES:
            yield b0, i, k0, k
            b0, k0, size = i, k, 0
        size += spec.nbytes
        k += -(-spec.nbytes // w.chunk)
    yield b0, len(w.bufs), k0, k


def batch_views(w, rep, b0, b1, window, slot, image):
    """Host arrays of buffers b0..b1-1 of the replica (views, writable)."""
    if image is not None:                       # shuffled placement: whole arena is on the host
        return [image[int(rep.offs[i]):int(rep.offs[i]) + w.bufs[i].nbytes] for i in range(b0, b1)]
    lo = int(rep.offs[b0])
    hi = int(rep.offs[b1 - 1]) + w.bufs[b1 - 1].nbytes
    host = window.fetch(slot, rep.arena[lo:hi])
    return [host[int(rep.offs[i]) - lo:int(rep.offs[i]) - lo + w.bufs[i].nbytes]
            for i in range(b0, b1)]


def whole_image(rep, window):
    """Host copy of a whole arena (used when list order is not memory order)."""
    n = rep.arena.numel()
    image = np.empty(n, dtype=np.uint8)
    slab = window.bufs[0].numel()
    for lo in range(0, n, slab):
        hi = min(n, lo + slab)
        image[lo:hi] = window.fetch(0, rep.arena[lo:hi])
    return image


class Snapshot:
    """Outputs of one GPU snapshot of `rep` against `ref`, by one of the two paths."""

    def __init__(self, rep, ref, path, prev=None):
        n = rep.plan.nchunks
        self.dig = torch.zeros(n, dtype=torch.int64, device="cuda")
        self.mask = torch.zeros(n, dtype=torch.uint8, device="cuda")
        self.counts = torch.zeros(3, dtype=torch.int64, device="cuda")
        if prev is None:               # a first look, to size staging and manifest
            ck.fingerprint(rep.plan, self.dig)
            ck.diff(rep.plan, self.dig, ref, self.mask, self.counts)
            torch.cuda.synchronize()
            self.ndirty, self.staged = int(self.counts[0]), int(self.counts[1])
            hint = self.mask.clone()
        else:                          # the previous snapshot's mask is the hint
            self.ndirty, self.staged = prev.ndirty, prev.staged
            hint = prev.mask.clone()
        self.staging = torch.full((max(16, self.staged),), 0xEE, dtype=torch.uint8, device="cuda")
        self.manifest = torch.full((max(1, self.ndirty) * 32,), 0xEE, dtype=torch.uint8,
                                   device="cuda")
        if path == "fused":
            misses = torch.full((1,), -1, dtype=torch.int64, device="cuda")
            ws = torch.empty(ck.snapshot_workspace_bytes(n), dtype=torch.uint8, device="cuda")
            self.dig.zero_()
            self.mask.zero_()
            ck.snapshot(rep.plan, ref, hint, self.dig, self.mask, self.staging, self.manifest,
                        self.counts, misses, ws, staging_cap=self.staged,
                        manifest_cap=self.ndirty)
            torch.cuda.synchronize()
            assert int(misses.item()) == 0
        else:
            self.dig.zero_()
            self.mask.zero_()
            ck.fingerprint(rep.plan, self.dig)
            ck.diff(rep.plan, self.dig, ref, self.mask, self.counts)
            ck.compact(rep.plan, self.mask, self.dig, self.staging, self.manifest, self.counts,
                       staging_cap=self.staged, manifest_cap=self.ndirty)
            torch.cuda.synchronize()
        c = self.counts.cpu().numpy().view(np.uint64)
        assert (int(c[0]), int(c[1]), int(c[2])) == (self.ndirty, self.staged, 0)
        self.h_dig = self.dig.cpu().numpy().view(np.uint64)
        self.h_mask = self.mask.cpu().numpy()
        self.h_man = ck.manifest_to_numpy(self.manifest, self.ndirty)


def compare_with_oracle(w, r_ref, r_new, g_ref, snaps, window, images=(None, None)):
    """Streams both replicas to the host batch by batch and compares every element of the
    GPU results (g_ref: reference digests on the host; snaps: {path: Snapshot}) with the
    oracle's.  Returns the number of chunks compared."""
    e0 = s0 = compared = 0
    for b0, b1, k0, k1 in batches(w):
        h_ref = batch_views(w, r_ref, b0, b1, window, 0, images[0])
        h_new = batch_views(w, r_new, b0, b1, window, 1, images[1])
        o_ref = oracle.fingerprint(h_ref, w.chunk, THREADS)
        o_dig = oracle.fingerprint(h_new, w.chunk, THREADS)
        assert o_ref.size == k1 - k0
        assert np.array_equal(g_ref[k0:k1], o_ref), ("reference digests", b0, b1)
        o_mask, o_cnt = oracle.diff(h_new, w.chunk, o_dig, o_ref)
        o_st, o_man, o_cnt2 = oracle.compact(h_new, w.chunk, o_mask, o_dig)
        nd, nst = int(o_cnt2["ndirty"]), int(o_cnt2["staged_bytes"])
        assert (nd, nst) == (int(o_cnt["ndirty"]), int(o_cnt["staged_bytes"]))
        for path, s in snaps.items():
            where = (path, b0, b1)
            assert np.array_equal(s.h_dig[k0:k1], o_dig), ("digests",) + where
            assert np.array_equal(s.h_mask[k0:k1], o_mask), ("mask",) + where
            assert e0 + nd <= s.ndirty and s0 + nst <= s.staged, ("counts",) + where
            man = s.h_man[e0:e0 + nd]
            assert np.array_equal(man["buf"], o_man["buf"] + np.uint32(b0)), ("buf",) + where
            assert np.array_equal(man["len"], o_man["len"]), ("len",) + where
            assert np.array_equal(man["buf_off"], o_man["buf_off"]), ("buf_off",) + where
            assert np.array_equal(man["stage_off"], o_man["stage_off"] + np.uint64(s0)), \
                ("stage_off",) + where
            assert np.array_equal(man["digest"], o_man["digest"]), ("digest field",) + where
            slab = window.bufs[2].numel()
            for lo in range(0, nst, slab):
                hi = min(nst, lo + slab)
                got = window.fetch(2, s.staging[s0 + lo:s0 + hi])
                assert np.array_equal(got, o_st[lo:hi]), ("staging bytes", lo) + where
        # the oracle's restore of this batch's delta into the reference's bytes
        assert oracle.restore(h_ref, w.chunk, o_st, o_man) == 0
        for a, b in zip(h_ref, h_new):
            assert np.array_equal(a, b), ("oracle restore", b0, b1)
        e0 += nd
        s0 += nst
        compared += k1 - k0
    for path, s in snaps.items():
        assert (e0, s0) == (s.ndirty, s.staged), ("totals", path)
    return compared


def device_equal(a, b):
    """Every buffer of replica a equals the same buffer of replica b (device compare)."""
    if a.arena.numel() == b.arena.numel() and np.array_equal(a.offs, b.offs):
        # same layout: compare the arenas in slabs (alignment gaps are never written)
        step = 1 << 32
        return all(torch.equal(a.arena[lo:lo + step], b.arena[lo:lo + step])
                   for lo in range(0, a.arena.numel(), step))
    for oa, ob, spec in zip(a.offs, b.offs, a.w.bufs):
        if not torch.equal(a.arena[int(oa):int(oa) + spec.nbytes],
                           b.arena[int(ob):int(ob) + spec.nbytes]):
            return False
    return True


def gpu_restore_check(r_ref, r_new, s):
    """Delta restore of the snapshot into the reference replica's buffers: byte-identical
    afterwards, and fingerprinting the result gives the snapshot's digests."""
    rejected = torch.zeros(1, dtype=torch.int64, device="cuda")
    ck.restore(r_ref.plan, s.staging, s.staged, s.manifest, s.ndirty, rejected)
    torch.cuda.synchronize()
    assert int(rejected.item()) == 0
    assert device_equal(r_ref, r_new)
    again = torch.zeros_like(s.dig)
    ck.fingerprint(r_ref.plan, again)
    torch.cuda.synchronize()
    assert torch.equal(again, s.dig)


def make_window(w):
    # a batch's arena range includes the alignment gaps between its buffers (< 256 bytes each)
    largest = max(sum(w.bufs[i].nbytes + 256 for i in range(b0, b1)) for b0, b1, _, _ in batches(w))
    return HostWindow(largest, largest, min(largest, 1 << 30))


@pytest.mark.parametrize("cfg", [1, 2, 5, 4])
def test_replica_configs_full_size_every_element(cfg):
    w = wl.config(cfg)
    window = make_window(w)
    a0, offs = wl.torch_replica(w, 0, "cuda")
    r0 = Rep(w, a0, offs)
    n = r0.plan.nchunks
    assert n == w.nchunks and r0.plan.nbytes == w.nbytes
    ref = torch.zeros(n, dtype=torch.int64, device="cuda")
    ck.fingerprint(r0.plan, ref)
    torch.cuda.synchronize()
    g_ref = ref.cpu().numpy().view(np.uint64)
    buf, _, _ = wl.chunk_table(w)
    expect = np.array([not b.shared for b in w.bufs])[buf].astype(np.uint8)
    compared = 0
    for r in range(1, w.nreplicas):
        a, _ = wl.torch_replica(w, r, "cuda", shared_from=a0)
        rep = Rep(w, a, offs)
        snaps = {}
        for path in PATHS:
            snaps[path] = Snapshot(rep, ref, path, snaps.get(PATHS[0]))
            # by construction the distinct chunks are exactly those of the per-replica buffers
            assert np.array_equal(snaps[path].h_mask, expect)
            assert snaps[path].staged == w.distinct_bytes
        got = compare_with_oracle(w, r0, rep, g_ref, snaps, window)
        assert got == n
        compared += got
        if r == w.nreplicas - 1:
            assert not device_equal(r0, rep)
            gpu_restore_check(r0, rep, snaps["fused"])
        del snaps, rep, a
        torch.cuda.empty_cache()
    print(f"config {cfg}: chunks compared with the oracle = {compared} "
          f"({w.nreplicas - 1} snapshot(s) x N = {n}, both paths)")
    assert compared == n * (w.nreplicas - 1)


@pytest.mark.parametrize("fraction", [0.01, 0.10, 0.50])
def test_config3_full_size_every_element(fraction):
    w = wl.config(3)
    window = HostWindow(1 << 30, 16, 1 << 30)
    a0, offs = wl.torch_replica(w, 0, "cuda")
    t0 = Rep(w, a0, offs)
    n = t0.plan.nchunks
    assert n == w.nchunks
    ref = torch.zeros(n, dtype=torch.int64, device="cuda")
    ck.fingerprint(t0.plan, ref)
    torch.cuda.synchronize()
    g_ref = ref.cpu().numpy().view(np.uint64)
    step = int(fraction * 100)
    ids = wl.dirty_chunk_ids(w, fraction, step)
    a1 = a0.clone()
    wl.torch_rewrite_chunks(w, a1, offs, ids, step)
    t1 = Rep(w, a1, offs)
    expect = np.zeros(n, dtype=np.uint8)
    expect[ids] = 1
    snaps = {}
    for path in PATHS:
        snaps[path] = Snapshot(t1, ref, path, snaps.get(PATHS[0]))
        assert snaps[path].ndirty == ids.size == round(fraction * n)
        assert np.array_equal(snaps[path].h_mask, expect)      # exactly the rewritten set
    # the all-zero 4 KiB chunks of t0 carry the stored vector for 4096 zero bytes
    buf, off, length = wl.chunk_table(w)
    zero_full = np.flatnonzero((np.array([b.kind == "zero" for b in w.bufs])[buf])
                               & (length == w.chunk))
    assert zero_full.size > 0 and np.all(g_ref[zero_full] == np.uint64(0xAC869B6F32D8BBDB))
    # list order is not memory order here (shuffled placement): whole arenas go to the host
    images = (whole_image(t0, window), whole_image(t1, window))
    got = compare_with_oracle(w, t0, t1, g_ref, snaps, window, images)
    print(f"config 3, {fraction:.0%} rewritten: chunks compared with the oracle = {got} "
          f"(N = {n}, both paths)")
    assert got == n
    gpu_restore_check(t0, t1, snaps["three_calls"])


def test_config4_chain_restore_full_size():
    """ckpt_restore_chain at config 4's size (paper sec. 4.6).  States: replica 0, replica 1,
    replica 2, then replica 2 with two shared buffers rewritten; every link is the delta against
    the state before it.  The links hold different chunk sets (all per-replica chunks twice, a
    few shared chunks once); restored in one pass into a copy of replica 0 the image must equal
    the last state byte for byte -- which no part of the library computed -- and its fingerprint
    the last state's digests; the counts follow from the construction."""
    w = wl.config(4)
    a0, offs = wl.torch_replica(w, 0, "cuda")
    r0 = Rep(w, a0, offs)
    n = r0.plan.nchunks
    prev = torch.zeros(n, dtype=torch.int64, device="cuda")
    ck.fingerprint(r0.plan, prev)
    image = Rep(w, a0.clone(), offs)
    buf, _, _ = wl.chunk_table(w)
    private = np.array([not b.shared for b in w.bufs])[buf]
    links, sets, state = [], [], None
    for step in (1, 2, 3):
        if step < 3:
            a, _ = wl.torch_replica(w, step, "cuda", shared_from=a0)
            state = Rep(w, a, offs)
            sets.append(private.copy())
        else:
            # two shared buffers of the last state change: a large one and a ragged small one
            shared = [i for i, b in enumerate(w.bufs) if b.shared]
            big = max(shared, key=lambda i: w.bufs[i].nbytes)
            small = next(i for i in shared if 0 < w.bufs[i].nbytes < w.chunk)
            for i in (big, small):
                state.arena[int(offs[i]):int(offs[i]) + w.bufs[i].nbytes] ^= 0x5C
            sets.append(np.isin(buf, [big, small]))
        s = Snapshot(state, prev, "three_calls")
        assert np.array_equal(s.h_mask, sets[-1].astype(np.uint8))
        links.append((s.staging, s.staged, s.manifest, s.ndirty, s.counts))
        prev = s.dig
    assert not device_equal(image, state)
    ws = torch.empty(ck.restore_chain_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    stats = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    ck.restore_chain(image.plan, links, ws, stats)
    torch.cuda.synchronize()
    assert device_equal(image, state)
    again = torch.zeros(n, dtype=torch.int64, device="cuda")
    ck.fingerprint(image.plan, again)
    torch.cuda.synchronize()
    assert torch.equal(again, prev)
    union = int(np.logical_or.reduce(sets).sum())
    total = int(sum(s.sum() for s in sets))
    assert [int(x) for x in stats.cpu().numpy().view(np.uint64)] == [union, total - union, 0]
    print(f"config 4 chain: {len(links)} links, {total} entries, {union} chunks written once")


@pytest.mark.parametrize("chunk", [1 << 20, 4096], ids=["1MiB_chunks", "4KiB_chunks"])
def test_one_buffer_larger_than_4_gib_every_element(chunk):
    """Offsets inside a buffer beyond 2^32: one 4.5 GiB + 4 321 byte buffer (and a small second
    one), as 4 613 chunks of 1 MiB or as 1.18 million chunks of 4 KiB in ONE buffer; reference = a copy that differs in a few chunks on both sides of the
    4 GiB line and in the ragged tail.  Every digest, mask byte, manifest entry and staged byte
    against the oracle, both call shapes, then the restore."""
    sizes = [(9 << 29) + 4321, 3 * (1 << 20) + 17]
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    offs = [0, (sizes[0] + 255) // 256 * 256]
    arena_ref = torch.randint(0, 256, (offs[1] + sizes[1],), dtype=torch.uint8, device="cuda",
                              generator=g)
    arena_new = arena_ref.clone()
    for off in (5, (1 << 32) - 3, (1 << 32) + chunk + 9, sizes[0] - 1, offs[1] + 2 * chunk + 1):
        arena_new[off] ^= 0x5A
    plans = [ck.Plan([(a.data_ptr() + o, n) for o, n in zip(offs, sizes)], chunk)
             for a in (arena_ref, arena_new)]
    n = plans[1].nchunks
    assert n == sum(-(-x // chunk) for x in sizes)
    host_ref, host_new = ([a[o:o + s].cpu().numpy() for o, s in zip(offs, sizes)]
                          for a in (arena_ref, arena_new))
    o_ref = oracle.fingerprint(host_ref, chunk, THREADS)
    o_dig = oracle.fingerprint(host_new, chunk, THREADS)
    o_mask, o_cnt = oracle.diff(host_new, chunk, o_dig, o_ref)
    o_st, o_man, _ = oracle.compact(host_new, chunk, o_mask, o_dig)
    assert o_cnt["ndirty"] == 5
    ref = torch.zeros(n, dtype=torch.int64, device="cuda")
    ck.fingerprint(plans[0], ref)
    torch.cuda.synchronize()
    assert np.array_equal(ref.cpu().numpy().view(np.uint64), o_ref)

    class View:                                   # what Snapshot() needs of a replica
        def __init__(self, plan):
            self.plan = plan

    prev = None
    for path in PATHS:
        s = Snapshot(View(plans[1]), ref, path, prev)
        assert np.array_equal(s.h_dig, o_dig) and np.array_equal(s.h_mask, o_mask)
        assert s.h_man.tolist() == o_man.tolist()
        assert np.array_equal(s.staging.cpu().numpy()[:s.staged], o_st)
        prev = s
    rejected = torch.zeros(1, dtype=torch.int64, device="cuda")
    ck.restore(plans[0], prev.staging, prev.staged, prev.manifest, prev.ndirty, rejected)
    torch.cuda.synchronize()
    assert int(rejected.item()) == 0 and torch.equal(arena_ref, arena_new)
