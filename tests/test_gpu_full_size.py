"""GPU parity at the full sizes of the five configurations, in the launch
configuration bench.py times (same workload builders, same plans, same calls).

The oracle cannot hash 65 GB in seconds, so the full-size checks are:
  * digests of a sample of chunks (first / last chunk of buffers, short last
    chunks, random ones) recomputed by the oracle from the device bytes;
  * the mask against the set that is dirty by construction, for every chunk;
  * the whole manifest against its closed form (entries = dirty chunks in
    ascending order, offsets = exclusive prefix sum of padded lengths, digest
    field = digest array), which holds at any size;
  * staging bytes of sampled entries against the source chunk bytes;
  * restore: device-side byte equality of every buffer with the snapshot.
Config 2 (3 GB per replica) is small enough to be compared with the oracle in
full."""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_07848_amd import binding as ck
from paper_2202_07848_amd import workloads as wl

pytestmark = pytest.mark.gpu


class Rep:
    def __init__(self, w, arena, offs):
        self.w, self.arena, self.offs = w, arena, offs
        base = arena.data_ptr()
        self.plan = ck.Plan([(base + int(o), b.nbytes) for o, b in zip(offs, w.bufs)], w.chunk)

    def chunk_bytes(self, buf, off, length):
        o = int(self.offs[buf]) + int(off)
        return self.arena[o:o + int(length)].cpu().numpy()

    def host_buffers(self):
        return [self.arena[int(o):int(o) + b.nbytes].cpu().numpy()
                for o, b in zip(self.offs, self.w.bufs)]


def snapshot(rep, ref, fused=False):
    """The launch configurations bench.py times: three calls, or (fused) one ckpt_snapshot whose
    hint is the mask of a previous snapshot of the same state."""
    n = rep.plan.nchunks
    dig = torch.zeros(n, dtype=torch.int64, device="cuda")
    mask = torch.zeros(n, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    ck.fingerprint(rep.plan, dig)
    ck.diff(rep.plan, dig, ref, mask, counts)
    torch.cuda.synchronize()
    ndirty, staged = int(counts[0]), int(counts[1])
    staging = torch.empty(max(16, staged), dtype=torch.uint8, device="cuda")
    manifest = torch.empty(max(1, ndirty) * 32, dtype=torch.uint8, device="cuda")
    if fused:
        misses = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        ws = torch.empty(ck.snapshot_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        dig.zero_()
        ck.snapshot(rep.plan, ref, mask, dig, mask, staging, manifest, counts, misses, ws,
                    staging_cap=staged, manifest_cap=ndirty)
        torch.cuda.synchronize()
        assert int(misses.item()) == 0
    else:
        ck.compact(rep.plan, mask, dig, staging, manifest, counts, staging_cap=staged,
                   manifest_cap=ndirty)
    torch.cuda.synchronize()
    c = counts.cpu().numpy().view(np.uint64)
    assert (int(c[0]), int(c[1]), int(c[2])) == (ndirty, staged, 0)
    return dig, mask, staging, manifest, ndirty, staged


def sample_ids(w, rng, extra=48):
    buf, off, length = wl.chunk_table(w)
    n = buf.size
    first = np.flatnonzero(off == 0)
    last = np.concatenate([first[1:] - 1, [n - 1]])
    short = np.flatnonzero(length < w.chunk)
    picks = [rng.choice(first, size=min(8, first.size), replace=False),
             rng.choice(last, size=min(8, last.size), replace=False),
             rng.integers(0, n, size=extra)]
    if short.size:
        picks.append(rng.choice(short, size=min(16, short.size), replace=False))
    return np.unique(np.concatenate(picks)), (buf, off, length)


def check_sampled(w, rep, dig, mask, staging, manifest, ndirty, staged, expect_dirty, seed):
    rng = np.random.default_rng(seed)
    ids, (buf, off, length) = sample_ids(w, rng)
    h_dig = dig.cpu().numpy().view(np.uint64)
    h_mask = mask.cpu().numpy()
    # sampled digests against the oracle's hash of the very bytes on the device
    for k in ids.tolist():
        data = rep.chunk_bytes(buf[k], off[k], length[k])
        assert int(h_dig[k]) == oracle.xxh64(data), ("digest", k)
    # mask: every chunk
    assert np.array_equal(h_mask, expect_dirty.astype(np.uint8))
    # manifest: closed form over every entry
    man = ck.manifest_to_numpy(manifest, ndirty)
    dirty = np.flatnonzero(expect_dirty)
    assert ndirty == dirty.size
    padded = (length[dirty] + 15) // 16 * 16
    assert staged == int(padded.sum())
    assert np.array_equal(man["buf"].astype(np.int64), buf[dirty])
    assert np.array_equal(man["buf_off"].astype(np.int64), off[dirty])
    assert np.array_equal(man["len"].astype(np.int64), length[dirty])
    assert np.array_equal(man["stage_off"].astype(np.int64),
                          np.concatenate([[0], np.cumsum(padded)[:-1]]))
    assert np.array_equal(man["digest"], h_dig[dirty])
    # staging bytes of sampled entries (first, last, random, and the sampled dirty chunks)
    pos = {int(k): e for e, k in enumerate(dirty.tolist())}
    ents = {0, ndirty - 1} | {int(e) for e in rng.integers(0, ndirty, size=24)} \
        | {pos[k] for k in ids.tolist() if k in pos}
    for e in sorted(ents):
        k = int(dirty[e])
        so, ln = int(man["stage_off"][e]), int(man["len"][e])
        got = staging[so:so + (ln + 15) // 16 * 16].cpu().numpy()
        want = rep.chunk_bytes(buf[k], off[k], ln)
        assert np.array_equal(got[:ln], want), ("staging", e)
        assert not got[ln:].any()


def device_equal(a, b):
    """Every buffer of replica a equals the same buffer of replica b (device compare)."""
    for oa, ob, spec in zip(a.offs, b.offs, a.w.bufs):
        if not torch.equal(a.arena[int(oa):int(oa) + spec.nbytes],
                           b.arena[int(ob):int(ob) + spec.nbytes]):
            return False
    return True


def test_config2_full_size_exact_against_oracle():
    w = wl.config(2)
    a0, offs = wl.torch_replica(w, 0, "cuda")
    a1, _ = wl.torch_replica(w, 1, "cuda", shared_from=a0)
    r0, r1 = Rep(w, a0, offs), Rep(w, a1, offs)
    n = r0.plan.nchunks
    ref = torch.zeros(n, dtype=torch.int64, device="cuda")
    ck.fingerprint(r0.plan, ref)
    dig, mask, staging, manifest, ndirty, staged = snapshot(r1, ref)
    h0, h1 = r0.host_buffers(), r1.host_buffers()
    o_ref = oracle.fingerprint(h0, w.chunk, 16)
    o_dig = oracle.fingerprint(h1, w.chunk, 16)
    o_mask, o_cnt = oracle.diff(h1, w.chunk, o_dig, o_ref)
    o_st, o_man, _ = oracle.compact(h1, w.chunk, o_mask, o_dig)
    assert np.array_equal(ref.cpu().numpy().view(np.uint64), o_ref)
    assert np.array_equal(dig.cpu().numpy().view(np.uint64), o_dig)
    assert np.array_equal(mask.cpu().numpy(), o_mask)
    assert (ndirty, staged) == (o_cnt["ndirty"], o_cnt["staged_bytes"])
    assert ndirty == w.distinct_chunks
    assert np.array_equal(staging[:staged].cpu().numpy(), o_st)
    assert np.array_equal(ck.manifest_to_numpy(manifest, ndirty), o_man)
    ck.restore(r0.plan, staging, staged, manifest, ndirty)
    torch.cuda.synchronize()
    assert oracle.restore(h0, w.chunk, o_st, o_man) == 0
    for got, want in zip(r0.host_buffers(), h0):
        assert np.array_equal(got, want)
    assert device_equal(r0, r1)


@pytest.mark.parametrize("fused", [False, True], ids=["three_calls", "fused"])
@pytest.mark.parametrize("cfg", [5, 4])
def test_replica_configs_full_size_sampled(cfg, fused):
    w = wl.config(cfg)
    a0, offs = wl.torch_replica(w, 0, "cuda")
    r0 = Rep(w, a0, offs)
    n = r0.plan.nchunks
    assert n == w.nchunks and r0.plan.nbytes == w.nbytes
    ref = torch.zeros(n, dtype=torch.int64, device="cuda")
    ck.fingerprint(r0.plan, ref)
    buf, _, _ = wl.chunk_table(w)
    expect = np.array([not b.shared for b in w.bufs])[buf]
    staged_sizes = []
    for r in range(1, w.nreplicas):
        a, _ = wl.torch_replica(w, r, "cuda", shared_from=a0)
        rep = Rep(w, a, offs)
        dig, mask, staging, manifest, ndirty, staged = snapshot(rep, ref, fused)
        check_sampled(w, rep, dig, mask, staging, manifest, ndirty, staged, expect, 100 * cfg + r)
        staged_sizes.append(staged)
        if r == w.nreplicas - 1:
            # delta restore of the last replica into replica 0's buffers: byte-identical after
            assert not device_equal(r0, rep)
            rejected = torch.zeros(1, dtype=torch.int64, device="cuda")
            ck.restore(r0.plan, staging, staged, manifest, ndirty, rejected)
            torch.cuda.synchronize()
            assert int(rejected.item()) == 0
            assert device_equal(r0, rep)
            again = torch.zeros(n, dtype=torch.int64, device="cuda")
            ck.fingerprint(r0.plan, again)
            torch.cuda.synchronize()
            assert torch.equal(again, dig)
        del rep, a, dig, mask, staging, manifest
        torch.cuda.empty_cache()
    assert set(staged_sizes) == {w.distinct_bytes}


@pytest.mark.parametrize("fraction", [0.01, 0.10, 0.50])
def test_config3_full_size_sampled(fraction):
    fused = fraction >= 0.2            # as bench.py chooses
    w = wl.config(3)
    a0, offs = wl.torch_replica(w, 0, "cuda")
    t0 = Rep(w, a0, offs)
    n = t0.plan.nchunks
    assert n == w.nchunks
    ref = torch.zeros(n, dtype=torch.int64, device="cuda")
    ck.fingerprint(t0.plan, ref)
    step = int(fraction * 100)
    ids = wl.dirty_chunk_ids(w, fraction, step)
    a1 = a0.clone()
    wl.torch_rewrite_chunks(w, a1, offs, ids, step)
    t1 = Rep(w, a1, offs)
    expect = np.zeros(n, dtype=bool)
    expect[ids] = True
    dig, mask, staging, manifest, ndirty, staged = snapshot(t1, ref, fused)
    assert ndirty == ids.size == round(fraction * n)
    check_sampled(w, t1, dig, mask, staging, manifest, ndirty, staged, expect, 300 + step)
    # the all-zero 4 KiB chunks of t0 carry the stored vector for 4096 zero bytes
    buf, off, length = wl.chunk_table(w)
    zero_full = np.flatnonzero((np.array([b.kind == "zero" for b in w.bufs])[buf])
                               & (length == w.chunk))
    h_ref = ref.cpu().numpy().view(np.uint64)
    assert zero_full.size > 0 and np.all(h_ref[zero_full] == np.uint64(0xAC869B6F32D8BBDB))
    ck.restore(t0.plan, staging, staged, manifest, ndirty)
    torch.cuda.synchronize()
    assert torch.equal(a0, a1)
