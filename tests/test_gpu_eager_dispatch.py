"""ckpt_restore_counted and the eager dispatch it allows (paper sec. 6): the
whole switch -- checksum, compare, swap-out of the outgoing rank's delta,
swap-in of the incoming rank's -- is enqueued without the host reading any
result, and the next rank's device work is dispatched at once on another stream
behind an event.  Results are compared with the oracle."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DeviceBuffers, counts_dict, run_compact, run_diff, run_fingerprint, u64
from paper_2202_07848_amd import binding as ck

pytestmark = pytest.mark.gpu

CHUNK = 1024
SIZES = [70000, 1024, 33333, 0, 2048, 5]


def states(seed):
    rng = np.random.default_rng(seed)
    a = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in SIZES]
    b = [x.copy() for x in a]
    for i, off in ((0, 100), (0, 69999), (2, 2048), (4, 1024), (5, 3)):
        b[i][off] ^= 0x11
    return a, b


@pytest.mark.parametrize("cap_delta", [0, 3, -2])
def test_restore_counted_applies_exactly_the_counted_entries(cap_delta):
    a, b = states(1)
    src, dst = DeviceBuffers(b, CHUNK), DeviceBuffers(a, CHUNK)
    n = src.plan.nchunks
    o_ref, o_dig = oracle.fingerprint(a, CHUNK), oracle.fingerprint(b, CHUNK)
    o_mask, o_cnt = oracle.diff(b, CHUNK, o_dig, o_ref)
    cap = o_cnt["ndirty"] + cap_delta
    o_st, o_man, o_c = oracle.compact(b, CHUNK, o_mask, o_dig, manifest_cap=cap)
    dig = run_fingerprint(src.plan)
    mask, _ = run_diff(src.plan, dig, torch.from_numpy(o_ref.view(np.int64)).cuda())
    staging, manifest, counts = run_compact(src.plan, mask, dig, o_cnt["staged_bytes"], cap, slack=0)
    assert counts_dict(counts) == o_c
    if cap_delta > 0:
        # entries past the count look valid (they would rewrite chunk 0 of buffer 0 with other
        # bytes) and must not be applied
        man = ck.manifest_to_numpy(manifest, cap).copy()
        man[o_cnt["ndirty"]:] = man[0]
        man["stage_off"][o_cnt["ndirty"]:] = man["stage_off"][1]
        manifest.copy_(torch.from_numpy(man.view(np.uint8).reshape(-1)).cuda())
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ck.restore_counted(dst.plan, staging, o_cnt["staged_bytes"], manifest, cap, counts, rejected)
    torch.cuda.synchronize()
    want = [x.copy() for x in a]
    applied = min(cap, o_cnt["ndirty"])
    assert oracle.restore(want, CHUNK, o_st, o_man[:applied]) == 0
    got, img = dst.host()
    assert int(rejected.item()) == 0
    assert all(np.array_equal(g, w) for g, w in zip(got, want))
    assert dst.canaries_intact(img)
    if cap_delta >= 0:
        assert all(np.array_equal(g, w) for g, w in zip(got, b))


def test_restore_counted_argument_errors():
    a, _ = states(2)
    dst = DeviceBuffers(a, CHUNK)
    st = torch.zeros(64, dtype=torch.uint8, device="cuda")
    man = torch.zeros(64, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    with pytest.raises(ck.CkptError) as e:
        ck.restore_counted(dst.plan, st, 64, man, 2, None)
    assert e.value.status == -1
    with pytest.raises(ck.CkptError) as e:
        ck.restore_counted(dst.plan, st, 64, None, 2, counts)
    assert e.value.status == -1
    with pytest.raises(ck.CkptError) as e:
        ck.restore_counted(dst.plan, st[8:], 56, man, 2, counts)
    assert e.value.status == -2
    ck.restore_counted(dst.plan, None, 0, None, 0, counts)          # nothing to do is fine
    torch.cuda.synchronize()


@pytest.mark.parametrize("where", ["device", "pinned_host"])
def test_switch_is_enqueued_without_host_reads_and_next_rank_waits_on_an_event(where):
    """Two ranks share one set of device buffers; the deltas that are swapped out and in live in
    device memory or in pinned host memory (then the kernels move them over the host link).  Rank A is resident; the switch saves A's delta
    against the common reference and brings in B's delta, on the switch stream.  Rank B's first
    device operation (here: a checksum pass over its state and a mutation of one buffer) is
    dispatched immediately on its own stream behind an event.  Nothing is synchronised until the
    end."""
    base, a_host = states(3)
    _, b_host = states(3)
    b_host[2][:4096] ^= 0x5A                       # B differs from base elsewhere than A does
    b_host[4][7] ^= 1
    n_ref = oracle.fingerprint(base, CHUNK)
    o_a, o_b = oracle.fingerprint(a_host, CHUNK), oracle.fingerprint(b_host, CHUNK)

    shared = DeviceBuffers(a_host, CHUNK)          # the device memory both ranks use: A is in it
    plan, n = shared.plan, shared.plan.nchunks
    ref = torch.from_numpy(n_ref.view(np.int64)).cuda()

    # B's delta against the reference, as an earlier switch left it (device-resident here)
    mb, cb = oracle.diff(b_host, CHUNK, o_b, n_ref)
    st_b, man_b, _ = oracle.compact(b_host, CHUNK, mb, o_b)
    def place(t):
        if where == "device":
            return t.cuda()
        p = torch.empty(t.shape, dtype=t.dtype, pin_memory=True)
        p.copy_(t)
        return p

    b_staging = place(torch.from_numpy(st_b))
    b_manifest = torch.from_numpy(man_b.view(np.uint8).reshape(-1).copy()).cuda()
    b_counts = torch.tensor([cb["ndirty"], cb["staged_bytes"], 0], dtype=torch.int64, device="cuda")

    dig = torch.zeros(n, dtype=torch.int64, device="cuda")
    mask = torch.zeros(n, dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    a_staging = place(torch.full((n * CHUNK,), 0xEE, dtype=torch.uint8))
    a_manifest = torch.full((n * 32,), 0xEE, dtype=torch.uint8, device="cuda")
    rejected = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    b_dig = torch.zeros(n, dtype=torch.int64, device="cuda")
    # the reference image (what both deltas are relative to) stays on the device, with its checksums
    base_dev = DeviceBuffers(base, CHUNK)
    base_staging = torch.zeros(n * CHUNK, dtype=torch.uint8, device="cuda")
    base_manifest = torch.zeros(n * 32, dtype=torch.uint8, device="cuda")
    base_counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()                       # end of set-up; no host wait from here on

    switch, nxt = torch.cuda.Stream(), torch.cuda.Stream()
    done = torch.cuda.Event()
    # --- the switch: out with A (its delta against the reference goes to a_staging) ...
    ck.fingerprint(plan, dig, stream=switch)
    ck.diff(plan, dig, ref, mask, counts, stream=switch)
    ck.compact(plan, mask, dig, a_staging, a_manifest, counts, stream=switch)
    # ... the chunks A had changed go back to the reference's bytes (B's delta assumes them) ...
    ck.compact(base_dev.plan, mask, ref, base_staging, base_manifest, base_counts, stream=switch)
    ck.restore_counted(plan, base_staging, base_staging.numel(), base_manifest, n, base_counts,
                       rejected[0:1], stream=switch)
    # ... and in with B
    ck.restore_counted(plan, b_staging, b_staging.numel(), b_manifest, man_b.size, b_counts,
                       rejected[1:2], stream=switch)
    done.record(switch)
    # --- rank B's first device operation, dispatched at once behind the event
    nxt.wait_event(done)
    ck.fingerprint(plan, b_dig, stream=nxt)
    torch.cuda.synchronize()

    assert rejected.tolist() == [0, 0]
    assert np.array_equal(u64(dig, n), o_a)        # the switch saw A's state
    ma, ca = oracle.diff(a_host, CHUNK, o_a, n_ref)
    st_a, man_a, _ = oracle.compact(a_host, CHUNK, ma, o_a)
    assert counts_dict(counts) == ca
    assert np.array_equal(a_staging[:st_a.size].cpu().numpy(), st_a)
    assert np.array_equal(ck.manifest_to_numpy(a_manifest, ca["ndirty"]), man_a)
    assert np.array_equal(u64(b_dig, n), o_b)      # rank B's first operation saw B's state
    got, img = shared.host()
    assert all(np.array_equal(g, w) for g, w in zip(got, b_host))
    assert shared.canaries_intact(img)


def test_graph_with_counted_restore_follows_a_changing_dirty_set():
    """A captured snapshot + counted restore is replayed after the snapshot's content (and with it
    the number of dirty chunks) changed: every replay must equal the oracle for that content."""
    base, b0 = states(4)
    src, dst = DeviceBuffers(b0, CHUNK), DeviceBuffers(base, CHUNK)
    n = src.plan.nchunks
    o_ref = oracle.fingerprint(base, CHUNK)
    ref = torch.from_numpy(o_ref.view(np.int64)).cuda()
    dig = torch.zeros(n, dtype=torch.int64, device="cuda")
    mask = torch.zeros(n, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    staging = torch.zeros(n * CHUNK, dtype=torch.uint8, device="cuda")
    manifest = torch.zeros(n * 32, dtype=torch.uint8, device="cuda")
    rejected = torch.zeros(1, dtype=torch.int64, device="cuda")

    def enqueue(stream):
        ck.fingerprint(src.plan, dig, stream=stream)
        ck.diff(src.plan, dig, ref, mask, counts, stream=stream)
        ck.compact(src.plan, mask, dig, staging, manifest, counts, stream=stream)
        ck.restore_counted(dst.plan, staging, staging.numel(), manifest, n, counts, rejected,
                           stream=stream)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue(side)
    torch.cuda.synchronize()

    rng = np.random.default_rng(5)
    seen = set()
    for replay in range(5):
        cur = [x.copy() for x in base]
        for _ in range(int(rng.integers(0, 12)) if replay else 0):    # replay 0: nothing dirty
            i = int(rng.choice([0, 1, 2, 4, 5]))
            cur[i][int(rng.integers(0, cur[i].size))] ^= 0x21
        src.arena.copy_(DeviceBuffers(cur, CHUNK).arena)
        dst.arena.copy_(DeviceBuffers(base, CHUNK).arena)
        staging.fill_(0xEE); manifest.fill_(0xEE); counts.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        o_dig = oracle.fingerprint(cur, CHUNK)
        o_mask, o_cnt = oracle.diff(cur, CHUNK, o_dig, o_ref)
        seen.add(o_cnt["ndirty"])
        assert counts_dict(counts) == o_cnt, replay
        assert np.array_equal(mask.cpu().numpy(), o_mask), replay
        assert int(rejected.item()) == 0
        got, img = dst.host()
        assert all(np.array_equal(g, w) for g, w in zip(got, cur)), replay
        assert dst.canaries_intact(img)
    assert len(seen) >= 3
