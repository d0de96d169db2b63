"""ckpt_snapshot_static (the snapshot call that allocates nothing: its workspace and scan scratch
are one static device array inside the library) against ckpt_snapshot on the same inputs, bit
for bit: digests, mask, counts, hint misses, manifest entries, staged bytes, and nothing written
past the capacities.  Two calls in a row share the array, the second on a smaller input, so
whatever the first left behind must not reach the second's results."""
import numpy as np
import pytest
import torch

from paper_2202_07848_amd import binding as ck

pytestmark = pytest.mark.gpu


def make_state(seed, sizes, chunk, flip_every, split):
    """Reference digests, a snapshot state that differs from the reference in some chunks, and
    an exact hint -- all produced by the existing entry points."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    ref_bufs = [torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda", generator=g)
                for n in sizes]
    bufs = [b.clone() for b in ref_bufs]
    for i, b in enumerate(bufs):
        if b.numel() and i % 2 == 0:
            b[::flip_every] ^= 0x5A
    p_ref, plan = ck.Plan(ref_bufs, chunk), ck.Plan(bufs, chunk)
    plan.split_threshold = split
    n = plan.nchunks
    ref = torch.zeros(n, dtype=torch.int64, device="cuda")
    dig = torch.zeros(n, dtype=torch.int64, device="cuda")
    hint = torch.zeros(n, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    ck.fingerprint(p_ref, ref)
    ck.fingerprint(plan, dig)
    ck.diff(plan, dig, ref, hint, counts)
    torch.cuda.synchronize()
    return plan, bufs, ref, hint, int(counts[0]), int(counts[1])


def outputs(n, ndirty, staged):
    return dict(dig=torch.zeros(n, dtype=torch.int64, device="cuda"),
                mask=torch.full((n,), 0x77, dtype=torch.uint8, device="cuda"),
                staging=torch.full((staged + 256,), 0xA5, dtype=torch.uint8, device="cuda"),
                manifest=torch.full((ndirty * 32 + 256,), 0xA5, dtype=torch.uint8, device="cuda"),
                counts=torch.full((3,), -1, dtype=torch.int64, device="cuda"),
                misses=torch.full((1,), -1, dtype=torch.int64, device="cuda"))


def both_ways(plan, ref, hint, ndirty, staged):
    n = plan.nchunks
    a, b = outputs(n, ndirty, staged), outputs(n, ndirty, staged)
    ws = torch.full((ck.snapshot_workspace_bytes(n),), 0x11, dtype=torch.uint8, device="cuda")
    ck.snapshot(plan, ref, hint, a["dig"], a["mask"], a["staging"], a["manifest"], a["counts"],
                a["misses"], ws, staging_cap=staged, manifest_cap=ndirty)
    ck.snapshot_static(plan, ref, hint, b["dig"], b["mask"], b["staging"], b["manifest"],
                       b["counts"], b["misses"], staging_cap=staged, manifest_cap=ndirty)
    torch.cuda.synchronize()
    for key in a:
        assert torch.equal(a[key], b[key]), key
    return a


@pytest.mark.parametrize("split", [0, 2**64 - 1], ids=["two_launches", "one_launch"])
def test_static_snapshot_equals_snapshot_twice_in_a_row(split):
    big = [3 << 20, 1 << 20, 4096 * 37 + 123, 0, 65536, 17, 2 << 20, 700_001]
    small = [4096 * 5 + 1, 300_000, 31]
    plan1, bufs1, ref1, hint1, nd1, st1 = make_state(11, big, 4096, 40_009, split)
    plan2, bufs2, ref2, hint2, nd2, st2 = make_state(12, small, 4096, 9_001, split)
    assert nd1 > nd2 > 0 and plan1.nchunks > plan2.nchunks
    r1 = both_ways(plan1, ref1, hint1, nd1, st1)        # first call: exact hint
    c = r1["counts"].cpu().numpy().view(np.uint64)
    assert (int(c[0]), int(c[1]), int(c[2])) == (nd1, st1, 0) and int(r1["misses"]) == 0
    r2 = both_ways(plan2, ref2, hint2, nd2, st2)        # second call: smaller input
    c = r2["counts"].cpu().numpy().view(np.uint64)
    assert (int(c[0]), int(c[1]), int(c[2])) == (nd2, st2, 0) and int(r2["misses"]) == 0
    # a wrong hint (gather path), no hint, and no reference, each after the other
    wrong = hint2.clone()
    wrong[plan2.nchunks // 2] ^= 1
    r3 = both_ways(plan2, ref2, wrong, nd2, st2)
    assert int(r3["misses"]) == 1
    assert torch.equal(r3["staging"][:st2], r2["staging"][:st2])
    both_ways(plan2, ref2, None, nd2, st2)
    both_ways(plan2, None, None, plan2.nchunks, plan2.nbytes + 16 * plan2.nchunks)
    # capacity limits are honoured the same way
    both_ways(plan1, ref1, hint1, nd1 // 2, st1 // 3)


def test_static_snapshot_refuses_plans_above_its_limit():
    limit = ck.snapshot_static_max_chunks()
    assert limit == 1 << 18
    buf = torch.zeros((limit + 1) * 256, dtype=torch.uint8, device="cuda")
    at_limit = ck.Plan([buf[: limit * 256]], 256)
    above = ck.Plan([buf], 256)
    assert at_limit.nchunks == limit and above.nchunks == limit + 1
    o = outputs(limit + 1, limit + 1, (limit + 1) * 256)
    with pytest.raises(ck.CkptError) as err:
        ck.snapshot_static(above, None, None, o["dig"], o["mask"], o["staging"], o["manifest"],
                           o["counts"], o["misses"], staging_cap=(limit + 1) * 256,
                           manifest_cap=limit + 1)
    assert err.value.status == -5
    torch.cuda.synchronize()
    assert int(o["counts"][0]) == -1                       # nothing was enqueued
    hint = torch.ones(limit, dtype=torch.uint8, device="cuda")
    both_ways(at_limit, None, hint, limit, limit * 256)    # the largest plan it takes
