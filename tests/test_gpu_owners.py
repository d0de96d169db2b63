"""GPU parity of ckpt_upload_owners (paper sec. 4.6) with the oracle, through
the C ABI: mask and counts bit-exact for every rank, the compacted uploads
byte-exact, argument errors, and config 4 at full size against the closed form
of its construction (shared state spread k mod 4, private state kept)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DeviceBuffers, counts_dict, run_compact, run_fingerprint, u64
from oracle_pins import worker_states
from paper_2202_07848_amd import binding as ck
from paper_2202_07848_amd import workloads as wl

pytestmark = pytest.mark.gpu


def run_owners(plan, gathered, world, rank):
    mask = torch.full((max(1, plan.nchunks),), 0x77, dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    ck.upload_owners(plan, gathered, world, rank, mask, counts)
    torch.cuda.synchronize()
    return mask, counts


@pytest.mark.parametrize("world,seed", [(1, 11), (2, 12), (3, 13), (5, 14), (8, 15)])
@pytest.mark.parametrize("chunk,sizes", [(256, (5000, 256, 0, 1300, 77)),
                                         (4096, (300000, 4096, 17, 0, 123457))])
def test_owner_masks_and_uploads_match_oracle(world, seed, chunk, sizes):
    states, _ = worker_states(world, seed, sizes=sizes, chunk=chunk)
    devs = [DeviceBuffers(st, chunk) for st in states]
    n = devs[0].plan.nchunks
    digs = torch.stack([run_fingerprint(d.plan)[:n] for d in devs]).contiguous()
    o_digs = np.stack([oracle.fingerprint(st, chunk) for st in states])
    assert np.array_equal(digs.cpu().numpy().view(np.uint64), o_digs)
    for r in range(world):
        o_mask, o_cnt = oracle.upload_owners(states[r], chunk, o_digs, r)
        mask, counts = run_owners(devs[r].plan, digs, world, r)
        assert np.array_equal(mask[:n].cpu().numpy(), o_mask), f"rank {r}"
        assert counts_dict(counts) == o_cnt
        o_st, o_man, _ = oracle.compact(states[r], chunk, o_mask, o_digs[r])
        st, man, c2 = run_compact(devs[r].plan, mask, digs[r], o_cnt["staged_bytes"], o_cnt["ndirty"])
        assert counts_dict(c2) == o_cnt
        assert np.array_equal(st[:o_cnt["staged_bytes"]].cpu().numpy(), o_st)
        assert np.array_equal(ck.manifest_to_numpy(man, o_cnt["ndirty"]), o_man)


def test_owner_argument_errors():
    dev = DeviceBuffers([np.arange(1000, dtype=np.uint8)], 256)
    n = dev.plan.nchunks
    g = torch.zeros((2, n), dtype=torch.int64, device="cuda")
    mask = torch.zeros(n, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    for world, rank in ((0, 0), (2, 2), (2, 7)):
        with pytest.raises(ck.CkptError) as e:
            ck.upload_owners(dev.plan, g, world, rank, mask, counts)
        assert e.value.status == -1
    with pytest.raises(ck.CkptError):
        ck.upload_owners(dev.plan, None, 2, 0, mask, counts)
    with pytest.raises(ck.CkptError) as e:
        ck.upload_owners(dev.plan, g.view(torch.uint8).reshape(-1)[4:], 2, 0, mask, counts)
    assert e.value.status == -2
    torch.cuda.synchronize()


def test_owner_empty_plan():
    dev = DeviceBuffers([np.zeros(0, dtype=np.uint8)], 256)
    assert dev.plan.nchunks == 0
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    ck.upload_owners(dev.plan, None, 3, 1, None, counts)
    torch.cuda.synchronize()
    assert counts_dict(counts) == {"ndirty": 0, "staged_bytes": 0, "overflow": 0}


def test_config4_full_size_four_workers():
    """Four replicas of the 1.3 B state (here on one device, as four ranks' digests gathered):
    parameters and optimizer state are identical, gradients and activations private, so worker r
    uploads the shared chunks with k mod 4 == r plus all its private chunks."""
    w = wl.config(4)
    world = w.nreplicas
    a0, offs = wl.torch_replica(w, 0, "cuda")
    base = a0.data_ptr()
    plan0 = ck.Plan([(base + int(o), b.nbytes) for o, b in zip(offs, w.bufs)], w.chunk)
    n = plan0.nchunks
    gathered = torch.zeros((world, n), dtype=torch.int64, device="cuda")
    ck.fingerprint(plan0, gathered[0])
    for r in range(1, world):
        a, _ = wl.torch_replica(w, r, "cuda", shared_from=a0)
        plan = ck.Plan([(a.data_ptr() + int(o), b.nbytes) for o, b in zip(offs, w.bufs)], w.chunk)
        ck.fingerprint(plan, gathered[r])
        torch.cuda.synchronize()
        del plan, a
        torch.cuda.empty_cache()
    buf, _, length = wl.chunk_table(w)
    private = np.array([not b.shared for b in w.bufs])[buf]
    padded = (length + 15) // 16 * 16
    total = 0
    for r in range(world):
        mask, counts = run_owners(plan0, gathered, world, r)
        want = private | (np.arange(n) % world == r)
        assert np.array_equal(mask.cpu().numpy().astype(bool), want)
        c = counts_dict(counts)
        assert c == {"ndirty": int(want.sum()), "staged_bytes": int(padded[want].sum()), "overflow": 0}
        total += c["staged_bytes"]
    # one copy of the shared state plus every worker's private state
    assert total == int(padded[~private].sum()) + world * int(padded[private].sum())
