"""ckpt_buffer_verdicts on the GPU against the oracle: per buffer of the caller's list, does any
chunk carry a mark (the paper's per-buffer comparison, sec. 5.2.1), and the two counts."""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_07848_amd import binding as ck
from paper_2202_07848_amd import workloads as wl
from gpu_util import DeviceBuffers, run_diff, run_fingerprint

pytestmark = pytest.mark.gpu


def gpu_verdicts(plan, mask, nbufs):
    dirty = torch.full((nbufs + 64,), 0x77, dtype=torch.uint8, device="cuda")
    counts = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    ck.buffer_verdicts(plan, mask, dirty, counts)
    torch.cuda.synchronize()
    d = dirty.cpu().numpy()
    assert np.all(d[nbufs:] == 0x77)                    # nothing written past the list
    c = counts.cpu().numpy().view(np.uint64)
    return d[:nbufs], {"buffers": int(c[0]), "bytes": int(c[1])}


def check(sizes, chunk, mask_host):
    dev = DeviceBuffers([np.zeros(n, np.uint8) for n in sizes], chunk)
    assert dev.plan.nchunks == mask_host.size
    mask = torch.from_numpy(np.concatenate([mask_host, np.full(16, 0xFF, np.uint8)])).cuda()
    got, got_counts = gpu_verdicts(dev.plan, mask, len(sizes))
    want, want_counts = oracle.buffer_verdicts(sizes, chunk, mask_host)
    assert np.array_equal(got, want) and got_counts == want_counts
    return want_counts


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
@pytest.mark.parametrize("density", [0.0, 0.001, 0.05, 0.5, 1.0])
def test_random_geometry_and_masks(seed, density):
    rng = np.random.default_rng(seed)
    chunk = int(rng.choice([256, 512, 4096]))
    sizes = [int(x) for x in rng.integers(0, 40 * chunk, size=300)]
    sizes += [0, 0, 1, chunk - 1, chunk, chunk + 1] + [int(x) for x in rng.integers(1, 64, size=100)]
    rng.shuffle(sizes)
    n = sum((s + chunk - 1) // chunk for s in sizes)
    mask = (rng.random(n) < density).astype(np.uint8)
    mask[mask != 0] = rng.integers(1, 256, size=int(mask.sum()), dtype=np.uint8)
    check(sizes, chunk, mask)


@pytest.mark.parametrize("nchunks", [1, 3, 4, 5, 1023, 1024, 1025, 4097])
def test_chunk_counts_around_the_thread_and_block_sizes(nchunks):
    """One buffer per chunk (every thread's four chunks lie in four buffers), then one buffer
    holding all chunks; a mark on the last chunk only, and on every chunk."""
    chunk = 256
    for sizes in ([chunk] * nchunks, [chunk * nchunks]):
        last = np.zeros(nchunks, np.uint8)
        last[-1] = 1
        assert check(sizes, chunk, last)["buffers"] == 1
        assert check(sizes, chunk, np.ones(nchunks, np.uint8))["buffers"] == len(sizes)


def test_through_the_path_a_buffer_differs_exactly_when_its_bytes_do():
    rng = np.random.default_rng(7)
    sizes, chunk = [50000, 4096, 0, 12345, 70001, 16, 300], 4096
    ref = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]
    new = [b.copy() for b in ref]
    new[0][49999] ^= 1
    new[4][0] ^= 1
    new[5][15] ^= 1
    a, b = DeviceBuffers(ref, chunk), DeviceBuffers(new, chunk)
    mask, _ = run_diff(b.plan, run_fingerprint(b.plan), run_fingerprint(a.plan))
    got, counts = gpu_verdicts(b.plan, mask, len(sizes))
    assert got.tolist() == [int(not np.array_equal(x, y)) for x, y in zip(ref, new)]
    assert counts == {"buffers": 3, "bytes": 50000 + 70001 + 16}


@pytest.mark.parametrize("cfg,shrink", [(1, 1), (2, 6), (4, 16), (5, 16)])
def test_replica_configs_per_replica_buffers_differ_and_nothing_else(cfg, shrink):
    w = wl.config(cfg, shrink)
    a0, offs = wl.torch_replica(w, 0, "cuda")
    a1, _ = wl.torch_replica(w, 1, "cuda", shared_from=a0)
    plans = [ck.Plan([(a.data_ptr() + int(o), b.nbytes) for o, b in zip(offs, w.bufs)], w.chunk)
             for a in (a0, a1)]
    mask, cnt = run_diff(plans[1], run_fingerprint(plans[1]), run_fingerprint(plans[0]))
    got, counts = gpu_verdicts(plans[1], mask, len(w.bufs))
    want, want_counts = oracle.buffer_verdicts([b.nbytes for b in w.bufs], w.chunk,
                                               mask[:plans[1].nchunks].cpu().numpy())
    assert np.array_equal(got, want) and counts == want_counts
    assert got.tolist() == [int(not b.shared and b.nbytes > 0) for b in w.bufs]
    assert counts["bytes"] == w.distinct_bytes          # whole buffers differ in these configs


def test_empty_plan_and_argument_checks():
    nothing = ck.Plan([], 256)
    counts = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    ck.buffer_verdicts(nothing, None, None, counts)
    torch.cuda.synchronize()
    assert counts.tolist() == [0, 0]
    dev = DeviceBuffers([np.zeros(1000, np.uint8)], 256)
    mask = torch.zeros(4, dtype=torch.uint8, device="cuda")
    dirty = torch.zeros(1, dtype=torch.uint8, device="cuda")
    for args in ((dev.plan, None, dirty, counts), (dev.plan, mask, None, counts),
                 (dev.plan, mask, dirty, None)):
        with pytest.raises(ck.CkptError) as e:
            ck.buffer_verdicts(*args)
        assert e.value.status == -1


@pytest.mark.parametrize("n", [1, 15, 16, 17, 4096, 100003])
@pytest.mark.parametrize("shift", [0, 1])
def test_mask_andnot_against_the_oracle(n, shift):
    """Every byte value counts as set; odd addresses take the bytewise path; the result may
    overwrite either input; nothing is written past N."""
    rng = np.random.default_rng(n + shift)
    dev = DeviceBuffers([np.zeros(n * 256, np.uint8)], 256)
    assert dev.plan.nchunks == n
    a = rng.integers(0, 3, size=n, dtype=np.uint8) * rng.integers(1, 128, size=n, dtype=np.uint8)
    b = rng.integers(0, 3, size=n, dtype=np.uint8) * rng.integers(1, 128, size=n, dtype=np.uint8)
    want = oracle.mask_andnot(a, b)
    pad = np.full(32, 0x77, np.uint8)
    da = torch.from_numpy(np.concatenate([pad, a, pad])).cuda()[32 - shift:]
    db = torch.from_numpy(np.concatenate([pad, b, pad])).cuda()[32 - shift:]
    out = torch.full((n + 64,), 0x55, dtype=torch.uint8, device="cuda")
    ck.mask_andnot(dev.plan, da[shift:], db[shift:], out[shift:])
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert np.array_equal(got[shift:shift + n], want)
    assert np.all(got[:shift] == 0x55) and np.all(got[shift + n:] == 0x55)
    ck.mask_andnot(dev.plan, da[shift:], db[shift:], da[shift:])          # in place
    torch.cuda.synchronize()
    assert np.array_equal(da.cpu().numpy()[shift:shift + n], want)
    assert np.all(da.cpu().numpy()[shift + n:] == 0x77)


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_marks_from_buffers_against_the_oracle(seed):
    rng = np.random.default_rng(70 + seed)
    chunk = int(rng.choice([256, 512, 4096]))
    sizes = [int(x) for x in rng.integers(0, 40 * chunk, size=200)]
    sizes += [0, 0, 1, chunk - 1, chunk, chunk + 1] + [int(x) for x in rng.integers(1, 64, size=100)]
    rng.shuffle(sizes)
    flags = (rng.random(len(sizes)) < 0.4).astype(np.uint8) * rng.integers(1, 256, size=len(sizes), dtype=np.uint8)
    dev = DeviceBuffers([np.zeros(n, np.uint8) for n in sizes], chunk)
    n = dev.plan.nchunks
    marks = torch.full((n + 64,), 0x77, dtype=torch.uint8, device="cuda")
    ck.marks_from_buffers(dev.plan, torch.from_numpy(flags).cuda(), marks)
    torch.cuda.synchronize()
    got = marks.cpu().numpy()
    assert np.array_equal(got[:n], oracle.marks_from_buffers(sizes, chunk, flags))
    assert np.all(got[n:] == 0x77)


def test_buffer_flags_as_the_hint_of_the_first_snapshot():
    """The use: per-replica buffers flagged by whoever owns the allocator, expanded to the hint
    of ckpt_snapshot -- exact when whole buffers differ, so no chunk is gathered afterwards and
    every output equals the oracle's."""
    w = wl.config(4, 16)
    a0, offs = wl.torch_replica(w, 0, "cuda")
    a1, _ = wl.torch_replica(w, 1, "cuda", shared_from=a0)
    p0, p1 = (ck.Plan([(a.data_ptr() + int(o), b.nbytes) for o, b in zip(offs, w.bufs)], w.chunk)
              for a in (a0, a1))
    n = p1.nchunks
    ref = run_fingerprint(p0)
    flags = torch.tensor([0 if b.shared else 1 for b in w.bufs], dtype=torch.uint8, device="cuda")
    hint = torch.zeros(n, dtype=torch.uint8, device="cuda")
    ck.marks_from_buffers(p1, flags, hint)
    dig = torch.zeros(n, dtype=torch.int64, device="cuda")
    mask = torch.zeros(n, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    misses = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    staging = torch.zeros(w.distinct_bytes, dtype=torch.uint8, device="cuda")
    manifest = torch.zeros(w.distinct_chunks * 32, dtype=torch.uint8, device="cuda")
    ws = torch.zeros(ck.snapshot_workspace_bytes(n), dtype=torch.uint8, device="cuda")
    ck.snapshot(p1, ref, hint, dig, mask, staging, manifest, counts, misses, ws)
    torch.cuda.synchronize()
    assert int(misses.item()) == 0 and ck.snapshot_stats(ws, n)["regathered_chunks"] == 0
    host0, host1 = ([a[int(o):int(o) + b.nbytes].cpu().numpy() for o, b in zip(offs, w.bufs)]
                    for a in (a0, a1))
    o_dig = oracle.fingerprint(host1, w.chunk, 8)
    o_mask, _ = oracle.diff(host1, w.chunk, o_dig, oracle.fingerprint(host0, w.chunk, 8))
    o_st, o_man, o_cnt = oracle.compact(host1, w.chunk, o_mask, o_dig)
    assert np.array_equal(dig.cpu().numpy().view(np.uint64), o_dig)
    assert np.array_equal(mask.cpu().numpy(), o_mask) and np.array_equal(hint.cpu().numpy(), o_mask)
    assert np.array_equal(staging.cpu().numpy(), o_st)
    assert np.array_equal(ck.manifest_to_numpy(manifest, o_cnt["ndirty"]), o_man)
