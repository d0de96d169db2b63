"""GPU parity: the HIP path against the CPU oracle, element by element, on the
same bytes.  Everything here is integer / byte work, so the bar is bit-exact:
digests, masks, counts, manifest entries, staging bytes, restored buffers."""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_07848_amd import binding as ck
from paper_2202_07848_amd import workloads as wl
from gpu_util import (DeviceBuffers, counts_dict, run_compact, run_diff, run_fingerprint, u64)

pytestmark = pytest.mark.gpu

# lengths around every boundary the kernel has: 16-byte load, 32-byte stripe,
# 256-byte tile, chunk size, empty buffers, groups of 16 chunks with mixed lengths
ODD_SIZES = [0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 288, 511, 512, 1000, 4095, 4096, 4097,
             8191, 8192, 12289, 0, 31, 100000, 7, 65536, 65537, 3, 262144 + 40, 5000]


def host_bufs(seed, sizes):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]


def full_pipeline_check(snap, ref_bufs, chunk, dst_init=None):
    """fingerprint -> diff -> compact -> restore on the GPU, compared with the oracle at
    every step.  ref_bufs: reference content (same geometry) or None."""
    dev = DeviceBuffers(snap, chunk)
    n = oracle.nchunks(snap, chunk)
    assert dev.plan.nchunks == n and dev.plan.nbytes == sum(b.size for b in snap)

    want_dig = oracle.fingerprint(snap, chunk, 8)
    dig = run_fingerprint(dev.plan)
    assert np.array_equal(u64(dig, n), want_dig)

    if ref_bufs is not None:
        want_ref = oracle.fingerprint(ref_bufs, chunk, 8)
        dev_ref = DeviceBuffers(ref_bufs, chunk)
        ref = run_fingerprint(dev_ref.plan)
        assert np.array_equal(u64(ref, n), want_ref)
    else:
        want_ref, ref = None, None

    want_mask, want_cnt = oracle.diff(snap, chunk, want_dig, want_ref)
    mask, counts = run_diff(dev.plan, dig, ref)
    assert np.array_equal(mask[:n].cpu().numpy(), want_mask)
    assert counts_dict(counts) == want_cnt

    want_st, want_man, want_cnt2 = oracle.compact(snap, chunk, want_mask, want_dig)
    staging, manifest, counts2 = run_compact(dev.plan, mask, dig, want_st.size, want_man.size)
    assert counts_dict(counts2) == want_cnt2
    st = staging.cpu().numpy()
    assert np.array_equal(st[:want_st.size], want_st)
    assert np.all(st[want_st.size:] == 0xA5)
    man_raw = manifest.cpu().numpy()
    assert np.array_equal(man_raw[:32 * want_man.size].view(oracle.ENTRY_DTYPE), want_man)
    assert np.all(man_raw[32 * want_man.size:] == 0xA5)
    assert dev.canaries_intact()

    # restore into a destination that holds the reference (or garbage when there is none)
    if dst_init is None:
        dst_init = ref_bufs if ref_bufs is not None else host_bufs(99, [b.size for b in snap])
    dst = DeviceBuffers(dst_init, chunk)
    want_dst = [b.copy() for b in dst_init]
    assert oracle.restore(want_dst, chunk, want_st, want_man) == 0
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ck.restore(dst.plan, staging, want_st.size, manifest, want_man.size, rejected)
    torch.cuda.synchronize()
    assert int(rejected.item()) == 0
    got, img = dst.host()
    for g, w, s in zip(got, want_dst, snap):
        assert np.array_equal(g, w)
        assert np.array_equal(g, s)
    assert dst.canaries_intact(img)
    return want_cnt2


@pytest.mark.parametrize("chunk", [256, 1024, 4096, 65536])
def test_odd_sizes_no_reference(chunk):
    snap = host_bufs(1, ODD_SIZES)
    cnt = full_pipeline_check(snap, None, chunk)
    assert cnt["ndirty"] == oracle.nchunks(snap, chunk)


@pytest.mark.parametrize("chunk", [256, 4096])
def test_odd_sizes_against_reference(chunk):
    ref = host_bufs(2, ODD_SIZES)
    snap = [b.copy() for b in ref]
    rng = np.random.default_rng(3)
    for i, b in enumerate(snap):          # touch single bytes in about a third of the buffers
        if b.size and i % 3 == 0:
            for off in rng.integers(0, b.size, size=3):
                b[off] ^= 0x5A
    snap[23][99999] ^= 1                  # last byte of a ragged last chunk
    cnt = full_pipeline_check(snap, ref, chunk)
    assert 0 < cnt["ndirty"] < oracle.nchunks(snap, chunk)


def sizes_with_chunks(total_chunks, chunk):
    """A ragged buffer list (odd sizes, empty buffers, short last chunks) with exactly
    total_chunks chunks."""
    sizes = [1, 255, 257, 1000, 70001, 0, 4097, 300, 123457, 31, 5 * chunk, 0, 999999, chunk + 1]
    have = sum(-(-n // chunk) for n in sizes)
    left = total_chunks - have
    assert left > 2
    half = left // 2
    return sizes[:7] + [half * chunk] + sizes[7:] + [(left - half) * chunk - 17]


@pytest.mark.parametrize("nchunks", [1 << 18, (1 << 18) + 1],
                         ids=["scan_in_one_kernel_at_its_limit", "scan_in_two_kernels"])
def test_both_scan_shapes_at_the_switch_over(nchunks):
    """Up to 2**18 chunks every workgroup of the manifest kernel counts the marked chunks in
    front of its block itself; above, block sums are scanned by the workgroup that finishes
    last and a second kernel writes the manifest.  One case on each side of the boundary."""
    chunk = 256
    sizes = sizes_with_chunks(nchunks, chunk)
    ref = host_bufs(21, sizes)
    assert oracle.nchunks(ref, chunk) == nchunks
    snap = [b.copy() for b in ref]
    rng = np.random.default_rng(22)
    for b in snap:                          # about 1 byte in 700 differs, everywhere
        if b.size:
            b[rng.integers(0, b.size, size=max(1, b.size // 700))] ^= 0x3C
    cnt = full_pipeline_check(snap, ref, chunk)
    assert nchunks // 8 < cnt["ndirty"] < nchunks
    cnt = full_pipeline_check(snap, None, chunk)
    assert cnt["ndirty"] == nchunks


def test_identical_replica_stages_nothing():
    ref = host_bufs(4, ODD_SIZES)
    cnt = full_pipeline_check([b.copy() for b in ref], ref, 1024)
    assert cnt == {"ndirty": 0, "staged_bytes": 0, "overflow": 0}


def test_empty_plans():
    for sizes in ([], [0, 0, 0]):
        cnt = full_pipeline_check(host_bufs(5, sizes), None, 4096)
        assert cnt == {"ndirty": 0, "staged_bytes": 0, "overflow": 0}


def test_many_tiny_buffers_one_group_spans_sixteen_buffers():
    sizes = [1 + (i * 37) % 700 for i in range(200)] + [0, 0] + [300] * 40
    full_pipeline_check(host_bufs(6, sizes), None, 256)


def test_single_long_ragged_chunk():
    # a 3 MiB + 5 byte buffer with 4 MiB chunks: one long chunk that ends mid-stripe
    full_pipeline_check(host_bufs(7, [3 * 1024 * 1024 + 5, 100]), None, 4 * 1024 * 1024)


def test_maximum_chunk_size():
    # the largest chunk the plan accepts (1 GiB): one full chunk hashed by a single quad of
    # lanes for 2**25 stripes, and a short second chunk that ends mid-stripe
    chunk = 1 << 30
    rng = np.random.default_rng(11)
    big = rng.integers(0, 256, size=chunk + 4096 + 5, dtype=np.uint8)
    dev = DeviceBuffers([big], chunk)
    assert dev.plan.nchunks == 2
    dig = run_fingerprint(dev.plan)
    assert np.array_equal(u64(dig, 2), oracle.fingerprint([big], chunk, 2))
    # only the short chunk is marked: compact and restore it
    mask = torch.tensor([0, 1], dtype=torch.uint8, device="cuda")
    staging, manifest, counts = run_compact(dev.plan, mask, dig, 4112, 1)
    assert counts_dict(counts) == {"ndirty": 1, "staged_bytes": 4112, "overflow": 0}
    st = staging.cpu().numpy()
    assert np.array_equal(st[:4101], big[chunk:]) and not st[4101:4112].any()
    man = ck.manifest_to_numpy(manifest, 1)
    assert (int(man["buf"][0]), int(man["len"][0]), int(man["buf_off"][0])) == (0, 4101, chunk)


def test_config1_tiny_spliced_pair_full_size():
    w = wl.config(1)
    rep0, rep1 = wl.numpy_replica(w, 0), wl.numpy_replica(w, 1)
    cnt = full_pipeline_check(rep1, rep0, w.chunk)
    assert cnt["ndirty"] == w.distinct_chunks
    assert cnt["staged_bytes"] == w.distinct_bytes


@pytest.mark.parametrize("cfg,shrink", [(2, 6), (4, 16), (5, 16)])
def test_replica_configs_reduced(cfg, shrink):
    w = wl.config(cfg, shrink)
    rep0 = wl.numpy_replica(w, 0)
    for r in range(1, w.nreplicas):
        cnt = full_pipeline_check(wl.numpy_replica(w, r), rep0, w.chunk)
        assert cnt["ndirty"] == w.distinct_chunks


@pytest.mark.parametrize("fraction", [0.01, 0.10, 0.50])
def test_config3_fragmented_reduced(fraction):
    w = wl.config(3, 100)       # 1000 buffers
    t0 = wl.numpy_replica(w, 0)
    step = int(fraction * 100)
    ids = wl.dirty_chunk_ids(w, fraction, step)
    t1 = [b.copy() for b in t0]
    wl.numpy_rewrite_chunks(w, t1, ids, step)
    cnt = full_pipeline_check(t1, t0, w.chunk)
    assert cnt["ndirty"] == ids.size


def test_compact_capacity_overflow_writes_nothing_out_of_bounds():
    snap = host_bufs(8, [1000, 1000, 5000, 4096 * 3 + 1])
    chunk = 256
    dev = DeviceBuffers(snap, chunk)
    n = dev.plan.nchunks
    want_dig = oracle.fingerprint(snap, chunk)
    dig = run_fingerprint(dev.plan)
    mask, _ = run_diff(dev.plan, dig, None)
    want_mask = np.ones(n, dtype=np.uint8)
    full_st, full_man, _ = oracle.compact(snap, chunk, want_mask, want_dig)
    for staging_cap, manifest_cap in [(full_st.size, 5), (700, n), (0, 0), (1024, 3),
                                      (full_st.size - 16, n), (full_st.size, n - 1)]:
        want_st, want_man, want_cnt = oracle.compact(snap, chunk, want_mask, want_dig,
                                                     staging_cap=staging_cap,
                                                     manifest_cap=manifest_cap)
        staging, manifest, counts = run_compact(dev.plan, mask, dig, staging_cap, manifest_cap)
        assert counts_dict(counts) == want_cnt
        assert want_cnt["overflow"] > 0
        st = staging.cpu().numpy()
        assert np.array_equal(st[:staging_cap], want_st)
        assert np.all(st[staging_cap:] == 0xA5)
        man_raw = manifest.cpu().numpy()
        assert np.array_equal(man_raw[:32 * manifest_cap].view(oracle.ENTRY_DTYPE), want_man)
        assert np.all(man_raw[32 * manifest_cap:] == 0xA5)


def test_restore_skips_entries_that_do_not_fit():
    chunk = 1024
    snap = host_bufs(9, [2048, 1000, 4096])
    dig = oracle.fingerprint(snap, chunk)
    mask = np.ones(dig.size, dtype=np.uint8)
    staging, man, _ = oracle.compact(snap, chunk, mask, dig)
    bad = man.copy()
    bad["stage_off"][0] += 8            # misaligned
    bad["len"][1] = 1025                # longer than a chunk
    bad["buf"][2] = 7                   # no such buffer
    bad["buf_off"][3] = 4096            # outside its buffer
    bad["stage_off"][4] = staging.size  # outside staging
    bad["buf_off"][5] = np.uint64(2**64 - 1024)   # would wrap
    dst_init = [np.zeros(b.size, dtype=np.uint8) for b in snap]
    want = [b.copy() for b in dst_init]
    want_rejected = oracle.restore(want, chunk, staging, bad)
    assert want_rejected == 6
    dst = DeviceBuffers(dst_init, chunk)
    d_staging = torch.from_numpy(staging).cuda()
    d_man = torch.from_numpy(bad.view(np.uint8).copy()).cuda()
    rejected = torch.zeros(1, dtype=torch.int64, device="cuda")
    ck.restore(dst.plan, d_staging, staging.size, d_man, bad.size, rejected)
    torch.cuda.synchronize()
    assert int(rejected.item()) == want_rejected
    got, img = dst.host()
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
    assert dst.canaries_intact(img)


def test_restore_into_other_replica_buffers_is_idempotent():
    w = wl.config(1)
    rep0, rep1 = wl.numpy_replica(w, 0), wl.numpy_replica(w, 1)
    d0, d1 = DeviceBuffers(rep0, w.chunk), DeviceBuffers(rep1, w.chunk)
    ref, dig = run_fingerprint(d0.plan), run_fingerprint(d1.plan)
    mask, counts = run_diff(d1.plan, dig, ref)
    c = counts_dict(counts)
    staging, manifest, _ = run_compact(d1.plan, mask, dig, c["staged_bytes"], c["ndirty"])
    for _ in range(2):
        ck.restore(d0.plan, staging, c["staged_bytes"], manifest, c["ndirty"])
    torch.cuda.synchronize()
    got, img = d0.host()
    assert all(np.array_equal(g, s) for g, s in zip(got, rep1))
    assert d0.canaries_intact(img)
    # and the restored replica now fingerprints like replica 1
    assert np.array_equal(u64(run_fingerprint(d0.plan), d0.plan.nchunks), u64(dig, d1.plan.nchunks))


def test_argument_errors_on_device():
    snap = host_bufs(10, [4096, 4096])
    dev = DeviceBuffers(snap, 1024)
    dig = run_fingerprint(dev.plan)
    mask = torch.zeros(8, dtype=torch.uint8, device="cuda")
    counts = torch.zeros(3, dtype=torch.int64, device="cuda")
    with pytest.raises(ck.CkptError) as e:
        ck.diff(dev.plan, dig, dig, mask, counts, n_ref=7)
    assert e.value.status == -4
    with pytest.raises(ck.CkptError) as e:
        ck.Plan([(dev.arena.data_ptr() + 8, 100)], 1024)
    assert e.value.status == -2
    with pytest.raises(ck.CkptError) as e:
        ck.Plan([(dev.arena.data_ptr(), 100)], 1000)
    assert e.value.status == -3
