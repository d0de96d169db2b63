"""GPU parity of swap-out to / swap-in from host memory (paper sec. 5.1, 5.2.1)
against the oracle: the host image must be the oracle's staging byte for byte,
the manifest its manifest, and swap-in must rebuild the buffers exactly --
through a device ring much smaller than the staged data, with chunks that span
many slices and slices that span many chunks."""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_07848_amd import binding as ck
from paper_2202_07848_amd import workloads as wl
from gpu_util import DeviceBuffers, run_diff, run_fingerprint

pytestmark = pytest.mark.gpu

ODD_SIZES = [0, 1, 15, 16, 17, 255, 256, 257, 1000, 4095, 4096, 4097, 70000, 0, 31, 300001, 7,
             65536, 65537, 262144 + 40, 5000]


def host_bufs(seed, sizes):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]


def swap_round_trip(snap, ref_bufs, chunk, slice_bytes):
    dev = DeviceBuffers(snap, chunk)
    n = dev.plan.nchunks
    dig = run_fingerprint(dev.plan)
    o_dig = oracle.fingerprint(snap, chunk, 8)
    if ref_bufs is not None:
        o_ref = oracle.fingerprint(ref_bufs, chunk, 8)
        ref = torch.from_numpy(o_ref.view(np.int64)).cuda()
    else:
        o_ref, ref = None, None
    mask, _ = run_diff(dev.plan, dig, ref)
    o_mask, _ = oracle.diff(snap, chunk, o_dig, o_ref)
    want_st, want_man, want_cnt = oracle.compact(snap, chunk, o_mask, o_dig)

    slack = 4096
    h_staging = torch.full((want_st.size + slack,), 0xA5, dtype=torch.uint8).pin_memory()
    manifest = torch.full((max(1, want_man.size) * 32 + 256,), 0xA5, dtype=torch.uint8,
                          device="cuda")
    sw = ck.Swapper(slice_bytes)
    cnt = sw.swap_out(dev.plan, mask, dig, h_staging, manifest, staging_cap=want_st.size,
                      manifest_cap=want_man.size)
    assert cnt == {**want_cnt, "status": 0}
    img = h_staging.numpy()
    assert np.array_equal(img[:want_st.size], want_st)
    assert np.all(img[want_st.size:] == 0xA5)
    man_raw = manifest.cpu().numpy()
    assert np.array_equal(man_raw[:32 * want_man.size].view(oracle.ENTRY_DTYPE), want_man)
    assert np.all(man_raw[32 * want_man.size:] == 0xA5)
    assert dev.canaries_intact()

    dst_init = ref_bufs if ref_bufs is not None else host_bufs(77, [b.size for b in snap])
    dst = DeviceBuffers(dst_init, chunk)
    rejected = sw.swap_in(dst.plan, h_staging, want_st.size, manifest, want_man.size)
    assert rejected == 0
    want_dst = [b.copy() for b in dst_init]
    assert oracle.restore(want_dst, chunk, want_st, want_man) == 0
    got, image = dst.host()
    for g, w, s in zip(got, want_dst, snap):
        assert np.array_equal(g, w) and np.array_equal(g, s)
    assert dst.canaries_intact(image)
    sw.close()
    return want_cnt


@pytest.mark.parametrize("chunk,slice_bytes", [(256, 65536), (4096, 65536), (65536, 131072),
                                               (1 << 20, 65536), (4096, 1 << 22)])
def test_swap_round_trip_no_reference(chunk, slice_bytes):
    cnt = swap_round_trip(host_bufs(1, ODD_SIZES), None, chunk, slice_bytes)
    assert cnt["staged_bytes"] > 2 * slice_bytes or slice_bytes >= (1 << 22)


def test_swap_round_trip_against_reference():
    ref = host_bufs(2, ODD_SIZES)
    snap = [b.copy() for b in ref]
    rng = np.random.default_rng(3)
    for i, b in enumerate(snap):
        if b.size and i % 2 == 0:
            b[rng.integers(0, b.size, size=5)] ^= 0x33
    cnt = swap_round_trip(snap, ref, 1024, 65536)
    assert 0 < cnt["ndirty"] < oracle.nchunks(snap, 1024)


def test_swap_nothing_dirty_and_empty_plan():
    ref = host_bufs(4, ODD_SIZES)
    assert swap_round_trip([b.copy() for b in ref], ref, 4096, 65536)["staged_bytes"] == 0
    assert swap_round_trip([], None, 4096, 65536)["ndirty"] == 0


def test_swap_config1_full_size():
    w = wl.config(1)
    cnt = swap_round_trip(wl.numpy_replica(w, 1), wl.numpy_replica(w, 0), w.chunk, 1 << 20)
    assert cnt["staged_bytes"] == w.distinct_bytes


def test_swap_out_capacity_error_leaves_host_buffer_untouched():
    snap = host_bufs(5, [100000, 5000])
    dev = DeviceBuffers(snap, 4096)
    dig = run_fingerprint(dev.plan)
    mask, _ = run_diff(dev.plan, dig, None)
    need = int(((oracle.chunk_lens(snap, 4096).astype(np.int64) + 15) // 16 * 16).sum())
    h = torch.full((need,), 0x5A, dtype=torch.uint8).pin_memory()
    manifest = torch.zeros(dev.plan.nchunks * 32, dtype=torch.uint8, device="cuda")
    sw = ck.Swapper(65536)
    cnt = sw.swap_out(dev.plan, mask, dig, h, manifest, staging_cap=need - 16)
    assert cnt["status"] == -5 and cnt["staged_bytes"] == need and cnt["overflow"] != 0
    assert bool((h == 0x5A).all())
    cnt = sw.swap_out(dev.plan, mask, dig, h, manifest, manifest_cap=dev.plan.nchunks - 1)
    assert cnt["status"] == -5 and cnt["overflow"] == 1
    assert bool((h == 0x5A).all())
    with pytest.raises(ck.CkptError):
        ck.Swapper(1000)


# ---- the same swap with no ring and no DMA: staging in pinned host memory -----------------
# ckpt_compact, ckpt_snapshot and ckpt_restore take a staging pointer the device can reach; pinned
# host memory is such a pointer, and then the kernels move the bytes over the host link
# themselves.  The calls stay asynchronous, which the ring cannot be.

def pinned(nbytes, fill):
    t = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    t.fill_(fill)
    assert t.is_pinned()
    return t


@pytest.mark.parametrize("chunk", [256, 4096, 65536, 1 << 20])
@pytest.mark.parametrize("fused", [False, True], ids=["compact", "snapshot"])
def test_staging_in_pinned_host_memory(chunk, fused):
    ref_bufs = host_bufs(5, ODD_SIZES)
    snap = [b.copy() for b in ref_bufs]
    rng = np.random.default_rng(6)
    for i in (6, 8, 12, 15, 19):
        off = int(rng.integers(0, snap[i].size))
        snap[i][off:off + 3000] ^= 0x3C
    dev = DeviceBuffers(snap, chunk)
    n = dev.plan.nchunks
    o_ref, o_dig = oracle.fingerprint(ref_bufs, chunk, 8), oracle.fingerprint(snap, chunk, 8)
    o_mask, _ = oracle.diff(snap, chunk, o_dig, o_ref)
    want_st, want_man, want_cnt = oracle.compact(snap, chunk, o_mask, o_dig)
    ref = torch.from_numpy(o_ref.view(np.int64)).cuda()
    slack = 4096
    h_staging = pinned(want_st.size + slack, 0xA5)
    manifest = torch.full((max(1, want_man.size) * 32,), 0xA5, dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    dig = torch.zeros(n, dtype=torch.int64, device="cuda")
    mask = torch.zeros(n, dtype=torch.uint8, device="cuda")
    if fused:
        hint = torch.from_numpy(o_mask).cuda()
        misses = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        ws = torch.empty(ck.snapshot_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        ck.snapshot(dev.plan, ref, hint, dig, mask, h_staging, manifest, counts, misses, ws,
                    staging_cap=want_st.size, manifest_cap=want_man.size)
        torch.cuda.synchronize()
        assert int(misses.item()) == 0
    else:
        ck.fingerprint(dev.plan, dig)
        ck.diff(dev.plan, dig, ref, mask, counts)
        ck.compact(dev.plan, mask, dig, h_staging, manifest, counts, staging_cap=want_st.size,
                   manifest_cap=want_man.size)
        torch.cuda.synchronize()
    c = counts.cpu().numpy().view(np.uint64)
    assert {"ndirty": int(c[0]), "staged_bytes": int(c[1]), "overflow": int(c[2])} == want_cnt
    img = h_staging.numpy()
    assert np.array_equal(img[:want_st.size], want_st)
    assert np.all(img[want_st.size:] == 0xA5)
    assert np.array_equal(ck.manifest_to_numpy(manifest, want_man.size), want_man)

    dst = DeviceBuffers(ref_bufs, chunk)
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ck.restore_counted(dst.plan, h_staging, want_st.size, manifest, want_man.size, counts, rejected)
    torch.cuda.synchronize()
    assert int(rejected.item()) == 0
    got, image = dst.host()
    assert all(np.array_equal(g, s) for g, s in zip(got, snap))
    assert dst.canaries_intact(image)
