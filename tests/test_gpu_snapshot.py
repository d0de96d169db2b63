"""GPU parity of the fused ckpt_snapshot (fingerprint + diff + compact in one
call, optionally in one pass over the data guided by a hint) against the
oracle's three separate steps: same digests, mask, counts, manifest and staging
bytes whatever the hint says -- exact, absent, wrong, all ones, all zeros -- and
under capacity limits."""
import numpy as np
import pytest
import torch

import oracle
from paper_2202_07848_amd import binding as ck
from paper_2202_07848_amd import workloads as wl
from gpu_util import DeviceBuffers, counts_dict, u64

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True, params=["two_launches", "one_launch"])
def fused_pass_shape(request):
    """Every test here runs with the hinted pass forced into each of its two launch shapes (the
    library picks by state size, and these inputs are all on the small side)."""
    import gpu_util
    gpu_util.SPLIT_THRESHOLD = 0 if request.param == "two_launches" else 2**64 - 1
    yield request.param
    gpu_util.SPLIT_THRESHOLD = None

ODD_SIZES = [0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 288, 511, 512, 1000, 4095, 4096, 4097,
             8191, 8192, 12289, 0, 31, 100000, 7, 65536, 65537, 3, 262144 + 40, 5000]


def host_bufs(seed, sizes):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]


def run_snapshot(dev, ref, hint, staging_cap, manifest_cap, alias_hint_and_mask=False):
    n = dev.plan.nchunks
    dig = torch.zeros(max(1, n), dtype=torch.int64, device="cuda")
    mask = torch.full((max(1, n),), 0x77, dtype=torch.uint8, device="cuda")
    if hint is not None and alias_hint_and_mask:
        mask[:n] = hint[:n]
        hint = mask
    staging = torch.full((staging_cap + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    manifest = torch.full((manifest_cap * 32 + 256,), 0xA5, dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    misses = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ws = torch.full((ck.snapshot_workspace_bytes(n),), 0x11, dtype=torch.uint8, device="cuda")
    ck.snapshot(dev.plan, ref, hint, dig, mask, staging, manifest, counts, misses, ws,
                staging_cap=staging_cap, manifest_cap=manifest_cap,
                n_ref=None if ref is None else n)
    torch.cuda.synchronize()
    stats = ck.snapshot_stats(ws, n) if hint is not None else None
    return dig, mask, staging, manifest, counts_dict(counts), int(misses.item()), stats


def expected_regather(lens, h, o_mask, staging_cap, manifest_cap):
    """Entries the corrective gather has to copy after a pass guided by hint h: those the pass
    did not already put at their final offset.  Host arithmetic on the definition: a chunk is in
    place iff it was hinted, its entry would have fitted the manifest in the hint's numbering,
    the hint's prefix sum gives it the offset the real mask's prefix sum gives it, and it fits."""
    pad = (lens.astype(np.int64) + 15) // 16 * 16
    hm, m = (h != 0), (o_mask != 0)
    if not np.any(hm != m):
        return 0
    hoff = np.cumsum(pad * hm) - pad * hm
    hcnt = np.cumsum(hm) - hm
    off = np.cumsum(pad * m) - pad * m
    cnt = np.cumsum(m) - m
    fits = m & (cnt < manifest_cap) & (off + pad <= staging_cap)
    in_place = fits & hm & (hcnt < manifest_cap) & (hoff == off)
    return int((fits & ~in_place).sum())


def check_against_oracle(snap, ref_bufs, chunk, hint_kind, staging_cap=None, manifest_cap=None,
                         alias=False):
    dev = DeviceBuffers(snap, chunk)
    n = dev.plan.nchunks
    o_dig = oracle.fingerprint(snap, chunk, 8)
    o_ref = None if ref_bufs is None else oracle.fingerprint(ref_bufs, chunk, 8)
    o_mask, o_cnt = oracle.diff(snap, chunk, o_dig, o_ref)
    o_st, o_man, o_cnt2 = oracle.compact(snap, chunk, o_mask, o_dig, staging_cap=staging_cap,
                                         manifest_cap=manifest_cap)
    rng = np.random.default_rng(n)
    if hint_kind == "exact":
        h = o_mask.copy()
    elif hint_kind == "none":
        h = None
    elif hint_kind == "ones":
        h = np.ones(n, dtype=np.uint8)
    elif hint_kind == "zeros":
        h = np.zeros(n, dtype=np.uint8)
    elif hint_kind == "one_flip":
        h = o_mask.copy()
        h[n // 2] ^= 1
    else:
        h = (rng.random(n) < 0.5).astype(np.uint8) * 7          # any non-zero byte marks
    hint = None if h is None else torch.from_numpy(h if h.size else np.zeros(1, np.uint8)).cuda()
    ref = None if o_ref is None else torch.from_numpy(o_ref.view(np.int64)).cuda()
    dig, mask, staging, manifest, cnt, misses, stats = run_snapshot(
        dev, ref, hint, o_st.size, o_man.size, alias_hint_and_mask=alias)
    assert np.array_equal(u64(dig, n), o_dig)
    assert np.array_equal(mask[:n].cpu().numpy(), o_mask)
    assert cnt == o_cnt2
    want_misses = 0 if h is None else int(((h != 0) != (o_mask != 0)).sum())
    assert misses == want_misses
    if h is not None:
        # the gather after a wrong hint copies exactly the chunks that are not yet in place
        assert stats["hint_misses"] == want_misses
        assert stats["regathered_chunks"] == expected_regather(
            oracle.chunk_lens(snap, chunk), h, o_mask, o_st.size, o_man.size)
    man_raw = manifest.cpu().numpy()
    assert np.array_equal(man_raw[:32 * o_man.size].view(oracle.ENTRY_DTYPE), o_man)
    assert np.all(man_raw[32 * o_man.size:] == 0xA5)
    st = staging.cpu().numpy()
    if want_misses == 0:
        # single pass: exactly the oracle's staging, unwritten bytes included
        assert np.array_equal(st[:o_st.size], o_st)
    elif staging_cap is None and manifest_cap is None:
        # wrong hint, enough room: the gather that followed made the staged range exact
        assert np.array_equal(st[:o_cnt2["staged_bytes"]], o_st)
    assert np.all(st[o_st.size:] == 0xA5)                      # never past the capacity
    assert dev.canaries_intact()
    return cnt, misses


HINTS = ["exact", "none", "ones", "zeros", "one_flip", "random"]


@pytest.mark.parametrize("hint_kind", HINTS)
@pytest.mark.parametrize("chunk", [256, 4096])
def test_snapshot_against_reference(chunk, hint_kind):
    ref = host_bufs(2, ODD_SIZES)
    snap = [b.copy() for b in ref]
    rng = np.random.default_rng(3)
    for i, b in enumerate(snap):
        if b.size and i % 3 == 0:
            for off in rng.integers(0, b.size, size=3):
                b[off] ^= 0x5A
    snap[23][99999] ^= 1
    cnt, misses = check_against_oracle(snap, ref, chunk, hint_kind)
    assert 0 < cnt["ndirty"] < oracle.nchunks(snap, chunk)
    assert (misses == 0) == (hint_kind in ("exact", "none"))


@pytest.mark.parametrize("hint_kind", ["exact", "none", "one_flip", "random"])
@pytest.mark.parametrize("nchunks", [1 << 18, (1 << 18) + 1],
                         ids=["scan_in_one_kernel_at_its_limit", "scan_in_two_kernels"])
def test_snapshot_both_scan_shapes_at_the_switch_over(nchunks, hint_kind):
    from test_gpu_parity import sizes_with_chunks
    chunk = 256
    ref = host_bufs(31, sizes_with_chunks(nchunks, chunk))
    snap = [b.copy() for b in ref]
    rng = np.random.default_rng(32)
    for b in snap:
        if b.size:
            b[rng.integers(0, b.size, size=max(1, b.size // 900))] ^= 0x11
    cnt, misses = check_against_oracle(snap, ref, chunk, hint_kind)
    assert nchunks // 8 < cnt["ndirty"] < nchunks
    assert (misses == 0) == (hint_kind in ("exact", "none"))


def test_one_wrong_hint_chunk_regathers_only_what_lies_behind_it():
    """A hint that is wrong in one chunk in the middle: the chunks staged before it stay as the
    pass wrote them, the gather copies the ones behind it (about half), and the result is exact."""
    chunk = 4096
    ref = host_bufs(41, [1 << 20, 3 << 20, 4096 * 9 + 5, 2 << 20])
    snap = [b.copy() for b in ref]
    for b in snap:
        b[::8192] ^= 0x7E                      # every second chunk differs
    dev = DeviceBuffers(snap, chunk)
    n = dev.plan.nchunks
    o_dig, o_ref = oracle.fingerprint(snap, chunk, 8), oracle.fingerprint(ref, chunk, 8)
    o_mask, _ = oracle.diff(snap, chunk, o_dig, o_ref)
    o_st, o_man, o_cnt = oracle.compact(snap, chunk, o_mask, o_dig)
    ref_t = torch.from_numpy(o_ref.view(np.int64)).cuda()
    for flip, lo, hi in ((n // 2, 0.4, 0.6), (n - 1, 0.0, 0.01), (0, 0.99, 1.01)):
        h = o_mask.copy()
        h[flip] ^= 1
        out = run_snapshot(dev, ref_t, torch.from_numpy(h).cuda(), o_st.size, o_man.size)
        dig, mask, staging, manifest, cnt, misses, stats = out
        assert misses == 1 and cnt == o_cnt
        assert np.array_equal(staging.cpu().numpy()[:o_st.size], o_st)
        assert np.array_equal(ck.manifest_to_numpy(manifest, o_man.size), o_man)
        assert lo * o_man.size <= stats["regathered_chunks"] <= hi * o_man.size, (flip, stats)


@pytest.mark.parametrize("hint_kind", ["exact", "ones", "zeros"])
def test_snapshot_without_reference(hint_kind):
    cnt, misses = check_against_oracle(host_bufs(1, ODD_SIZES), None, 1024, hint_kind)
    assert cnt["ndirty"] == oracle.nchunks(host_bufs(1, ODD_SIZES), 1024)
    assert (misses == 0) == (hint_kind != "zeros")


def test_snapshot_hint_and_mask_in_one_buffer():
    ref = host_bufs(4, ODD_SIZES)
    snap = [b.copy() for b in ref]
    snap[15][7] ^= 1
    snap[28][200000] ^= 1
    check_against_oracle(snap, ref, 4096, "exact", alias=True)
    check_against_oracle(snap, ref, 4096, "random", alias=True)


@pytest.mark.parametrize("caps", [(700, None), (None, 5), (0, 0), (1024, 3)])
@pytest.mark.parametrize("hint_kind", ["exact", "ones"])
def test_snapshot_capacity_limits(caps, hint_kind):
    snap = host_bufs(8, [1000, 1000, 5000, 4096 * 3 + 1])
    n = oracle.nchunks(snap, 256)
    staging_cap, manifest_cap = caps
    full_st, full_man, _ = oracle.compact(snap, 256, np.ones(n, np.uint8),
                                          oracle.fingerprint(snap, 256))
    check_against_oracle(snap, None, 256, hint_kind,
                         staging_cap=full_st.size if staging_cap is None else staging_cap,
                         manifest_cap=n if manifest_cap is None else manifest_cap)


def test_snapshot_config1_full_size_exact_hint_single_pass():
    w = wl.config(1)
    rep0, rep1 = wl.numpy_replica(w, 0), wl.numpy_replica(w, 1)
    cnt, misses = check_against_oracle(rep1, rep0, w.chunk, "exact")
    assert misses == 0 and cnt["staged_bytes"] == w.distinct_bytes


def test_snapshot_empty_plan_and_argument_errors():
    check_against_oracle([], None, 4096, "exact")
    dev = DeviceBuffers(host_bufs(9, [4096]), 1024)
    t = lambda n, dt=torch.uint8: torch.zeros(n, dtype=dt, device="cuda")
    with pytest.raises(ck.CkptError) as e:     # workspace too small for a hinted call
        ck.snapshot(dev.plan, None, t(4), t(4, torch.int64), t(4), t(4096), t(4 * 32),
                    t(3, torch.int64), None, t(16))
    assert e.value.status == -5
    with pytest.raises(ck.CkptError) as e:     # reference of another geometry
        ck.snapshot(dev.plan, t(3, torch.int64), None, t(4, torch.int64), t(4), t(4096),
                    t(4 * 32), t(3, torch.int64), n_ref=3)
    assert e.value.status == -4


def test_thousands_of_buffers_shorter_than_a_chunk():
    """Nearly every chunk is a short last chunk: the one-kernel manifest path gets its byte
    offsets from the plan's short-chunk list, which here is as long as the chunk list itself."""
    rng = np.random.default_rng(51)
    sizes = rng.integers(0, 5000, size=6000).tolist() + [4096 * 3, 4096, 1]
    ref = host_bufs(52, sizes)
    snap = [b.copy() for b in ref]
    for i in rng.choice(len(snap), size=2500, replace=False).tolist():
        if snap[i].size:
            snap[i][int(rng.integers(0, snap[i].size))] ^= 0x80
    for kind in ("exact", "none", "random", "one_flip"):
        cnt, misses = check_against_oracle(snap, ref, 4096, kind)
        assert 2000 < cnt["ndirty"] < 3000


@pytest.mark.parametrize("nchunks", [1, 2, 1023, 1024, 1025, 2048, 4097])
def test_chunk_counts_around_the_scan_block(nchunks):
    """One scan block is 1024 chunks: plans with exactly, one fewer and one more, and a single
    chunk."""
    ref = host_bufs(60 + nchunks, [256 * (nchunks - 1) + 77])
    snap = [ref[0].copy()]
    snap[0][::512] ^= 1                                   # every second chunk differs
    for kind in ("exact", "zeros"):
        cnt, _ = check_against_oracle(snap, ref, 256, kind)
        assert cnt["ndirty"] == (nchunks + 1) // 2


def test_mask_and_hint_at_odd_addresses():
    """The mask and the hint are byte arrays with no alignment requirement; the manifest kernel
    reads them 16 bytes at a time where it can and bytewise at the ragged ends."""
    ref = host_bufs(71, [256 * 5000 + 3, 100, 256 * 300])
    snap = [b.copy() for b in ref]
    rng = np.random.default_rng(72)
    for b in snap:
        b[rng.integers(0, b.size, size=b.size // 600)] ^= 0x22
    chunk = 256
    dev = DeviceBuffers(snap, chunk)
    n = dev.plan.nchunks
    o_dig, o_ref = oracle.fingerprint(snap, chunk, 8), oracle.fingerprint(ref, chunk, 8)
    o_mask, _ = oracle.diff(snap, chunk, o_dig, o_ref)
    o_st, o_man, o_cnt = oracle.compact(snap, chunk, o_mask, o_dig)
    ref_t = torch.from_numpy(o_ref.view(np.int64)).cuda()
    dig_t = torch.from_numpy(o_dig.view(np.int64)).cuda()
    for shift in (1, 3, 15, 17):
        mask = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")[shift:shift + n]
        hint = torch.zeros(n + 64, dtype=torch.uint8, device="cuda")[shift + 4:shift + 4 + n]
        assert mask.data_ptr() % 16 == shift % 16
        hint.copy_(torch.from_numpy(o_mask).cuda())
        staging = torch.full((o_st.size + 256,), 0xA5, dtype=torch.uint8, device="cuda")
        manifest = torch.full((o_man.size * 32 + 256,), 0xA5, dtype=torch.uint8, device="cuda")
        counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
        dig = torch.zeros(n, dtype=torch.int64, device="cuda")
        misses = torch.full((1,), -1, dtype=torch.int64, device="cuda")
        ws = torch.empty(ck.snapshot_workspace_bytes(n), dtype=torch.uint8, device="cuda")
        ck.snapshot(dev.plan, ref_t, hint, dig, mask, staging, manifest, counts, misses, ws,
                    staging_cap=o_st.size, manifest_cap=o_man.size)
        torch.cuda.synchronize()
        assert np.array_equal(mask.cpu().numpy(), o_mask) and int(misses.item()) == 0
        assert counts_dict(counts) == o_cnt
        assert np.array_equal(staging.cpu().numpy()[:o_st.size], o_st)
        assert np.array_equal(ck.manifest_to_numpy(manifest, o_man.size), o_man)
        # the three-call path with the same odd mask address
        staging.fill_(0xA5)
        manifest.fill_(0xA5)
        ck.compact(dev.plan, mask, dig_t, staging, manifest, counts, staging_cap=o_st.size,
                   manifest_cap=o_man.size)
        torch.cuda.synchronize()
        assert counts_dict(counts) == o_cnt
        assert np.array_equal(staging.cpu().numpy()[:o_st.size], o_st)
        assert np.array_equal(ck.manifest_to_numpy(manifest, o_man.size), o_man)
        assert bool((staging[o_st.size:] == 0xA5).all())
