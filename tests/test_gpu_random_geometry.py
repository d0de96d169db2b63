"""Seeded random buffer lists, chunk sizes, mutations, hints and capacity limits: the whole path
(fused call in both launch shapes, and the three calls, then restore) against the oracle,
element by element.  Breadth beside the hand-picked lists of the other parity tests."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import DeviceBuffers, counts_dict, run_compact, run_diff, run_fingerprint, u64
from paper_2202_07848_amd import binding as ck
from test_gpu_snapshot import check_against_oracle, fused_pass_shape  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = np.random.default_rng(1000 + seed)
    chunk = int(rng.choice([256, 512, 1024, 4096, 16384, 65536]))
    nbufs = int(rng.integers(1, 41))
    sizes = []
    for _ in range(nbufs):
        kind = rng.integers(0, 6)
        if kind == 0:
            n = 0
        elif kind == 1:
            n = int(rng.integers(1, 64))                         # shorter than two stripes
        elif kind == 2:
            n = int(rng.integers(1, 9)) * chunk                  # whole chunks only
        elif kind == 3:
            n = int(rng.integers(0, 9)) * chunk + int(rng.choice([1, 15, 16, 17, 31, 32, 33, 255,
                                                                  256, 257, chunk - 1]))
        else:
            n = int(rng.integers(1, 40 * chunk if chunk <= 4096 else 6 * chunk))
        sizes.append(n)
    ref = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in sizes]
    snap = [b.copy() for b in ref]
    style = rng.integers(0, 4)
    for i, b in enumerate(snap):
        if b.size == 0:
            continue
        if style == 0 and rng.random() < 0.4:                    # whole buffers differ
            b[:] = rng.integers(0, 256, size=b.size, dtype=np.uint8)
        elif style == 1:                                         # scattered single bytes
            for off in rng.integers(0, b.size, size=int(rng.integers(0, 4))):
                b[off] ^= 0x41
        elif style == 2 and rng.random() < 0.5:                  # a run in the middle
            lo = int(rng.integers(0, b.size))
            b[lo:lo + int(rng.integers(1, 3 * chunk))] ^= 0x99
    hint = str(rng.choice(["exact", "none", "ones", "zeros", "one_flip", "random"]))
    return chunk, ref, snap, hint, rng


@pytest.mark.parametrize("seed", range(24))
def test_random_case_against_oracle(seed):
    chunk, ref, snap, hint, rng = random_case(seed)
    n = oracle.nchunks(snap, chunk)
    if n == 0:
        hint = "none"
    # the fused call, whatever the hint
    use_ref = ref if rng.random() < 0.85 else None
    check_against_oracle(snap, use_ref, chunk, hint)
    # ... and under capacity limits every third case
    if seed % 3 == 0 and n:
        lens = oracle.chunk_lens(snap, chunk)
        check_against_oracle(snap, use_ref, chunk, "exact" if hint == "none" else hint,
                             staging_cap=int(lens.sum()) // 3, manifest_cap=max(1, n // 2))

    # the three calls and the restore
    dev = DeviceBuffers(snap, chunk)
    o_dig = oracle.fingerprint(snap, chunk, 4)
    o_ref = None if use_ref is None else oracle.fingerprint(use_ref, chunk, 4)
    o_mask, o_cnt = oracle.diff(snap, chunk, o_dig, o_ref)
    o_st, o_man, _ = oracle.compact(snap, chunk, o_mask, o_dig)
    dig = run_fingerprint(dev.plan)
    assert np.array_equal(u64(dig, n), o_dig)
    d_ref = None if o_ref is None else torch.from_numpy(
        (o_ref if o_ref.size else np.zeros(1, np.uint64)).view(np.int64)).cuda()
    mask, counts = run_diff(dev.plan, dig, d_ref)
    assert np.array_equal(mask[:n].cpu().numpy(), o_mask) and counts_dict(counts) == o_cnt
    staging, manifest, c2 = run_compact(dev.plan, mask, dig, o_st.size, o_man.size)
    assert counts_dict(c2) == o_cnt
    assert np.array_equal(staging[:o_st.size].cpu().numpy(), o_st)
    assert np.array_equal(ck.manifest_to_numpy(manifest, o_man.size), o_man)
    base = use_ref if use_ref is not None else [np.full(b.size, 0x3D, np.uint8) for b in snap]
    dst = DeviceBuffers(base, chunk)
    rejected = torch.full((1,), -1, dtype=torch.int64, device="cuda")
    ck.restore_counted(dst.plan, staging, o_st.size, manifest, max(1, o_man.size), c2, rejected)
    torch.cuda.synchronize()
    assert int(rejected.item()) == 0
    got, img = dst.host()
    assert all(np.array_equal(g, s) for g, s in zip(got, snap))
    assert dst.canaries_intact(img)
