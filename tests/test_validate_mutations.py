"""Squashing validation (paper sec. 5.2.3): mutations inferred from checksum
differences must be identical across the ranks sharing a GPU.  The oracle is
pinned by construction -- buffers are mutated at known chunks with known bytes,
so the expected verdict never comes from the formula under test -- and the GPU
kernel must agree with it exactly."""
import numpy as np
import pytest

import oracle

CHUNK = 512
SIZES = [4096, 1000, 0, 8192 + 40, 512]


def state(seed):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, 256, size=n, dtype=np.uint8) for n in SIZES]


def write(bufs, chunk_id, value):
    """Overwrite global chunk `chunk_id` with `value` bytes."""
    k = chunk_id
    for b in bufs:
        n = -(-b.size // CHUNK)
        if k < n:
            b[k * CHUNK:(k + 1) * CHUNK] = value
            return
        k -= n
    raise IndexError(chunk_id)


def chunk_of(bufs, chunk_id):
    k = chunk_id
    for b in bufs:
        n = -(-b.size // CHUNK)
        if k < n:
            return b[k * CHUNK:(k + 1) * CHUNK].copy()
        k -= n
    raise IndexError(chunk_id)


def scenario(kind):
    """Two ranks with identical P/O state before the optimizer step (the squashing
    window); returns (before_a, after_a, before_b, after_b, expected verdict)."""
    a0, b0 = state(1), state(1)
    if kind == "untouched_state_differs":                # e.g. a per-rank buffer nobody writes
        write(b0, 14, 200)
    a1, b1 = [x.copy() for x in a0], [x.copy() for x in b0]
    for k, v in ((0, 11), (9, 12), (27, 13)):          # the update every rank performs
        write(a1, k, v)
        write(b1, k, v)
    exp = {"changed_a": 3, "changed_b": 3, "mismatches": 0, "first_mismatch": 2**64 - 1}
    if kind == "b_extra_write":                          # rank b also touches chunk 5
        write(b1, 5, 99)
        exp.update(changed_b=4, mismatches=1, first_mismatch=5)
    elif kind == "different_value":                      # same address, different content
        write(b1, 9, 77)
        exp.update(mismatches=1, first_mismatch=9)
    elif kind == "a_skips_one":                          # rank a misses one of the updates
        write(a1, 27, chunk_of(a0, 27))                  # back to the old bytes
        exp.update(changed_a=2, mismatches=1, first_mismatch=27)
    elif kind == "both_wrong_twice":
        write(a1, 3, 1)
        write(b1, 3, 2)
        write(b1, 20, 5)
        exp.update(changed_a=4, changed_b=5, mismatches=2, first_mismatch=3)
    return a0, a1, b0, b1, exp


KINDS = ["identical", "b_extra_write", "different_value", "a_skips_one", "both_wrong_twice",
         "untouched_state_differs"]


@pytest.mark.parametrize("kind", KINDS)
def test_oracle_verdict_matches_construction(kind):
    a0, a1, b0, b1, exp = scenario(kind)
    digs = [oracle.fingerprint(x, CHUNK) for x in (a0, a1, b0, b1)]
    assert oracle.validate_mutations(*digs) == exp


def test_oracle_no_mutation_at_all_and_empty():
    d = oracle.fingerprint(state(2), CHUNK)
    assert oracle.validate_mutations(d, d, d, d) == {"changed_a": 0, "changed_b": 0,
                                                     "mismatches": 0,
                                                     "first_mismatch": 2**64 - 1}
    e = np.zeros(0, dtype=np.uint64)
    assert oracle.validate_mutations(e, e, e, e)["mismatches"] == 0


@pytest.mark.gpu
@pytest.mark.parametrize("kind", KINDS)
def test_gpu_verdict_equals_oracle(kind):
    import torch
    from paper_2202_07848_amd import binding as ck
    from gpu_util import DeviceBuffers, run_fingerprint

    a0, a1, b0, b1, exp = scenario(kind)
    devs = [DeviceBuffers(x, CHUNK) for x in (a0, a1, b0, b1)]
    digs = [run_fingerprint(d.plan) for d in devs]
    res = torch.full((4,), 7, dtype=torch.int64, device="cuda")
    ck.validate_mutations(devs[0].plan, *digs, res)
    torch.cuda.synchronize()
    got = dict(zip(ck.VALIDATION_FIELDS, (int(v) for v in res.cpu().numpy().view(np.uint64))))
    want = oracle.validate_mutations(*[oracle.fingerprint(x, CHUNK) for x in (a0, a1, b0, b1)])
    assert got == want == exp


@pytest.mark.gpu
def test_gpu_verdict_on_large_random_digest_arrays():
    import torch
    from paper_2202_07848_amd import binding as ck
    from gpu_util import DeviceBuffers

    n = 300_001
    rng = np.random.default_rng(5)
    host = [np.zeros(n * 256 - 7, dtype=np.uint8)]
    dev = DeviceBuffers(host, 256)
    assert dev.plan.nchunks == n
    before = rng.integers(0, 2**63, size=n, dtype=np.uint64)
    after_a = before.copy()
    touched = rng.choice(n, size=5000, replace=False)
    after_a[touched] = rng.integers(0, 2**63, size=touched.size, dtype=np.uint64)
    after_b = after_a.copy()
    odd = rng.choice(n, size=37, replace=False)
    after_b[odd] ^= np.uint64(1)
    want = oracle.validate_mutations(before, after_a, before, after_b)
    assert want["mismatches"] == 37 and want["first_mismatch"] == int(odd.min())
    t = [torch.from_numpy(x.view(np.int64)).cuda() for x in (before, after_a, before, after_b)]
    res = torch.zeros(4, dtype=torch.int64, device="cuda")
    ck.validate_mutations(dev.plan, *t, res)
    torch.cuda.synchronize()
    got = dict(zip(ck.VALIDATION_FIELDS, (int(v) for v in res.cpu().numpy().view(np.uint64))))
    assert got == want
