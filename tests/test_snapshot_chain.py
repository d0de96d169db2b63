"""Incremental snapshot chains (paper sec. 4.6: successive checkpoints of one
process mostly coincide, so later ones are deltas against the previous): a full
snapshot followed by deltas, each diffed against the digests of the one before,
restores to the latest state when the manifests are applied in order.  Oracle
first (CPU), then the same chain on the GPU compared with it step by step."""
import numpy as np
import pytest

import oracle

CHUNK = 4096          # host-page granularity
SIZES = [40000, 4096, 123457, 0, 8192, 70001]


def evolve(rng, state, nwrites):
    new = [b.copy() for b in state]
    for _ in range(nwrites):
        i = int(rng.choice([k for k, b in enumerate(new) if b.size]))
        off = int(rng.integers(0, new[i].size))
        new[i][off:off + int(rng.integers(1, 3000))] ^= 0x6B
    return new


def make_chain(seed, steps=4):
    rng = np.random.default_rng(seed)
    states = [[rng.integers(0, 256, size=n, dtype=np.uint8) for n in SIZES]]
    for s in range(steps):
        states.append(evolve(rng, states[-1], 3 + 2 * s))
    return states


def oracle_chain(states):
    out, prev = [], None
    for st in states:
        dig = oracle.fingerprint(st, CHUNK)
        mask, cnt = oracle.diff(st, CHUNK, dig, prev)
        staging, man, _ = oracle.compact(st, CHUNK, mask, dig)
        out.append((dig, mask, staging, man))
        prev = dig
    return out


def test_oracle_chain_restores_latest_state_and_deltas_are_small():
    states = make_chain(1)
    chain = oracle_chain(states)
    assert chain[0][1].all()                                  # first snapshot: everything
    full = chain[0][2].size
    for dig, mask, staging, man in chain[1:]:
        assert 0 < mask.sum() < mask.size // 2 and staging.size < full // 2
    dst = [np.zeros(n, dtype=np.uint8) for n in SIZES]
    for upto, (_, _, staging, man) in enumerate(chain):
        assert oracle.restore(dst, CHUNK, staging, man) == 0
        assert all(np.array_equal(d, s) for d, s in zip(dst, states[upto]))
    # a delta applied to the wrong base does not give the right state
    wrong = [np.zeros(n, dtype=np.uint8) for n in SIZES]
    assert oracle.restore(wrong, CHUNK, chain[2][2], chain[2][3]) == 0
    assert not all(np.array_equal(d, s) for d, s in zip(wrong, states[2]))


@pytest.mark.gpu
def test_gpu_chain_matches_oracle_step_by_step():
    import torch
    from paper_2202_07848_amd import binding as ck
    from gpu_util import DeviceBuffers, counts_dict, run_compact, run_diff, run_fingerprint, u64

    states = make_chain(2)
    chain = oracle_chain(states)
    dst = DeviceBuffers([np.zeros(n, dtype=np.uint8) for n in SIZES], CHUNK)
    prev = None
    for upto, (st, (o_dig, o_mask, o_staging, o_man)) in enumerate(zip(states, chain)):
        dev = DeviceBuffers(st, CHUNK)
        n = dev.plan.nchunks
        dig = run_fingerprint(dev.plan)
        mask, counts = run_diff(dev.plan, dig, prev)
        assert np.array_equal(u64(dig, n), o_dig) and np.array_equal(mask[:n].cpu().numpy(), o_mask)
        c = counts_dict(counts)
        staging, manifest, _ = run_compact(dev.plan, mask, dig, c["staged_bytes"], c["ndirty"])
        assert np.array_equal(staging.cpu().numpy()[:o_staging.size], o_staging)
        assert np.array_equal(ck.manifest_to_numpy(manifest, c["ndirty"]), o_man)
        ck.restore(dst.plan, staging, c["staged_bytes"], manifest, c["ndirty"])
        torch.cuda.synchronize()
        got, img = dst.host()
        assert all(np.array_equal(g, s) for g, s in zip(got, st))
        assert dst.canaries_intact(img)
        prev = dig
