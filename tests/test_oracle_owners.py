"""Cross-worker upload ownership of the oracle (paper sec. 4.6) against its
pins; the pins themselves live in oracle_pins.py so that the mutation test can
run them against deliberately broken builds."""
import numpy as np
import pytest

import oracle
from oracle_pins import owner_pins, worker_states


def test_owner_pins_hold():
    owner_pins()


def test_rank_outside_world_is_an_error():
    states, chunk = worker_states(2, 1)
    digs = np.stack([oracle.fingerprint(st, chunk) for st in states])
    with pytest.raises(ValueError):
        oracle.upload_owners(states[0], chunk, digs, 2)
    with pytest.raises(ValueError):
        oracle.upload_owners(states[0], chunk, digs[:, :-1], 0)


def test_total_upload_shrinks_to_one_copy_plus_private_state():
    """The point of the method: with W replicas sharing P and O, the sum of uploads over all workers
    is one copy of the shared bytes plus each worker's private bytes."""
    world, chunk = 4, 256
    rng = np.random.default_rng(3)
    shared = [rng.integers(0, 256, size=n, dtype=np.uint8) for n in (4096, 1000)]
    total, lens = 0, None
    states = [shared + [rng.integers(0, 256, size=700, dtype=np.uint8)] for _ in range(world)]
    digs = np.stack([oracle.fingerprint(st, chunk) for st in states])
    for r in range(world):
        _, cnt = oracle.upload_owners(states[r], chunk, digs, r)
        total += cnt["staged_bytes"]
    pad = lambda b: sum((min(chunk, b.size - o) + 15) // 16 * 16 for o in range(0, b.size, chunk))
    assert total == sum(pad(b) for b in shared) + world * pad(states[0][2])
