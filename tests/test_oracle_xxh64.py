"""Pins of the oracle's XXH64 to things other than itself: the stored vectors
of the public function (tests/golden), the installed xxHash library, a
separately written big-integer implementation, and structural properties."""
import os

import numpy as np
import pytest

import oracle
from oracle import xxh64_bigint

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden",
                      "xxh64_seed0_vectors.txt")


def pattern(n):
    i = np.arange(n, dtype=np.uint64)
    return (((i * np.uint64(2654435761)) & np.uint64(0xFFFFFFFF)) >> np.uint64(24)).astype(
        np.uint8).tobytes()


def golden_vectors():
    out = []
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            kind, arg, dig = line.split()
            if kind == "pat":
                data = pattern(int(arg))
            elif kind == "zeros":
                data = bytes(int(arg))
            else:
                data = arg.encode()
            out.append((f"{kind}-{arg}", data, int(dig, 16)))
    return out


VECTORS = golden_vectors()


def test_golden_file_covers_every_branch():
    lens = {len(d) for _, d, _ in VECTORS}
    assert 0 in lens and any(0 < n < 4 for n in lens) and any(4 <= n < 8 for n in lens)
    assert any(8 <= n < 32 for n in lens) and 32 in lens
    assert any(n > 32 and n % 32 == 31 for n in lens)
    for c in (4096, 65536, 262144, 1048576):
        assert c in lens


@pytest.mark.parametrize("name,data,want", VECTORS, ids=[v[0] for v in VECTORS])
def test_oracle_matches_published_vectors(name, data, want):
    assert oracle.xxh64(data) == want


@pytest.mark.parametrize("name,data,want", [v for v in VECTORS if len(v[1]) <= 4096],
                         ids=[v[0] for v in VECTORS if len(v[1]) <= 4096])
def test_bigint_matches_published_vectors(name, data, want):
    assert xxh64_bigint.xxh64(data) == want


def test_oracle_matches_bigint_on_every_short_length():
    rng = np.random.default_rng(7)
    for n in range(0, 300):
        data = rng.integers(0, 256, size=n, dtype=np.uint8).tobytes()
        assert oracle.xxh64(data) == xxh64_bigint.xxh64(data), n


def test_oracle_matches_bigint_with_seed():
    rng = np.random.default_rng(8)
    for n in (0, 5, 31, 32, 100, 1000):
        data = rng.integers(0, 256, size=n, dtype=np.uint8).tobytes()
        for seed in (1, 0x9E3779B185EBCA87, (1 << 64) - 1):
            assert oracle.xxh64(data, seed) == xxh64_bigint.xxh64(data, seed)


def test_oracle_matches_installed_library():
    xxhash = pytest.importorskip("xxhash")
    rng = np.random.default_rng(9)
    big = rng.integers(0, 256, size=1 << 20, dtype=np.uint8)
    for n in list(range(0, 4098)) + [65536, 262144, 1 << 20]:
        start = int(rng.integers(0, big.size - n + 1))
        data = big[start:start + n].tobytes()
        assert oracle.xxh64(data) == xxhash.xxh64_intdigest(data, 0), n


def test_word_order_and_lane_order_matter():
    """Swapping two 8-byte words (a transposed lane) or two stripes changes the digest."""
    rng = np.random.default_rng(10)
    base = rng.integers(0, 256, size=128, dtype=np.uint8)
    h0 = oracle.xxh64(base.tobytes())
    swapped_words = base.copy()
    swapped_words[0:8], swapped_words[8:16] = base[8:16], base[0:8]
    swapped_stripes = base.copy()
    swapped_stripes[0:32], swapped_stripes[32:64] = base[32:64], base[0:32]
    assert oracle.xxh64(swapped_words.tobytes()) != h0
    assert oracle.xxh64(swapped_stripes.tobytes()) != h0


def test_every_single_bit_flip_changes_digest():
    rng = np.random.default_rng(11)
    for n in (1, 7, 33, 100):
        base = rng.integers(0, 256, size=n, dtype=np.uint8)
        h0 = oracle.xxh64(base.tobytes())
        for byte in range(n):
            for bit in range(8):
                x = base.copy()
                x[byte] ^= 1 << bit
                assert oracle.xxh64(x.tobytes()) != h0


def test_length_is_hashed_not_padded():
    """A short chunk and the same bytes zero-padded hash differently."""
    for n in (1, 31, 32, 100, 4000):
        data = pattern(n)
        assert oracle.xxh64(data) != oracle.xxh64(data + b"\0")
        assert oracle.xxh64(data) != oracle.xxh64(data + bytes(4096 - n if n < 4096 else 1))
