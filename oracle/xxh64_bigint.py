"""XXH64 on Python's unbounded integers -- TEST INFRASTRUCTURE ONLY.

A second, separately written statement of the public XXH64 definition, used
to cross-check ``ckpt_oracle.c`` on small inputs.  Every intermediate value is
an exact integer that is reduced mod 2**64 explicitly, so a missed wrap-around
or a wrong rotate in the C code shows up as a disagreement.  Slow on purpose.
"""
from __future__ import annotations

M64 = (1 << 64) - 1
PRIME = (
    None,
    0x9E3779B185EBCA87,
    0xC2B2AE3D27D4EB4F,
    0x165667B19E3779F9,
    0x85EBCA77C2B2AE63,
    0x27D4EB2F165667C5,
)
LANE_ROT = (1, 7, 12, 18)


def _rol(x: int, r: int) -> int:
    return ((x << r) & M64) | (x >> (64 - r))


def _mix(acc: int, word: int) -> int:
    return (_rol((acc + word * PRIME[2]) & M64, 31) * PRIME[1]) & M64


def xxh64(data: bytes, seed: int = 0) -> int:
    n = len(data)
    pos = 0
    if n >= 32:
        lanes = [
            (seed + PRIME[1] + PRIME[2]) & M64,
            (seed + PRIME[2]) & M64,
            seed & M64,
            (seed - PRIME[1]) & M64,
        ]
        for pos in range(0, n - n % 32, 32):
            for t in range(4):
                w = int.from_bytes(data[pos + 8 * t: pos + 8 * t + 8], "little")
                lanes[t] = _mix(lanes[t], w)
        pos = n - n % 32
        h = sum(_rol(v, r) for v, r in zip(lanes, LANE_ROT)) & M64
        for v in lanes:
            h = ((h ^ _mix(0, v)) * PRIME[1] + PRIME[4]) & M64
    else:
        h = (seed + PRIME[5]) & M64
    h = (h + n) & M64
    while n - pos >= 8:
        w = int.from_bytes(data[pos: pos + 8], "little")
        h = (_rol(h ^ _mix(0, w), 27) * PRIME[1] + PRIME[4]) & M64
        pos += 8
    if n - pos >= 4:
        w = int.from_bytes(data[pos: pos + 4], "little")
        h = (_rol(h ^ ((w * PRIME[1]) & M64), 23) * PRIME[2] + PRIME[3]) & M64
        pos += 4
    while pos < n:
        h = (_rol(h ^ ((data[pos] * PRIME[5]) & M64), 11) * PRIME[1]) & M64
        pos += 1
    h ^= h >> 33
    h = (h * PRIME[2]) & M64
    h ^= h >> 29
    h = (h * PRIME[3]) & M64
    h ^= h >> 32
    return h
