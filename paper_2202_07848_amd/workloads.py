"""Seeded synthetic training-state workloads (inputs only -- no hashing, no
diffing, no copying logic lives here).

The Singularity paper measures on real training jobs (its Table 2; two of the
models are proprietary).  These generators stand in for them: buffer lists with
the shapes of the paper's memory taxonomy (sec. 5.2.1): parameters P and
optimizer state O, identical across the data-parallel replicas that share a
GPU, gradients G and activations A, different per replica -- plus an
allocator-fragmentation case (a rank's state is spread over thousands of
buffers, sec. 5.2.1).

A workload is a list of ``BufSpec`` (size, value distribution, shared or
per-replica) and a chunk size.  It can be materialised two ways, both seeded:
``numpy_replica`` (host arrays, small cases and CPU tests) and
``torch_replica`` (one device arena per replica, full-size runs).  The two
back-ends do not produce the same bytes and do not need to: a parity test
always hands the very same bytes to both implementations under test.

Seed scheme: ``0x5EED0000 + 0x100 * config + replica`` (+ ``0x10000 * step``
for the dirty-fraction sweep); shared buffers always use replica 0's stream.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

KiB = 1024
MiB = 1024 * KiB
GiB = 1024 * MiB


@dataclass(frozen=True)
class BufSpec:
    name: str
    nbytes: int
    kind: str      # bf16_normal | f32_normal | f32_absnormal | u8_uniform | zero
    scale: float   # standard deviation for the normal kinds
    shared: bool   # True: same bytes in every replica (P and O); False: per replica (G, A)


@dataclass
class Workload:
    name: str
    config: int
    chunk: int
    nreplicas: int
    bufs: List[BufSpec] = field(default_factory=list)
    place_shuffled: bool = False   # arena placement order differs from list order

    @property
    def nbytes(self) -> int:
        return sum(b.nbytes for b in self.bufs)

    @property
    def nchunks(self) -> int:
        return sum(-(-b.nbytes // self.chunk) for b in self.bufs)

    @property
    def distinct_bytes(self) -> int:
        return sum(b.nbytes for b in self.bufs if not b.shared)

    @property
    def distinct_chunks(self) -> int:
        return sum(-(-b.nbytes // self.chunk) for b in self.bufs if not b.shared)

    def seed(self, replica: int, step: int = 0) -> int:
        return 0x5EED0000 + 0x100 * self.config + replica + 0x10000 * step


def _round512(x: float) -> int:
    return max(512, int(round(x / 512.0)) * 512)


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

def tiny_spliced_pair(total: int = 64 * MiB, nbufs: int = 16, ndistinct: int = 4,
                      chunk: int = 4 * KiB) -> Workload:
    """Config 1: two replicas, 16 buffers, log-uniform 256 KiB - 8 MiB."""
    w = Workload("tiny_spliced_pair", 1, chunk, 2)
    rng = np.random.default_rng(w.seed(0) ^ 0xC0FFEE)
    lo, hi = 256 * KiB * total / (64 * MiB), 8 * MiB * total / (64 * MiB)
    raw = lo * (hi / lo) ** rng.random(nbufs)
    raw = np.clip(raw * (total / raw.sum()), lo, hi)
    sizes = [_round512(x) for x in raw]
    sizes[-1] = max(512, total - sum(sizes[:-1]))
    distinct = set(rng.choice(nbufs, size=ndistinct, replace=False).tolist())
    for i, s in enumerate(sizes):
        if i in distinct:
            w.bufs.append(BufSpec(f"distinct{i}", s, "u8_uniform", 0.0, False))
        else:
            w.bufs.append(BufSpec(f"same{i}", s, "bf16_normal", 0.02, True))
    return w


def _gpt_tensor_shapes(layers: int, d: int, vocab: int, ctx: int) -> List[Tuple[str, int]]:
    """Per-tensor element counts of a GPT-2-style decoder (tied embedding)."""
    t = [("wte", vocab * d), ("wpe", ctx * d)]
    for l in range(layers):
        t += [(f"h{l}.ln_1.w", d), (f"h{l}.ln_1.b", d),
              (f"h{l}.attn.qkv.w", d * 3 * d), (f"h{l}.attn.qkv.b", 3 * d),
              (f"h{l}.attn.proj.w", d * d), (f"h{l}.attn.proj.b", d),
              (f"h{l}.ln_2.w", d), (f"h{l}.ln_2.b", d),
              (f"h{l}.mlp.fc.w", d * 4 * d), (f"h{l}.mlp.fc.b", 4 * d),
              (f"h{l}.mlp.proj.w", 4 * d * d), (f"h{l}.mlp.proj.b", d)]
    t += [("ln_f.w", d), ("ln_f.b", d)]
    return t


def gpt_replica_state(name: str, config: int, layers: int, d: int, vocab: int, ctx: int,
                      act_bytes: int, act_bufs: int, chunk: int, nreplicas: int) -> Workload:
    """Mixed-precision Adam training state of one data-parallel replica.

    Per tensor: bf16 parameter, fp32 master copy, fp32 Adam m and v (all four
    identical across replicas), bf16 gradient (per replica).  Then ``act_bufs``
    activation buffers of ``act_bytes / act_bufs`` bytes (per replica)."""
    w = Workload(name, config, chunk, nreplicas)
    for tname, n in _gpt_tensor_shapes(layers, d, vocab, ctx):
        w.bufs.append(BufSpec(tname + ".param", 2 * n, "bf16_normal", 0.02, True))
        w.bufs.append(BufSpec(tname + ".master", 4 * n, "f32_normal", 0.02, True))
        w.bufs.append(BufSpec(tname + ".adam_m", 4 * n, "f32_normal", 1e-3, True))
        w.bufs.append(BufSpec(tname + ".adam_v", 4 * n, "f32_absnormal", 1e-6, True))
        w.bufs.append(BufSpec(tname + ".grad", 2 * n, "bf16_normal", 1e-3, False))
    per = act_bytes // act_bufs
    for a in range(act_bufs):
        w.bufs.append(BufSpec(f"act{a}", per, "bf16_normal", 1.0, False))
    return w


def gpt2_small_pair(shrink: int = 1) -> Workload:
    """Config 2: GPT-2-small-shaped state x2, 1 GiB activations, 64 KiB chunks.
    ``shrink`` > 1 divides depth, vocabulary and activation size for CPU tests
    (d stays 768 so the many small bias/LayerNorm tensors keep their sizes)."""
    return gpt_replica_state("gpt2_small_pair", 2, max(1, 12 // shrink), 768,
                             50257 // shrink, 1024, GiB // (shrink * shrink), 1, 64 * KiB, 2)


def fragmented_allocator(nbufs: int = 100_000, chunk: int = 4 * KiB,
                         zero_fraction: float = 0.2) -> Workload:
    """Config 3: many buffers, sizes 512 B * 4096**u, 20 % all-zero; one
    replica, diffed against its own earlier snapshot."""
    w = Workload("fragmented_allocator", 3, chunk, 1, place_shuffled=True)
    rng = np.random.default_rng(w.seed(0) ^ 0xF4A6)
    sizes = 512.0 * 4096.0 ** rng.random(nbufs)
    zero = rng.random(nbufs) < zero_fraction
    for i in range(nbufs):
        kind = "zero" if zero[i] else "u8_uniform"
        w.bufs.append(BufSpec(f"blk{i}", _round512(sizes[i]), kind, 0.0, False))
    return w


def gpt_1p3b_x4(shrink: int = 1) -> Workload:
    """Config 4: 1.3 B parameters, four replicas on one GPU, 8 GiB activations
    each (64 x 128 MiB), 256 KiB chunks."""
    return gpt_replica_state("gpt_1p3b_x4", 4, max(1, 24 // shrink), 2048 // shrink,
                             50257 // shrink, 2048 // shrink, 8 * GiB // (shrink ** 3),
                             64 // min(shrink, 16), 256 * KiB, 4)


def gpt_3b_x2(shrink: int = 1) -> Workload:
    """Config 5: 3 B parameters (36 layers, d = 2560, context 4096), two
    replicas, 16 GiB activations each (128 x 128 MiB), 1 MiB chunks."""
    return gpt_replica_state("gpt_3b_x2", 5, max(1, 36 // shrink), 2560 // shrink,
                             50257 // shrink, 4096 // shrink, 16 * GiB // (shrink ** 3),
                             128 // min(shrink, 16), 1 * MiB, 2)


def config(index: int, shrink: int = 1) -> Workload:
    """Workload ``index`` (1-5).  ``shrink`` > 1 gives a reduced version with
    the same structure for CPU-sized runs."""
    if index == 1:
        return tiny_spliced_pair(total=64 * MiB // (shrink if shrink > 1 else 1))
    if index == 2:
        return gpt2_small_pair(shrink)
    if index == 3:
        return fragmented_allocator(nbufs=max(16, 100_000 // shrink))
    if index == 4:
        return gpt_1p3b_x4(shrink)
    if index == 5:
        return gpt_3b_x2(shrink)
    raise ValueError("config index must be 1..5")


# --------------------------------------------------------------------------
# host materialisation (NumPy)
# --------------------------------------------------------------------------

def _np_fill(spec: BufSpec, rng: np.random.Generator) -> np.ndarray:
    n = spec.nbytes
    if spec.kind == "zero":
        return np.zeros(n, dtype=np.uint8)
    if spec.kind == "u8_uniform":
        return rng.integers(0, 256, size=n, dtype=np.uint8)
    if spec.kind == "bf16_normal":
        f = (rng.standard_normal(n // 2, dtype=np.float32) * np.float32(spec.scale))
        u = (f.view(np.uint32) + np.uint32(0x8000)) >> np.uint32(16)
        out = np.zeros(n, dtype=np.uint8)
        out[: 2 * (n // 2)] = u.astype(np.uint16).view(np.uint8)
        return out
    if spec.kind in ("f32_normal", "f32_absnormal"):
        f = (rng.standard_normal(n // 4, dtype=np.float32) * np.float32(spec.scale))
        if spec.kind == "f32_absnormal":
            f = np.abs(f)
        out = np.zeros(n, dtype=np.uint8)
        out[: 4 * (n // 4)] = f.view(np.uint8)
        return out
    raise ValueError(spec.kind)


def numpy_replica(w: Workload, replica: int) -> List[np.ndarray]:
    """Host bytes of one replica: a list of uint8 arrays in buffer-list order."""
    out = []
    for i, spec in enumerate(w.bufs):
        seed = w.seed(0 if spec.shared else replica)
        out.append(_np_fill(spec, np.random.default_rng([seed, i])))
    return out


def dirty_chunk_ids(w: Workload, fraction: float, step: int) -> np.ndarray:
    """Exactly round(fraction * N) distinct global chunk ids, seeded, sorted."""
    n = w.nchunks
    k = int(round(fraction * n))
    rng = np.random.default_rng(w.seed(0, step) ^ 0xD1)
    return np.sort(rng.permutation(n)[:k]).astype(np.int64)


def chunk_table(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(buffer index, offset in buffer, length) of every chunk, global order."""
    counts = np.array([-(-b.nbytes // w.chunk) for b in w.bufs], dtype=np.int64)
    buf = np.repeat(np.arange(len(w.bufs), dtype=np.int64), counts)
    first = np.concatenate([[0], np.cumsum(counts)[:-1]])
    j = np.arange(counts.sum(), dtype=np.int64) - np.repeat(first, counts)
    off = j * w.chunk
    sizes = np.array([b.nbytes for b in w.bufs], dtype=np.int64)
    length = np.minimum(w.chunk, sizes[buf] - off)
    return buf, off, length


def numpy_rewrite_chunks(w: Workload, bufs: Sequence[np.ndarray], ids: np.ndarray,
                         step: int) -> None:
    """Overwrite the chunks ``ids`` with fresh uniform bytes, in place."""
    buf, off, length = chunk_table(w)
    rng = np.random.default_rng(w.seed(0, step) ^ 0xD2)
    for k in ids.tolist():
        b, o, n = int(buf[k]), int(off[k]), int(length[k])
        old = bufs[b][o:o + n].copy()
        new = rng.integers(0, 256, size=n, dtype=np.uint8)
        if np.array_equal(old, new):       # must really differ
            new[0] ^= 0xFF
        bufs[b][o:o + n] = new


# --------------------------------------------------------------------------
# device materialisation (PyTorch, one arena per replica)
# --------------------------------------------------------------------------

def arena_layout(w: Workload, align: int = 256) -> Tuple[np.ndarray, int]:
    """Byte offset of every buffer inside a replica's arena.  With
    ``place_shuffled`` the placement order is a seeded permutation of the list
    order, so neighbours in the list are not neighbours in memory."""
    n = len(w.bufs)
    order = np.arange(n)
    if w.place_shuffled:
        order = np.random.default_rng(w.seed(0) ^ 0xA11).permutation(n)
    sizes = np.array([b.nbytes for b in w.bufs], dtype=np.int64)
    padded = (sizes + align - 1) // align * align
    offs = np.zeros(n, dtype=np.int64)
    offs[order] = np.concatenate([[0], np.cumsum(padded[order])[:-1]])
    return offs, int(padded.sum())


def torch_replica(w: Workload, replica: int, device, shared_from=None):
    """Fill one replica's arena on ``device``.

    Returns (arena uint8 tensor, offsets).  Buffers marked shared are copied
    from ``shared_from`` (another replica's arena with the same layout) when it
    is given, otherwise generated from replica 0's seed."""
    import torch

    offs, total = arena_layout(w)
    arena = torch.empty(total, dtype=torch.uint8, device=device)
    gen = torch.Generator(device=device)

    if all(b.kind in ("zero", "u8_uniform") for b in w.bufs):
        # allocator-fragmentation case: one pass of random bytes, then zero the
        # all-zero buffers (100k tiny per-buffer fills would take minutes)
        gen.manual_seed(w.seed(replica))
        step = 1 << 30
        for lo in range(0, total, step):
            hi = min(total, lo + step)
            arena[lo:hi] = torch.randint(0, 256, (hi - lo,), dtype=torch.uint8, device=device,
                                         generator=gen)
        zoff = [int(offs[i]) for i, b in enumerate(w.bufs) if b.kind == "zero"]
        zlen = [b.nbytes for b in w.bufs if b.kind == "zero"]
        _torch_fill_ranges(arena, zoff, zlen, None, gen)
        return arena, offs

    for i, spec in enumerate(w.bufs):
        o, n = int(offs[i]), spec.nbytes
        dst = arena[o:o + n]
        if spec.shared and shared_from is not None:
            dst.copy_(shared_from[o:o + n])
            continue
        gen.manual_seed((w.seed(0 if spec.shared else replica) * 1_000_003 + i) % (1 << 63))
        if spec.kind == "zero":
            dst.zero_()
        elif spec.kind == "u8_uniform":
            dst.copy_(torch.randint(0, 256, (n,), dtype=torch.uint8, device=device, generator=gen))
        elif spec.kind == "bf16_normal":
            t = torch.randn(n // 2, dtype=torch.float32, device=device, generator=gen)
            dst[: 2 * (n // 2)].copy_((t * spec.scale).to(torch.bfloat16).view(torch.uint8))
        else:
            t = torch.randn(n // 4, dtype=torch.float32, device=device, generator=gen) * spec.scale
            if spec.kind == "f32_absnormal":
                t = t.abs()
            dst[: 4 * (n // 4)].copy_(t.view(torch.uint8))
    return arena, offs


def _torch_fill_ranges(arena, offsets, lengths, seed: Optional[int], gen) -> None:
    """Zero (seed None) or re-randomise the byte ranges, in 256-byte granules
    (every offset and length here is a multiple of 256)."""
    import torch

    if not offsets:
        return
    g = 256
    off = torch.tensor(offsets, dtype=torch.int64) // g
    cnt = torch.tensor(lengths, dtype=torch.int64) // g
    if int((torch.tensor(lengths, dtype=torch.int64) % g).sum()) or \
            int((torch.tensor(offsets, dtype=torch.int64) % g).sum()):
        raise ValueError("ranges must be multiples of 256 bytes")
    view = arena[: arena.numel() // g * g].view(-1, g)
    batch = 1 << 20   # granules per pass, bounds the temporary index/random tensors
    start = torch.repeat_interleave(off, cnt)
    first = torch.repeat_interleave(torch.cumsum(cnt, 0) - cnt, cnt)
    idx = (start + torch.arange(start.numel(), dtype=torch.int64) - first)
    if seed is not None:
        gen.manual_seed(seed)
    for lo in range(0, idx.numel(), batch):
        sel = idx[lo:lo + batch].to(arena.device)
        if seed is None:
            view[sel] = 0
        else:
            view[sel] = torch.randint(0, 256, (sel.numel(), g), dtype=torch.uint8,
                                      device=arena.device, generator=gen)


def torch_rewrite_chunks(w: Workload, arena, offs: np.ndarray, ids: np.ndarray,
                         step: int) -> None:
    """Device version of ``numpy_rewrite_chunks`` (fresh uniform bytes; a
    rewritten chunk equals its old content with probability 256**-len)."""
    import torch

    buf, off, length = chunk_table(w)
    a = (offs[buf[ids]] + off[ids]).tolist()
    n = length[ids].tolist()
    gen = torch.Generator(device=arena.device)
    _torch_fill_ranges(arena, a, n, w.seed(0, step) ^ 0xD2, gen)


def describe(w: Workload) -> dict:
    return {"name": w.name, "config": w.config, "chunk": w.chunk, "replicas": w.nreplicas,
            "buffers": len(w.bufs), "bytes_per_replica": w.nbytes, "chunks": w.nchunks,
            "distinct_bytes": w.distinct_bytes,
            "distinct_fraction": w.distinct_bytes / max(1, w.nbytes)}


if __name__ == "__main__":
    for c in range(1, 6):
        d = describe(config(c))
        print(d)
