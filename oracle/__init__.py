"""CPU oracle for the device-state snapshot path -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline
leg may import this package.  The product (``paper_2202_07848_amd``) never
does, and this package never imports the product.

The arithmetic lives in ``ckpt_oracle.c`` (plain C, built with gcc into
``libckpt_oracle.so`` next to it).  This module only marshals NumPy arrays
into that library: every function takes a list of ``uint8`` arrays (one per
live buffer, list order = global chunk order) and the chunk size.

Operation names follow the Singularity paper: content checksums of live
buffers and their comparison (sec. 5.2.1, sec. 6), swap-out of what is not
de-duplicated (sec. 5.2.1, sec. 4.6) and restore to the same addresses
(sec. 4.5).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ckpt_oracle.c")
_LIB = os.path.join(_HERE, "libckpt_oracle.so")

ENTRY_DTYPE = np.dtype(
    [("buf", "<u4"), ("len", "<u4"), ("buf_off", "<u8"), ("stage_off", "<u8"), ("digest", "<u8")]
)
assert ENTRY_DTYPE.itemsize == 32


class _Buf(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("nbytes", ctypes.c_uint64)]


class _Link(ctypes.Structure):
    _fields_ = [("staging", ctypes.c_void_p), ("staging_bytes", ctypes.c_uint64),
                ("manifest", ctypes.c_void_p), ("nentries", ctypes.c_uint64)]


class _Counts(ctypes.Structure):
    _fields_ = [("ndirty", ctypes.c_uint64), ("staged_bytes", ctypes.c_uint64),
                ("overflow", ctypes.c_uint64)]


def build(force: bool = False) -> str:
    """Compile ckpt_oracle.c with gcc.  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        # built under a private name and renamed into place, so that a process loading the
        # library while another one rebuilds it never sees a half-written file
        tmp = "%s.%d.tmp" % (_LIB, os.getpid())
        cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fPIC", "-shared", "-pthread",
               _SRC, "-o", tmp]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, vp = ctypes.c_uint64, ctypes.c_void_p
        lib.ora_xxh64.restype = u64
        lib.ora_xxh64.argtypes = [vp, u64, u64]
        lib.ora_nchunks.restype = u64
        lib.ora_nchunks.argtypes = [vp, u64, u64]
        lib.ora_chunk_lens.restype = None
        lib.ora_chunk_lens.argtypes = [vp, u64, u64, vp]
        lib.ora_fingerprint.restype = ctypes.c_int
        lib.ora_fingerprint.argtypes = [vp, u64, u64, vp, ctypes.c_int]
        lib.ora_diff.restype = None
        lib.ora_diff.argtypes = [vp, u64, u64, vp, vp, vp, vp]
        lib.ora_compact.restype = None
        lib.ora_compact.argtypes = [vp, u64, u64, vp, vp, vp, u64, vp, u64, vp]
        lib.ora_match.restype = ctypes.c_int
        lib.ora_match.argtypes = [vp, u64, u64, vp, vp, u64, vp, vp, vp]
        lib.ora_apply_matches.restype = u64
        lib.ora_apply_matches.argtypes = [vp, u64, vp, u64, u64, vp]
        lib.ora_validate_mutations.restype = None
        lib.ora_validate_mutations.argtypes = [u64, vp, vp, vp, vp, vp]
        lib.ora_upload_owners.restype = ctypes.c_int
        lib.ora_upload_owners.argtypes = [vp, u64, u64, vp, ctypes.c_uint32, ctypes.c_uint32, vp, vp]
        lib.ora_restore.restype = ctypes.c_uint64
        lib.ora_restore.argtypes = [vp, u64, u64, vp, u64, vp, u64]
        lib.ora_restore_chain.restype = ctypes.c_int
        lib.ora_restore_chain.argtypes = [vp, u64, u64, vp, u64, vp, vp]
        lib.ora_marks_from_buffers.restype = None
        lib.ora_marks_from_buffers.argtypes = [vp, u64, u64, vp, vp]
        lib.ora_mask_andnot.restype = None
        lib.ora_mask_andnot.argtypes = [u64, vp, vp, vp]
        lib.ora_buffer_verdicts.restype = None
        lib.ora_buffer_verdicts.argtypes = [vp, u64, u64, vp, vp, vp]
        lib.ora_merge_chain.restype = ctypes.c_int
        lib.ora_merge_chain.argtypes = [vp, u64, u64, vp, u64, vp, u64, vp, u64, vp, vp]
        _lib = lib
    return _lib


def _desc(bufs: Sequence[np.ndarray]):
    """ctypes descriptor array over a list of contiguous uint8 arrays."""
    arr = (_Buf * max(1, len(bufs)))()
    for i, b in enumerate(bufs):
        if b.dtype != np.uint8 or not b.flags["C_CONTIGUOUS"] or b.ndim != 1:
            raise TypeError("oracle buffers must be 1-D contiguous uint8 arrays")
        arr[i].ptr = b.ctypes.data if b.size else None
        arr[i].nbytes = b.size
    return arr


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def xxh64(data: bytes | np.ndarray, seed: int = 0) -> int:
    """XXH64 of a byte string."""
    a = np.frombuffer(bytes(data), dtype=np.uint8) if not isinstance(data, np.ndarray) else data
    a = np.ascontiguousarray(a.view(np.uint8).reshape(-1))
    return int(_load().ora_xxh64(_p(a) if a.size else None, a.size, seed))


def nchunks(bufs: Sequence[np.ndarray], chunk: int) -> int:
    return int(_load().ora_nchunks(_desc(bufs), len(bufs), chunk))


def chunk_lens(bufs: Sequence[np.ndarray], chunk: int) -> np.ndarray:
    n = nchunks(bufs, chunk)
    lens = np.zeros(n, dtype=np.uint32)
    _load().ora_chunk_lens(_desc(bufs), len(bufs), chunk, _p(lens))
    return lens


def fingerprint(bufs: Sequence[np.ndarray], chunk: int, nthreads: int = 1) -> np.ndarray:
    """dig[k] = XXH64(chunk k, seed 0) for every chunk in global order."""
    n = nchunks(bufs, chunk)
    dig = np.zeros(n, dtype=np.uint64)
    rc = _load().ora_fingerprint(_desc(bufs), len(bufs), chunk, _p(dig), int(nthreads))
    if rc != 0:
        raise RuntimeError("oracle: could not start worker threads")
    return dig


def diff(bufs: Sequence[np.ndarray], chunk: int, dig: np.ndarray,
         ref: Optional[np.ndarray]) -> Tuple[np.ndarray, dict]:
    """Positional comparison of checksums; ref=None marks every chunk."""
    n = nchunks(bufs, chunk)
    dig = np.ascontiguousarray(dig, dtype=np.uint64)
    if dig.size != n:
        raise ValueError("digest count does not match the buffer list")
    if ref is not None:
        ref = np.ascontiguousarray(ref, dtype=np.uint64)
        if ref.size != n:
            raise ValueError("reference has a different chunk geometry")
    mask = np.zeros(n, dtype=np.uint8)
    c = _Counts()
    _load().ora_diff(_desc(bufs), len(bufs), chunk, _p(dig), _p(ref), _p(mask), ctypes.byref(c))
    return mask, {"ndirty": c.ndirty, "staged_bytes": c.staged_bytes, "overflow": c.overflow}


def compact(bufs: Sequence[np.ndarray], chunk: int, mask: np.ndarray, dig: np.ndarray,
            staging_cap: Optional[int] = None, manifest_cap: Optional[int] = None,
            fill: int = 0xA5) -> Tuple[np.ndarray, np.ndarray, dict]:
    """Gather the marked chunks.  Returns (staging[staging_cap], manifest[manifest_cap],
    counts).  Bytes / entries the call does not write keep the ``fill`` pattern."""
    n = nchunks(bufs, chunk)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    dig = np.ascontiguousarray(dig, dtype=np.uint64)
    if mask.size != n or dig.size != n:
        raise ValueError("mask/digest count does not match the buffer list")
    lens = chunk_lens(bufs, chunk).astype(np.uint64)
    need = int((((lens + 15) // 16) * 16)[mask != 0].sum())
    if staging_cap is None:
        staging_cap = need
    if manifest_cap is None:
        manifest_cap = int((mask != 0).sum())
    staging = np.full(staging_cap, fill, dtype=np.uint8)
    manifest = np.frombuffer(bytes([fill]) * (32 * manifest_cap), dtype=ENTRY_DTYPE).copy()
    c = _Counts()
    _load().ora_compact(_desc(bufs), len(bufs), chunk, _p(mask), _p(dig), _p(staging),
                        staging_cap, _p(manifest), manifest_cap, ctypes.byref(c))
    return staging, manifest, {"ndirty": c.ndirty, "staged_bytes": c.staged_bytes,
                               "overflow": c.overflow}


class _MatchCounts(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in
                ("nsame", "nmoved", "ndup", "nnew", "staged_bytes", "table_full")]


def match(bufs: Sequence[np.ndarray], chunk: int, dig: np.ndarray,
          ref: np.ndarray) -> Tuple[np.ndarray, np.ndarray, dict]:
    """Content-addressed lookup of every snapshot checksum in the reference's
    checksums (any geometry).  Returns (src int64[N], mask uint8[N], counts)."""
    n = nchunks(bufs, chunk)
    dig = np.ascontiguousarray(dig, dtype=np.uint64)
    ref = np.ascontiguousarray(ref, dtype=np.uint64)
    if dig.size != n:
        raise ValueError("digest count does not match the buffer list")
    src = np.zeros(n, dtype=np.int64)
    mask = np.zeros(n, dtype=np.uint8)
    c = _MatchCounts()
    rc = _load().ora_match(_desc(bufs), len(bufs), chunk, _p(dig), _p(ref), ref.size, _p(src),
                           _p(mask), ctypes.byref(c))
    if rc != 0:
        raise MemoryError("oracle: match scratch allocation failed")
    return src, mask, {f: int(getattr(c, f)) for f, _ in _MatchCounts._fields_}


def apply_matches(dst: List[np.ndarray], ref: Sequence[np.ndarray], chunk: int,
                  src: np.ndarray) -> int:
    """Copies matched chunks from ``ref`` and duplicates from ``dst`` itself
    into ``dst`` (in place).  Returns the number of chunks skipped."""
    src = np.ascontiguousarray(src, dtype=np.int64)
    if src.size != nchunks(dst, chunk):
        raise ValueError("src length does not match the destination geometry")
    return int(_load().ora_apply_matches(_desc(dst), len(dst), _desc(ref), len(ref), chunk,
                                         _p(src)))


def validate_mutations(before_a, after_a, before_b, after_b) -> dict:
    """Squashing validation over four checksum arrays of one geometry."""
    arrs = [np.ascontiguousarray(x, dtype=np.uint64) for x in (before_a, after_a, before_b, after_b)]
    if len({a.size for a in arrs}) != 1:
        raise ValueError("the four checksum arrays must have one length")
    res = np.zeros(4, dtype=np.uint64)
    _load().ora_validate_mutations(arrs[0].size, *[_p(a) for a in arrs], _p(res))
    return {"changed_a": int(res[0]), "changed_b": int(res[1]), "mismatches": int(res[2]),
            "first_mismatch": int(res[3])}


def upload_owners(bufs: Sequence[np.ndarray], chunk: int, gathered: np.ndarray,
                  rank: int) -> Tuple[np.ndarray, dict]:
    """Which chunks worker ``rank`` uploads, from the checksums of all workers
    (``gathered`` has shape (world, N)).  Returns (mask[N], counts)."""
    n = nchunks(bufs, chunk)
    gathered = np.ascontiguousarray(gathered, dtype=np.uint64)
    if gathered.ndim != 2 or gathered.shape[1] != n:
        raise ValueError("gathered checksums must have shape (world, N)")
    mask = np.zeros(n, dtype=np.uint8)
    c = _Counts()
    rc = _load().ora_upload_owners(_desc(bufs), len(bufs), chunk, _p(gathered), gathered.shape[0],
                                   rank, _p(mask), ctypes.byref(c))
    if rc != 0:
        raise ValueError("rank outside the world")
    return mask, {"ndirty": c.ndirty, "staged_bytes": c.staged_bytes, "overflow": c.overflow}


def restore(dst: List[np.ndarray], chunk: int, staging: np.ndarray, manifest: np.ndarray,
            staging_bytes: Optional[int] = None) -> int:
    """Scatter staging back into ``dst`` (modified in place).  Returns the
    number of entries skipped because they do not fit ``dst`` or staging."""
    staging = np.ascontiguousarray(staging, dtype=np.uint8)
    manifest = np.ascontiguousarray(manifest, dtype=ENTRY_DTYPE)
    if staging_bytes is None:
        staging_bytes = staging.size
    for b in dst:
        if not b.flags["WRITEABLE"]:
            raise TypeError("destination buffers must be writable")
    return int(_load().ora_restore(_desc(dst), len(dst), chunk, _p(staging), staging_bytes,
                                   _p(manifest), manifest.size))


def _links(links):
    keep = []
    arr = (_Link * max(1, len(links)))()
    for i, (staging, manifest) in enumerate(links):
        staging = np.ascontiguousarray(staging, dtype=np.uint8)
        manifest = np.ascontiguousarray(manifest, dtype=ENTRY_DTYPE)
        keep.append((staging, manifest))
        arr[i] = _Link(_p(staging), staging.size, _p(manifest), manifest.size)
    return arr, keep


def merge_chain(sizes: Sequence[int], chunk: int, links: Sequence[Tuple[np.ndarray, np.ndarray]],
                staging_cap: Optional[int] = None, manifest_cap: Optional[int] = None,
                fill: int = 0xA5) -> Tuple[np.ndarray, np.ndarray, dict, dict]:
    """Fold a chain (oldest first) into one link for buffers of the given sizes.  Returns
    (staging, manifest, counts, stats); without capacities both are sized to the need, found by
    a first call with none.  Bytes / entries the call does not write keep ``fill``."""
    arr, keep = _links(links)
    sz = np.ascontiguousarray(sizes, dtype=np.uint64)
    c, stats = _Counts(), (ctypes.c_uint64 * 3)()

    def call(staging, scap, manifest, mcap):
        if _load().ora_merge_chain(_p(sz), sz.size, chunk, arr, len(links), _p(staging), scap,
                                   _p(manifest), mcap, ctypes.byref(c), stats) != 0:
            raise MemoryError("ora_merge_chain")

    if staging_cap is None or manifest_cap is None:
        call(None, 0, None, 0)
        staging_cap = c.staged_bytes if staging_cap is None else staging_cap
        manifest_cap = c.ndirty if manifest_cap is None else manifest_cap
    staging = np.full(staging_cap, fill, dtype=np.uint8)
    manifest = np.frombuffer(bytes([fill]) * (32 * manifest_cap), dtype=ENTRY_DTYPE).copy()
    call(staging, staging_cap, manifest, manifest_cap)
    return (staging, manifest,
            {"ndirty": c.ndirty, "staged_bytes": c.staged_bytes, "overflow": c.overflow},
            {"written": int(stats[0]), "superseded": int(stats[1]), "rejected": int(stats[2])})


def restore_chain(dst: List[np.ndarray], chunk: int,
                  links: Sequence[Tuple[np.ndarray, np.ndarray]],
                  only: Optional[np.ndarray] = None) -> dict:
    """Apply a chain of incremental snapshots, oldest first, to ``dst`` (modified in
    place): ``links`` holds one (staging, manifest) pair per snapshot (sec. 4.6).
    Only entries that are whole chunks of ``dst`` are applied, and with ``only`` (one
    byte per chunk) only those of chunks it marks.  Returns the numbers of chunks
    written, of applied entries a later one overwrote, and of entries skipped."""
    if only is not None:
        only = np.ascontiguousarray(only, dtype=np.uint8)
        if only.size != nchunks(dst, chunk):
            raise ValueError("one byte per chunk of the destination is needed")
    for b in dst:
        if not b.flags["WRITEABLE"]:
            raise TypeError("destination buffers must be writable")
    arr, keep = _links(links)
    stats = (ctypes.c_uint64 * 3)()
    if _load().ora_restore_chain(_desc(dst), len(dst), chunk, arr, len(links), _p(only), stats) != 0:
        raise MemoryError("ora_restore_chain")
    return {"written": int(stats[0]), "superseded": int(stats[1]), "rejected": int(stats[2])}


def buffer_verdicts(sizes: Sequence[int], chunk: int, mask: np.ndarray) -> Tuple[np.ndarray, dict]:
    """Per buffer: does any of its chunks carry a mark (the paper's per-buffer comparison,
    sec. 5.2.1, derived from the chunk verdicts).  Returns (dirty[B] uint8, counts)."""
    sz = np.ascontiguousarray(sizes, dtype=np.uint64)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.size != int(((sz + np.uint64(chunk - 1)) // np.uint64(chunk)).sum()):
        raise ValueError("mask length does not match the buffer list")
    dirty = np.full(sz.size, 0xA5, dtype=np.uint8)
    res = (ctypes.c_uint64 * 2)()
    _load().ora_buffer_verdicts(_p(sz), sz.size, chunk, _p(mask), _p(dirty), res)
    return dirty, {"buffers": int(res[0]), "bytes": int(res[1])}


def mask_andnot(mask: np.ndarray, without: np.ndarray) -> np.ndarray:
    """1 where ``mask`` is set and ``without`` is not (any non-zero byte counts as set)."""
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    without = np.ascontiguousarray(without, dtype=np.uint8)
    if mask.size != without.size:
        raise ValueError("the two masks must have one byte per chunk each")
    out = np.full(mask.size, 0xA5, dtype=np.uint8)
    _load().ora_mask_andnot(mask.size, _p(mask), _p(without), _p(out))
    return out


def marks_from_buffers(sizes: Sequence[int], chunk: int, flags: np.ndarray) -> np.ndarray:
    """One mark per chunk: 1 for every chunk of a buffer whose flag is non-zero."""
    sz = np.ascontiguousarray(sizes, dtype=np.uint64)
    flags = np.ascontiguousarray(flags, dtype=np.uint8)
    if flags.size != sz.size:
        raise ValueError("one flag per buffer is needed")
    n = int(((sz + np.uint64(chunk - 1)) // np.uint64(chunk)).sum())
    marks = np.full(n, 0xA5, dtype=np.uint8)
    _load().ora_marks_from_buffers(_p(sz), sz.size, chunk, _p(flags), _p(marks))
    return marks
