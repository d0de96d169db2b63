"""ctypes binding of libckpt.so -- argument marshalling only.

Same names as the C ABI (include/ckpt.h): ``fingerprint``, ``diff``,
``compact``, ``restore`` over a ``Plan`` built from a buffer-descriptor list.
PyTorch supplies device memory and the HIP stream; every step of the path runs
in the library's kernels.  There is no CPU fallback: if the library is missing
the import of this module's functions fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libckpt.so")

ENTRY_DTYPE = np.dtype(
    [("buf", "<u4"), ("len", "<u4"), ("buf_off", "<u8"), ("stage_off", "<u8"), ("digest", "<u8")]
)
ENTRY_BYTES = 32
COUNTS_WORDS = 3          # ndirty, staged_bytes, overflow

EXPORTS = (
    "ckpt_plan_create", "ckpt_plan_destroy", "ckpt_plan_nchunks", "ckpt_plan_nbytes",
    "ckpt_plan_nbufs", "ckpt_plan_chunk_bytes", "ckpt_fingerprint", "ckpt_diff", "ckpt_compact", "ckpt_manifest", "ckpt_exchange",
    "ckpt_restore", "ckpt_restore_counted", "ckpt_restore_chain_workspace_bytes", "ckpt_restore_chain",
    "ckpt_merge_chain_workspace_bytes", "ckpt_merge_chain",
    "ckpt_snapshot_workspace_bytes", "ckpt_snapshot_stats_offset", "ckpt_snapshot",
    "ckpt_snapshot_static", "ckpt_snapshot_static_max_chunks",
    "ckpt_plan_split_threshold", "ckpt_plan_set_split_threshold", "ckpt_match_workspace_bytes", "ckpt_match", "ckpt_apply_matches", "ckpt_moves_workspace_bytes", "ckpt_apply_moves_inplace",
    "ckpt_validate_mutations", "ckpt_upload_owners", "ckpt_buffer_verdicts", "ckpt_mask_andnot",
    "ckpt_marks_from_buffers",
    "ckpt_swapper_create", "ckpt_swapper_destroy", "ckpt_swap_out", "ckpt_swap_in",
    "ckpt_bw_copy", "ckpt_bw_read", "ckpt_bw_streams", "ckpt_alu_xxh64", "ckpt_strerror", "ckpt_last_device_error",
    "ckpt_version",
)


class CkptError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().ckpt_strerror(status).decode()
        if status == -6:
            msg += " (hipError %d)" % _lib().ckpt_last_device_error()
        super().__init__(f"{where}: {msg} [{status}]")


class _Buf(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("nbytes", ctypes.c_uint64)]


class _Link(ctypes.Structure):
    _fields_ = [("d_staging", ctypes.c_void_p), ("staging_bytes", ctypes.c_uint64),
                ("d_manifest", ctypes.c_void_p), ("manifest_cap", ctypes.c_uint64),
                ("d_counts", ctypes.c_void_p)]


_handle = None


def _lib():
    global _handle
    if _handle is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is not built; run `python -m paper_2202_07848_amd.build` "
                "(there is no CPU fallback)")
        # PyTorch must load its HIP runtime first: the library then binds to that
        # same runtime (same SONAME) instead of bringing a second copy into the
        # process, which would not share torch's device context.
        import torch  # noqa: F401
        lib = ctypes.CDLL(LIB_PATH)
        u64, vp, ci = ctypes.c_uint64, ctypes.c_void_p, ctypes.c_int
        lib.ckpt_plan_create.restype = ci
        lib.ckpt_plan_create.argtypes = [vp, u64, u64, ctypes.POINTER(vp)]
        lib.ckpt_plan_destroy.restype = ci
        lib.ckpt_plan_destroy.argtypes = [vp]
        for name in ("ckpt_plan_nchunks", "ckpt_plan_nbytes", "ckpt_plan_nbufs",
                     "ckpt_plan_chunk_bytes"):
            getattr(lib, name).restype = u64
            getattr(lib, name).argtypes = [vp]
        lib.ckpt_fingerprint.restype = ci
        lib.ckpt_fingerprint.argtypes = [vp, vp, vp]
        lib.ckpt_diff.restype = ci
        lib.ckpt_diff.argtypes = [vp, vp, vp, u64, vp, vp, vp]
        lib.ckpt_upload_owners.restype = ci
        lib.ckpt_upload_owners.argtypes = [vp, vp, ctypes.c_uint32, ctypes.c_uint32, vp, vp, vp]
        lib.ckpt_compact.restype = ci
        lib.ckpt_compact.argtypes = [vp, vp, vp, vp, u64, vp, u64, vp, vp]
        lib.ckpt_manifest.restype = ci
        lib.ckpt_manifest.argtypes = [vp, vp, vp, u64, vp, u64, vp, vp]
        lib.ckpt_exchange.restype = ci
        lib.ckpt_exchange.argtypes = [vp, vp, vp, vp, u64, vp, vp, vp, u64, u64, vp, vp, vp]
        lib.ckpt_restore.restype = ci
        lib.ckpt_restore.argtypes = [vp, vp, u64, vp, u64, vp, vp]
        lib.ckpt_restore_counted.restype = ci
        lib.ckpt_restore_counted.argtypes = [vp, vp, u64, vp, u64, vp, vp, vp]
        lib.ckpt_restore_chain_workspace_bytes.restype = u64
        lib.ckpt_restore_chain_workspace_bytes.argtypes = [u64]
        lib.ckpt_restore_chain.restype = ci
        lib.ckpt_restore_chain.argtypes = [vp, vp, u64, vp, vp, u64, vp, vp]
        lib.ckpt_merge_chain_workspace_bytes.restype = u64
        lib.ckpt_merge_chain_workspace_bytes.argtypes = [u64]
        lib.ckpt_merge_chain.restype = ci
        lib.ckpt_merge_chain.argtypes = [vp, vp, u64, vp, u64, vp, u64, vp, vp, u64, vp, vp]
        lib.ckpt_plan_split_threshold.restype = u64
        lib.ckpt_plan_split_threshold.argtypes = [vp]
        lib.ckpt_plan_set_split_threshold.restype = ci
        lib.ckpt_plan_set_split_threshold.argtypes = [vp, u64]
        lib.ckpt_snapshot_workspace_bytes.restype = u64
        lib.ckpt_snapshot_workspace_bytes.argtypes = [u64]
        lib.ckpt_snapshot_stats_offset.restype = u64
        lib.ckpt_snapshot_stats_offset.argtypes = [u64]
        lib.ckpt_snapshot.restype = ci
        lib.ckpt_snapshot.argtypes = [vp, vp, u64, vp, vp, vp, vp, u64, vp, u64, vp, vp, vp, u64, vp]
        lib.ckpt_snapshot_static_max_chunks.restype = u64
        lib.ckpt_snapshot_static_max_chunks.argtypes = []
        lib.ckpt_snapshot_static.restype = ci
        lib.ckpt_snapshot_static.argtypes = [vp, vp, u64, vp, vp, vp, vp, u64, vp, u64, vp, vp, vp]
        lib.ckpt_match_workspace_bytes.restype = u64
        lib.ckpt_match_workspace_bytes.argtypes = [u64, u64]
        lib.ckpt_match.restype = ci
        lib.ckpt_match.argtypes = [vp, vp, vp, u64, vp, u64, vp, vp, vp, vp]
        lib.ckpt_apply_matches.restype = ci
        lib.ckpt_apply_matches.argtypes = [vp, vp, vp, vp, vp]
        lib.ckpt_moves_workspace_bytes.restype = u64
        lib.ckpt_moves_workspace_bytes.argtypes = [u64]
        lib.ckpt_apply_moves_inplace.restype = ci
        lib.ckpt_apply_moves_inplace.argtypes = [vp, vp, vp, u64, vp, u64, vp, vp, vp]
        lib.ckpt_marks_from_buffers.restype = ci
        lib.ckpt_marks_from_buffers.argtypes = [vp, vp, vp, vp]
        lib.ckpt_mask_andnot.restype = ci
        lib.ckpt_mask_andnot.argtypes = [vp, vp, vp, vp, vp]
        lib.ckpt_buffer_verdicts.restype = ci
        lib.ckpt_buffer_verdicts.argtypes = [vp, vp, vp, vp, vp]
        lib.ckpt_validate_mutations.restype = ci
        lib.ckpt_validate_mutations.argtypes = [vp, vp, vp, vp, vp, vp, vp]
        lib.ckpt_swapper_create.restype = ci
        lib.ckpt_swapper_create.argtypes = [u64, ctypes.POINTER(vp)]
        lib.ckpt_swapper_destroy.restype = ci
        lib.ckpt_swapper_destroy.argtypes = [vp]
        lib.ckpt_swap_out.restype = ci
        lib.ckpt_swap_out.argtypes = [vp, vp, vp, vp, vp, u64, vp, u64, vp, vp]
        lib.ckpt_swap_in.restype = ci
        lib.ckpt_swap_in.argtypes = [vp, vp, vp, u64, vp, u64, vp, vp]
        lib.ckpt_bw_copy.restype = ci
        lib.ckpt_bw_copy.argtypes = [vp, vp, u64, vp]
        lib.ckpt_bw_read.restype = ci
        lib.ckpt_bw_read.argtypes = [vp, u64, vp, vp]
        lib.ckpt_bw_streams.restype = ci
        lib.ckpt_bw_streams.argtypes = [vp, vp, u64, u64, u64, vp, vp]
        lib.ckpt_alu_xxh64.restype = u64
        lib.ckpt_alu_xxh64.argtypes = [u64, vp, vp]
        lib.ckpt_strerror.restype = ctypes.c_char_p
        lib.ckpt_strerror.argtypes = [ci]
        lib.ckpt_last_device_error.restype = ci
        lib.ckpt_version.restype = ci
        _handle = lib
    return _handle


def _check(status: int, where: str) -> None:
    if status != 0:
        raise CkptError(status, where)


def _stream(stream) -> Optional[int]:
    """hipStream_t of a torch stream (None = torch's current stream)."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr(t) -> Optional[int]:
    return None if t is None else ctypes.c_void_p(t.data_ptr())


class Plan:
    """Chunk geometry of a list of live device buffers (``ckpt_plan_create``).

    ``buffers``: sequence of (device pointer, nbytes) pairs or of torch tensors
    (their storage bytes are the buffer).  Tensors are kept alive by the plan.
    """

    def __init__(self, buffers: Sequence, chunk_bytes: int):
        self._keep = []
        descs = (_Buf * max(1, len(buffers)))()
        for i, b in enumerate(buffers):
            if isinstance(b, tuple):
                ptr, nbytes = b
            else:
                if not b.is_contiguous():
                    raise ValueError("buffer tensors must be contiguous")
                ptr, nbytes = b.data_ptr(), b.numel() * b.element_size()
                self._keep.append(b)
            descs[i].ptr = ptr if nbytes else None
            descs[i].nbytes = nbytes
        handle = ctypes.c_void_p()
        _check(_lib().ckpt_plan_create(descs, len(buffers), chunk_bytes, ctypes.byref(handle)),
               "ckpt_plan_create")
        self._h = handle

    def close(self) -> None:
        if getattr(self, "_h", None):
            _check(_lib().ckpt_plan_destroy(self._h), "ckpt_plan_destroy")
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def nchunks(self) -> int:
        return int(_lib().ckpt_plan_nchunks(self._h))

    @property
    def nbytes(self) -> int:
        return int(_lib().ckpt_plan_nbytes(self._h))

    @property
    def nbufs(self) -> int:
        return int(_lib().ckpt_plan_nbufs(self._h))

    @property
    def chunk_bytes(self) -> int:
        return int(_lib().ckpt_plan_chunk_bytes(self._h))

    @property
    def split_threshold(self) -> int:
        """``ckpt_plan_split_threshold``: state size from which the hinted pass runs as two launches."""
        return int(_lib().ckpt_plan_split_threshold(self._h))

    @split_threshold.setter
    def split_threshold(self, nbytes: int) -> None:
        _check(_lib().ckpt_plan_set_split_threshold(self._h, nbytes), "ckpt_plan_set_split_threshold")


def fingerprint(plan: Plan, digests, stream=None) -> None:
    """``ckpt_fingerprint``: digests (int64/uint64 CUDA tensor, N elements) <- XXH64 per chunk."""
    _check(_lib().ckpt_fingerprint(plan._h, _ptr(digests), _stream(stream)), "ckpt_fingerprint")


def diff(plan: Plan, digests, ref, mask, counts, stream=None, n_ref: Optional[int] = None) -> None:
    """``ckpt_diff``: mask (uint8, N) and counts (3 x int64) from digests vs ref (or None)."""
    if n_ref is None:
        n_ref = 0 if ref is None else ref.numel()
    _check(_lib().ckpt_diff(plan._h, _ptr(digests), _ptr(ref), n_ref, _ptr(mask), _ptr(counts),
                            _stream(stream)), "ckpt_diff")


def upload_owners(plan: Plan, gathered, world: int, rank: int, mask, counts, stream=None) -> None:
    """``ckpt_upload_owners``: gathered is int64 (world, N) checksums of all workers; mask (uint8, N)
    marks the chunks worker ``rank`` uploads; counts as for ``diff``."""
    _check(_lib().ckpt_upload_owners(plan._h, _ptr(gathered), world, rank, _ptr(mask), _ptr(counts),
                                     _stream(stream)), "ckpt_upload_owners")


def compact(plan: Plan, mask, digests, staging, manifest, counts, stream=None,
            staging_cap: Optional[int] = None, manifest_cap: Optional[int] = None) -> None:
    """``ckpt_compact``: staging (uint8) and manifest (uint8 view of 32-byte entries)."""
    if staging_cap is None:
        staging_cap = 0 if staging is None else staging.numel() * staging.element_size()
    if manifest_cap is None:
        manifest_cap = 0 if manifest is None else \
            manifest.numel() * manifest.element_size() // ENTRY_BYTES
    _check(_lib().ckpt_compact(plan._h, _ptr(mask), _ptr(digests), _ptr(staging), staging_cap,
                               _ptr(manifest), manifest_cap, _ptr(counts), _stream(stream)),
           "ckpt_compact")


def manifest(plan: Plan, mask, digests, manifest_t, counts, staging_cap: int,
             manifest_cap: Optional[int] = None, stream=None) -> None:
    """``ckpt_manifest``: manifest entries and counts for a mask, no chunk bytes moved."""
    if manifest_cap is None:
        manifest_cap = manifest_t.numel() * manifest_t.element_size() // ENTRY_BYTES
    _check(_lib().ckpt_manifest(plan._h, _ptr(mask), _ptr(digests), staging_cap, _ptr(manifest_t),
                                manifest_cap, _ptr(counts), _stream(stream)), "ckpt_manifest")


def exchange(plan: Plan, manifest_out, counts_out, staging_out, staging_out_cap: int, manifest_in,
             counts_in, staging_in, staging_in_bytes: int, manifest_cap: int, serial=None,
             rejected=None, stream=None) -> None:
    """``ckpt_exchange``: swap-out of one rank's chunks and swap-in of another's as one pass."""
    _check(_lib().ckpt_exchange(plan._h, _ptr(manifest_out), _ptr(counts_out), _ptr(staging_out),
                                staging_out_cap, _ptr(manifest_in), _ptr(counts_in),
                                _ptr(staging_in), staging_in_bytes, manifest_cap, _ptr(serial),
                                _ptr(rejected), _stream(stream)), "ckpt_exchange")


def snapshot_workspace_bytes(nchunks: int) -> int:
    return int(_lib().ckpt_snapshot_workspace_bytes(nchunks))


def snapshot_stats(workspace, nchunks: int) -> dict:
    """Diagnostics a hinted ``snapshot`` left in its workspace (synchronise first)."""
    off = int(_lib().ckpt_snapshot_stats_offset(nchunks))
    words = workspace.view(-1)[off:off + 32].cpu().numpy().view(np.uint64)
    return {"hint_misses": int(words[0]), "regathered_chunks": int(words[3])}


def snapshot(plan: Plan, ref, hint, digests, mask, staging, manifest, counts, hint_misses=None,
             workspace=None, stream=None, staging_cap: Optional[int] = None,
             manifest_cap: Optional[int] = None, n_ref: Optional[int] = None) -> None:
    """``ckpt_snapshot``: fingerprint + diff + compact in one call; with ``hint`` (uint8, N) the
    predicted chunks are staged during the fingerprint pass."""
    if n_ref is None:
        n_ref = 0 if ref is None else ref.numel()
    if staging_cap is None:
        staging_cap = 0 if staging is None else staging.numel() * staging.element_size()
    if manifest_cap is None:
        manifest_cap = 0 if manifest is None else \
            manifest.numel() * manifest.element_size() // ENTRY_BYTES
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(_lib().ckpt_snapshot(plan._h, _ptr(ref), n_ref, _ptr(hint), _ptr(digests), _ptr(mask),
                                _ptr(staging), staging_cap, _ptr(manifest), manifest_cap,
                                _ptr(counts), _ptr(hint_misses), _ptr(workspace), ws_bytes,
                                _stream(stream)), "ckpt_snapshot")


def snapshot_static_max_chunks() -> int:
    return int(_lib().ckpt_snapshot_static_max_chunks())


def snapshot_static(plan: Plan, ref, hint, digests, mask, staging, manifest, counts,
                    hint_misses=None, stream=None, staging_cap: Optional[int] = None,
                    manifest_cap: Optional[int] = None, n_ref: Optional[int] = None) -> None:
    """``ckpt_snapshot_static``: ``snapshot`` without a workspace argument (the library's static
    device scratch serves; plans up to ``snapshot_static_max_chunks()`` chunks)."""
    if n_ref is None:
        n_ref = 0 if ref is None else ref.numel()
    if staging_cap is None:
        staging_cap = 0 if staging is None else staging.numel() * staging.element_size()
    if manifest_cap is None:
        manifest_cap = 0 if manifest is None else \
            manifest.numel() * manifest.element_size() // ENTRY_BYTES
    _check(_lib().ckpt_snapshot_static(plan._h, _ptr(ref), n_ref, _ptr(hint), _ptr(digests),
                                       _ptr(mask), _ptr(staging), staging_cap, _ptr(manifest),
                                       manifest_cap, _ptr(counts), _ptr(hint_misses),
                                       _stream(stream)), "ckpt_snapshot_static")


def restore(dst_plan: Plan, staging, staging_bytes: int, manifest, nentries: int,
            rejected=None, stream=None) -> None:
    """``ckpt_restore``: scatter the first nentries manifest entries into dst_plan's buffers."""
    _check(_lib().ckpt_restore(dst_plan._h, _ptr(staging), staging_bytes, _ptr(manifest), nentries,
                               _ptr(rejected), _stream(stream)), "ckpt_restore")


def restore_counted(dst_plan: Plan, staging, staging_bytes: int, manifest, manifest_cap: int, counts,
                    rejected=None, stream=None) -> None:
    """``ckpt_restore_counted``: as ``restore``, the entry count taken from ``counts`` on the device."""
    _check(_lib().ckpt_restore_counted(dst_plan._h, _ptr(staging), staging_bytes, _ptr(manifest),
                                       manifest_cap, _ptr(counts), _ptr(rejected), _stream(stream)),
           "ckpt_restore_counted")


CHAIN_MAX = 16
CHAIN_STAT_FIELDS = ("written", "superseded", "rejected")


def restore_chain_workspace_bytes(nchunks: int) -> int:
    return int(_lib().ckpt_restore_chain_workspace_bytes(nchunks))


def _links(links):
    arr = (_Link * max(1, len(links)))()
    for i, (staging, staging_bytes, manifest, cap, counts) in enumerate(links):
        arr[i] = _Link(_ptr(staging), staging_bytes, _ptr(manifest), cap, _ptr(counts))
    return arr


def merge_chain_workspace_bytes(nchunks: int) -> int:
    return int(_lib().ckpt_merge_chain_workspace_bytes(nchunks))


def merge_chain(plan: Plan, links, staging, manifest, counts, workspace, stats=None, stream=None,
                staging_cap: Optional[int] = None, manifest_cap: Optional[int] = None) -> None:
    """``ckpt_merge_chain``: links as for ``restore_chain``; staging / manifest / counts as for
    ``compact``."""
    if staging_cap is None:
        staging_cap = 0 if staging is None else staging.numel() * staging.element_size()
    if manifest_cap is None:
        manifest_cap = 0 if manifest is None else \
            manifest.numel() * manifest.element_size() // ENTRY_BYTES
    _check(_lib().ckpt_merge_chain(plan._h, _links(links), len(links), _ptr(staging), staging_cap,
                                   _ptr(manifest), manifest_cap, _ptr(counts), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _ptr(stats),
                                   _stream(stream)), "ckpt_merge_chain")


def restore_chain(dst_plan: Plan, links, workspace, stats=None, stream=None, only=None) -> None:
    """``ckpt_restore_chain``: ``links`` is a sequence, oldest first, of
    (staging, staging_bytes, manifest, manifest_cap, counts or None); workspace is a uint8
    tensor, stats (optional) 3 x int64, only (optional) one uint8 per chunk: 0 = leave alone."""
    arr = _links(links)
    _check(_lib().ckpt_restore_chain(dst_plan._h, arr, len(links), _ptr(only), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _ptr(stats),
                                     _stream(stream)), "ckpt_restore_chain")


def marks_from_buffers(plan: Plan, buf_flags, marks, stream=None) -> None:
    """``ckpt_marks_from_buffers``: marks (uint8, N) = 1 for every chunk of a flagged buffer."""
    _check(_lib().ckpt_marks_from_buffers(plan._h, _ptr(buf_flags), _ptr(marks), _stream(stream)),
           "ckpt_marks_from_buffers")


def mask_andnot(plan: Plan, mask, without, out, stream=None) -> None:
    """``ckpt_mask_andnot``: out[k] = 1 where mask[k] is set and without[k] is not (uint8, N)."""
    _check(_lib().ckpt_mask_andnot(plan._h, _ptr(mask), _ptr(without), _ptr(out), _stream(stream)),
           "ckpt_mask_andnot")


def buffer_verdicts(plan: Plan, mask, buf_dirty, counts, stream=None) -> None:
    """``ckpt_buffer_verdicts``: buf_dirty (uint8, one per buffer of the plan's list), counts
    (2 x int64: buffers that differ, their bytes)."""
    _check(_lib().ckpt_buffer_verdicts(plan._h, _ptr(mask), _ptr(buf_dirty), _ptr(counts),
                                       _stream(stream)), "ckpt_buffer_verdicts")


MATCH_COUNT_FIELDS = ("nsame", "nmoved", "ndup", "nnew", "staged_bytes", "table_full")


def match_workspace_bytes(n_ref: int, nchunks: int) -> int:
    return int(_lib().ckpt_match_workspace_bytes(n_ref, nchunks))


def match(plan: Plan, digests, ref, workspace, src, mask, counts, stream=None,
          n_ref: Optional[int] = None) -> None:
    """``ckpt_match``: src (int64, N), mask (uint8, N), counts (6 x int64) from a
    content-addressed lookup of digests in ref (any length); workspace is a uint8 tensor."""
    if n_ref is None:
        n_ref = 0 if ref is None else ref.numel()
    _check(_lib().ckpt_match(plan._h, _ptr(digests), _ptr(ref), n_ref, _ptr(workspace),
                             workspace.numel() * workspace.element_size(), _ptr(src), _ptr(mask),
                             _ptr(counts), _stream(stream)), "ckpt_match")


def apply_matches(dst_plan: Plan, ref_plan: Optional[Plan], src, rejected=None,
                  stream=None) -> None:
    """``ckpt_apply_matches``: device-to-device moves of the matched chunks into dst_plan
    (ref_plan None: only the duplicates)."""
    _check(_lib().ckpt_apply_matches(dst_plan._h, None if ref_plan is None else ref_plan._h,
                                     _ptr(src), _ptr(rejected), _stream(stream)),
           "ckpt_apply_matches")


def moves_workspace_bytes(nchunks: int) -> int:
    return int(_lib().ckpt_moves_workspace_bytes(nchunks))


def apply_moves_inplace(plan: Plan, src, temp, workspace, counts, rejected=None, stream=None,
                        temp_cap: Optional[int] = None) -> None:
    """``ckpt_apply_moves_inplace``: two-phase moves inside the memory that holds the reference."""
    if temp_cap is None:
        temp_cap = 0 if temp is None else temp.numel() * temp.element_size()
    _check(_lib().ckpt_apply_moves_inplace(plan._h, _ptr(src), _ptr(temp), temp_cap,
                                           _ptr(workspace),
                                           workspace.numel() * workspace.element_size(),
                                           _ptr(counts), _ptr(rejected), _stream(stream)),
           "ckpt_apply_moves_inplace")


class Swapper:
    """``ckpt_swapper_create``: device ring + copy stream for host swap-out / swap-in."""

    def __init__(self, slice_bytes: int):
        h = ctypes.c_void_p()
        _check(_lib().ckpt_swapper_create(slice_bytes, ctypes.byref(h)), "ckpt_swapper_create")
        self._h = h

    def close(self) -> None:
        if getattr(self, "_h", None):
            _lib().ckpt_swapper_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def swap_out(self, plan: Plan, mask, digests, host_staging, manifest, stream=None,
                 staging_cap: Optional[int] = None, manifest_cap: Optional[int] = None) -> dict:
        """``ckpt_swap_out``: host_staging is a (pinned) CPU uint8 tensor.  Returns the counts."""
        if staging_cap is None:
            staging_cap = host_staging.numel()
        if manifest_cap is None:
            manifest_cap = manifest.numel() * manifest.element_size() // ENTRY_BYTES
        counts = (ctypes.c_uint64 * 3)()
        status = _lib().ckpt_swap_out(self._h, plan._h, _ptr(mask), _ptr(digests),
                                      _ptr(host_staging), staging_cap, _ptr(manifest),
                                      manifest_cap, counts, _stream(stream))
        out = {"ndirty": int(counts[0]), "staged_bytes": int(counts[1]), "overflow": int(counts[2])}
        if status == -5:
            out["status"] = status
            return out
        _check(status, "ckpt_swap_out")
        out["status"] = 0
        return out

    def swap_in(self, dst_plan: Plan, host_staging, staged_bytes: int, manifest, nentries: int,
                stream=None) -> int:
        """``ckpt_swap_in``: returns the number of rejected entries."""
        rejected = ctypes.c_uint64(0)
        _check(_lib().ckpt_swap_in(self._h, dst_plan._h, _ptr(host_staging), staged_bytes,
                                   _ptr(manifest), nentries, ctypes.byref(rejected),
                                   _stream(stream)), "ckpt_swap_in")
        return int(rejected.value)


VALIDATION_FIELDS = ("changed_a", "changed_b", "mismatches", "first_mismatch")


def validate_mutations(plan: Plan, before_a, after_a, before_b, after_b, result,
                       stream=None) -> None:
    """``ckpt_validate_mutations``: result (4 x int64) from four digest arrays of plan's geometry."""
    _check(_lib().ckpt_validate_mutations(plan._h, _ptr(before_a), _ptr(after_a), _ptr(before_b),
                                          _ptr(after_b), _ptr(result), _stream(stream)),
           "ckpt_validate_mutations")


def bw_copy(dst, src, nbytes: int, stream=None) -> None:
    _check(_lib().ckpt_bw_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "ckpt_bw_copy")


def bw_read(src, nbytes: int, sink, stream=None) -> None:
    _check(_lib().ckpt_bw_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)), "ckpt_bw_read")


def bw_streams(dst, src, nstreams: int, stream_bytes: int, sink, stream=None,
               tile_bytes: int = 256) -> None:
    """``ckpt_bw_streams``: copy (or, with dst None, read) nstreams streams of stream_bytes bytes
    with the fingerprint pass's access pattern, tile_bytes (256 or 1024) of a stream per step."""
    _check(_lib().ckpt_bw_streams(_ptr(dst), _ptr(src), nstreams, stream_bytes, tile_bytes,
                                  _ptr(sink), _stream(stream)), "ckpt_bw_streams")


def alu_xxh64(rounds_per_lane: int, sink, stream=None) -> int:
    """``ckpt_alu_xxh64``: hash arithmetic only; returns the bytes the steps stand for."""
    n = int(_lib().ckpt_alu_xxh64(rounds_per_lane, _ptr(sink), _stream(stream)))
    if n == 0:
        raise CkptError(-1, "ckpt_alu_xxh64")
    return n


def version() -> int:
    return int(_lib().ckpt_version())


def manifest_to_numpy(manifest, nentries: int) -> np.ndarray:
    """Host copy of the first nentries manifest entries as a structured array."""
    raw = manifest.view(-1)[: nentries * ENTRY_BYTES].cpu().numpy()
    return raw.view(ENTRY_DTYPE)
