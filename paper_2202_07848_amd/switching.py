"""Time-slicing several ranks over one device-memory image: the context switch of
replica splicing (Singularity paper sec. 5.1, 5.2.1, 6), as a sequence of library
calls.  Orchestration only -- every step runs in the library's kernels.

All ranks of a data-parallel job that share a GPU have the same buffer list
(consistent allocation, sec. 5.2.2), so one plan describes the image whichever
rank is resident.  The host keeps, per rank, the delta of that rank's state
against a common base (the content every rank shares: parameters and optimizer
state); `ref_digests` are the base's checksums.  A switch

    outgoing rank:  checksum every live buffer, compare with the base, swap the
                    chunks that differ out to that rank's pinned host area
    incoming rank:  swap its delta in from its host area, at the same addresses

is enqueued on one stream without the host reading any result (the entry count
of the swap-in is read on the device), so the incoming rank's first kernel can
be dispatched at once behind an event (sec. 6).  Since both deltas normally
cover the same chunks, the two halves run as one exchange pass that keeps both
directions of the host link busy (``ckpt_exchange``).

Precondition, as in the paper's setting: the chunks in which a rank differs from
the base are the same set for every rank (its gradients and activations), so
swapping a delta in leaves no chunk of the previous rank behind.  `same_dirty_set`
checks it on the device.
"""
from __future__ import annotations

from typing import List, Optional

from . import binding as ck


class TimeSlicedRanks:
    def __init__(self, plan: ck.Plan, ref_digests, nranks: int, staging_cap: int,
                 manifest_cap: int, device="cuda"):
        import torch

        self.plan, self.ref, self.nranks = plan, ref_digests, nranks
        self.staging_cap, self.manifest_cap = staging_cap, manifest_cap
        n = plan.nchunks
        self.digests = torch.zeros(max(1, n), dtype=torch.int64, device=device)
        self.rejected = torch.zeros(1, dtype=torch.int64, device=device)
        self.serial = torch.zeros(1, dtype=torch.int64, device=device)   # last switch: 0 = one pass
        # per rank: delta bytes in pinned host memory, manifest / mask / counts on the device
        self.host: List = [torch.empty(max(16, staging_cap), dtype=torch.uint8, pin_memory=True)
                           for _ in range(nranks)]
        self.manifest = [torch.zeros(max(1, manifest_cap) * ck.ENTRY_BYTES, dtype=torch.uint8,
                                     device=device) for _ in range(nranks)]
        self.mask = [torch.zeros(max(1, n), dtype=torch.uint8, device=device)
                     for _ in range(nranks)]
        self.counts = [torch.zeros(ck.COUNTS_WORDS, dtype=torch.int64, device=device)
                       for _ in range(nranks)]

    def swap_out(self, rank: int, stream=None) -> None:
        """Checksums of the resident image, comparison with the base, and the chunks that
        differ written to the rank's host area by the gather kernel itself."""
        ck.snapshot(self.plan, self.ref, None, self.digests, self.mask[rank], self.host[rank],
                    self.manifest[rank], self.counts[rank], stream=stream,
                    staging_cap=self.staging_cap, manifest_cap=self.manifest_cap)

    def swap_in(self, rank: int, stream=None) -> None:
        """The rank's delta back to the addresses it came from; the entry count is the one its
        swap-out left on the device."""
        ck.restore_counted(self.plan, self.host[rank], self.staging_cap, self.manifest[rank],
                           self.manifest_cap, self.counts[rank], self.rejected, stream=stream)

    def switch(self, outgoing: int, incoming: int, stream=None, exchange: bool = True) -> None:
        """Enqueue one context switch; nothing is read on the host.

        exchange=True: checksums, comparison and manifest of the outgoing rank, then
        ``ckpt_exchange``: where both ranks' deltas cover the same chunks (the usual case) every
        chunk is swapped out and in by one pass, both directions of the host link busy at once;
        otherwise the library falls back, on the device, to swap-out followed by swap-in.
        exchange=False: swap-out, then swap-in."""
        if not exchange:
            self.swap_out(outgoing, stream)
            self.swap_in(incoming, stream)
            return
        ck.fingerprint(self.plan, self.digests, stream)
        ck.diff(self.plan, self.digests, self.ref, self.mask[outgoing], self.counts[outgoing],
                stream)
        ck.manifest(self.plan, self.mask[outgoing], self.digests, self.manifest[outgoing],
                    self.counts[outgoing], self.staging_cap, self.manifest_cap, stream)
        ck.exchange(self.plan, self.manifest[outgoing], self.counts[outgoing], self.host[outgoing],
                    self.staging_cap, self.manifest[incoming], self.counts[incoming],
                    self.host[incoming], self.staging_cap, self.manifest_cap, self.serial,
                    self.rejected, stream)

    def same_dirty_set(self, ranks: Optional[List[int]] = None) -> bool:
        """True if the given ranks (default: all) differ from the base in the same chunks."""
        import torch

        ranks = list(range(self.nranks)) if ranks is None else ranks
        return all(bool(torch.equal(self.mask[ranks[0]], self.mask[r])) for r in ranks[1:])
