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

Precondition of `switch`, as in the paper's setting: the chunks in which a rank
differs from the base are the same set for every rank (its gradients and
activations), so swapping a delta in leaves no chunk of the previous rank behind.
`same_dirty_set` checks it on the device.

`switch_exact` drops that precondition.  The host also keeps one full copy of the
base (the first rank is swapped out whole, sec. 5.2.1; the copy is cut into a few
pinned allocations) and the device keeps every
rank's checksums from its last swap-out.  The incoming rank's chunks are then
compared, by checksum, with what is resident, and exactly the chunks that differ
come in (the paper's rule: no swap-in of content the device already holds): from
the incoming rank's delta where it has the chunk, else from the base copy
(``ckpt_restore_chain`` over [base slices..., delta], restricted to the chunks that
differ).
Ranks may differ from the base in any chunks; when they differ in the same ones the
base copy is never read.  With exchange=True the exchange pass runs first and only
the chunks the outgoing rank alone changed are then repaired from the base copy,
so the usual case costs what `switch(exchange=True)` costs.
"""
from __future__ import annotations

from typing import List, Optional

from . import binding as ck


class TimeSlicedRanks:
    def __init__(self, plan: ck.Plan, ref_digests, nranks: int, staging_cap: int,
                 manifest_cap: int, device="cuda", exact: bool = False):
        import torch

        self.plan, self.ref, self.nranks = plan, ref_digests, nranks
        self.staging_cap, self.manifest_cap = staging_cap, manifest_cap
        n = plan.nchunks
        self.exact = exact
        if exact:
            # every rank's checksums at its last swap-out, the mask of what has to come in,
            # scratch of the chain restore; the base copy is made by capture_base()
            self.rank_digests = [torch.zeros(max(1, n), dtype=torch.int64, device=device)
                                 for _ in range(nranks)]
            self.incoming = torch.zeros(max(1, n), dtype=torch.uint8, device=device)
            self.incoming_counts = torch.zeros(ck.COUNTS_WORDS, dtype=torch.int64, device=device)
            self.chain_ws = torch.empty(ck.restore_chain_workspace_bytes(n), dtype=torch.uint8,
                                        device=device)
            self.chain_stats = torch.zeros(3, dtype=torch.int64, device=device)
            self.base_links = None
            self.base_bytes = 0
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

    def capture_base(self, max_slice_bytes: int = 8 << 30, pinned_host: bool = True) -> None:
        """Exact mode, set-up: the resident image IS the base (its checksums are ref_digests);
        a full copy goes to pinned host memory, cut into consecutive runs of chunks of at most
        max_slice_bytes each (one pinned allocation and one manifest per run; at most
        CHAIN_MAX - 1 runs, each of which becomes a link of the chain restore).  Synchronous.
        pinned_host=False keeps the copy in device memory instead (for machines whose limit on
        pinned memory the copy would exceed)."""
        import numpy as np
        import torch

        assert self.exact
        n = self.plan.nchunks
        dev = self.digests.device
        ones = torch.ones(max(1, n), dtype=torch.uint8, device=dev)
        counts = torch.zeros(ck.COUNTS_WORDS, dtype=torch.int64, device=dev)
        full = torch.zeros(max(1, n) * ck.ENTRY_BYTES, dtype=torch.uint8, device=dev)
        ck.manifest(self.plan, ones, self.ref, full, counts, 1 << 62, n)
        torch.cuda.synchronize()
        total = int(counts[1])
        offs = ck.manifest_to_numpy(full, n)["stage_off"].astype(np.int64) if n else np.zeros(0, np.int64)
        nslices = max(1, -(-total // max_slice_bytes))
        if nslices > ck.CHAIN_MAX - 1:
            raise ValueError("the base needs more slices than a chain has links; raise max_slice_bytes")
        # slice i starts at the first chunk whose offset reaches i / nslices of the total
        starts = [int(np.searchsorted(offs, total * i // nslices, side="left")) for i in range(nslices)]
        starts.append(n)
        self.base_links = []
        for lo, hi in zip(starts[:-1], starts[1:]):
            if hi <= lo:
                continue
            mask = torch.zeros(max(1, n), dtype=torch.uint8, device=dev)
            mask[lo:hi] = 1
            nbytes = (int(offs[hi]) if hi < n else total) - int(offs[lo])
            if pinned_host:
                host = torch.empty(max(16, nbytes), dtype=torch.uint8, pin_memory=True)
            else:
                host = torch.empty(max(16, nbytes), dtype=torch.uint8, device=dev)
            manifest = torch.zeros((hi - lo) * ck.ENTRY_BYTES, dtype=torch.uint8, device=dev)
            ck.compact(self.plan, mask, self.ref, host, manifest, counts, staging_cap=nbytes,
                       manifest_cap=hi - lo)
            torch.cuda.synchronize()
            assert [int(x) for x in counts] == [hi - lo, nbytes, 0]
            self.base_links.append((host, nbytes, manifest, hi - lo, None))
        self.base_bytes = total

    def switch_exact(self, outgoing: int, incoming: int, stream=None,
                     exchange: bool = False) -> None:
        """Enqueue one context switch that is exact whatever chunks the two ranks changed;
        nothing is read on the host.

        exchange=False: the outgoing rank's delta against the base goes out; then the chunks
        whose checksum differs between the incoming rank (at its last swap-out) and what is
        resident come in, from the incoming rank's delta or, where that rank never changed the
        chunk, from the base copy.  Chunks both ranks changed to the same content stay.

        exchange=True: `switch` with the exchange pass first (one pass over both directions of
        the host link when the two deltas cover the same chunks, else swap-out then swap-in of
        the incoming delta); afterwards the chunks only the outgoing rank changed -- marked for
        it, not for the incoming rank -- get the base's bytes back.  When the deltas line up
        there are none, and the switch costs what the exchange pass costs."""
        assert self.exact and self.base_links is not None, "exact mode needs capture_base()"
        if exchange:
            self.switch(outgoing, incoming, stream, exchange=True)
            ck.mask_andnot(self.plan, self.mask[outgoing], self.mask[incoming], self.incoming,
                           stream)
            ck.restore_chain(self.plan, self.base_links, self.chain_ws, self.chain_stats, stream,
                             only=self.incoming)
            return
        self.swap_out(outgoing, stream)
        ck.diff(self.plan, self.rank_digests[incoming], self.rank_digests[outgoing], self.incoming,
                self.incoming_counts, stream)
        ck.restore_chain(self.plan,
                         self.base_links + [(self.host[incoming], self.staging_cap,
                                             self.manifest[incoming], self.manifest_cap,
                                             self.counts[incoming])],
                         self.chain_ws, self.chain_stats, stream, only=self.incoming)

    def swap_out(self, rank: int, stream=None) -> None:
        """Checksums of the resident image, comparison with the base, and the chunks that
        differ written to the rank's host area by the gather kernel itself."""
        digests = self.rank_digests[rank] if self.exact else self.digests
        ck.snapshot(self.plan, self.ref, None, digests, self.mask[rank], self.host[rank],
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
        digests = self.rank_digests[outgoing] if self.exact else self.digests
        ck.fingerprint(self.plan, digests, stream)
        ck.diff(self.plan, digests, self.ref, self.mask[outgoing], self.counts[outgoing], stream)
        ck.manifest(self.plan, self.mask[outgoing], digests, self.manifest[outgoing],
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
