"""Helpers for the GPU parity tests: put host byte arrays on the device inside
one arena with canary gaps, run the library through its binding, fetch results."""
from __future__ import annotations

import numpy as np
import torch

from paper_2202_07848_amd import binding as ck

CANARY = 0xC7
GAP = 64          # canary bytes between buffers (keeps 16-byte alignment)
# When not None, every plan DeviceBuffers creates gets this split threshold (the state size from
# which the hinted snapshot pass runs as two launches): tests force both launch shapes with it.
SPLIT_THRESHOLD = None


class DeviceBuffers:
    """Host arrays -> one device arena: [gap][buf0][pad][gap][buf1]..."""

    def __init__(self, host_bufs, chunk):
        self.sizes = [int(b.size) for b in host_bufs]
        offs, cur = [], GAP
        for n in self.sizes:
            offs.append(cur)
            cur += (n + 15) // 16 * 16 + GAP
        self.offs = offs
        image = np.full(cur, CANARY, dtype=np.uint8)
        for o, b in zip(offs, host_bufs):
            image[o:o + b.size] = b
        self.arena = torch.from_numpy(image).cuda()
        base = self.arena.data_ptr()
        assert base % 16 == 0
        self.plan = ck.Plan([(base + o, n) for o, n in zip(offs, self.sizes)], chunk)
        if SPLIT_THRESHOLD is not None:
            self.plan.split_threshold = SPLIT_THRESHOLD

    def host(self):
        """Current device bytes of every buffer plus the whole arena image."""
        img = self.arena.cpu().numpy()
        return [img[o:o + n] for o, n in zip(self.offs, self.sizes)], img

    def canaries_intact(self, img=None):
        if img is None:
            img = self.arena.cpu().numpy()
        keep = np.ones(img.size, dtype=bool)
        for o, n in zip(self.offs, self.sizes):
            keep[o:o + n] = False
        return bool(np.all(img[keep] == CANARY))


def run_fingerprint(plan):
    dig = torch.zeros(max(1, plan.nchunks), dtype=torch.int64, device="cuda")
    ck.fingerprint(plan, dig)
    torch.cuda.synchronize()
    return dig


def run_diff(plan, dig, ref):
    mask = torch.full((max(1, plan.nchunks),), 0x77, dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    ck.diff(plan, dig, ref, mask, counts, n_ref=None if ref is None else plan.nchunks)
    torch.cuda.synchronize()
    return mask, counts


def run_compact(plan, mask, dig, staging_cap, manifest_cap, fill=0xA5, slack=256):
    """Staging and manifest are followed by `slack` canary bytes."""
    staging = torch.full((staging_cap + slack,), fill, dtype=torch.uint8, device="cuda")
    manifest = torch.full((manifest_cap * 32 + slack,), fill, dtype=torch.uint8, device="cuda")
    counts = torch.full((3,), -1, dtype=torch.int64, device="cuda")
    ck.compact(plan, mask, dig, staging, manifest, counts, staging_cap=staging_cap,
               manifest_cap=manifest_cap)
    torch.cuda.synchronize()
    return staging, manifest, counts


def u64(t, n):
    return t[:n].cpu().numpy().view(np.uint64)


def counts_dict(c):
    v = c.cpu().numpy().view(np.uint64)
    return {"ndirty": int(v[0]), "staged_bytes": int(v[1]), "overflow": int(v[2])}
