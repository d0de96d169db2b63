"""MI355X-native device-state snapshot path: chunk, XXH64-fingerprint, diff,
compact and restore of a training job's live device buffers (the checksum
de-duplicated swap-out / swap-in of the Singularity paper, sec. 4.5, 4.6,
5.2.1).  ``binding`` wraps the C-ABI library; ``workloads`` holds the seeded
synthetic inputs.  Nothing here computes on the CPU."""

__all__ = ["binding", "workloads"]
