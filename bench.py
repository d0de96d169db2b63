#!/usr/bin/env python3
"""Benchmark of the device-state snapshot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--dirty F]

One step = one pass of the whole path over the configuration's synthetic
training state, everything already resident in HBM:

    replica configs (1, 2, 4, 5):  fingerprint(replica 0) -> reference digests,
        then for every other replica r: fingerprint(r), diff against the
        reference, compact, restore (back into r's own buffers, so the state is
        the same for the next step);
    config 3 (one fragmented replica, previous-snapshot diff):  fingerprint(t1),
        diff against the digests of t0, compact, restore.

Prints ONE JSON line.  `value` is device-state GB/s over fingerprint + diff +
compact (all bytes fingerprinted in the step / the time of those three phases,
from HIP events on the launch stream); restore is timed inside the same step
and reported beside it; `ms_per_step` is the wall time of the whole step.
The default workload is config 5 (3B-parameter replicas x2, 1 MiB chunks), the
configuration the throughput target is quoted on.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--shrink", type=int, default=1, help="reduced workload (debugging only)")
    ap.add_argument("--dirty", type=float, default=0.10, help="config 3: rewritten chunk fraction")
    ap.add_argument("--fused-from", type=float, default=0.2,
                    help="staged fraction from which the fused ckpt_snapshot is used (default 0.2)")
    ap.add_argument("--separate", action="store_true",
                    help="time ckpt_fingerprint, ckpt_diff and ckpt_compact as three calls instead "
                         "of the fused ckpt_snapshot (hint = the previous step's mask)")
    ap.add_argument("--hint-cases", action="store_true",
                    help="time ckpt_snapshot with an exact hint, no hint and a hint with one wrong "
                         "chunk also when the main path is the three calls")
    ap.add_argument("--no-hint-cases", action="store_true",
                    help="skip the three-hint comparison (keeps a profiler's per-kernel averages "
                         "to the main path)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-gib", type=float, default=8.0)
    ap.add_argument("--match", action="store_true",
                    help="config 3 only: also run the content-addressed match on a snapshot whose "
                         "buffer list is rotated by one (every unchanged chunk sits at another "
                         "position), and the device-to-device moves that rebuild it")
    ap.add_argument("--swap", action="store_true",
                    help="also swap the last replica's delta out to pinned host memory and back in "
                         "(ckpt_swap_out / ckpt_swap_in through a small device ring)")
    ap.add_argument("--swap-slice-mib", type=int, default=256)
    ap.add_argument("--switch", action="store_true",
                    help="config 4 only: also time whole context switches between four time-sliced "
                         "ranks that share one device image (swap-out of the outgoing rank's delta "
                         "to pinned host memory, swap-in of the incoming rank's, no host read)")
    ap.add_argument("--chain", action="store_true",
                    help="--config 4 or --config 3: also restore a chain of three deltas, one "
                         "ckpt_restore_counted per link against one ckpt_restore_chain over all of "
                         "them, and fold the chain into one link (ckpt_merge_chain)")
    ap.add_argument("--graph", action="store_true",
                    help="also capture the step in HIP graphs (snapshot part, restore part) and "
                         "time their replays: what a launch-bound small state gains")
    ap.add_argument("--probe", action="store_true",
                    help="also run the side measurements the design notes cite: the hinted pass as "
                         "one launch against two, plain and 16-streams-per-wavefront copy and read "
                         "rates, and the fingerprint over one buffer for chunk sizes 256 B - 64 MiB")
    ap.add_argument("--calibrate", action="store_true",
                    help="also time the plain read and copy kernels on 8 GiB (HBM ceiling, and "
                         "the known-size dispatches that scale the rocprofv3 byte counters) and "
                         "the XXH64 arithmetic alone (integer ceiling)")
    return ap.parse_args()


class Replica:
    plan_create_ms = []        # one entry per plan built (host geometry + table upload)

    def __init__(self, w, arena, offs, ck):
        self.arena = arena
        base = arena.data_ptr()
        self.desc = [(base + int(o), b.nbytes) for o, b in zip(offs, w.bufs)]
        self.offs = offs
        t0 = time.perf_counter()
        self.plan = ck.Plan(self.desc, w.chunk)
        Replica.plan_create_ms.append((time.perf_counter() - t0) * 1e3)


def read_traffic_note(kernel: str, workload: str):
    """HBM bytes per launch of `kernel` measured with rocprofv3 --pmc (FETCH_SIZE and
    WRITE_SIZE runs), kept as text under profiles/.  None when no such record exists."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{kernel}_{workload}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1]), os.path.relpath(path, ROOT)
    except OSError:
        pass
    return None, None


def cpu_baseline(w, rep_ref, rep_new, sample_bytes, torch):
    """The oracle, as it stands, on a bounded sample of the same workload: every
    s-th buffer of the list (so shared and per-replica buffers keep their mix)."""
    import numpy as np
    import oracle

    total = w.nbytes
    stride = max(1, int(round(total / max(1, sample_bytes))))
    idx = list(range(0, len(w.bufs), stride))
    if w.distinct_bytes and not any(not w.bufs[i].shared for i in idx):
        idx.append(next(i for i, b in enumerate(w.bufs) if not b.shared))
        idx.sort()

    def fetch(rep):
        out = []
        for i in idx:
            o, n = int(rep.offs[i]), w.bufs[i].nbytes
            out.append(rep.arena[o:o + n].cpu().numpy())
        return out

    h_ref, h_new = fetch(rep_ref), fetch(rep_new)
    nbytes = sum(b.size for b in h_new)
    threads = len(os.sched_getaffinity(0))
    t0 = time.perf_counter()
    ref = oracle.fingerprint(h_ref, w.chunk, threads)
    dig = oracle.fingerprint(h_new, w.chunk, threads)
    mask, cnt = oracle.diff(h_new, w.chunk, dig, ref)
    staging, man, cnt2 = oracle.compact(h_new, w.chunk, mask, dig)
    dt = time.perf_counter() - t0
    hashed = sum(b.size for b in h_ref) + nbytes
    return {
        "value": hashed / dt / 1e9,
        "unit": "GB/s of device state (fingerprint on all threads + diff + compact on one thread)",
        "cores": threads, "kind": "oracle",
        "sample": f"every {stride}th buffer of both replicas: {len(idx)} buffers, "
                  f"{hashed / 2**30:.2f} GiB fingerprinted, {cnt2['staged_bytes'] / 2**30:.2f} GiB "
                  f"staged, {dt:.2f} s wall (fingerprint on {threads} threads, rest on one)",
    }, (idx, dig, mask)


def host_swap_leg(w, rep, dig, mask, manifest, d_staging, staged, ndirty, ck, torch, slice_bytes):
    """Swap-out of the replica's delta to pinned host memory and swap-in back, each timed on
    the host clock (the calls block until the data has landed).  The host image must equal
    the device staging buffer that ckpt_compact produced for the same mask."""
    host = torch.empty(max(16, staged), dtype=torch.uint8, pin_memory=True)
    # the device staging buffer is the yardstick below; other legs use it as scratch, so fill it
    fresh = torch.zeros(3, dtype=torch.int64, device=mask.device)
    ck.compact(rep.plan, mask, dig, d_staging, manifest, fresh, staging_cap=staged,
               manifest_cap=ndirty)
    sw = ck.Swapper(slice_bytes)
    t = {}
    for name in ("warm", "timed"):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        cnt = sw.swap_out(rep.plan, mask, dig, host, manifest, staging_cap=staged,
                          manifest_cap=ndirty)
        t[name + "_out"] = time.perf_counter() - t0
        assert cnt["status"] == 0 and cnt["staged_bytes"] == staged
        t0 = time.perf_counter()
        rejected = sw.swap_in(rep.plan, host, staged, manifest, ndirty)
        t[name + "_in"] = time.perf_counter() - t0
        assert rejected == 0
    same = True
    step = 1 << 30
    for lo in range(0, staged, step):
        hi = min(staged, lo + step)
        same = same and bool(torch.equal(host[lo:hi], d_staging[lo:hi].cpu()))
    assert same, "host image differs from the device staging buffer"
    sw.close()
    # the same swap with no ring: the staging pointer of ckpt_compact / ckpt_restore is the
    # pinned host buffer itself, the kernels move the bytes over the host link
    host.fill_(0)
    counts = torch.zeros(3, dtype=torch.int64, device=mask.device)
    rejected = torch.zeros(1, dtype=torch.int64, device=mask.device)
    for name in ("warm", "timed"):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ck.compact(rep.plan, mask, dig, host, manifest, counts, staging_cap=staged,
                   manifest_cap=ndirty)
        torch.cuda.synchronize()
        t[name + "_zc_out"] = time.perf_counter() - t0
        t0 = time.perf_counter()
        ck.restore(rep.plan, host, staged, manifest, ndirty, rejected)
        torch.cuda.synchronize()
        t[name + "_zc_in"] = time.perf_counter() - t0
    assert int(rejected.item()) == 0 and int(counts[1].item()) == staged
    for lo in range(0, staged, step):
        hi = min(staged, lo + step)
        same = same and bool(torch.equal(host[lo:hi], d_staging[lo:hi].cpu()))
    assert same, "host image written by ckpt_compact differs from the device staging buffer"
    return {
        "staged_bytes": staged, "state_bytes": w.nbytes, "slice_bytes": slice_bytes,
        "device_ring_bytes": 2 * slice_bytes,
        "swap_out_ms": round(t["timed_out"] * 1e3, 1), "swap_in_ms": round(t["timed_in"] * 1e3, 1),
        "swap_out_GBps": round(staged / t["timed_out"] / 1e9, 1),
        "swap_in_GBps": round(staged / t["timed_in"] / 1e9, 1),
        "naive_full_state_ms_at_same_rate": round(w.nbytes / (staged / t["timed_out"]) * 1e3, 1),
        "kernel_writes_pinned_host": {
            "swap_out_ms": round(t["timed_zc_out"] * 1e3, 1),
            "swap_in_ms": round(t["timed_zc_in"] * 1e3, 1),
            "swap_out_GBps": round(staged / t["timed_zc_out"] / 1e9, 1),
            "swap_in_GBps": round(staged / t["timed_zc_in"] / 1e9, 1)},
        "host_image_equals_device_staging": same,
    }


def graph_leg(step_calls, restore_calls, bytes_fp, args, torch):
    """The same calls captured in two HIP graphs and replayed: the library only enqueues kernels,
    so a whole snapshot is one graph launch.  Times are per replay, from events around it."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graphs = []
    with torch.cuda.stream(side):
        for calls in (step_calls, restore_calls):
            calls()                                   # eager once on the capture stream
            side.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=side):
                calls()
            graphs.append(g)
    torch.cuda.synchronize()
    times = {"snapshot": [], "restore": []}
    for it in range(args.warmup + args.steps):
        for name, g in zip(("snapshot", "restore"), graphs):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            g.replay()
            e1.record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                times[name].append(e0.elapsed_time(e1))
    snap = sum(times["snapshot"]) / len(times["snapshot"])
    return {"snapshot_ms": round(snap, 4),
            "restore_ms": round(sum(times["restore"]) / len(times["restore"]), 4),
            "value_GBps": round(bytes_fp / snap / 1e6, 1)}


def content_addressed_leg(w, t0, t1, ref, ck, torch, np, steps):
    """Snapshot = t1's bytes described by a buffer list rotated by one buffer, so the
    positional diff against t0 finds almost nothing while every unchanged chunk is
    still present in t0 at another position.  Times ckpt_match, then rebuilds the
    snapshot in a fresh arena from staging + moves and checks it byte for byte."""
    dev = t1.arena.device
    order = list(range(1, len(w.bufs))) + [0]
    base1 = t1.arena.data_ptr()
    rot = ck.Plan([(base1 + int(t1.offs[i]), w.bufs[i].nbytes) for i in order], w.chunk)
    n = rot.nchunks
    dig = torch.zeros(n, dtype=torch.int64, device=dev)
    mask = torch.zeros(n, dtype=torch.uint8, device=dev)
    pmask = torch.zeros(n, dtype=torch.uint8, device=dev)
    src = torch.zeros(n, dtype=torch.int64, device=dev)
    cnt = torch.zeros(3, dtype=torch.int64, device=dev)
    mcnt = torch.zeros(6, dtype=torch.int64, device=dev)
    ws = torch.empty(ck.match_workspace_bytes(n, n), dtype=torch.uint8, device=dev)
    ck.fingerprint(rot, dig)
    ck.diff(rot, dig, ref, pmask, cnt)
    ck.match(rot, dig, ref, ws, src, mask, mcnt)
    torch.cuda.synchronize()
    positional = cnt.cpu().numpy().view(np.uint64)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        ck.match(rot, dig, ref, ws, src, mask, mcnt)
    e1.record()
    torch.cuda.synchronize()
    match_ms = e0.elapsed_time(e1) / steps
    m = dict(zip(ck.MATCH_COUNT_FIELDS, (int(v) for v in mcnt.cpu().numpy().view(np.uint64))))
    staging = torch.empty(max(16, m["staged_bytes"]), dtype=torch.uint8, device=dev)
    manifest = torch.empty(max(1, m["nnew"]) * 32, dtype=torch.uint8, device=dev)
    ck.compact(rot, mask, dig, staging, manifest, cnt, staging_cap=m["staged_bytes"],
               manifest_cap=m["nnew"])
    fresh = torch.full_like(t1.arena, 0x5C)
    dst = ck.Plan([(fresh.data_ptr() + int(t1.offs[i]), w.bufs[i].nbytes) for i in order], w.chunk)
    rej = torch.zeros(1, dtype=torch.int64, device=dev)
    torch.cuda.synchronize()
    e0.record()
    ck.restore(dst, staging, m["staged_bytes"], manifest, m["nnew"])
    ck.apply_matches(dst, t0.plan, src, rej)
    e1.record()
    torch.cuda.synchronize()
    rebuild_ms = e0.elapsed_time(e1)
    assert int(rej.item()) == 0 and m["table_full"] == 0
    assert torch.equal(fresh, t1.arena), "content-addressed rebuild differs from the snapshot"
    moved_bytes = w.nbytes - m["staged_bytes"]
    return {
        "chunks": n, "match_ms": round(match_ms, 3),
        "match_Mchunks_per_s": round(n / match_ms / 1e3, 1),
        "classes": {k: m[k] for k in ("nsame", "nmoved", "ndup", "nnew")},
        "staged_bytes_content_addressed": m["staged_bytes"],
        "staged_bytes_positional": int(positional[1]),
        "rebuild_ms": round(rebuild_ms, 3),
        "rebuild_GBps_read_plus_write": round(2 * w.nbytes / rebuild_ms / 1e6, 1),
        "moved_or_duplicated_bytes": moved_bytes, "rebuild_matches_snapshot": True,
    }


def hint_cases_leg(w, rep, ref, staged, ndirty, ck, torch, np, args):
    """ckpt_snapshot of one replica under the three hints a caller can have, each timed on its
    own with events around the call: (i) the exact hint (the steady state of a context switch),
    (ii) no hint (the first snapshot: plain pass + gather), (iii) the exact hint with one wrong
    chunk in the middle (the pass, then a gather of the staged chunks behind the miss).
    Fractions: `of_peak_on_moved_bytes` counts the bytes each case really moves,
    `of_peak_vs_two_pass` the (1 + 2d) S a fingerprint followed by a gather has to move."""
    dev = rep.arena.device
    n, S = w.nchunks, w.nbytes
    dig = torch.zeros(n, dtype=torch.int64, device=dev)
    mask = torch.zeros(n, dtype=torch.uint8, device=dev)
    cnt = torch.zeros(3, dtype=torch.int64, device=dev)
    miss = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = torch.empty(ck.snapshot_workspace_bytes(n), dtype=torch.uint8, device=dev)
    staging = torch.empty(max(16, staged), dtype=torch.uint8, device=dev)
    manifest = torch.empty(max(1, ndirty) * 32, dtype=torch.uint8, device=dev)
    ck.fingerprint(rep.plan, dig)
    ck.diff(rep.plan, dig, ref, mask, cnt)
    exact = mask.clone()
    wrong = exact.clone()
    wrong[n // 2] ^= 1
    ev = torch.cuda.Event
    out = {}
    for name, hint in (("exact_hint", exact), ("no_hint", None), ("one_wrong_chunk_mid", wrong)):
        ms = []
        for it in range(args.warmup + args.steps):
            e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
            e0.record()
            ck.snapshot(rep.plan, ref, hint, dig, mask, staging, manifest, cnt, miss,
                        ws if hint is not None else None, staging_cap=staged, manifest_cap=ndirty)
            e1.record()
            torch.cuda.synchronize()
            if it >= args.warmup:
                ms.append(e0.elapsed_time(e1))
        c = cnt.cpu().numpy().view(np.uint64)
        assert (int(c[0]), int(c[1]), int(c[2])) == (ndirty, staged, 0), (name, c)
        stats = ck.snapshot_stats(ws, n) if hint is not None else \
            {"hint_misses": 0, "regathered_chunks": ndirty}
        regathered_bytes = staged * stats["regathered_chunks"] / max(1, ndirty)
        moved = S + (staged if hint is not None else 0) + 2 * regathered_bytes
        mean = float(np.mean(ms))
        out[name] = {
            "snapshot_ms_mean": round(mean, 4), "snapshot_ms_min": round(min(ms), 4),
            "hint_misses": stats["hint_misses"], "regathered_chunks": stats["regathered_chunks"],
            "bytes_moved": int(moved),
            "of_peak_on_moved_bytes": round(moved / mean / 1e6 / HBM_PEAK_GBPS, 4),
            "of_peak_vs_two_pass": round((S + 2 * staged) / mean / 1e6 / HBM_PEAK_GBPS, 4),
        }
    return out


def context_switch_leg(w, replicas, ref, ck, wl, torch, np, args):
    """Round robin of four time-sliced ranks over ONE device image (paper sec. 5.1, 5.2.1, 6):
    per switch the outgoing rank's delta against the shared base goes to pinned host memory
    (checksum, compare, gather kernel writing over the host link) and the incoming rank's delta
    comes back (counted restore reading from pinned host memory); the next rank's first kernel
    waits on another stream behind one event; the host reads nothing.  Ranks = replicas 1..3
    and a fourth generated here; base = replica 0 (the state all ranks share)."""
    from paper_2202_07848_amd.switching import TimeSlicedRanks

    dev = replicas[0].arena.device
    nranks = 4
    S, n = w.nbytes, w.nchunks
    cap_bytes, cap_entries = w.distinct_bytes, w.distinct_chunks
    # the image starts as a copy of rank 0 (= replica 1); the library sees only this arena
    image = replicas[1].arena.clone()
    offs = replicas[1].offs
    plan = ck.Plan([(image.data_ptr() + int(o), b.nbytes) for o, b in zip(offs, w.bufs)], w.chunk)
    sw = TimeSlicedRanks(plan, ref, nranks, cap_bytes, cap_entries, dev, exact=True)
    # exact mode keeps a full copy of the base in host memory: taken while the base is resident
    image.copy_(replicas[0].arena)
    base_copy = "pinned host memory"
    try:
        sw.capture_base()
    except RuntimeError:        # the machine's limit on pinned memory (four rank areas are pinned too)
        torch.cuda.synchronize()
        sw.capture_base(pinned_host=False)
        base_copy = "device memory (pinned host allocation refused); not read in this workload"
    image.copy_(replicas[1].arena)
    states = [replicas[1].arena, replicas[2].arena, replicas[3].arena]
    extra, _ = wl.torch_replica(w, 4, dev, shared_from=replicas[0].arena)
    states.append(extra)
    # every rank has been resident once: its delta is in its host area
    for r in range(1, nranks):
        image.copy_(states[r])
        sw.swap_out(r)
    image.copy_(states[0])
    torch.cuda.synchronize()
    assert sw.same_dirty_set(list(range(1, nranks)))
    side = torch.cuda.Stream()
    token = torch.zeros(1, dtype=torch.int64, device=dev)
    ev = torch.cuda.Event
    rounds, ok, modes = 2, True, {}
    for mode, exchange in (("swap_out_then_swap_in", False), ("exchange_pass", True),
                           ("exact_for_any_change_sets", None),
                           ("exact_exchange_then_repair", "exact")):
        ms, wall_ms, enq_ms, serial = [], [], [], 0
        resident = 0
        for step in range(rounds * nranks):
            nxt = (resident + 1) % nranks
            e0, e1, e2 = ev(enable_timing=True), ev(enable_timing=True), ev(enable_timing=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            e0.record()
            if exchange is None:
                sw.switch_exact(resident, nxt)
            elif exchange == "exact":
                sw.switch_exact(resident, nxt, exchange=True)
            else:
                sw.switch(resident, nxt, exchange=exchange)
            e1.record()
            with torch.cuda.stream(side):
                side.wait_event(e1)
                token.add_(1)                 # the incoming rank's first kernel
                e2.record()
            enq_ms.append((time.perf_counter() - t0) * 1e3)
            torch.cuda.synchronize()
            wall_ms.append((time.perf_counter() - t0) * 1e3)
            ms.append(e0.elapsed_time(e1))
            serial += int(sw.serial.item()) if exchange is not None else 0
            if step < nranks:             # first rotation: the image is the incoming rank's state
                ok = ok and bool(torch.equal(image, states[nxt]))
            resident = nxt
        assert ok and int(sw.rejected.item()) == 0 and serial == 0
        staged = int(sw.counts[0].cpu().numpy().view(np.uint64)[1])
        timed = ms[nranks:]                   # second rotation: everything warm
        mean = float(np.mean(timed))
        modes[mode] = {
            "switch_ms_mean": round(mean, 2), "switch_ms_min": round(min(timed), 2),
            "switch_wall_ms_mean": round(float(np.mean(wall_ms[nranks:])), 2),
            "host_enqueue_ms_mean": round(float(np.mean(enq_ms[nranks:])), 3),
            "host_link_GBps_both_directions": round(2 * staged / mean / 1e6, 1),
        }
    assert int(token.item()) == len(modes) * rounds * nranks
    slow = modes["swap_out_then_swap_in"]["switch_ms_mean"]
    return {
        "workload": f"config{w.config}_{w.name}: {nranks} ranks round robin on one device image",
        "state_bytes_per_rank": S, "delta_bytes_per_rank": staged,
        "host_link_bytes_per_switch": 2 * staged,
        **modes,
        "full_state_swap_ms_at_the_one_way_rate": round(2 * S / (2 * staged / slow), 1),
        "image_equals_incoming_rank_after_each_switch": ok,
        "exact_mode_base_copy": base_copy,
        "paper_context": "sec. 5.2: swapping 32 GB out and in without de-duplication costs 2-4 s "
                         "per mini-batch on the paper's V100 hosts",
    }


def chain_leg(w, replicas, pairs, ref, stagings, manifests, ck, wl, torch, np, args):
    """Restore from a chain of incremental snapshots (paper sec. 4.6), link by link against
    ckpt_restore_chain, which writes every chunk once, and ckpt_merge_chain.
    Replica configurations: the links are the deltas of replicas 1, 2, ... against the reference;
    every link holds the same chunks (the per-replica gradients and activations), as the steps
    of one job do.  Config 3: three more rounds of scattered rewrites (--dirty of the chunks each,
    a fresh seeded set per round) on a copy of the rewritten state; every link is the delta
    against the state before it, so the links hold different, partly overlapping chunk sets."""
    dev = ref.device
    n = w.nchunks
    dig = torch.zeros(n, dtype=torch.int64, device=dev)
    mask = torch.zeros(n, dtype=torch.uint8, device=dev)
    links, staged = [], []
    if w.nreplicas >= 3:
        final = pairs[-1][1].arena
        for (_, rep), staging, manifest in zip(pairs, stagings, manifests):
            cnt = torch.zeros(3, dtype=torch.int64, device=dev)
            ck.fingerprint(rep.plan, dig)
            ck.diff(rep.plan, dig, ref, mask, cnt)
            ck.compact(rep.plan, mask, dig, staging, manifest, cnt, staging_cap=staging.numel(),
                       manifest_cap=manifest.numel() // 32)
            torch.cuda.synchronize()
            assert int(cnt[2]) == 0
            staged.append(int(cnt[1]))
            links.append((staging, int(cnt[1]), manifest, manifest.numel() // 32, cnt))
    else:
        final = replicas[0].arena.clone()
        state = Replica(w, final, replicas[0].offs, ck)
        prev = ref.clone()
        for rnd in range(3):
            step = int(args.dirty * 100) + 1000 * (rnd + 1)
            ids = wl.dirty_chunk_ids(w, args.dirty, step)
            wl.torch_rewrite_chunks(w, final, replicas[0].offs, ids, step)
            cnt = torch.zeros(3, dtype=torch.int64, device=dev)
            ck.fingerprint(state.plan, dig)
            ck.diff(state.plan, dig, prev, mask, cnt)
            torch.cuda.synchronize()
            nd, nb = int(cnt[0]), int(cnt[1])
            assert nd == ids.size
            staging = torch.empty(max(16, nb), dtype=torch.uint8, device=dev)
            manifest = torch.empty(max(1, nd) * 32, dtype=torch.uint8, device=dev)
            ck.compact(state.plan, mask, dig, staging, manifest, cnt, staging_cap=nb, manifest_cap=nd)
            torch.cuda.synchronize()
            staged.append(nb)
            links.append((staging, nb, manifest, nd, cnt))
            prev.copy_(dig)
    image = replicas[0].arena.clone()
    plan = ck.Plan([(image.data_ptr() + int(o), b.nbytes) for o, b in zip(replicas[0].offs, w.bufs)],
                   w.chunk)
    ws = torch.empty(ck.restore_chain_workspace_bytes(n), dtype=torch.uint8, device=dev)
    stats = torch.zeros(3, dtype=torch.int64, device=dev)

    def one_by_one():
        for staging, nbytes, manifest, cap, cnt in links:
            ck.restore_counted(plan, staging, nbytes, manifest, cap, cnt)

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        assert torch.equal(image, final)
        image.copy_(replicas[0].arena)
        fn()
        e0, e1 = (torch.cuda.Event(enable_timing=True) for _ in range(2))
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ms_each = timed(one_by_one)
    ms_chain = timed(lambda: ck.restore_chain(plan, links, ws, stats))
    written, superseded, rejected = (int(x) for x in stats.cpu().numpy().view(np.uint64))
    assert rejected == 0 and superseded == sum(int(l[4][0]) for l in links) - written

    # the same chain folded into one link (ckpt_merge_chain), then that link restored
    m_staging = torch.empty(sum(staged), dtype=torch.uint8, device=dev)
    m_manifest = torch.empty(written * 32, dtype=torch.uint8, device=dev)
    m_counts = torch.zeros(3, dtype=torch.int64, device=dev)
    m_ws = torch.empty(ck.merge_chain_workspace_bytes(n), dtype=torch.uint8, device=dev)

    def merge():
        ck.merge_chain(plan, links, m_staging, m_manifest, m_counts, m_ws)

    merge()
    e0, e1 = (torch.cuda.Event(enable_timing=True) for _ in range(2))
    e0.record()
    for _ in range(5):
        merge()
    e1.record()
    torch.cuda.synchronize()
    ms_merge = e0.elapsed_time(e1) / 5
    mc = [int(x) for x in m_counts.cpu().numpy().view(np.uint64)]
    assert mc[0] == written and mc[2] == 0 and mc[1] <= sum(staged), mc
    image.copy_(replicas[0].arena)
    ck.restore_counted(plan, m_staging, mc[1], m_manifest, written, m_counts)
    torch.cuda.synchronize()
    assert torch.equal(image, final)
    return {
        "workload": f"config{w.config}_{w.name}: chain of {len(links)} deltas restored into a copy "
                    "of the reference state",
        "links": len(links), "bytes_per_link": staged,
        "chunks_written": written, "entries_superseded": superseded,
        "one_restore_per_link_ms": round(ms_each, 3),
        "restore_chain_ms": round(ms_chain, 3),
        "speedup": round(ms_each / ms_chain, 2),
        "restore_chain_hbm_GBps_read_plus_write": round(2 * mc[1] / ms_chain / 1e6, 1),
        "merge_chain_ms": round(ms_merge, 3),
        "merge_chain_hbm_GBps_read_plus_write": round(2 * mc[1] / ms_merge / 1e6, 1),
        "merged_link_bytes": mc[1],
        "image_equals_last_state": True,
    }


def probe_leg(w, rep, ref, staging, staged, ndirty, ck, torch, np, args):
    """The measurements the design notes lean on, each through the C ABI so that they can be
    repeated from this file: (a) the hinted snapshot pass as one launch against two (staging
    groups first, then the rest); (b) copy and read rates of plain streaming kernels against
    the fingerprint pass's access pattern (16 streams per wavefront, 256 bytes of each per
    step), on as many streams of one chunk's size as the snapshot stages chunks; (c) the plain
    fingerprint over one large buffer for chunk sizes from 256 B to 64 MiB."""
    dev = rep.arena.device
    ev = torch.cuda.Event
    n = w.nchunks

    def timed(fn, reps=5):
        fn()
        e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    out = {}
    # (a) one launch against two
    dig = torch.zeros(n, dtype=torch.int64, device=dev)
    mask = torch.zeros(n, dtype=torch.uint8, device=dev)
    cnt = torch.zeros(3, dtype=torch.int64, device=dev)
    ws = torch.empty(ck.snapshot_workspace_bytes(n), dtype=torch.uint8, device=dev)
    manifest = torch.empty(max(1, ndirty) * 32, dtype=torch.uint8, device=dev)
    ck.fingerprint(rep.plan, dig)
    ck.diff(rep.plan, dig, ref, mask, cnt)
    hint = mask.clone()
    before = rep.plan.split_threshold
    shapes = {}
    for name, thr in (("one_launch", 2**64 - 1), ("two_launches", 0)):
        rep.plan.split_threshold = thr
        shapes[name + "_ms"] = round(timed(lambda: ck.snapshot(
            rep.plan, ref, hint, dig, mask, staging, manifest, cnt, None, ws,
            staging_cap=staged, manifest_cap=ndirty)), 4)
    rep.plan.split_threshold = before
    out["hinted_pass_launch_shape"] = shapes

    # (b) access patterns; the copy goes from the replica's arena into the staging buffer
    stream_bytes = max(2048, w.chunk)
    nstreams = min(staged, rep.arena.numel()) // stream_bytes // 16 * 16
    if nstreams:
        nb = nstreams * stream_bytes
        sink = torch.zeros(4096, dtype=torch.int64, device=dev)
        pat = {"bytes": nb, "streams": nstreams, "stream_bytes": stream_bytes}
        for name, fn, factor in (
                ("sweep_copy", lambda: ck.bw_copy(staging, rep.arena, nb), 2),
                ("stream_copy", lambda: ck.bw_streams(staging, rep.arena, nstreams, stream_bytes,
                                                      sink), 2),
                ("sweep_read", lambda: ck.bw_read(rep.arena, nb, sink), 1),
                ("stream_read", lambda: ck.bw_streams(None, rep.arena, nstreams, stream_bytes,
                                                      sink), 1),
                ("stream_copy_1KiB_tiles", lambda: ck.bw_streams(
                    staging, rep.arena, nstreams, stream_bytes, sink, tile_bytes=1024), 2),
                ("stream_read_1KiB_tiles", lambda: ck.bw_streams(
                    None, rep.arena, nstreams, stream_bytes, sink, tile_bytes=1024), 1)):
            ms = timed(fn)
            pat[name] = {"ms": round(ms, 4), "GBps_read_plus_write": round(factor * nb / ms / 1e6, 1)}
        out["access_patterns"] = pat

    # (c) chunk size against parallelism: one buffer, every chunk size
    big = min(rep.arena.numel(), 24 << 30) // (64 << 20) * (64 << 20)
    if big:
        sweep = {}
        base = rep.arena.data_ptr()
        for log2 in (8, 10, 12, 14, 16, 18, 20, 22, 24, 26):
            c = 1 << log2
            plan = ck.Plan([(base, big)], c)
            d = torch.zeros(plan.nchunks, dtype=torch.int64, device=dev)
            ms = timed(lambda: ck.fingerprint(plan, d), reps=3)
            sweep[str(c)] = {"chunks": plan.nchunks, "ms": round(ms, 3),
                             "GBps": round(big / ms / 1e6, 1)}
            plan.close()
        out["fingerprint_chunk_size_sweep"] = {"buffer_bytes": big, "by_chunk_bytes": sweep}
    return out


def phase_names(d, fused):
    """With the fused call there is one snapshot phase instead of three."""
    if not fused:
        return d
    return {"fingerprint_ref": d["fingerprint_ref"], "snapshot_fused": d["fingerprint"],
            "restore": d["restore"]}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path shards per device with no "
              "exchange); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2202_07848_amd import binding as ck
    from paper_2202_07848_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = wl.config(args.config, args.shrink)
    t_gen = time.perf_counter()

    Replica.plan_create_ms.clear()
    replicas = []
    if w.nreplicas >= 2:
        for r in range(w.nreplicas):
            arena, offs = wl.torch_replica(w, r, dev, shared_from=replicas[0].arena if r else None)
            replicas.append(Replica(w, arena, offs, ck))
        pairs = [(replicas[0], replicas[r]) for r in range(1, w.nreplicas)]
        fingerprinted = w.nreplicas
        expect_dirty = w.distinct_chunks
    else:
        arena0, offs = wl.torch_replica(w, 0, dev)
        t0 = Replica(w, arena0, offs, ck)
        arena1 = arena0.clone()
        t1 = Replica(w, arena1, offs, ck)
        ids = wl.dirty_chunk_ids(w, args.dirty, int(args.dirty * 100))
        wl.torch_rewrite_chunks(w, arena1, offs, ids, int(args.dirty * 100))
        replicas = [t0, t1]
        pairs = [(t0, t1)]
        fingerprinted = 1
        expect_dirty = int(ids.size)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen

    n = w.nchunks
    S = w.nbytes
    ref = torch.zeros(n, dtype=torch.int64, device=dev)
    digs = [torch.zeros(n, dtype=torch.int64, device=dev) for _ in pairs]
    masks = [torch.zeros(n, dtype=torch.uint8, device=dev) for _ in pairs]
    counts = [torch.zeros(3, dtype=torch.int64, device=dev) for _ in pairs]

    # size staging from a first diff (part of set-up, like plan creation)
    ck.fingerprint(pairs[0][0].plan, ref)
    staged, ndirty = [], []
    for (a, b), dig, mask, cnt in zip(pairs, digs, masks, counts):
        ck.fingerprint(b.plan, dig)
        ck.diff(b.plan, dig, ref, mask, cnt)
    torch.cuda.synchronize()
    for cnt in counts:
        ndirty.append(int(cnt[0]))
        staged.append(int(cnt[1]))
    assert all(x == expect_dirty for x in ndirty), (ndirty, expect_dirty)
    stagings = [torch.empty(max(16, s), dtype=torch.uint8, device=dev) for s in staged]
    manifests = [torch.empty(max(1, k) * 32, dtype=torch.uint8, device=dev) for k in ndirty]

    ev = torch.cuda.Event
    # The single-pass snapshot (hint = the previous snapshot's mask) pays off when a good part
    # of the state is staged: measured against the three separate calls it is ahead from 10 %
    # when whole buffers differ (configs 2, 4, 5) and from somewhere between 10 % and 50 % when
    # the dirty 4 KiB chunks are scattered (config 3).  Use it from 20 % upwards, which the
    # caller knows from the previous snapshot's counts.
    fused = not args.separate and sum(staged) >= args.fused_from * S * len(pairs)
    misses = [torch.zeros(1, dtype=torch.int64, device=dev) for _ in pairs]
    spaces = [torch.empty(ck.snapshot_workspace_bytes(n), dtype=torch.uint8, device=dev)
              for _ in pairs] if fused else None

    nmarks = 2 + 4 * len(pairs)

    def step(marks):
        """One step; marks: pre-created events, recorded in order (a phase boundary each)."""
        it = iter(marks)
        next(it).record()
        if w.nreplicas >= 2:
            ck.fingerprint(pairs[0][0].plan, ref)
        next(it).record()
        for i, (a, b) in enumerate(pairs):
            if fused:
                # one call; the mask of the previous step (same buffer) is the hint
                ck.snapshot(b.plan, ref, masks[i], digs[i], masks[i], stagings[i], manifests[i],
                            counts[i], misses[i], spaces[i], staging_cap=staged[i],
                            manifest_cap=ndirty[i])
                next(it).record()
                next(it).record()
            else:
                ck.fingerprint(b.plan, digs[i])
                next(it).record()
                ck.diff(b.plan, digs[i], ref, masks[i], counts[i])
                next(it).record()
                ck.compact(b.plan, masks[i], digs[i], stagings[i], manifests[i], counts[i],
                           staging_cap=staged[i], manifest_cap=ndirty[i])
            next(it).record()
            ck.restore(b.plan, stagings[i], staged[i], manifests[i], ndirty[i])
            next(it).record()
        return marks

    def step_calls():          # the measured part of a step, no events: for graph capture
        if w.nreplicas >= 2:
            ck.fingerprint(pairs[0][0].plan, ref)
        for i, (a, b) in enumerate(pairs):
            if fused:
                ck.snapshot(b.plan, ref, masks[i], digs[i], masks[i], stagings[i], manifests[i],
                            counts[i], misses[i], spaces[i], staging_cap=staged[i],
                            manifest_cap=ndirty[i])
            else:
                ck.fingerprint(b.plan, digs[i])
                ck.diff(b.plan, digs[i], ref, masks[i], counts[i])
                ck.compact(b.plan, masks[i], digs[i], stagings[i], manifests[i], counts[i],
                           staging_cap=staged[i], manifest_cap=ndirty[i])

    def restore_calls():
        for i, (a, b) in enumerate(pairs):
            ck.restore(b.plan, stagings[i], staged[i], manifests[i], ndirty[i])

    # events exist (and have been recorded once, in the warm-up) before the timed region, and the
    # collector stays out of it: a host hiccup between two enqueues would be timed as GPU work
    import gc
    all_marks = [[ev(enable_timing=True) for _ in range(nmarks)] for _ in range(args.steps)]
    for i in range(max(args.warmup, 1)):
        step(all_marks[i % args.steps])
    for marks in all_marks[max(args.warmup, 1):]:
        for e in marks:
            e.record()
    torch.cuda.synchronize()
    gc.collect()
    gc.disable()
    wall0 = time.perf_counter()
    for marks in all_marks:
        step(marks)
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    gc.enable()

    ph = {"fingerprint_ref": [], "fingerprint": [], "diff": [], "compact": [], "restore": []}
    for marks in all_marks:
        ph["fingerprint_ref"].append(marks[0].elapsed_time(marks[1]))
        fp = df = cp = rs = 0.0
        for i in range(len(pairs)):
            m = marks[1 + 4 * i: 6 + 4 * i]      # end of the previous phase + this pair's four
            fp += m[0].elapsed_time(m[1]); df += m[1].elapsed_time(m[2])
            cp += m[2].elapsed_time(m[3]); rs += m[3].elapsed_time(m[4])
        ph["fingerprint"].append(fp); ph["diff"].append(df)
        ph["compact"].append(cp); ph["restore"].append(rs)
    if fused:   # one call: its whole time sits in the first interval
        ph["fingerprint"] = [a + b + c for a, b, c in zip(ph["fingerprint"], ph["diff"], ph["compact"])]
        ph["diff"] = [0.0] * len(ph["diff"])
        ph["compact"] = [0.0] * len(ph["compact"])
    mean = {k: float(np.mean(v)) for k, v in ph.items()}
    med = {k: float(np.median(v)) for k, v in ph.items()}
    low = {k: float(np.min(v)) for k, v in ph.items()}

    for cnt, k, s in zip(counts, ndirty, staged):
        c = cnt.cpu().numpy().view(np.uint64)
        assert (int(c[0]), int(c[1]), int(c[2])) == (k, s, 0), c
    if fused:
        assert all(int(m.item()) == 0 for m in misses), "the hint was not exact in the last step"

    bytes_fp = S * fingerprinted if w.nreplicas >= 2 else S
    dirty_bytes = sum(staged)
    t_fdc = (mean["fingerprint_ref"] + mean["fingerprint"] + mean["diff"] + mean["compact"]) / 1e3
    value = bytes_fp / t_fdc / 1e9
    # what a fingerprint followed by a gather has to move, (1 + 2d) S per snapshot, and what the
    # path really moves: the fused pass reads S and writes d S, nothing twice
    two_pass_bytes = bytes_fp + 2 * dirty_bytes
    moved_path = bytes_fp + (dirty_bytes if fused else 2 * dirty_bytes)
    workload = f"config{w.config}_{w.name}"
    if fused:
        # dominant kernel: the fused fingerprint + stage pass, which the library runs as two
        # launches from 256 MiB of state (k_fingerprint<1>: the groups that stage chunks,
        # k_fingerprint<2>: the rest) and as one below (k_fingerprint<3>).  Its time is the
        # snapshot phase, which also holds the hint-offset, manifest and (idle) gather kernels:
        # events cannot separate kernels inside one call, and those are microseconds (profiles/).
        split = S >= pairs[0][1].plan.split_threshold
        kernel = "k_fingerprint<1>+k_fingerprint<2>" if split else "k_fingerprint<3>"
        launches = len(pairs)
        kernel_bytes = S + dirty_bytes / launches             # read S, write d S
        two_pass_kernel_bytes = S + 2 * dirty_bytes / launches
        fp_launch_ms = mean["fingerprint"] / launches
    else:
        kernel = "k_fingerprint<0>"
        launches = fingerprinted if w.nreplicas >= 2 else 1
        kernel_bytes = two_pass_kernel_bytes = S
        fp_launch_ms = (mean["fingerprint_ref"] + mean["fingerprint"]) / launches
    achieved = kernel_bytes / (fp_launch_ms / 1e3) / 1e9
    # counter-measured traffic of the same launches, from the rocprofv3 summaries under profiles/
    # (config 3's are per rewritten fraction)
    profiled = workload + (f"_dirty{int(round(args.dirty * 100)):02d}" if w.nreplicas == 1 else "")
    notes = [read_traffic_note(k.replace("<", "_").replace(">", ""), profiled)
             for k in kernel.split("+")]
    traffic = None if any(x[0] is None for x in notes) else sum(x[0] for x in notes)
    traffic_source = None if traffic is None else [x[1] for x in notes]

    out = {
        "metric": "device-state GB/s (fingerprint+diff+compact) and % of MI355X HBM peak",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(wall / args.steps * 1e3, 3),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {
            "workload": workload, "chunk_bytes": w.chunk, "replicas": w.nreplicas,
            "buffers": len(w.bufs), "bytes_per_replica": S, "chunks_per_replica": n,
            "dirty_chunks": ndirty, "staged_bytes": staged,
            "dirty_fraction": round(dirty_bytes / (S * len(pairs)), 4),
            "shrink": args.shrink,
            "path": "fused ckpt_snapshot, hint = previous mask (exact every step)" if fused else
                    "ckpt_fingerprint + ckpt_diff + ckpt_compact (three calls)",
        },
        # fraction of the 8 TB/s peak over fingerprint + diff + compact: on the bytes the path
        # really moves, and on the (1 + 2d) S of a fingerprint followed by a gather (equal
        # for the three calls; the fused pass moves less, so its second figure is an
        # effective rate, not a bandwidth)
        "hbm_frac_fp_diff_compact": round(moved_path / t_fdc / 1e9 / HBM_PEAK_GBPS, 4),
        "effective_hbm_frac_vs_two_pass": round(two_pass_bytes / t_fdc / 1e9 / HBM_PEAK_GBPS, 4),
        "bytes_moved": moved_path,
        "bytes_moved_two_pass": two_pass_bytes,
        # XXH64 costs two 64-bit multiplies per 8 input bytes; the rate the pass achieves, to set
        # beside the arithmetic-only ceiling that --calibrate measures
        "xxh64_u64_mul_per_s": round(bytes_fp / 4 / t_fdc, 0),
        "phases_ms_mean": phase_names({k: round(v, 4) for k, v in mean.items()}, fused),
        "phases_ms_median": phase_names({k: round(v, 4) for k, v in med.items()}, fused),
        "phases_ms_min": phase_names({k: round(v, 4) for k, v in low.items()}, fused),
        "restore_GBps_read_plus_write": round(2 * dirty_bytes / (mean["restore"] / 1e3) / 1e9, 1)
        if dirty_bytes else None,
        "compact_GBps_read_plus_write": round(2 * dirty_bytes / (mean["compact"] / 1e3) / 1e9, 1)
        if dirty_bytes and not fused else None,
        # set-up, outside the timed region: data generation, and plan creation on its own
        # (host chunk geometry + one table upload per plan; it matters for 100 000 buffers)
        "setup_s": round(t_gen, 1),
        "plan_create_ms": {"per_plan_mean": round(float(np.mean(Replica.plan_create_ms)), 3),
                           "per_plan_min": round(float(np.min(Replica.plan_create_ms)), 3),
                           "plans": len(Replica.plan_create_ms), "buffers_per_plan": len(w.bufs)},
        "roofline": {
            "kernel": kernel, "bound": "hbm", "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": traffic, "traffic_source": traffic_source,
            "algorithmic_bytes_per_launch": int(kernel_bytes), "launch_ms": round(fp_launch_ms, 4),
            "effective_frac_vs_two_pass": round(two_pass_kernel_bytes / (fp_launch_ms / 1e3) / 1e9
                                                / HBM_PEAK_GBPS, 4),
        },
    }
    if S < (1 << 30):
        # a state this small is bound by the chain of dependent kernels, not by bandwidth
        # (64 MiB also sits in the 256 MB last-level cache): report it as latency
        out["latency_us"] = {k: round(v * 1e3, 1) for k, v in
                             phase_names({k: v for k, v in low.items()}, fused).items()}
        out["latency_us"]["basis"] = "min over timed steps, per phase of one step"

    if (fused or args.hint_cases) and not args.no_hint_cases:
        out["hint_cases"] = hint_cases_leg(w, pairs[0][1], ref, staged[0], ndirty[0], ck, torch, np,
                                           args)

    # the paper's granularity next to ours: what a swap of whole differing buffers would move
    bdirty = torch.zeros(max(1, len(w.bufs)), dtype=torch.uint8, device=dev)
    bcounts = torch.zeros(2, dtype=torch.int64, device=dev)
    ck.buffer_verdicts(pairs[0][1].plan, masks[0], bdirty, bcounts)
    e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
    e0.record()
    for _ in range(5):
        ck.buffer_verdicts(pairs[0][1].plan, masks[0], bdirty, bcounts)
    e1.record()
    torch.cuda.synchronize()
    nb_diff, nb_bytes = (int(x) for x in bcounts.cpu().numpy().view(np.uint64))
    out["buffer_granularity"] = {
        "buffers_that_differ": nb_diff, "of_buffers": len(w.bufs),
        "bytes_if_whole_buffers_were_swapped": nb_bytes,
        "bytes_staged_at_chunk_granularity": staged[0],
        "chunking_saves": round(1.0 - staged[0] / nb_bytes, 4) if nb_bytes else 0.0,
        "verdicts_ms": round(e0.elapsed_time(e1) / 5, 4),
    }

    if args.graph:
        out["hip_graph"] = graph_leg(step_calls, restore_calls, bytes_fp, args, torch)

    if args.calibrate:
        nb = min(8 * 2**30, pairs[0][1].arena.numel() // 16 * 16, stagings[0].numel() // 16 * 16)
        src, dst = pairs[0][1].arena, stagings[0]
        sink = torch.zeros(4096, dtype=torch.int64, device=dev)
        cal = {}
        for name, fn in (("copy", lambda: ck.bw_copy(dst, src, nb)),
                         ("read", lambda: ck.bw_read(src, nb, sink))):
            fn()
            e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
            e0.record()
            for _ in range(5):
                fn()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 5
            cal[name] = {"bytes": nb, "ms": round(ms, 3),
                         "GBps": round((2 if name == "copy" else 1) * nb / ms / 1e6, 1)}
        # the hash arithmetic alone (no memory traffic): the integer units' ceiling for the pass
        hashed = ck.alu_xxh64(1 << 14, sink)
        e0, e1 = ev(enable_timing=True), ev(enable_timing=True)
        e0.record()
        for _ in range(5):
            ck.alu_xxh64(1 << 14, sink)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        cal["xxh64_alu_only"] = {"bytes_stood_for": hashed, "ms": round(ms, 3),
                                 "GBps": round(hashed / ms / 1e6, 1),
                                 "u64_mul_per_s": round(hashed / 4 / (ms / 1e3), 0)}
        out["calibration"] = cal

    if args.swap:
        out["host_swap"] = host_swap_leg(w, pairs[-1][1], digs[-1], masks[-1], manifests[-1],
                                         stagings[-1], staged[-1], ndirty[-1], ck, torch,
                                         args.swap_slice_mib << 20)

    if args.switch:
        if w.nreplicas < 4:
            raise SystemExit("--switch needs a configuration with four replicas (--config 4)")
        out["context_switch"] = context_switch_leg(w, replicas, ref, ck, wl, torch, np, args)

    if args.chain:
        if w.nreplicas == 2:
            raise SystemExit("--chain needs three or more replicas (--config 4) or config 3")
        out["restore_chain"] = chain_leg(w, replicas, pairs, ref, stagings, manifests, ck, wl, torch,
                                         np, args)

    if args.match and w.nreplicas == 1:
        out["content_addressed"] = content_addressed_leg(w, pairs[0][0], pairs[0][1], ref, ck, torch,
                                                         np, args.steps)

    if args.probe:        # last of the GPU legs: it uses the staging buffer as a copy target
        out["probe"] = probe_leg(w, pairs[0][1], ref, stagings[0], staged[0], ndirty[0], ck, torch,
                                 np, args)

    if not args.no_cpu_baseline:
        base, (idx, o_dig, o_mask) = cpu_baseline(w, pairs[0][0], pairs[0][1],
                                                  args.cpu_sample_gib * 2**30, torch)
        out["cpu_baseline"] = base
        # the sampled buffers' digests and masks must equal what the GPU produced
        buf, off, length = wl.chunk_table(w)
        sel = np.flatnonzero(np.isin(buf, np.array(idx)))
        g_dig = digs[0].cpu().numpy().view(np.uint64)[sel]
        g_mask = masks[0].cpu().numpy()[sel]
        out["cpu_baseline"]["sample_matches_gpu"] = bool(
            np.array_equal(g_dig, o_dig) and np.array_equal(g_mask, o_mask))
        assert out["cpu_baseline"]["sample_matches_gpu"], "GPU and oracle disagree on the sample"

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
