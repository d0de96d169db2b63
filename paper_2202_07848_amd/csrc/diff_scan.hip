// Checksum comparison and the prefix scan that orders the swap-out.
//
// diff: the comparison of a rank's checksums with the other rank's copy that
// the Singularity paper does on the host (sec. 6; sec. 5.2.1, 5.2.3) -- here a
// device kernel, one thread per four chunks.
//
// compact, metadata half: stable compaction.  Staging order must be ascending
// chunk id, so offsets come from an exclusive prefix sum over
// (mask, mask * pad16(len)) pairs, in deterministic steps with no workgroup
// ever waiting for another and no memory fence inside a kernel (a device-scope
// fence writes back and invalidates the L2 of the XCD that issues it: measured
// with 6 000 workgroups, one fence each turned a 50 us kernel into 500 us):
//   * above SMALL_SCAN_CHUNKS chunks: per-workgroup sums, a single-workgroup
//     scan of those sums, then a per-workgroup rescan that writes the manifest;
//   * up to SMALL_SCAN_CHUNKS chunks one kernel does it all: a workgroup gets
//     its offset by counting the mask bytes in front of its block itself (at
//     most 256 KiB, out of L2), so nothing has to be handed over; the last
//     workgroup's offset plus its own sum are the totals; the few counters that
//     need every workgroup's share are added with plain atomics into words an
//     earlier kernel of the same call has cleared.
#include "ckpt_internal.h"

namespace ckpt {

namespace {

struct Pair {
  uint64_t cnt;
  uint64_t bytes;
};

__device__ __forceinline__ Pair operator+(Pair a, Pair b) { return {a.cnt + b.cnt, a.bytes + b.bytes}; }

__device__ __forceinline__ Pair shfl_up(Pair v, int delta) {
  Pair r;
  r.cnt = __shfl_up(v.cnt, delta, 64);
  r.bytes = __shfl_up(v.bytes, delta, 64);
  return r;
}

// Exclusive scan of one Pair per thread across a workgroup of SCAN_THREADS
// threads; `total` receives the workgroup sum in every thread.
__device__ Pair block_exclusive_scan(Pair v, Pair *total) {
  __shared__ Pair s_wave[SCAN_THREADS / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  Pair incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    Pair o = shfl_up(incl, d);
    if (lane >= d) incl = incl + o;
  }
  __syncthreads();                 // s_wave may still be read from a previous call
  if (lane == 63) s_wave[wave] = incl;
  __syncthreads();
  Pair before = {0, 0}, all = {0, 0};
#pragma unroll
  for (int w = 0; w < SCAN_THREADS / 64; ++w) {
    if (w < wave) before = before + s_wave[w];
    all = all + s_wave[w];
  }
  *total = all;
  Pair excl = before + incl;
  excl.cnt -= v.cnt;
  excl.bytes -= v.bytes;
  return excl;
}

__device__ __forceinline__ uint64_t thread_first_chunk() {
  return (uint64_t)blockIdx.x * SCAN_BLOCK + (uint64_t)threadIdx.x * SCAN_PER_THREAD;
}

// Pair of the marked chunks among a thread's n consecutive ones; refs receives all n.
__device__ __forceinline__ Pair sum_marked(const PlanDev &p, uint64_t k0, const uint8_t *m, int n,
                                           ChunkRef *refs) {
  locate_run(p, k0, n, refs);
  Pair s = {0, 0};
  for (int i = 0; i < n; ++i) {
    if (m[i]) {
      s.cnt += 1;
      s.bytes += pad16(refs[i].len);
    }
  }
  return s;
}

// Stores the workgroup's pair where the scan kernel finds it.
__device__ __forceinline__ void store_block_pair(uint64_t *pairs, Pair total) {
  if (threadIdx.x == 0) {
    pairs[2 * (uint64_t)blockIdx.x] = total.cnt;
    pairs[2 * (uint64_t)blockIdx.x + 1] = total.bytes;
  }
}

// One workgroup: turns pairs[0..nblocks) into their exclusive prefix sums
// (when `rewrite`) and writes the grand totals to counts, overflow = 0.
// Fused snapshot: *publish_dst (when not null) receives *publish_src, or 0
// when there is no source -- the hint-miss count, complete once the kernel
// before this one is.
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_blocks(
    uint64_t *__restrict__ pairs, uint64_t nblocks, int rewrite,
    ckpt_counts_t *__restrict__ counts, const unsigned long long *publish_src,
    unsigned long long *publish_dst) {
  Pair carry = {0, 0};
  for (uint64_t base = 0; base < nblocks; base += SCAN_THREADS) {
    const uint64_t b = base + threadIdx.x;
    Pair v = {0, 0};
    if (b < nblocks) v = {pairs[2 * b], pairs[2 * b + 1]};
    Pair total;
    Pair excl = block_exclusive_scan(v, &total);
    if (rewrite && b < nblocks) {
      pairs[2 * b] = carry.cnt + excl.cnt;
      pairs[2 * b + 1] = carry.bytes + excl.bytes;
    }
    carry = carry + total;
  }
  if (threadIdx.x == 0) {
    counts->ndirty = carry.cnt;
    counts->staged_bytes = carry.bytes;
    counts->overflow = 0;
    if (publish_dst != nullptr) *publish_dst = publish_src != nullptr ? *publish_src : 0ull;
  }
}

// mask[k] = (ref == nullptr || dig[k] != ref[k]); per-workgroup sums of the marked chunks.
__global__ __launch_bounds__(SCAN_THREADS) void k_diff(PlanDev p, const uint64_t *__restrict__ dig,
                                                       const uint64_t *__restrict__ ref,
                                                       uint8_t *__restrict__ mask,
                                                       uint64_t *__restrict__ pairs) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  int n = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    if (k < p.nchunks) {
      m[i] = (ref == nullptr || dig[k] != ref[k]) ? 1 : 0;
      mask[k] = m[i];
      n = i + 1;
    }
  }
  ChunkRef refs[SCAN_PER_THREAD];
  Pair mine = sum_marked(p, k0, m, n, refs), total;
  block_exclusive_scan(mine, &total);
  store_block_pair(pairs, total);
}

// Cross-worker upload ownership (sec. 4.6): gathered holds `world` rows of N
// checksums.  The workers whose checksum at k equals this worker's form a
// group in rank order; member number (k mod group size) uploads the chunk.
// A thread reads `world` values per chunk, each row access coalesced over k.
__global__ __launch_bounds__(SCAN_THREADS) void k_upload_owners(
    PlanDev p, const uint64_t *__restrict__ gathered, uint32_t world, uint32_t rank,
    uint8_t *__restrict__ mask, uint64_t *__restrict__ pairs) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  int n = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    if (k < p.nchunks) {
      const uint64_t mine = gathered[(uint64_t)rank * p.nchunks + k];
      uint32_t size = 0, place = 0;
      for (uint32_t r = 0; r < world; ++r) {
        const bool same = gathered[(uint64_t)r * p.nchunks + k] == mine;
        place += (same && r < rank) ? 1u : 0u;
        size += same ? 1u : 0u;
      }
      m[i] = (uint32_t)(k % size) == place ? 1 : 0;   // size >= 1: the worker's own row matches
      mask[k] = m[i];
      n = i + 1;
    }
  }
  ChunkRef refs[SCAN_PER_THREAD];
  Pair mine = sum_marked(p, k0, m, n, refs), total;
  block_exclusive_scan(mine, &total);
  store_block_pair(pairs, total);
}

// Per-workgroup sums for a caller-supplied mask (any non-zero byte marks a chunk).
// Fused snapshot, first use (the hint): the mask is also copied to `keep`, and
// the snapshot's counters zero_me[0 .. SNAPSHOT_COUNTERS) are cleared.  Second
// use (the real mask): chunks whose mask differs from `hint` are added to
// *misses (k_scan_blocks publishes the sum).
__global__ __launch_bounds__(SCAN_THREADS) void k_block_sums(
    PlanDev p, const uint8_t *__restrict__ mask, uint64_t *__restrict__ pairs,
    uint8_t *__restrict__ keep, unsigned long long *zero_me, const uint8_t *__restrict__ hint,
    unsigned long long *misses) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  int n = 0;
  uint32_t bad = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    if (k < p.nchunks) {
      const uint8_t v = mask[k];
      if (keep != nullptr) keep[k] = v;
      m[i] = v != 0;
      if (hint != nullptr) bad += (hint[k] != 0) != (m[i] != 0);
      n = i + 1;
    }
  }
  if (zero_me != nullptr && blockIdx.x == 0 && threadIdx.x < SNAPSHOT_COUNTERS)
    zero_me[threadIdx.x] = 0;
  if (hint != nullptr) {
    for (int o = 32; o > 0; o >>= 1) bad += __shfl_down(bad, o, 64);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(misses, (unsigned long long)bad);
  }
  ChunkRef refs[SCAN_PER_THREAD];
  Pair mine = sum_marked(p, k0, m, n, refs), total;
  block_exclusive_scan(mine, &total);
  store_block_pair(pairs, total);
}

// Sum over the workgroup of one pair per thread, returned in every thread.
__device__ Pair block_sum(Pair v) {
  __shared__ Pair s_part[SCAN_THREADS / 64];
  for (int o = 32; o > 0; o >>= 1) {
    v.cnt += __shfl_down(v.cnt, o, 64);
    v.bytes += __shfl_down(v.bytes, o, 64);
  }
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = v;
  __syncthreads();
  Pair all = {0, 0};
#pragma unroll
  for (int w = 0; w < SCAN_THREADS / 64; ++w) all = all + s_part[w];
  return all;
}

// Non-zero bytes among the four of a word.
__device__ __forceinline__ uint32_t nonzero_bytes(uint32_t w) {
  return __popc((((w & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | w) & 0x80808080u);
}

// The pair of all marked chunks with id < k0, computed by the calling workgroup
// from the mask bytes themselves: their number by counting non-zero bytes, and
// their padded bytes as number * C minus what the marked short last chunks fall
// short of C (the plan lists those: at most one per buffer).
__device__ Pair pair_before(const PlanDev &p, const uint8_t *__restrict__ mask, uint64_t k0) {
  uint64_t cnt = 0, lost = 0;
  uint64_t head = (16 - (reinterpret_cast<uintptr_t>(mask) & 15)) & 15;   // bytes before 16-byte alignment
  if (head > k0) head = k0;
  if (threadIdx.x < head) cnt += mask[threadIdx.x] != 0;
  const uint64_t nvec = (k0 - head) / 16;
  const uint4 *v = reinterpret_cast<const uint4 *>(mask + head);
  for (uint64_t i = threadIdx.x; i < nvec; i += SCAN_THREADS) {
    const uint4 w = v[i];
    cnt += nonzero_bytes(w.x) + nonzero_bytes(w.y) + nonzero_bytes(w.z) + nonzero_bytes(w.w);
  }
  const uint64_t tail = head + 16 * nvec;
  if (tail + threadIdx.x < k0) cnt += mask[tail + threadIdx.x] != 0;     // fewer than 16 left
  const uint64_t c = 1ull << p.chunk_log2;
  for (uint64_t s = threadIdx.x; s < p.nshort; s += SCAN_THREADS) {
    const uint64_t k = p.short_chunk[s];
    if (k < k0 && mask[k] != 0) lost += c - pad16(p.short_len[s]);
  }
  Pair r = block_sum(Pair{cnt, lost});
  r.bytes = r.cnt * c - r.bytes;
  return r;
}

// End of the one-kernel manifest path.  The last workgroup's offset plus its own sum are the
// totals.  Entries that missed a capacity, hint misses and entries left for the gather are
// added to their counters by whichever workgroups have any: those words (counts->overflow,
// misses[0], misses[3], *misses_out) were cleared by an earlier kernel of the same call.
__device__ void finish_small(Pair before, Pair total, uint32_t missed, uint32_t bad, uint32_t todo,
                             ckpt_counts_t *counts, unsigned long long *misses,
                             unsigned long long *misses_out) {
  // the three small counts share one reduction: 16-bit fields, none can exceed SCAN_BLOCK
  const uint64_t small =
      block_sum(Pair{(uint64_t)missed | ((uint64_t)bad << 16) | ((uint64_t)todo << 32), 0}).cnt;
  if (threadIdx.x != 0) return;
  if (blockIdx.x == gridDim.x - 1) {
    counts->ndirty = before.cnt + total.cnt;
    counts->staged_bytes = before.bytes + total.bytes;
  }
  const unsigned long long over = small & 0xFFFF, wrong = (small >> 16) & 0xFFFF, left = small >> 32;
  if (over) atomicAdd(reinterpret_cast<unsigned long long *>(&counts->overflow), over);
  if (wrong && misses != nullptr) atomicAdd(misses, wrong);
  if (wrong && misses_out != nullptr) atomicAdd(misses_out, wrong);
  if (left && misses != nullptr) atomicAdd(misses + 3, left);
}

// Final pass: every marked chunk learns its entry index and staging offset and
// writes its manifest entry.  !SMALL: `pairs` holds the exclusive block sums and
// counts the totals (k_scan_blocks).  SMALL: the workgroup computes its own
// offset (pair_before), the last one writes the totals.  Either way entries that
// miss a capacity are added to counts->overflow, which an earlier kernel cleared.
// Fused snapshot (hint, hoff, need not null): entry e gets need[e] = 0 if the
// fingerprint pass has already staged the chunk at this very offset (it was
// hinted, its hinted offset equals the real one, and it fitted), else 1 -- the
// gather that follows a wrong hint copies only those.  SMALL also counts the
// chunks where hint and mask differ.
template <bool SMALL>
__global__ __launch_bounds__(SCAN_THREADS) void k_emit_manifest(
    PlanDev p, const uint8_t *__restrict__ mask, const uint64_t *__restrict__ dig,
    const uint64_t *__restrict__ pairs, ckpt_entry_t *__restrict__ manifest, uint64_t manifest_cap,
    uint64_t staging_cap, ckpt_counts_t *__restrict__ counts, const uint8_t *__restrict__ hint,
    const uint64_t *__restrict__ hoff, uint8_t *__restrict__ need, unsigned long long *misses,
    unsigned long long *misses_out) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  uint64_t d[SCAN_PER_THREAD], ho[SCAN_PER_THREAD];
  bool hinted[SCAN_PER_THREAD];
  ChunkRef refs[SCAN_PER_THREAD];
  int n = 0;
  uint32_t bad = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    hinted[i] = false;
    ho[i] = 0;
    if (k < p.nchunks) {
      // everything the entries need is read up front: no load waits behind the scan
      m[i] = mask[k] != 0;
      d[i] = dig[k];
      if (hint != nullptr) {          // hoff comes with hint
        hinted[i] = hint[k] != 0;
        ho[i] = hoff[k];
        bad += hinted[i] != (m[i] != 0);
      }
      n = i + 1;
    }
  }
  Pair mine = sum_marked(p, k0, m, n, refs), total;
  Pair pos = block_exclusive_scan(mine, &total);
  Pair before;
  if (SMALL) {
    before = pair_before(p, mask, (uint64_t)blockIdx.x * SCAN_BLOCK);
  } else {
    before = {pairs[2 * (uint64_t)blockIdx.x], pairs[2 * (uint64_t)blockIdx.x + 1]};
  }
  pos = pos + before;
  uint32_t missed = 0, todo = 0;
  for (int i = 0; i < n; ++i) {
    if (!m[i]) continue;
    const ChunkRef r = refs[i];
    const uint64_t padded = pad16(r.len);
    const bool fits_manifest = pos.cnt < manifest_cap;
    const bool fits_staging = fits_manifest && pos.bytes + padded <= staging_cap;
    if (fits_manifest) {
      ckpt_entry_t e;
      e.buf = p.dense_orig[r.row];
      e.len = r.len;
      e.buf_off = r.off;
      e.stage_off = pos.bytes;
      e.digest = d[i];
      manifest[pos.cnt] = e;
      if (need != nullptr) {
        const bool in_place = fits_staging && hinted[i] && ho[i] == pos.bytes;
        need[pos.cnt] = !in_place;
        todo += fits_staging && !in_place;
      }
    }
    if (!fits_staging) ++missed;
    pos.cnt += 1;
    pos.bytes += padded;
  }
  if (SMALL) {
    finish_small(before, total, missed, bad, todo, counts, misses, misses_out);
  } else {
    if (missed)
      atomicAdd(reinterpret_cast<unsigned long long *>(&counts->overflow), (unsigned long long)missed);
    if (need != nullptr) {         // one atomic per wavefront that has something to report
      for (int o = 32; o > 0; o >>= 1) todo += __shfl_down(todo, o, 64);
      if ((threadIdx.x & 63) == 0 && todo) atomicAdd(misses + 3, (unsigned long long)todo);
    }
  }
}

// Fused snapshot, before the pass: staging offset of every hinted chunk (the
// exclusive prefix sum over the hint, as k_emit_manifest computes it for a
// mask).  SMALL: one kernel does it all -- reads the caller's hint, keeps a
// private copy (hint and mask may be one buffer), clears the snapshot's
// counters; otherwise k_block_sums has done those and left the block offsets.
template <bool SMALL>
__global__ __launch_bounds__(SCAN_THREADS) void k_hint_offsets(
    PlanDev p, const uint8_t *__restrict__ hint, const uint64_t *__restrict__ pairs,
    uint64_t manifest_cap, uint64_t *__restrict__ hoff, uint8_t *__restrict__ keep,
    unsigned long long *zero_me, unsigned long long *zero_a, unsigned long long *zero_b) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  ChunkRef refs[SCAN_PER_THREAD];
  int n = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    if (k < p.nchunks) {
      const uint8_t v = hint[k];
      if (SMALL) keep[k] = v;
      m[i] = v != 0;
      n = i + 1;
    }
  }
  if (SMALL && blockIdx.x == 0) {
    // everything the manifest kernel later adds to starts at zero
    if (threadIdx.x < SNAPSHOT_COUNTERS) zero_me[threadIdx.x] = 0;
    if (threadIdx.x == 0 && zero_a != nullptr) *zero_a = 0;
    if (threadIdx.x == 0 && zero_b != nullptr) *zero_b = 0;
  }
  Pair mine = sum_marked(p, k0, m, n, refs), total;
  Pair pos = block_exclusive_scan(mine, &total);
  Pair before;
  if (SMALL) {
    before = pair_before(p, hint, (uint64_t)blockIdx.x * SCAN_BLOCK);
  } else {
    before = {pairs[2 * (uint64_t)blockIdx.x], pairs[2 * (uint64_t)blockIdx.x + 1]};
  }
  pos = pos + before;
  for (int i = 0; i < n; ++i) {
    // a chunk whose entry would not fit the manifest is not staged either (all-ones = never fits)
    hoff[k0 + i] = pos.cnt < manifest_cap ? pos.bytes : ~0ull;
    if (m[i]) {
      pos.cnt += 1;
      pos.bytes += pad16(refs[i].len);
    }
  }
}

// Zero counts and miss counters: what a call over no chunks reports, and the cleared state the
// one-kernel manifest path adds to when no earlier kernel of the call could do the clearing.
__global__ void k_clear_counts(ckpt_counts_t *counts, unsigned long long *misses,
                               unsigned long long *misses_out) {
  counts->ndirty = counts->staged_bytes = counts->overflow = 0;
  if (misses != nullptr) misses[0] = misses[3] = 0;
  if (misses_out != nullptr) *misses_out = 0;
}

// Squashing validation (paper sec. 5.2.3): per chunk, did rank a and rank b
// change it alike?  Counters are zeroed by k_validate_init on the same stream.
__global__ void k_validate_init(ckpt_validation_t *r) {
  r->changed_a = r->changed_b = r->mismatches = 0;
  r->first_mismatch = ~0ull;
}

__global__ __launch_bounds__(SCAN_THREADS) void k_validate(uint64_t n,
                                                           const uint64_t *__restrict__ b_a,
                                                           const uint64_t *__restrict__ a_a,
                                                           const uint64_t *__restrict__ b_b,
                                                           const uint64_t *__restrict__ a_b,
                                                           ckpt_validation_t *__restrict__ r) {
  uint32_t ca = 0, cb = 0, bad = 0;
  uint64_t first = ~0ull;
  const uint64_t stride = (uint64_t)gridDim.x * SCAN_THREADS;
  for (uint64_t k = (uint64_t)blockIdx.x * SCAN_THREADS + threadIdx.x; k < n; k += stride) {
    const uint64_t after_a = a_a[k], after_b = a_b[k];
    const bool xa = b_a[k] != after_a, xb = b_b[k] != after_b;
    ca += xa;
    cb += xb;
    if (xa != xb || (xa && after_a != after_b)) {
      bad += 1;
      if (k < first) first = k;
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    ca += __shfl_down(ca, o, 64);
    cb += __shfl_down(cb, o, 64);
    bad += __shfl_down(bad, o, 64);
    const uint64_t f = __shfl_down(first, o, 64);
    first = f < first ? f : first;
  }
  // one set of atomics per workgroup: every workgroup adds to the same four words
  __shared__ uint32_t s_ca[SCAN_THREADS / 64], s_cb[SCAN_THREADS / 64], s_bad[SCAN_THREADS / 64];
  __shared__ uint64_t s_first[SCAN_THREADS / 64];
  if ((threadIdx.x & 63) == 0) {
    s_ca[threadIdx.x >> 6] = ca;
    s_cb[threadIdx.x >> 6] = cb;
    s_bad[threadIdx.x >> 6] = bad;
    s_first[threadIdx.x >> 6] = first;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int v = 1; v < SCAN_THREADS / 64; ++v) {
      ca += s_ca[v];
      cb += s_cb[v];
      bad += s_bad[v];
      first = s_first[v] < first ? s_first[v] : first;
    }
    if (ca) atomicAdd(reinterpret_cast<unsigned long long *>(&r->changed_a), (unsigned long long)ca);
    if (cb) atomicAdd(reinterpret_cast<unsigned long long *>(&r->changed_b), (unsigned long long)cb);
    if (bad) {
      atomicAdd(reinterpret_cast<unsigned long long *>(&r->mismatches), (unsigned long long)bad);
      atomicMin(reinterpret_cast<unsigned long long *>(&r->first_mismatch),
                (unsigned long long)first);
    }
  }
}

// Per-buffer verdicts (the paper compares whole buffers, sec. 5.2.1): a buffer differs when any
// of its chunks is marked.  k_verdict_clear zeroes the flags and the counts; k_verdict_mark has
// every thread look at its four consecutive chunks and set the flag of each marked chunk's
// buffer (all writers of a flag store the same 1); k_verdict_count adds up the buffers that
// differ and their sizes.
__global__ __launch_bounds__(256) void k_verdict_clear(uint8_t *__restrict__ dirty, uint64_t nbufs,
                                                       unsigned long long *counts) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < nbufs; i += stride) dirty[i] = 0;
  if (blockIdx.x == 0 && threadIdx.x < 2) counts[threadIdx.x] = 0;
}

__global__ __launch_bounds__(SCAN_THREADS) void k_verdict_mark(PlanDev p,
                                                               const uint8_t *__restrict__ mask,
                                                               uint8_t *__restrict__ dirty) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  int n = 0;
  bool any = false;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    m[i] = 0;
    if (k < p.nchunks) {
      m[i] = mask[k];
      any = any || m[i] != 0;
      n = i + 1;
    }
  }
  if (!any) return;
  ChunkRef refs[SCAN_PER_THREAD];
  locate_run(p, k0, n, refs);
  for (int i = 0; i < n; ++i)
    if (m[i] != 0) dirty[p.dense_orig[refs[i].row]] = 1;
}

__global__ __launch_bounds__(256) void k_verdict_count(PlanDev p, const uint8_t *__restrict__ dirty,
                                                       unsigned long long *counts) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  unsigned long long differing = 0, bytes = 0;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < p.nbufs; i += stride) {
    if (dirty[i] != 0) {
      differing += 1;
      bytes += p.list_nbytes[i];
    }
  }
  for (int o = 32; o > 0; o >>= 1) {
    differing += __shfl_down(differing, o, 64);
    bytes += __shfl_down(bytes, o, 64);
  }
  if ((threadIdx.x & 63) == 0 && differing != 0) {
    atomicAdd(&counts[0], differing);
    atomicAdd(&counts[1], bytes);
  }
}

// marks[k] = 1 for every chunk of a buffer whose flag is set: the reverse of the verdicts, one
// thread per four consecutive chunks.
__global__ __launch_bounds__(SCAN_THREADS) void k_marks_from_buffers(
    PlanDev p, const uint8_t *__restrict__ flags, uint8_t *__restrict__ marks) {
  const uint64_t k0 = thread_first_chunk();
  if (k0 >= p.nchunks) return;
  const uint64_t left = p.nchunks - k0;
  const int n = left < SCAN_PER_THREAD ? (int)left : SCAN_PER_THREAD;
  ChunkRef refs[SCAN_PER_THREAD];
  locate_run(p, k0, n, refs);
  for (int i = 0; i < n; ++i) marks[k0 + i] = flags[p.dense_orig[refs[i].row]] != 0 ? 1 : 0;
}

// out[k] = 1 where mask[k] is set and without[k] is not.  Sixteen chunks per thread when the
// three arrays allow 16-byte accesses, else one.
__global__ __launch_bounds__(256) void k_mask_andnot(uint64_t n, const uint8_t *mask,
                                                     const uint8_t *without, uint8_t *out,
                                                     bool wide) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  const uint64_t tid = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  uint64_t done = 0;
  if (wide) {
    const uint64_t n16 = n / 16;
    for (uint64_t i = tid; i < n16; i += stride) {
      const uint4 a = reinterpret_cast<const uint4 *>(mask)[i];
      const uint4 b = reinterpret_cast<const uint4 *>(without)[i];
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
      uint32_t r[4];
      for (int w = 0; w < 4; ++w) {
        r[w] = 0;
        for (int byte = 0; byte < 4; ++byte) {
          const uint32_t m = (aw[w] >> (8 * byte)) & 0xFF, x = (bw[w] >> (8 * byte)) & 0xFF;
          r[w] |= (uint32_t)(m != 0 && x == 0) << (8 * byte);
        }
      }
      reinterpret_cast<uint4 *>(out)[i] = make_uint4(r[0], r[1], r[2], r[3]);
    }
    done = n16 * 16;
  }
  for (uint64_t k = done + tid; k < n; k += stride) out[k] = (mask[k] != 0 && without[k] == 0) ? 1 : 0;
}

inline uint32_t scan_blocks(uint64_t nchunks) {
  return (uint32_t)((nchunks + SCAN_BLOCK - 1) / SCAN_BLOCK);
}

typedef unsigned long long ull;

}  // namespace

hipError_t launch_diff(const PlanDev &p, const uint64_t *d_dig, const uint64_t *d_ref,
                       uint8_t *d_mask, uint64_t *d_pairs, ckpt_counts_t *d_counts, hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  if (nblocks)
    hipLaunchKernelGGL(k_diff, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_dig, d_ref, d_mask,
                       d_pairs);
  hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_pairs, (uint64_t)nblocks, 0,
                     d_counts, (const ull *)nullptr, (ull *)nullptr);
  return hipGetLastError();
}

hipError_t launch_upload_owners(const PlanDev &p, const uint64_t *d_gathered, uint32_t world,
                                uint32_t rank, uint8_t *d_mask, uint64_t *d_pairs,
                                ckpt_counts_t *d_counts, hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  if (nblocks)
    hipLaunchKernelGGL(k_upload_owners, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_gathered,
                       world, rank, d_mask, d_pairs);
  hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_pairs, (uint64_t)nblocks, 0,
                     d_counts, (const ull *)nullptr, (ull *)nullptr);
  return hipGetLastError();
}

// The metadata half of compact for a given mask: one kernel up to SMALL_SCAN_CHUNKS chunks,
// three above.  With h (fused snapshot) the hint misses are counted and the entries the pass has
// already staged are marked in h->need.  cleared: an earlier kernel of the same call has zeroed
// d_counts->overflow, *d_misses_out and h's counters (see launch_hint_offsets and the
// fingerprint pass); otherwise the one-kernel path clears them with a kernel of its own.
hipError_t launch_compact_scan(const PlanDev &p, const uint8_t *d_mask, const uint64_t *d_dig,
                               uint64_t staging_cap, ckpt_entry_t *d_manifest,
                               uint64_t manifest_cap, uint64_t *d_pairs, ckpt_counts_t *d_counts,
                               const HintState *h, uint64_t *d_misses_out, bool cleared,
                               hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  const uint8_t *hint = h ? h->copy : nullptr;
  const uint64_t *hoff = h ? h->hoff : nullptr;
  uint8_t *need = h ? h->need : nullptr;
  ull *misses = h ? reinterpret_cast<ull *>(h->misses) : nullptr;
  ull *misses_out = reinterpret_cast<ull *>(d_misses_out);
  if (nblocks == 0) {
    hipLaunchKernelGGL(k_clear_counts, dim3(1), dim3(1), 0, s, d_counts, misses, misses_out);
  } else if (p.nchunks <= SMALL_SCAN_CHUNKS) {
    if (!cleared)
      hipLaunchKernelGGL(k_clear_counts, dim3(1), dim3(1), 0, s, d_counts, misses, misses_out);
    hipLaunchKernelGGL(k_emit_manifest<true>, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_mask,
                       d_dig, (const uint64_t *)nullptr, d_manifest, manifest_cap, staging_cap,
                       d_counts, hint, hoff, need, misses, misses_out);
  } else {
    hipLaunchKernelGGL(k_block_sums, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_mask, d_pairs,
                       (uint8_t *)nullptr, (ull *)nullptr, hint, misses);
    hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_pairs, (uint64_t)nblocks,
                       1, d_counts, (const ull *)misses, misses_out);
    hipLaunchKernelGGL(k_emit_manifest<false>, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_mask,
                       d_dig, (const uint64_t *)d_pairs, d_manifest, manifest_cap, staging_cap,
                       d_counts, hint, hoff, need, misses, (ull *)nullptr);
  }
  return hipGetLastError();
}

// Staging offsets of the hinted chunks, the private copy of the hint, cleared counters; in the
// one-kernel shape also d_counts->overflow and *d_misses_out, for the manifest kernel to add to.
hipError_t launch_hint_offsets(const PlanDev &p, const uint8_t *d_hint_in, const HintState &h,
                               uint64_t *d_pairs, ckpt_counts_t *d_tmp_counts, uint64_t manifest_cap,
                               ckpt_counts_t *d_counts, uint64_t *d_misses_out, hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  ull *zero_me = reinterpret_cast<ull *>(h.misses);
  if (nblocks == 0) {
    hipLaunchKernelGGL(k_clear_counts, dim3(1), dim3(1), 0, s, d_tmp_counts, zero_me, (ull *)nullptr);
  } else if (p.nchunks <= SMALL_SCAN_CHUNKS) {
    hipLaunchKernelGGL(k_hint_offsets<true>, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_hint_in,
                       (const uint64_t *)nullptr, manifest_cap, h.hoff, h.copy, zero_me,
                       reinterpret_cast<ull *>(&d_counts->overflow),
                       reinterpret_cast<ull *>(d_misses_out));
  } else {
    hipLaunchKernelGGL(k_block_sums, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_hint_in, d_pairs,
                       h.copy, zero_me, (const uint8_t *)nullptr, (ull *)nullptr);
    hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_pairs, (uint64_t)nblocks,
                       1, d_tmp_counts, (const ull *)nullptr, (ull *)nullptr);
    hipLaunchKernelGGL(k_hint_offsets<false>, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p,
                       (const uint8_t *)h.copy, (const uint64_t *)d_pairs, manifest_cap, h.hoff,
                       (uint8_t *)nullptr, (ull *)nullptr, (ull *)nullptr, (ull *)nullptr);
  }
  return hipGetLastError();
}

hipError_t launch_validate(uint64_t n, const uint64_t *b_a, const uint64_t *a_a, const uint64_t *b_b,
                           const uint64_t *a_b, ckpt_validation_t *d_result, hipStream_t s) {
  hipLaunchKernelGGL(k_validate_init, dim3(1), dim3(1), 0, s, d_result);
  if (n) {
    uint64_t groups = (n + SCAN_THREADS - 1) / SCAN_THREADS;
    if (groups > 2048) groups = 2048;
    hipLaunchKernelGGL(k_validate, dim3((uint32_t)groups), dim3(SCAN_THREADS), 0, s, n, b_a, a_a,
                       b_b, a_b, d_result);
  }
  return hipGetLastError();
}

hipError_t launch_marks_from_buffers(const PlanDev &p, const uint8_t *d_flags, uint8_t *d_marks,
                                     hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  if (nblocks == 0) return hipSuccess;
  hipLaunchKernelGGL(k_marks_from_buffers, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_flags,
                     d_marks);
  return hipGetLastError();
}

hipError_t launch_mask_andnot(uint64_t n, const uint8_t *d_mask, const uint8_t *d_without,
                              uint8_t *d_out, hipStream_t s) {
  if (n == 0) return hipSuccess;
  const bool wide = ((reinterpret_cast<uintptr_t>(d_mask) | reinterpret_cast<uintptr_t>(d_without) |
                      reinterpret_cast<uintptr_t>(d_out)) & 15) == 0;
  uint64_t groups = ((wide ? n / 16 + 16 : n) + 255) / 256;
  if (groups > 4096) groups = 4096;
  hipLaunchKernelGGL(k_mask_andnot, dim3((uint32_t)groups), dim3(256), 0, s, n, d_mask, d_without,
                     d_out, wide);
  return hipGetLastError();
}

hipError_t launch_buffer_verdicts(const PlanDev &p, const uint8_t *d_mask, uint8_t *d_dirty,
                                  uint64_t *d_counts, hipStream_t s) {
  ull *counts = reinterpret_cast<ull *>(d_counts);
  uint64_t groups = (p.nbufs + 255) / 256;
  if (groups > 4096) groups = 4096;
  if (groups == 0) groups = 1;
  hipLaunchKernelGGL(k_verdict_clear, dim3((uint32_t)groups), dim3(256), 0, s, d_dirty, p.nbufs,
                     counts);
  const uint32_t nblocks = scan_blocks(p.nchunks);
  if (nblocks != 0) {
    hipLaunchKernelGGL(k_verdict_mark, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_mask, d_dirty);
    hipLaunchKernelGGL(k_verdict_count, dim3((uint32_t)groups), dim3(256), 0, s, p,
                       (const uint8_t *)d_dirty, counts);
  }
  return hipGetLastError();
}

}  // namespace ckpt
