// Checksum comparison and the prefix scan that orders the swap-out.
//
// diff: the comparison of a rank's checksums "with the other rank's copy" that
// the Singularity paper does on the host (sec. 6; sec. 5.2.1, 5.2.3) -- here a
// device kernel, one thread per four chunks.
//
// compact, metadata half: stable compaction.  Staging order must be ascending
// chunk id, so offsets come from an exclusive prefix sum over
// (mask, mask * pad16(len)) pairs, done in three deterministic steps with no
// inter-workgroup waiting: per-workgroup sums, a single-workgroup scan of
// those sums, then a per-workgroup rescan that writes the manifest.
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

__device__ __forceinline__ Pair sum_marked(const PlanDev &p, uint64_t k0, const uint8_t *m, int n,
                                           ChunkRef *refs) {
  Pair s = {0, 0};
  for (int i = 0; i < n; ++i) {
    if (m[i]) {
      ChunkRef r = locate_chunk(p, k0 + i);
      if (refs) refs[i] = r;
      s.cnt += 1;
      s.bytes += pad16(r.len);
    }
  }
  return s;
}

// mask[k] = (ref == nullptr || dig[k] != ref[k]); per-workgroup sums of the
// marked chunks go to blocksums[2*b], [2*b+1].
//
// Fused snapshot: with `hint` (a private copy of the caller's hint, so that hint
// and mask may be one buffer) the chunks whose mask differs from the hint are
// counted into *misses.
__global__ __launch_bounds__(SCAN_THREADS) void k_diff(PlanDev p, const uint64_t *__restrict__ dig,
                                                       const uint64_t *__restrict__ ref,
                                                       uint8_t *__restrict__ mask,
                                                       uint64_t *__restrict__ blocksums,
                                                       const uint8_t *__restrict__ hint,
                                                       unsigned long long *misses) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  int n = 0;
  uint32_t bad = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    if (k < p.nchunks) {
      m[i] = (ref == nullptr || dig[k] != ref[k]) ? 1 : 0;
      if (hint != nullptr) bad += (hint[k] != 0) != (m[i] != 0);
      mask[k] = m[i];
      n = i + 1;
    }
  }
  if (hint != nullptr) {
    for (int o = 32; o > 0; o >>= 1) bad += __shfl_down(bad, o, 64);
    if ((threadIdx.x & 63) == 0 && bad) atomicAdd(misses, (unsigned long long)bad);
  }
  Pair mine = sum_marked(p, k0, m, n, nullptr), total;
  block_exclusive_scan(mine, &total);
  if (threadIdx.x == 0) {
    blocksums[2 * (uint64_t)blockIdx.x] = total.cnt;
    blocksums[2 * (uint64_t)blockIdx.x + 1] = total.bytes;
  }
}

// Cross-worker upload ownership (sec. 4.6): gathered holds `world` rows of N
// checksums.  The workers whose checksum at k equals this worker's form a
// group in rank order; member number (k mod group size) uploads the chunk.
// A thread reads `world` values per chunk, each row access coalesced over k.
__global__ __launch_bounds__(SCAN_THREADS) void k_upload_owners(
    PlanDev p, const uint64_t *__restrict__ gathered, uint32_t world, uint32_t rank,
    uint8_t *__restrict__ mask, uint64_t *__restrict__ blocksums) {
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
  Pair mine = sum_marked(p, k0, m, n, nullptr), total;
  block_exclusive_scan(mine, &total);
  if (threadIdx.x == 0) {
    blocksums[2 * (uint64_t)blockIdx.x] = total.cnt;
    blocksums[2 * (uint64_t)blockIdx.x + 1] = total.bytes;
  }
}

// Same sums for a caller-supplied mask (any non-zero byte marks a chunk).
// Fused snapshot: the mask (there: the hint) is also copied to `keep`, and the
// snapshot's counters zero_me[0 .. SNAPSHOT_COUNTERS) are cleared (hint misses,
// which k_diff adds to later; scratch counts; the lengths of the group lists).
__global__ __launch_bounds__(SCAN_THREADS) void k_block_sums(PlanDev p,
                                                             const uint8_t *__restrict__ mask,
                                                             uint64_t *__restrict__ blocksums,
                                                             uint8_t *__restrict__ keep,
                                                             unsigned long long *zero_me) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  int n = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    if (k < p.nchunks) {
      const uint8_t v = mask[k];
      if (keep != nullptr) keep[k] = v;
      m[i] = v != 0;
      n = i + 1;
    }
  }
  if (zero_me != nullptr && blockIdx.x == 0 && threadIdx.x < SNAPSHOT_COUNTERS)
    zero_me[threadIdx.x] = 0;
  Pair mine = sum_marked(p, k0, m, n, nullptr), total;
  block_exclusive_scan(mine, &total);
  if (threadIdx.x == 0) {
    blocksums[2 * (uint64_t)blockIdx.x] = total.cnt;
    blocksums[2 * (uint64_t)blockIdx.x + 1] = total.bytes;
  }
}

// One workgroup: turns blocksums[0..nblocks) into their exclusive prefix sums
// (when `rewrite`) and writes the grand totals to counts, overflow = 0.
// Fused snapshot: *publish_dst (when not null) receives *publish_src, or 0
// when there is no source -- the hint-miss count, complete once k_diff is.
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_blocks(
    uint64_t *__restrict__ blocksums, uint64_t nblocks, int rewrite,
    ckpt_counts_t *__restrict__ counts, const unsigned long long *publish_src,
    unsigned long long *publish_dst) {
  Pair carry = {0, 0};
  for (uint64_t base = 0; base < nblocks; base += SCAN_THREADS) {
    const uint64_t b = base + threadIdx.x;
    Pair v = {0, 0};
    if (b < nblocks) v = {blocksums[2 * b], blocksums[2 * b + 1]};
    Pair total;
    Pair excl = block_exclusive_scan(v, &total);
    if (rewrite && b < nblocks) {
      blocksums[2 * b] = carry.cnt + excl.cnt;
      blocksums[2 * b + 1] = carry.bytes + excl.bytes;
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

// Final pass: every marked chunk learns its entry index and staging offset and
// writes its manifest entry.  blockoff holds the exclusive sums from
// k_scan_blocks.  Entries that miss a capacity are counted in counts->overflow.
__global__ __launch_bounds__(SCAN_THREADS) void k_emit_manifest(
    PlanDev p, const uint8_t *__restrict__ mask, const uint64_t *__restrict__ dig,
    const uint64_t *__restrict__ blockoff, ckpt_entry_t *__restrict__ manifest,
    uint64_t manifest_cap, uint64_t staging_cap, ckpt_counts_t *__restrict__ counts) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  ChunkRef refs[SCAN_PER_THREAD];
  int n = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    if (k < p.nchunks) {
      m[i] = mask[k] != 0;
      n = i + 1;
    }
  }
  Pair mine = sum_marked(p, k0, m, n, refs), total;
  Pair pos = block_exclusive_scan(mine, &total);
  pos.cnt += blockoff[2 * (uint64_t)blockIdx.x];
  pos.bytes += blockoff[2 * (uint64_t)blockIdx.x + 1];
  uint32_t missed = 0;
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
      e.digest = dig[k0 + i];
      manifest[pos.cnt] = e;
    }
    if (!fits_staging) ++missed;
    pos.cnt += 1;
    pos.bytes += padded;
  }
  if (missed) atomicAdd(reinterpret_cast<unsigned long long *>(&counts->overflow),
                        (unsigned long long)missed);
}

// Fused snapshot, before the pass: staging offset of every hinted chunk (the
// exclusive prefix sum over the hint, as k_emit_manifest computes it for a mask).
__global__ __launch_bounds__(SCAN_THREADS) void k_hint_offsets(PlanDev p,
                                                               const uint8_t *__restrict__ hint,
                                                               const uint64_t *__restrict__ blockoff,
                                                               uint64_t manifest_cap,
                                                               uint64_t *__restrict__ hoff) {
  const uint64_t k0 = thread_first_chunk();
  uint8_t m[SCAN_PER_THREAD];
  ChunkRef refs[SCAN_PER_THREAD];
  int n = 0;
  for (int i = 0; i < SCAN_PER_THREAD; ++i) {
    const uint64_t k = k0 + i;
    if (k < p.nchunks) {
      m[i] = hint[k] != 0;
      n = i + 1;
    }
  }
  Pair mine = sum_marked(p, k0, m, n, refs), total;
  Pair pos = block_exclusive_scan(mine, &total);
  pos.cnt += blockoff[2 * (uint64_t)blockIdx.x];
  pos.bytes += blockoff[2 * (uint64_t)blockIdx.x + 1];
  for (int i = 0; i < n; ++i) {
    // a chunk whose entry would not fit the manifest is not staged either (all-ones = never fits)
    hoff[k0 + i] = pos.cnt < manifest_cap ? pos.bytes : ~0ull;
    if (m[i]) {
      pos.cnt += 1;
      pos.bytes += pad16(refs[i].len);
    }
  }
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
  if ((threadIdx.x & 63) == 0) {
    if (ca) atomicAdd(reinterpret_cast<unsigned long long *>(&r->changed_a), (unsigned long long)ca);
    if (cb) atomicAdd(reinterpret_cast<unsigned long long *>(&r->changed_b), (unsigned long long)cb);
    if (bad) {
      atomicAdd(reinterpret_cast<unsigned long long *>(&r->mismatches), (unsigned long long)bad);
      atomicMin(reinterpret_cast<unsigned long long *>(&r->first_mismatch),
                (unsigned long long)first);
    }
  }
}

inline uint32_t scan_blocks(uint64_t nchunks) {
  return (uint32_t)((nchunks + SCAN_BLOCK - 1) / SCAN_BLOCK);
}

}  // namespace

hipError_t launch_diff(const PlanDev &p, const uint64_t *d_dig, const uint64_t *d_ref,
                       uint8_t *d_mask, uint64_t *d_blocksums, ckpt_counts_t *d_counts,
                       hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  if (nblocks)
    hipLaunchKernelGGL(k_diff, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_dig, d_ref, d_mask,
                       d_blocksums, (const uint8_t *)nullptr, (unsigned long long *)nullptr);
  hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_blocksums,
                     (uint64_t)nblocks, 0, d_counts, (const unsigned long long *)nullptr,
                     (unsigned long long *)nullptr);
  return hipGetLastError();
}

// diff and the metadata half of compact as one sequence of three kernels (the
// workgroup sums k_diff leaves behind are the ones the compaction scan needs).
hipError_t launch_diff_compact_scan(const PlanDev &p, const uint64_t *d_dig, const uint64_t *d_ref,
                                    uint8_t *d_mask, const uint8_t *d_hint_copy, uint64_t *d_misses,
                                    uint64_t *d_misses_out, uint64_t staging_cap,
                                    ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                                    uint64_t *d_blocksums, ckpt_counts_t *d_counts, hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  unsigned long long *misses = reinterpret_cast<unsigned long long *>(d_misses);
  if (nblocks)
    hipLaunchKernelGGL(k_diff, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_dig, d_ref, d_mask,
                       d_blocksums, d_hint_copy, misses);
  hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_blocksums,
                     (uint64_t)nblocks, 1, d_counts, (const unsigned long long *)misses,
                     reinterpret_cast<unsigned long long *>(d_misses_out));
  if (nblocks)
    hipLaunchKernelGGL(k_emit_manifest, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_mask, d_dig,
                       d_blocksums, d_manifest, manifest_cap, staging_cap, d_counts);
  return hipGetLastError();
}

hipError_t launch_upload_owners(const PlanDev &p, const uint64_t *d_gathered, uint32_t world,
                                uint32_t rank, uint8_t *d_mask, uint64_t *d_blocksums,
                                ckpt_counts_t *d_counts, hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  if (nblocks)
    hipLaunchKernelGGL(k_upload_owners, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_gathered,
                       world, rank, d_mask, d_blocksums);
  hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_blocksums,
                     (uint64_t)nblocks, 0, d_counts, (const unsigned long long *)nullptr,
                     (unsigned long long *)nullptr);
  return hipGetLastError();
}

hipError_t launch_hint_offsets(const PlanDev &p, const uint8_t *d_hint_in, uint8_t *d_hint_copy,
                               uint64_t *d_blocksums, ckpt_counts_t *d_tmp_counts,
                               uint64_t manifest_cap, uint64_t *d_hoff, uint64_t *d_misses,
                               hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  if (nblocks)
    hipLaunchKernelGGL(k_block_sums, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_hint_in,
                       d_blocksums, d_hint_copy, reinterpret_cast<unsigned long long *>(d_misses));
  // with no chunks the scan kernel clears the miss counter instead
  hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_blocksums,
                     (uint64_t)nblocks, 1, d_tmp_counts, (const unsigned long long *)nullptr,
                     nblocks ? (unsigned long long *)nullptr
                             : reinterpret_cast<unsigned long long *>(d_misses));
  if (nblocks)
    hipLaunchKernelGGL(k_hint_offsets, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_hint_copy,
                       d_blocksums, manifest_cap, d_hoff);
  return hipGetLastError();
}

hipError_t launch_validate(uint64_t n, const uint64_t *b_a, const uint64_t *a_a, const uint64_t *b_b,
                           const uint64_t *a_b, ckpt_validation_t *d_result, hipStream_t s) {
  hipLaunchKernelGGL(k_validate_init, dim3(1), dim3(1), 0, s, d_result);
  if (n) {
    uint64_t groups = (n + SCAN_THREADS - 1) / SCAN_THREADS;
    if (groups > 4096) groups = 4096;
    hipLaunchKernelGGL(k_validate, dim3((uint32_t)groups), dim3(SCAN_THREADS), 0, s, n, b_a, a_a,
                       b_b, a_b, d_result);
  }
  return hipGetLastError();
}

hipError_t launch_compact_scan(const PlanDev &p, const uint8_t *d_mask, const uint64_t *d_dig,
                               uint64_t staging_cap, ckpt_entry_t *d_manifest,
                               uint64_t manifest_cap, uint64_t *d_blocksums,
                               ckpt_counts_t *d_counts, hipStream_t s) {
  const uint32_t nblocks = scan_blocks(p.nchunks);
  if (nblocks)
    hipLaunchKernelGGL(k_block_sums, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_mask,
                       d_blocksums, (uint8_t *)nullptr, (unsigned long long *)nullptr);
  hipLaunchKernelGGL(k_scan_blocks, dim3(1), dim3(SCAN_THREADS), 0, s, d_blocksums,
                     (uint64_t)nblocks, 1, d_counts, (const unsigned long long *)nullptr,
                     (unsigned long long *)nullptr);
  if (nblocks)
    hipLaunchKernelGGL(k_emit_manifest, dim3(nblocks), dim3(SCAN_THREADS), 0, s, p, d_mask, d_dig,
                       d_blocksums, d_manifest, manifest_cap, staging_cap, d_counts);
  return hipGetLastError();
}

}  // namespace ckpt
