// Internal declarations shared by the HIP translation units of libckpt.so.
// Nothing here is part of the ABI (that is include/ckpt.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ckpt.h"

namespace ckpt {

// Chunks handled by one wavefront of the fingerprint kernel: 16 chunks x 4
// lanes, one XXH64 accumulator per lane.  The plan's group table has one entry
// per GROUP consecutive chunk ids.
constexpr int GROUP = 16;
constexpr int GROUP_LOG2 = 4;

// Chunk geometry on the device.  The "dense" arrays skip empty buffers so that
// every table row owns at least one chunk; `orig` maps a row back to the
// caller's buffer index.  The "list" arrays are indexed by the caller's buffer
// index (manifest entries carry that index).
struct PlanDev {
  const uint64_t *dense_ptr;     // [nb]   device address of the buffer
  const uint64_t *dense_nbytes;  // [nb]
  const uint64_t *dense_base;    // [nb+1] global id of the buffer's first chunk; [nb] = N
  const uint32_t *dense_orig;    // [nb]   index in the caller's list
  const uint32_t *group_first;   // [ceil(N/GROUP)] dense row that holds chunk GROUP*g
  const uint64_t *list_ptr;      // [nbufs]
  const uint64_t *list_nbytes;   // [nbufs]
  const uint64_t *list_base;     // [nbufs] global id of the buffer's first chunk
  const uint8_t *spare;          // 256 readable bytes (zero), 256-byte aligned
  // Work lists of the fingerprint kernel.  Full chunks (length C) and last
  // chunks shorter than C are grouped separately so that the 16 chunks a
  // wavefront hashes together have the same length (full) or nearly the same
  // (short ones are sorted by length, longest first).
  const uint64_t *full_ptr;      // [nf]   address of a buffer that has >= 1 full chunk
  const uint64_t *full_chunk0;   // [nf]   global id of that buffer's first chunk
  const uint64_t *full_base;     // [nf+1] full chunks in earlier rows; [nf] = nfull
  const uint32_t *full_group_first;  // [ceil(nfull/GROUP)] row holding full chunk GROUP*g
  const uint64_t *short_ptr;     // [nshort] address of the short chunk
  const uint64_t *short_chunk;   // [nshort] its global id
  const uint32_t *short_len;     // [nshort] its length, descending
  uint64_t nfull;                // chunks of length C
  uint64_t nshort;               // chunks shorter than C (at most one per buffer)
  uint64_t nchunks;              // N
  uint64_t nbufs;                // B (caller's list length)
  uint32_t nb;                   // dense rows
  uint32_t chunk_log2;           // log2(C)
};

struct ChunkRef {
  uint32_t row;   // dense row
  uint32_t len;   // chunk length in bytes
  uint64_t off;   // offset inside the buffer
};

// Buffer row, offset and length of global chunk k (k < N).  The group table
// gives the row of the group's first chunk; at most GROUP-1 rows follow before
// the one that owns k, because every dense row owns at least one chunk.
__device__ __forceinline__ ChunkRef locate_chunk(const PlanDev &p, uint64_t k) {
  uint32_t row = p.group_first[k >> GROUP_LOG2];
  while (k >= p.dense_base[row + 1]) ++row;   // ends: dense_base[nb] = N > k
  ChunkRef r;
  r.row = row;
  r.off = (k - p.dense_base[row]) << p.chunk_log2;
  uint64_t rem = p.dense_nbytes[row] - r.off;
  uint64_t c = 1ull << p.chunk_log2;
  r.len = (uint32_t)(rem < c ? rem : c);
  return r;
}

// The same for n consecutive chunks k0 .. k0+n-1 (all < N), for small n: one walk from the
// group table instead of n, since a chain of dependent loads per chunk is what the scan kernels
// spend their time on.  From one chunk to the next the row advances by at most one (every row
// owns at least one chunk).
__device__ __forceinline__ void locate_run(const PlanDev &p, uint64_t k0, int n, ChunkRef *refs) {
  if (n <= 0) return;
  uint32_t row = p.group_first[k0 >> GROUP_LOG2];
  uint64_t next = p.dense_base[row + 1];
  while (k0 >= next) next = p.dense_base[++row + 1];          // ends: dense_base[nb] = N > k0
  uint64_t base = p.dense_base[row], nbytes = p.dense_nbytes[row];
  const uint64_t c = 1ull << p.chunk_log2;
  for (int i = 0; i < n; ++i) {
    const uint64_t k = k0 + i;
    if (k >= next) {
      base = next;
      next = p.dense_base[++row + 1];
      nbytes = p.dense_nbytes[row];
    }
    refs[i].row = row;
    refs[i].off = (k - base) << p.chunk_log2;
    const uint64_t rem = nbytes - refs[i].off;
    refs[i].len = (uint32_t)(rem < c ? rem : c);
  }
}

__device__ __forceinline__ uint64_t pad16(uint64_t x) { return (x + 15) & ~15ull; }

// Scan geometry: one workgroup of SCAN_THREADS threads covers SCAN_BLOCK
// consecutive chunk ids, SCAN_PER_THREAD each.
constexpr int SCAN_THREADS = 256;
constexpr int SCAN_PER_THREAD = 4;
constexpr int SCAN_BLOCK = SCAN_THREADS * SCAN_PER_THREAD;
// Scan scratch (owned by a plan): one (count, bytes) pair per SCAN_BLOCK chunks, and one spare
// pair whose first word ckpt_exchange uses.
// Up to this many chunks a workgroup finds its own scan offset by counting the mask bytes in
// front of its block (at most 256 KiB per workgroup), which makes the scan a single kernel.
constexpr uint64_t SMALL_SCAN_CHUNKS = 1ull << 18;

// Fused snapshot: where the hint's derived state lives in the caller's workspace.
struct HintState {
  uint64_t *hoff;     // [N] staging offset every chunk would get if the hint were the mask
  uint64_t *misses;   // counter block, SNAPSHOT_COUNTERS words: [0] chunks where hint != mask
  uint8_t *copy;      // [N] private copy of the hint
  uint8_t *need;      // [entries] 1 = the gather after a wrong hint must copy this entry
};

// Copy geometry: one wavefront moves one piece of one staged chunk per
// iteration; a piece is min(C, COPY_PIECE) bytes.
constexpr int COPY_PIECE_LOG2 = 14;
constexpr int COPY_THREADS = 256;
constexpr int COPY_MAX_GROUPS = 65536;

// launchers (each returns the hipError_t of the launch)
hipError_t launch_fingerprint(const PlanDev &p, uint64_t *d_digests, hipStream_t s);
// The same pass, also writing d_mask[k] = (d_ref == null || digest != d_ref[k]) and clearing
// d_counts->overflow and *d_misses_out (may be null) for the manifest kernel that follows.
hipError_t launch_fingerprint_diff(const PlanDev &p, uint64_t *d_digests, const uint64_t *d_ref,
                                   uint8_t *d_mask, ckpt_counts_t *d_counts, uint64_t *d_misses_out,
                                   hipStream_t s);
hipError_t launch_diff(const PlanDev &p, const uint64_t *d_dig, const uint64_t *d_ref,
                       uint8_t *d_mask, uint64_t *d_pairs, ckpt_counts_t *d_counts, hipStream_t s);
// Manifest and counts for a mask.  h (fused snapshot, may be null): hint misses are counted into
// h->misses[0] and entries the pass has already staged in place are marked in h->need;
// *d_misses_out (may be null) receives the miss count, 0 without h.  cleared: an earlier kernel
// of the same call has zeroed d_counts->overflow, *d_misses_out and h's counters.
hipError_t launch_compact_scan(const PlanDev &p, const uint8_t *d_mask, const uint64_t *d_dig,
                               uint64_t staging_cap, ckpt_entry_t *d_manifest,
                               uint64_t manifest_cap, uint64_t *d_pairs, ckpt_counts_t *d_counts,
                               const HintState *h, uint64_t *d_misses_out, bool cleared,
                               hipStream_t s);
// d_only_if_nonzero (may be null): the kernel does nothing when it points to 0;  d_need (may be
// null): entries e with d_need[e] == 0 are skipped.
hipError_t launch_gather(const PlanDev &p, const ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                         const ckpt_counts_t *d_counts, void *d_staging, uint64_t staging_cap,
                         const uint64_t *d_only_if_nonzero, const uint8_t *d_need, hipStream_t s);
// The fused pass: fingerprint + mask + staging of the hinted chunks.  d_list: one uint32, d_flags:
// one byte per fingerprint group; d_list_counts: two uint64, zero on entry; split: staging groups
// and the rest in two launches (pays off from a few hundred MB of state).
hipError_t launch_fingerprint_staging(const PlanDev &p, uint64_t *d_digests, const uint64_t *d_ref,
                                      uint8_t *d_mask, const uint8_t *d_hint,
                                      const uint64_t *d_hint_off, void *d_staging,
                                      uint64_t staging_cap, uint32_t *d_list, uint8_t *d_flags,
                                      uint64_t *d_list_counts, bool split, hipStream_t s);
uint64_t fingerprint_groups(const PlanDev &p);
// 64-bit words at the head of the fused snapshot's counter block, cleared by
// launch_hint_offsets: [0] hint misses, [1..3] scratch counts of the hint (word 3 ends up zero and
// then receives the number of chunks the corrective gather has to copy), [4..5] group list lengths.
constexpr int SNAPSHOT_COUNTERS = 6;
hipError_t launch_hint_offsets(const PlanDev &p, const uint8_t *d_hint_in, const HintState &h,
                               uint64_t *d_pairs, ckpt_counts_t *d_tmp_counts, uint64_t manifest_cap,
                               ckpt_counts_t *d_counts, uint64_t *d_misses_out, hipStream_t s);
// Applies min(nentries, d_counts->ndirty) entries when d_counts is not null, else nentries.
hipError_t launch_scatter(const PlanDev &p, const ckpt_entry_t *d_manifest, uint64_t nentries,
                          const ckpt_counts_t *d_counts, const void *d_staging,
                          uint64_t staging_bytes, uint64_t *d_rejected, hipStream_t s);
// As launch_scatter, but the kernel does nothing when *d_only_if_nonzero == 0, and d_rejected
// (may be null) is added to, not cleared first.
hipError_t launch_scatter_gated(const PlanDev &p, const ckpt_entry_t *d_manifest, uint64_t nentries,
                                const ckpt_counts_t *d_counts, const void *d_staging,
                                uint64_t staging_bytes, uint64_t *d_rejected,
                                const uint64_t *d_only_if_nonzero, hipStream_t s);
// Swap-out of one manifest's chunks and swap-in of another's in one pass when the two describe
// the same places, else one after the other; *d_differs (scratch word) receives the number of
// places where they differ, *d_serial (may be null) a copy of it.
hipError_t launch_exchange(const PlanDev &p, const ckpt_entry_t *d_manifest_out,
                           const ckpt_counts_t *d_counts_out, void *d_stage_out, uint64_t out_cap,
                           const ckpt_entry_t *d_manifest_in, const ckpt_counts_t *d_counts_in,
                           const void *d_stage_in, uint64_t in_bytes, uint64_t manifest_cap,
                           uint64_t *d_differs, uint64_t *d_serial, uint64_t *d_rejected,
                           hipStream_t s);
// A chain of incremental snapshots, oldest first, as the kernels take it (by value).
struct ChainArgs {
  const uint8_t *staging[CKPT_CHAIN_MAX];
  uint64_t staging_bytes[CKPT_CHAIN_MAX];
  const ckpt_entry_t *manifest[CKPT_CHAIN_MAX];
  uint64_t cap[CKPT_CHAIN_MAX];                 // entries the manifest can hold
  const ckpt_counts_t *counts[CKPT_CHAIN_MAX];  // null: cap entries; else min(cap, ndirty)
  uint32_t nlinks;
};
// d_only (may be null): chunks with d_only[k] == 0 are left alone; d_workspace: 2 N + 1 uint64
// (scratch); d_stats (may be null): written, superseded, skipped.
hipError_t launch_restore_chain(const PlanDev &p, const ChainArgs &a, const uint8_t *d_only,
                                uint64_t *d_workspace, uint64_t *d_stats, hipStream_t s);
// Folds the chain into one link laid out like a snapshot's.  d_workspace: 2 N + 2 uint64 and N
// bytes (scratch); d_pairs: the plan's scan scratch.
hipError_t launch_merge_chain(const PlanDev &p, const ChainArgs &a, void *d_staging,
                              uint64_t staging_cap, ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                              ckpt_counts_t *d_counts, uint64_t *d_workspace, uint64_t *d_pairs,
                              uint64_t *d_stats, hipStream_t s);
hipError_t launch_upload_owners(const PlanDev &p, const uint64_t *d_gathered, uint32_t world,
                                uint32_t rank, uint8_t *d_mask, uint64_t *d_blocksums,
                                ckpt_counts_t *d_counts, hipStream_t s);
// d_flags: one byte per buffer of the caller's list; d_marks: one per chunk.
hipError_t launch_marks_from_buffers(const PlanDev &p, const uint8_t *d_flags, uint8_t *d_marks,
                                     hipStream_t s);
// d_out may be d_mask or d_without itself.
hipError_t launch_mask_andnot(uint64_t n, const uint8_t *d_mask, const uint8_t *d_without,
                              uint8_t *d_out, hipStream_t s);
// d_dirty: one byte per buffer of the caller's list; d_counts: buffers that differ, their bytes.
hipError_t launch_buffer_verdicts(const PlanDev &p, const uint8_t *d_mask, uint8_t *d_dirty,
                                  uint64_t *d_counts, hipStream_t s);
hipError_t launch_validate(uint64_t n, const uint64_t *b_a, const uint64_t *a_a, const uint64_t *b_b,
                           const uint64_t *a_b, ckpt_validation_t *d_result, hipStream_t s);
uint64_t match_workspace_bytes(uint64_t n_ref, uint64_t n);
hipError_t launch_match(const PlanDev &p, const uint64_t *d_dig, const uint64_t *d_ref,
                        uint64_t n_ref, void *d_workspace, int64_t *d_src, uint8_t *d_mask,
                        ckpt_match_counts_t *d_counts, hipStream_t s);
hipError_t launch_apply_matches(const PlanDev &dstp, const PlanDev *refp, const int64_t *d_src,
                                uint64_t *d_rejected, hipStream_t s);
uint64_t moves_workspace_bytes(uint64_t n);
hipError_t launch_moves_inplace(const PlanDev &p, const int64_t *d_src, void *d_temp,
                                uint64_t temp_cap, void *d_workspace, uint64_t *d_blocksums,
                                ckpt_counts_t *d_counts, uint64_t *d_rejected, hipStream_t s);
hipError_t launch_slice(bool gather, const PlanDev &p, const ckpt_entry_t *d_manifest,
                        uint64_t nentries, void *d_ring, uint64_t b0, uint64_t b1,
                        uint64_t *d_rejected, hipStream_t s);
hipError_t launch_zero_u64(uint64_t *d_value, hipStream_t s);
hipError_t launch_bw_copy(void *d_dst, const void *d_src, uint64_t nbytes, hipStream_t s);
hipError_t launch_bw_read(const void *d_src, uint64_t nbytes, uint64_t *d_sink, hipStream_t s);
hipError_t launch_bw_streams(void *d_dst, const void *d_src, uint64_t nstreams,
                             uint64_t stream_bytes, uint32_t tile_bytes, uint64_t *d_sink,
                             hipStream_t s);
constexpr uint32_t ALU_PROBE_GROUPS = 2048;   // workgroups of 256 lanes in the hash-only probe
hipError_t launch_alu_xxh64(uint64_t rounds_per_lane, uint64_t *d_sink, hipStream_t s);

// access to the opaque plan from the other host translation units
const PlanDev *plan_dev(const ckpt_plan_t *plan);
uint64_t *plan_scratch(const ckpt_plan_t *plan);
void set_last_device_error(hipError_t e);

}  // namespace ckpt
