/*
 * ckpt.h -- C ABI of the MI355X device-state snapshot library (libckpt.so).
 *
 * The path it implements is the checksum-deduplicated swap-out / swap-in of a
 * training job's live device buffers described in the Singularity paper:
 *   sec. 5.2.1  content checksums of every live buffer at a context switch;
 *               a buffer whose checksum is already known is not swapped out;
 *               with 4 ranks on a GPU only the first swaps out P and O;
 *   sec. 4.6    the same checksum de-dup across workers before a checkpoint
 *               upload, and across time (incremental checkpoints);
 *   sec. 5.2.3  mutations between two points = difference of checksum state;
 *   sec. 4.5    restore copies the tensors back to the addresses they had;
 *   sec. 6      the checksum kernels are ordinary stream work, the comparison
 *               used to be host work -- here it runs on the device too.
 * The paper names no checksum function and works per buffer; this library
 * fingerprints fixed-size chunks inside each buffer with XXH64, seed 0.
 *
 * Model
 *   A plan describes a list of B live buffers (device pointer, size) and a
 *   chunk size C.  Buffer i is cut into n_i = ceil(nbytes_i / C) chunks; the
 *   last one may be short; an empty buffer has none.  Chunks are numbered
 *   globally in list order: k = (sum of n_i' for i' < i) + j.  N = sum n_i.
 *
 * Conventions for every call
 *   - Pointers named d_* are DEVICE pointers owned by the caller; everything
 *     else is host memory.  The library allocates device memory only inside
 *     ckpt_plan_create (descriptor tables and a small scan scratch) and frees
 *     it in ckpt_plan_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     The four data calls only enqueue kernels on it and return; outputs are
 *     valid once the caller has synchronised the stream.  Calls on one stream
 *     are ordered.  A plan must not be used by two streams at once (its scan
 *     scratch is shared).
 *   - Return value: 0 (CKPT_OK) or a negative ckpt_status.  Argument errors
 *     are reported synchronously and nothing is enqueued.  Nothing is ever
 *     written outside the ranges described below, also on capacity overflow.
 *   - The current HIP device must be the one that owns the buffers.
 */
#ifndef CKPT_H_
#define CKPT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ckpt_status {
  CKPT_OK = 0,
  CKPT_ERR_INVALID_ARG = -1, /* NULL where a pointer is required, size overflow */
  CKPT_ERR_ALIGNMENT = -2,   /* a buffer / staging / digest / manifest pointer is misaligned */
  CKPT_ERR_CHUNK = -3,       /* chunk size not a power of two in [256 B, 1 GiB], or two plans differ */
  CKPT_ERR_GEOMETRY = -4,    /* reference digest count differs from the plan's N */
  CKPT_ERR_CAPACITY = -5,    /* workspace too small (ckpt_match, ckpt_restore_chain,
                                ckpt_merge_chain), plan too large (ckpt_snapshot_static); also
                                free for callers that turn counts.overflow into a status */
  CKPT_ERR_DEVICE = -6,      /* a HIP call failed (see ckpt_last_device_error) */
  CKPT_ERR_NOMEM = -7        /* host or device allocation failed in ckpt_plan_create */
} ckpt_status;

/* One live buffer.  ptr: device address, 16-byte aligned (unless nbytes == 0,
 * then it is ignored).  The buffers of one list may not overlap. */
typedef struct ckpt_buf {
  void *ptr;
  uint64_t nbytes;
} ckpt_buf_t;

/* One staged chunk; 32 bytes, device-resident array written by ckpt_compact in
 * ascending global chunk order. */
typedef struct ckpt_entry {
  uint32_t buf;       /* index of the chunk's buffer in the plan's list */
  uint32_t len;       /* chunk length in bytes (C, or less for a last chunk) */
  uint64_t buf_off;   /* offset of the chunk in its buffer (multiple of C) */
  uint64_t stage_off; /* offset of the chunk in staging (multiple of 16) */
  uint64_t digest;    /* XXH64 of the chunk */
} ckpt_entry_t;

typedef struct ckpt_counts {
  uint64_t ndirty;       /* chunks with mask 1 */
  uint64_t staged_bytes; /* sum over those chunks of len rounded up to 16 */
  uint64_t overflow;     /* dirty chunks ckpt_compact could not stage (0 = complete) */
} ckpt_counts_t;

typedef struct ckpt_plan ckpt_plan_t; /* opaque, library-owned */

/* ---- plan --------------------------------------------------------------- */

/* Builds the chunk geometry of a buffer list (the paper's device proxy knows
 * every live buffer because it owns the allocator, sec. 3.2.1 / 5.2.1) and
 * uploads the descriptor tables to the current device.  Synchronous.
 *   bufs        host array of nbufs descriptors (may be NULL when nbufs == 0)
 *   chunk_bytes C: power of two, 256 <= C <= 2^30.  A chunk is hashed by four
 *               lanes (XXH64 has four independent accumulators), so speed needs
 *               many chunks: keep at least about 10 000 of them (1 KiB..2 MiB
 *               chunks for states of 100 MB..100 GB); with a few hundred the
 *               fingerprint runs at a fraction of the memory bandwidth
 *   out         receives the plan; destroy it with ckpt_plan_destroy
 * A plan also owns a small scan scratch that ckpt_diff, ckpt_compact,
 * ckpt_snapshot, ckpt_manifest, ckpt_exchange, ckpt_merge_chain,
 * ckpt_upload_owners, ckpt_swap_out and ckpt_apply_moves_inplace write: calls of
 * these on ONE plan must be ordered (one stream, or events); issued on two
 * streams at once they race.  ckpt_fingerprint, ckpt_restore,
 * ckpt_restore_chain and the other calls only read the plan and may overlap
 * freely.
 * Two non-empty buffers that share a byte are refused (INVALID_ARG): restoring
 * into such a list has no defined result, and an allocator never hands out
 * overlapping live buffers.
 * Errors: INVALID_ARG, CHUNK, ALIGNMENT (ptr not 16-byte aligned),
 * NOMEM, DEVICE. */
int ckpt_plan_create(const ckpt_buf_t *bufs, uint64_t nbufs, uint64_t chunk_bytes,
                     ckpt_plan_t **out);

/* Frees the plan's host and device memory.  The caller must have synchronised
 * every stream that used it.  NULL is accepted. */
int ckpt_plan_destroy(ckpt_plan_t *plan);

uint64_t ckpt_plan_nchunks(const ckpt_plan_t *plan);     /* N */
uint64_t ckpt_plan_nbytes(const ckpt_plan_t *plan);      /* S = sum nbytes_i */
uint64_t ckpt_plan_nbufs(const ckpt_plan_t *plan);       /* B */
uint64_t ckpt_plan_chunk_bytes(const ckpt_plan_t *plan); /* C */

/* Tuning of ckpt_snapshot with a hint, per plan: a plan of at least this many
 * bytes runs the pass as two launches (the chunks that are staged, then the
 * rest: read/write traffic and pure reads do not mix, which is faster from a
 * few hundred MB of state), a smaller one as a single launch (fewer kernels).
 * Results are identical either way.  Default 256 MiB; 0 = always two launches,
 * UINT64_MAX = never.  Set it while no call on the plan is being issued. */
uint64_t ckpt_plan_split_threshold(const ckpt_plan_t *plan);
int ckpt_plan_set_split_threshold(ckpt_plan_t *plan, uint64_t nbytes);

/* ---- the four data calls ------------------------------------------------- */

/* Content checksum of every chunk (sec. 5.2.1, sec. 6: checksums of all live
 * buffers are computed at every context switch):
 *   d_digests[k] = XXH64(bytes of chunk k, length len_k, seed 0), k in [0, N).
 * A short last chunk is hashed at its true length.  Reads every buffer byte
 * once and nothing else; writes N native-endian uint64.
 *   d_digests   device array of N uint64, 8-byte aligned
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_fingerprint(const ckpt_plan_t *plan, uint64_t *d_digests, void *stream);

/* Positional comparison with a reference replica's or an earlier snapshot's
 * checksums (sec. 5.2.1: a buffer whose checksum is already known is not
 * swapped; sec. 4.6; sec. 5.2.3):
 *   d_mask[k] = 1 if d_ref == NULL or d_digests[k] != d_ref[k], else 0.
 *   d_counts->ndirty = number of ones, ->staged_bytes = staging size
 *   ckpt_compact will need for them, ->overflow = 0.
 *   d_ref   device array of n_ref uint64, or NULL (no reference: the first
 *           rank really swaps everything out); n_ref must equal N otherwise
 *   d_mask  device array of N bytes
 *   d_counts device ckpt_counts_t, 8-byte aligned
 * Errors: INVALID_ARG, GEOMETRY (n_ref != N), ALIGNMENT, DEVICE. */
int ckpt_diff(const ckpt_plan_t *plan, const uint64_t *d_digests, const uint64_t *d_ref,
              uint64_t n_ref, uint8_t *d_mask, ckpt_counts_t *d_counts, void *stream);

/* Which chunks this worker uploads into a checkpoint when `world` workers hold
 * replicas of the job (sec. 4.6: a worker uploads a buffer only if no other
 * worker uploads the same content).  d_gathered holds the checksums of all
 * workers, row r = worker r's N checksums (one chunk geometry for all workers,
 * as consistent allocation gives, sec. 5.2.2; how the rows were exchanged is
 * the caller's business).  Per chunk k the workers whose checksum equals this
 * worker's form a group in ascending rank order, and member number
 * (k mod group size) uploads:
 *   d_mask[k] = 1 if that member is `rank`, else 0;  d_counts as ckpt_diff.
 * Every distinct content at every position is uploaded by exactly one worker;
 * content shared by all is spread evenly.  The mask feeds ckpt_compact.
 *   d_gathered  device array of world*N uint64, row-major, 8-byte aligned
 * Errors: INVALID_ARG (world == 0, rank >= world, NULL), ALIGNMENT, DEVICE. */
int ckpt_upload_owners(const ckpt_plan_t *plan, const uint64_t *d_gathered, uint32_t world,
                       uint32_t rank, uint8_t *d_mask, ckpt_counts_t *d_counts, void *stream);

/* Swap-out of what is not de-duplicated (sec. 5.2.1), as a gather into one
 * contiguous staging buffer: walking k upwards, each chunk with d_mask[k] != 0
 * gets the next manifest entry e and the next pad16(len_k) bytes of staging
 * (its bytes, then zeros up to a multiple of 16), so
 *   stage_off[0] = 0, stage_off[e+1] = stage_off[e] + pad16(len[e]).
 * d_counts receives ndirty, staged_bytes (both the full need, whatever the
 * capacities) and overflow.
 *   d_staging    buffer of staging_cap bytes the device can address, 16-byte
 *                aligned, not overlapping any plan buffer: device memory, or
 *                pinned host memory (hipHostMalloc) -- then the kernel writes
 *                the bytes over the host link itself and the call is the
 *                paper's swap-out to host memory, still asynchronous.  The
 *                same holds for ckpt_snapshot and, reading, for ckpt_restore
 *   d_manifest   device array of manifest_cap entries, 8-byte aligned
 * Capacity: entry e is written only if e < manifest_cap; its bytes are written
 * only if also stage_off + pad16(len) <= staging_cap.  Every dirty chunk that
 * is not fully staged adds 1 to d_counts->overflow; nothing is written past
 * either capacity.  (The prefix that fits is complete and usable.)
 * The call is stream-ordered and reads nothing back, so it cannot know on the
 * host whether the capacities sufficed and never returns CKPT_ERR_CAPACITY
 * itself: the caller reads d_counts->overflow after synchronising (non-zero =
 * incomplete) and may map that to CKPT_ERR_CAPACITY.
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_compact(const ckpt_plan_t *plan, const uint8_t *d_mask, const uint64_t *d_digests,
                 void *d_staging, uint64_t staging_cap, ckpt_entry_t *d_manifest,
                 uint64_t manifest_cap, ckpt_counts_t *d_counts, void *stream);

/* The metadata half of ckpt_compact alone: d_manifest and d_counts exactly as
 * ckpt_compact writes them for the same arguments (staging_cap only decides
 * which entries count as overflow), and not a byte of chunk data moved.  For
 * callers that move the bytes another way: ckpt_exchange below.
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_manifest(const ckpt_plan_t *plan, const uint8_t *d_mask, const uint64_t *d_digests,
                  uint64_t staging_cap, ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                  ckpt_counts_t *d_counts, void *stream);

/* A whole context switch between two ranks that share the plan's buffers
 * (sec. 5.1, 5.2.1): the outgoing rank's chunks (d_manifest_out, from
 * ckpt_manifest or ckpt_compact on its mask, d_counts_out->ndirty entries) go to
 * d_staging_out as ckpt_compact would stage them, and the incoming rank's
 * chunks (d_manifest_in, d_counts_in->ndirty entries, bytes in d_staging_in)
 * come into the buffers as ckpt_restore_counted would put them -- the same
 * result as those two calls one after the other.
 * Ranks of a data-parallel job that are time-sliced on one GPU differ from
 * their shared base in the same chunks, so the two manifests normally name the
 * same buffer ranges and staging offsets entry by entry.  The call checks that
 * on the device; if it holds, one kernel exchanges each chunk in place (reads
 * the outgoing bytes from the buffer and the incoming bytes from d_staging_in,
 * writes each where the other came from): with both staging areas in pinned
 * host memory the host link carries both directions at once.  If it does not
 * hold, the swap-out and the swap-in run one after the other instead.  Nothing
 * is read on the host either way.
 *   staging_out_cap   bytes d_staging_out can hold; staging_in_bytes: valid
 *                     bytes of d_staging_in.  The two areas must not overlap
 *                     each other or the buffers.
 *   manifest_cap      entries each manifest can hold (upper bound on reads)
 *   d_serial          optional device uint64: 0 if the single exchange pass
 *                     ran, else the number of places where the manifests differ
 *   d_rejected        optional device uint64: entries skipped because they do
 *                     not fit the plan or a staging area (0 = none)
 * Writes one word of the plan's scratch: order it like ckpt_diff / ckpt_compact.
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_exchange(const ckpt_plan_t *plan, const ckpt_entry_t *d_manifest_out,
                  const ckpt_counts_t *d_counts_out, void *d_staging_out, uint64_t staging_out_cap,
                  const ckpt_entry_t *d_manifest_in, const ckpt_counts_t *d_counts_in,
                  const void *d_staging_in, uint64_t staging_in_bytes, uint64_t manifest_cap,
                  uint64_t *d_serial, uint64_t *d_rejected, void *stream);

/* The three calls above as one, with the same outputs bit for bit (d_digests,
 * d_mask, d_staging, d_manifest, d_counts), optionally in a single pass over the
 * data.  d_hint (N bytes, or NULL) predicts the mask -- at a context switch the
 * previous switch's mask is the natural prediction, since which buffers are
 * per-replica state does not change (sec. 5.2.1).  With a hint, the staging
 * offsets of the predicted chunks are computed first and the fingerprint pass
 * writes each predicted chunk to its staging place while hashing it, so no byte
 * is read twice.  Afterwards the real mask is compared with the hint: if they are
 * equal staging is complete; if not, a gather copies the chunks that are not yet
 * at their final staging offset -- those behind the first chunk the hint got
 * wrong; the ones before it stay as the pass wrote them -- so a wrong hint costs
 * time, never correctness, and a late miss costs little.  (Measured on MI355X the
 * single pass wins once the hint marks more than about a fifth of the bytes; below
 * that, mixing the staging writes into the read stream costs more than the second
 * read it saves -- pass NULL then.)
 *   d_hint          may be the same buffer as d_mask (it is copied first)
 *   d_hint_misses   optional device uint64: chunks where hint and mask differ
 *                   (0 = the single pass sufficed; always 0 without a hint)
 *   d_workspace     device scratch, ckpt_snapshot_workspace_bytes(N) bytes, 16-byte
 *                   aligned; needed only with a hint
 * d_staging must not overlap d_hint or d_workspace.  Note that without
 * synchronising, a wrong hint may have written bytes of clean chunks into
 * staging beyond the final staged_bytes (never beyond staging_cap).
 * Errors: INVALID_ARG, GEOMETRY, ALIGNMENT, CAPACITY (workspace too small), DEVICE. */
uint64_t ckpt_snapshot_workspace_bytes(uint64_t nchunks);
/* Diagnostics of a hinted ckpt_snapshot, readable once the stream is synchronised:
 * at this byte offset of d_workspace sit four uint64 -- [0] the hint misses (as
 * *d_hint_misses), [1] and [2] unspecified, [3] the number of chunks the
 * corrective gather copies after the pass (0 with an exact hint; with one wrong
 * chunk, the staged chunks behind it). */
uint64_t ckpt_snapshot_stats_offset(uint64_t nchunks);
int ckpt_snapshot(const ckpt_plan_t *plan, const uint64_t *d_ref, uint64_t n_ref,
                  const uint8_t *d_hint, uint64_t *d_digests, uint8_t *d_mask, void *d_staging,
                  uint64_t staging_cap, ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                  ckpt_counts_t *d_counts, uint64_t *d_hint_misses, void *d_workspace,
                  uint64_t workspace_bytes, void *stream);

/* ckpt_snapshot for callers that cannot allocate device memory or carry a
 * workspace around: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * ckpt_snapshot minus the workspace: the hint offsets, counters, group lists
 * and the scan scratch (which ckpt_snapshot takes from d_workspace and from
 * the plan) live in one static device array inside the library, about 2.6 MiB,
 * which every GPU the library runs on holds until the process ends.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine);
 * its only set-up is one symbol-address lookup per device on the first call
 * there.
 *   Limit: plans of at most ckpt_snapshot_static_max_chunks() = 262 144 chunks;
 *   larger ones are refused with CKPT_ERR_CAPACITY and nothing is enqueued.
 *   The current device must be the plan's (INVALID_ARG otherwise).
 * All calls on one GPU share that array, which keeps the last call's contents
 * (every word a call reads it has written first): calls must be ordered on the
 * GPU -- one stream, or events -- also across plans; two that overlap race.
 * Errors: as ckpt_snapshot, plus CAPACITY for a plan above the limit. */
uint64_t ckpt_snapshot_static_max_chunks(void);
int ckpt_snapshot_static(const ckpt_plan_t *plan, const uint64_t *d_ref, uint64_t n_ref,
                         const uint8_t *d_hint, uint64_t *d_digests, uint8_t *d_mask,
                         void *d_staging, uint64_t staging_cap, ckpt_entry_t *d_manifest,
                         uint64_t manifest_cap, ckpt_counts_t *d_counts, uint64_t *d_hint_misses,
                         void *stream);

/* Swap-in / restore (sec. 4.5, sec. 5.2.1): for each of the first nentries
 * manifest entries, copy len bytes from d_staging + stage_off to buffer
 * entry.buf of dst_plan at offset buf_off.  Chunks without an entry are not
 * touched (the caller guarantees they already hold the reference's bytes).
 * An entry that names a buffer outside dst_plan, a range outside that buffer,
 * a range outside [0, staging_bytes), offsets that are not multiples of 16, or
 * a length above the chunk size is skipped, never partially applied.  Whether
 * an entry fits is only known when the kernel reads it, so a bad manifest is
 * not a host-side CKPT_ERR_GEOMETRY: the count of skipped entries is the
 * report, and a caller that must fail hard checks it after synchronising.
 *   d_rejected  optional device uint64 that receives the number of skipped
 *               entries (0 = all applied); may be NULL
 * dst_plan may be the snapshot's own plan or another one with compatible
 * geometry (e.g. the buffers of a different replica).
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_restore(const ckpt_plan_t *dst_plan, const void *d_staging, uint64_t staging_bytes,
                 const ckpt_entry_t *d_manifest, uint64_t nentries, uint64_t *d_rejected,
                 void *stream);

/* ckpt_restore whose entry count is read on the device when the kernel runs:
 * the first min(manifest_cap, d_counts->ndirty) entries are applied, d_counts
 * being what ckpt_compact / ckpt_snapshot wrote earlier on the stream.  With
 * it a whole switch (checksum, compare, swap-out, swap-in) is enqueued without
 * the host ever reading a result, so the next rank's operations can be
 * dispatched at once behind an event (the eager dispatch of sec. 6), and a
 * captured graph replays correctly when the number of dirty chunks changes.
 *   manifest_cap  entries d_manifest can hold (upper bound on what is read)
 *   d_counts      device ckpt_counts_t, 8-byte aligned; only ndirty is read
 * Everything else as ckpt_restore.
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_restore_counted(const ckpt_plan_t *dst_plan, const void *d_staging, uint64_t staging_bytes,
                         const ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                         const ckpt_counts_t *d_counts, uint64_t *d_rejected, void *stream);

/* ---- restore from a chain of incremental snapshots ------------------------ */

/* Sec. 4.6 de-duplicates successive checkpoints of one process against each
 * other, so every checkpoint after the first holds only what changed since the
 * one before, and a restore applies a chain of them.  ckpt_restore_chain gives
 * the result of calling ckpt_restore_counted for links[0], links[1], ... in that
 * order (links[0] is the oldest), but writes every chunk of the destination once,
 * from the last entry of the chain that holds it: state that changes in every
 * link (gradients, activations) is not copied once per link.
 * An entry is applied only if it is a whole chunk of dst_plan -- every link was
 * taken with dst_plan's geometry: buf < B, buf_off a multiple of C inside the
 * buffer, len equal to that chunk's length, stage_off a multiple of 16 and
 * [stage_off, stage_off + len) inside the link's staging area.  Other entries
 * are skipped and counted, and a chunk only they name keeps what an earlier
 * link, or the caller, put there.
 *   links        HOST array of nlinks descriptors (read during the call); every
 *                pointer inside is a device pointer the caller owns
 *     d_staging, staging_bytes   the link's staging area (16-byte aligned)
 *     d_manifest, manifest_cap   its manifest and how many entries it can hold
 *     d_counts   optional device ckpt_counts_t: min(manifest_cap, ndirty)
 *                entries are applied, read on the device when the kernels run;
 *                NULL: manifest_cap entries
 *   nlinks       at most CKPT_CHAIN_MAX; a longer chain is restored by
 *                consecutive calls, oldest links first
 *   d_only       optional device array of N bytes that restricts the restore:
 *                a chunk with d_only[k] == 0 keeps its bytes whatever the links
 *                hold, and entries naming it are counted nowhere.  At a context
 *                switch (sec. 5.2.1 skips the swap-in of what the device already
 *                holds) this is ckpt_diff of the incoming rank's digests against
 *                the resident rank's, and the chain is [a full copy of the
 *                common base, the incoming rank's delta]: exactly the chunks in
 *                which the two ranks differ come in, from the delta where it has
 *                them and from the base where the incoming rank never changed
 *                what the resident one did
 *   d_workspace  device scratch of at least
 *                ckpt_restore_chain_workspace_bytes(N) bytes, 16-byte aligned
 *   d_stats      optional device ckpt_chain_stats_t, 8-byte aligned
 * Stream-ordered, no allocation, nothing read back.
 * Errors: INVALID_ARG (NULL, nlinks > CKPT_CHAIN_MAX, manifest_cap >= 2^40),
 * ALIGNMENT, CAPACITY (workspace too small), DEVICE. */
#define CKPT_CHAIN_MAX 16
typedef struct ckpt_link {
  const void *d_staging;
  uint64_t staging_bytes;
  const ckpt_entry_t *d_manifest;
  uint64_t manifest_cap;
  const ckpt_counts_t *d_counts;
} ckpt_link_t;
typedef struct ckpt_chain_stats {
  uint64_t written;    /* chunks of the destination written (each once) */
  uint64_t superseded; /* whole-chunk entries not copied because a later entry holds the chunk */
  uint64_t rejected;   /* entries skipped because they are not whole chunks of dst_plan */
} ckpt_chain_stats_t;
uint64_t ckpt_restore_chain_workspace_bytes(uint64_t nchunks);
int ckpt_restore_chain(const ckpt_plan_t *dst_plan, const ckpt_link_t *links, uint64_t nlinks,
                       const uint8_t *d_only, void *d_workspace, uint64_t workspace_bytes,
                       ckpt_chain_stats_t *d_stats, void *stream);

/* Folds a chain into ONE link that restores to the same result, so that a chain
 * of increments (sec. 4.6) can be kept short: what a later link replaced is
 * dropped.  The chunks any link holds (rule and order as ckpt_restore_chain: the
 * last whole-chunk entry of the chain wins) are laid out exactly as
 * ckpt_compact lays out a snapshot: ascending chunk id, entry e at
 *   stage_off[0] = 0, stage_off[e+1] = stage_off[e] + pad16(len[e]),
 * bytes followed by zeros up to a multiple of 16, the entry carrying the
 * winning entry's digest.  The plan supplies the geometry only; its buffers are
 * neither read nor written, so the state itself need not be resident.
 *   d_staging, staging_cap     receives the merged bytes; 16-byte aligned, must
 *                              not overlap a link's staging area
 *   d_manifest, manifest_cap   receives the merged entries
 *   d_counts     ndirty = chunks held, staged_bytes = bytes needed (both the
 *                full need), overflow = chunks not fully staged; capacity rule
 *                as ckpt_compact
 *   d_workspace  at least ckpt_merge_chain_workspace_bytes(N) bytes, 16-byte
 *                aligned
 *   d_stats      optional, as ckpt_restore_chain (written = chunks held)
 * Uses the plan's scan scratch like ckpt_compact.
 * Errors: INVALID_ARG, ALIGNMENT, CAPACITY (workspace too small), DEVICE. */
uint64_t ckpt_merge_chain_workspace_bytes(uint64_t nchunks);
int ckpt_merge_chain(const ckpt_plan_t *plan, const ckpt_link_t *links, uint64_t nlinks,
                     void *d_staging, uint64_t staging_cap, ckpt_entry_t *d_manifest,
                     uint64_t manifest_cap, ckpt_counts_t *d_counts, void *d_workspace,
                     uint64_t workspace_bytes, ckpt_chain_stats_t *d_stats, void *stream);

/* ---- content-addressed comparison (the paper's own rule) ------------------- */

/* Sec. 5.2.1 looks a checksum up by content wherever it lives: a hit at the same
 * address needs nothing, a hit at another address becomes a device-to-device
 * move, only a miss is swapped.  ckpt_match does that lookup for every chunk of
 * the snapshot against the reference's digests (any geometry, n_ref chunks) and
 * against the snapshot itself:
 *   d_src[k] =  k         if k < n_ref and d_ref[k] == d_digests[k]   (same place)
 *               j >= 0    else the lowest j with d_ref[j] == d_digests[k] (moved)
 *               -2 - k0   else, if an earlier snapshot chunk has the same digest,
 *                         k0 being the first such chunk        (duplicate of new data)
 *               -1        else                                  (new: must be staged)
 *   d_mask[k] = 1 exactly when d_src[k] == -1, so ckpt_compact(d_mask) stages the
 *   new chunks only;  d_counts receives how many chunks fell in each class and
 *   the staging bytes the new ones need.
 *   d_workspace  device scratch of at least ckpt_match_workspace_bytes(n_ref, N)
 *                bytes, 16-byte aligned; contents are overwritten
 *   d_src        device array of N int64;  d_mask  device array of N bytes
 * table_full in the counts stays 0 (the tables are sized so that every insert
 * finds a slot); a non-zero value means the result must not be used.
 * Errors: INVALID_ARG, ALIGNMENT, CAPACITY (workspace too small), DEVICE. */
typedef struct ckpt_match_counts {
  uint64_t nsame, nmoved, ndup, nnew; /* chunks per class; they sum to N */
  uint64_t staged_bytes;              /* sum of pad16(len) over the new chunks */
  uint64_t table_full;                /* inserts that found no slot (always 0) */
} ckpt_match_counts_t;

uint64_t ckpt_match_workspace_bytes(uint64_t n_ref, uint64_t nchunks);

int ckpt_match(const ckpt_plan_t *plan, const uint64_t *d_digests, const uint64_t *d_ref,
               uint64_t n_ref, void *d_workspace, uint64_t workspace_bytes, int64_t *d_src,
               uint8_t *d_mask, ckpt_match_counts_t *d_counts, void *stream);

/* Puts the matched content into dst_plan's buffers (the device-to-device move of
 * sec. 5.2.1): a chunk with d_src[k] >= 0 is copied from chunk d_src[k] of
 * ref_plan's buffers, then a chunk with d_src[k] <= -2 from chunk -2 - d_src[k]
 * of dst_plan itself (so the new chunks must already have been restored from
 * staging on the same stream).  Chunks with -1 are not touched; a copy whose
 * source and destination address coincide is skipped.  A chunk whose source
 * does not exist, is not earlier (duplicates), or has another length is skipped
 * and counted in *d_rejected (optional, device uint64).
 * ref_plan's buffers must not overlap dst_plan's unless every match is in place
 * (for moves inside one memory image use ckpt_apply_moves_inplace).  ref_plan may
 * be NULL: then only the duplicates are filled in.  d_src must come from ckpt_match.
 * Errors: INVALID_ARG, CHUNK (the plans' chunk sizes differ), ALIGNMENT, DEVICE. */
int ckpt_apply_matches(const ckpt_plan_t *dst_plan, const ckpt_plan_t *ref_plan,
                       const int64_t *d_src, uint64_t *d_rejected, void *stream);

/* The moves when the destination IS the reference's memory (sec. 5.2.1: the
 * buffers of the rank that ran before are turned into those of the rank that runs
 * next; moves may depend on each other in cycles, which is why the paper copies
 * in phases).  plan's buffers hold the reference image, chunk for
 * chunk (n_ref == N); afterwards every chunk k with d_src[k] = j >= 0, j != k holds
 * what chunk j held BEFORE the call.  Two phases through d_temp break every cycle:
 * all sources are gathered, then all destinations written.  Chunks with
 * d_src[k] == k, -1 or <= -2 are not touched: call this first, then ckpt_restore
 * (new chunks), then ckpt_apply_matches(plan, NULL, ...) (duplicates).
 *   d_temp       device buffer of temp_cap bytes, 16-byte aligned, not overlapping
 *                the buffers; needs sum of pad16(len) over the moved chunks
 *   d_workspace  device scratch, ckpt_moves_workspace_bytes(N) bytes, 16-byte aligned
 *   d_counts     ndirty = chunks to move, staged_bytes = temp bytes they need,
 *                overflow != 0 if temp_cap is too small -- then NOTHING is moved
 *                (half a permutation would lose data)
 *   d_rejected   optional: moves whose source is no chunk or has another length
 * Errors: INVALID_ARG, ALIGNMENT, CAPACITY (workspace too small), DEVICE. */
uint64_t ckpt_moves_workspace_bytes(uint64_t nchunks);
int ckpt_apply_moves_inplace(const ckpt_plan_t *plan, const int64_t *d_src, void *d_temp,
                             uint64_t temp_cap, void *d_workspace, uint64_t workspace_bytes,
                             ckpt_counts_t *d_counts, uint64_t *d_rejected, void *stream);

/* ---- swap-out to / swap-in from host memory --------------------------------- */

/* The paper's context switch copies what is not de-duplicated to host memory and
 * back (sec. 5.1, 5.2.1).  These two calls do ckpt_compact / ckpt_restore through
 * host memory without a full-size device staging buffer: staging is cut into
 * slices; a slice is gathered into one half of a two-slot device ring and copied
 * to the host on a second stream while the next slice is gathered (the reverse
 * for swap-in).  The swapper owns the ring (2 x slice_bytes of device memory,
 * allocated once in ckpt_swapper_create), the copy stream and the events.
 *   slice_bytes  multiple of 64 KiB, 64 KiB .. 16 GiB
 * A swapper serves one call at a time. */
typedef struct ckpt_swapper ckpt_swapper_t;
int ckpt_swapper_create(uint64_t slice_bytes, ckpt_swapper_t **out);
int ckpt_swapper_destroy(ckpt_swapper_t *swapper);

/* Swap-out: same result as ckpt_compact, except that the staged bytes land in
 * h_staging (HOST memory; pinned memory is needed for the copies to overlap) and
 * the counts in *h_counts (host).  The manifest stays on the device.  Blocks the
 * calling thread until the last byte is in host memory; work is ordered after
 * what `stream` already holds.  If the manifest or h_staging is too small the
 * call returns CKPT_ERR_CAPACITY with the full need in *h_counts
 * (overflow != 0) and h_staging untouched.
 * Errors: INVALID_ARG, ALIGNMENT, CAPACITY, DEVICE. */
int ckpt_swap_out(ckpt_swapper_t *swapper, const ckpt_plan_t *plan, const uint8_t *d_mask,
                  const uint64_t *d_digests, void *h_staging, uint64_t h_staging_cap,
                  ckpt_entry_t *d_manifest, uint64_t manifest_cap, ckpt_counts_t *h_counts,
                  void *stream);

/* Swap-in: same result as ckpt_restore from a staging image in host memory.
 * d_manifest must be a manifest as ckpt_compact / ckpt_swap_out write it (entries
 * cover [0, staged_bytes) without gaps, in order); an entry that breaks that, or
 * does not fit dst_plan, ends the 64 KiB window it was met in and is counted in
 * *h_rejected (host, optional).  Blocks until the buffers are written.
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_swap_in(ckpt_swapper_t *swapper, const ckpt_plan_t *dst_plan, const void *h_staging,
                 uint64_t staged_bytes, const ckpt_entry_t *d_manifest, uint64_t nentries,
                 uint64_t *h_rejected, void *stream);

/* ---- the paper's granularity: whole buffers -------------------------------- */

/* Sec. 5.2.1 compares checksums per buffer and swaps a buffer as a whole.  The
 * same verdict from the chunk marks: buffer i differs when any of its chunks
 * has d_mask[k] != 0 (d_mask from ckpt_diff, ckpt_snapshot, ckpt_match or
 * ckpt_upload_owners).
 *   d_buf_dirty  device array of B bytes, indexed like the plan's buffer list:
 *                1 = differs, 0 = identical (also for a buffer without bytes)
 *   d_counts     buffers that differ and the sum of their sizes: what a swap at
 *                buffer granularity moves, to set against ckpt_counts_t's
 *                staged_bytes for the marked chunks alone
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
typedef struct ckpt_buffer_counts {
  uint64_t buffers; /* buffers with at least one marked chunk */
  uint64_t bytes;   /* sum of nbytes over those buffers */
} ckpt_buffer_counts_t;
int ckpt_buffer_verdicts(const ckpt_plan_t *plan, const uint8_t *d_mask, uint8_t *d_buf_dirty,
                         ckpt_buffer_counts_t *d_counts, void *stream);

/* The reverse of ckpt_buffer_verdicts: d_marks[k] = 1 for every chunk of a
 * buffer with d_buf_flags[i] != 0, else 0.  Which buffers hold per-replica state
 * is stable from switch to switch (sec. 5.2.1), so the prediction ckpt_snapshot
 * takes as d_hint can be kept as one byte per buffer -- the d_buf_dirty of the
 * previous switch, or what the allocator's owner knows -- and expanded here.
 *   d_buf_flags  device array of B bytes;  d_marks  device array of N bytes
 * Errors: INVALID_ARG, DEVICE. */
int ckpt_marks_from_buffers(const ckpt_plan_t *plan, const uint8_t *d_buf_flags, uint8_t *d_marks,
                            void *stream);

/* d_out[k] = 1 where d_mask[k] != 0 and d_without[k] == 0, else 0, for the N
 * chunks of the plan.  With d_mask the chunks in which the outgoing rank of a
 * context switch differs from the common base and d_without those of the
 * incoming rank (sec. 5.2.1), the result marks what the incoming rank's own
 * delta does not bring back -- the chunks only the outgoing rank changed -- and
 * is the d_only of a ckpt_restore_chain over a copy of the base.  d_out may be
 * d_mask or d_without.  No alignment requirement.
 * Errors: INVALID_ARG, DEVICE. */
int ckpt_mask_andnot(const ckpt_plan_t *plan, const uint8_t *d_mask, const uint8_t *d_without,
                     uint8_t *d_out, void *stream);

/* ---- squashing validation -------------------------------------------------- */

/* Sec. 5.2.3 validates operation squashing by inferring mutations from
 * checksums: what a rank changed between two points is the set of chunks whose
 * digest changed, and two ranks sharing the GPU may be squashed only if their
 * mutations are identical in address, checksum and size.  All four arrays are
 * fingerprints over ONE plan geometry (same addresses by consistent allocation,
 * hence same sizes), so the rule per chunk k is
 *   changed_a(k) == changed_b(k)  and, where changed,  after_a[k] == after_b[k]
 * with changed_x(k) = (before_x[k] != after_x[k]).
 * d_result receives { chunks a changed, chunks b changed, chunks that break the
 * rule (0 = squashing is safe), lowest such chunk id or UINT64_MAX }.
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
typedef struct ckpt_validation {
  uint64_t changed_a, changed_b, mismatches, first_mismatch;
} ckpt_validation_t;

int ckpt_validate_mutations(const ckpt_plan_t *plan, const uint64_t *d_before_a,
                            const uint64_t *d_after_a, const uint64_t *d_before_b,
                            const uint64_t *d_after_b, ckpt_validation_t *d_result, void *stream);

/* ---- helpers -------------------------------------------------------------- */

/* Plain streaming kernels used to calibrate HBM counters and the achievable
 * bandwidth next to the path's own kernels: copy nbytes (multiple of 16,
 * 16-byte aligned pointers) from d_src to d_dst; or read nbytes and write one
 * 8-byte XOR checksum per workgroup into d_sink (at least 16 KiB).
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_bw_copy(void *d_dst, const void *d_src, uint64_t nbytes, void *stream);
int ckpt_bw_read(const void *d_src, uint64_t nbytes, uint64_t *d_sink, void *stream);

/* The same two yardsticks with the fingerprint pass's access pattern: nstreams
 * (multiple of 16) streams of stream_bytes bytes each (a multiple of
 * 2 * tile_bytes), stream i at d_src + i * stream_bytes; every wavefront walks
 * 16 streams front to back, tile_bytes of each per step -- as it walks 16
 * chunks when it hashes.  tile_bytes is 256 (the fingerprint kernel's tile: one
 * load instruction takes 256 bytes from each of four streams) or 1024 (one load
 * instruction takes one kibibyte of one stream; the comparison shows what a
 * larger tile could gain).  With d_dst each tile is stored to the same offset
 * of d_dst (the staging writes of ckpt_snapshot with a hint); with d_dst == NULL
 * the streams are only read.  d_sink: at least 16 KiB.  The caller provides
 * nstreams * stream_bytes readable (and writable) bytes.
 * Errors: INVALID_ARG, ALIGNMENT, DEVICE. */
int ckpt_bw_streams(void *d_dst, const void *d_src, uint64_t nstreams, uint64_t stream_bytes,
                    uint64_t tile_bytes, uint64_t *d_sink, void *stream);

/* The other yardstick: the XXH64 accumulator arithmetic alone, on words made
 * up in registers, no memory traffic -- what the integer units allow the
 * fingerprint kernel.  Every lane of a fixed grid runs rounds_per_lane steps
 * (rounded up to a multiple of 8, at most 2^32); d_sink receives one word per
 * workgroup (at least 16 KiB).  Returns the number of input bytes those steps
 * stand for (8 per step), or 0 on an argument or launch error. */
uint64_t ckpt_alu_xxh64(uint64_t rounds_per_lane, uint64_t *d_sink, void *stream);

const char *ckpt_strerror(int status);
/* hipError_t of the last failed HIP call on this thread (0 if none). */
int ckpt_last_device_error(void);
/* 1000 * major + minor */
int ckpt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CKPT_H_ */
