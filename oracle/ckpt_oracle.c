/*
 * ckpt_oracle.c -- plain CPU oracle for the device-state snapshot path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke
 * check and the benchmark's cpu_baseline leg may call it.  It shares no code
 * with the HIP library: its own types, its own hash, its own loops.
 *
 * What it computes (Singularity paper, sections 4.5, 4.6, 5.2.1 and 6):
 *   - a content checksum of every live device buffer (sec. 5.2.1, sec. 6),
 *     here at the granularity of fixed-size chunks inside each buffer, with
 *     XXH64 (seed 0) as the checksum function -- the paper names none;
 *   - a comparison of those checksums with another rank's / an earlier
 *     snapshot's checksums (sec. 5.2.1 equal checksum = equal content, sec. 4.6
 *     de-dup across workers and across time, sec. 5.2.3 mutation = difference
 *     of checksum state);
 *   - the swap-out of only the non-deduplicated data (sec. 5.2.1), here a
 *     gather into one contiguous staging area plus a manifest;
 *   - the swap-in / restore that puts the data back at the addresses it came
 *     from (sec. 4.5), here a scatter driven by the manifest;
 *   - the paper's own content-addressed form of the comparison (sec. 5.2.1):
 *     a checksum found at another position means a device-to-device move, not
 *     a swap (ora_match, ora_apply_matches);
 *   - restore from a chain of incremental snapshots (sec. 4.6: de-dup across
 *     time), the links applied oldest first (ora_restore_chain), and the
 *     folding of such a chain into one link (ora_merge_chain);
 *   - the paper's own granularity, whole buffers, derived from the chunk
 *     verdicts (ora_buffer_verdicts).
 *
 * Every function is the definition written out: one loop over buffers, one
 * over chunks, memcpy for copies.  No blocking, no fusion.  The only
 * concession to run time is ora_fingerprint's optional static split of the
 * chunk range over pthreads (chunks are independent by definition).
 *
 * Pins (tests/test_oracle_*.py): XXH64 vectors under tests/golden/, agreement
 * with the installed xxHash library and with a separate big-integer
 * implementation, brute-force byte comparison, prefix-sum and round-trip
 * invariants, NumPy closed forms for staging and manifest, pair-by-pair
 * brute force for the content-addressed match, a per-chunk "latest link that
 * holds it" composition in NumPy for the chain restore.
 */
#include <pthread.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  void *ptr;       /* host pointer to the buffer's bytes */
  uint64_t nbytes; /* may be 0: such a buffer has no chunks */
} ora_buf_t;

/* One staged chunk.  32 bytes, little-endian fields, no padding. */
typedef struct {
  uint32_t buf;       /* index into the buffer list */
  uint32_t len;       /* true chunk length in bytes (<= chunk size) */
  uint64_t buf_off;   /* byte offset of the chunk inside its buffer */
  uint64_t stage_off; /* byte offset of the chunk inside staging */
  uint64_t digest;    /* the chunk's XXH64 */
} ora_entry_t;

typedef struct {
  uint64_t ndirty;       /* chunks whose mask is 1 */
  uint64_t staged_bytes; /* sum of pad16(len) over those chunks */
  uint64_t overflow;     /* entries that did not fit the given capacities */
} ora_counts_t;

/* ------------------------------------------------------------------ XXH64 */
/* The public XXH64 definition, seed passed in.  All arithmetic is unsigned
 * 64-bit with wrap-around; input words are little-endian. */

#define P1 0x9E3779B185EBCA87ULL
#define P2 0xC2B2AE3D27D4EB4FULL
#define P3 0x165667B19E3779F9ULL
#define P4 0x85EBCA77C2B2AE63ULL
#define P5 0x27D4EB2F165667C5ULL

static uint64_t rotl64(uint64_t x, int r) { return (x << r) | (x >> (64 - r)); }

static uint64_t le64(const uint8_t *p) {
  uint64_t v = 0;
  for (int i = 7; i >= 0; --i) v = (v << 8) | p[i];
  return v;
}

static uint64_t le32(const uint8_t *p) {
  uint64_t v = 0;
  for (int i = 3; i >= 0; --i) v = (v << 8) | p[i];
  return v;
}

/* One accumulator step: fold one 8-byte word into an accumulator. */
static uint64_t xxh_round(uint64_t acc, uint64_t word) {
  acc += word * P2;
  acc = rotl64(acc, 31);
  return acc * P1;
}

/* Fold a finished accumulator into the converged hash. */
static uint64_t xxh_merge(uint64_t h, uint64_t acc) {
  h ^= xxh_round(0, acc);
  return h * P1 + P4;
}

uint64_t ora_xxh64(const void *data, uint64_t len, uint64_t seed) {
  const uint8_t *p = (const uint8_t *)data;
  uint64_t left = len;
  uint64_t h;

  if (len >= 32) {
    /* four accumulators, each eats one 8-byte word of every 32-byte stripe */
    uint64_t v1 = seed + P1 + P2;
    uint64_t v2 = seed + P2;
    uint64_t v3 = seed;
    uint64_t v4 = seed - P1;
    while (left >= 32) {
      v1 = xxh_round(v1, le64(p + 0));
      v2 = xxh_round(v2, le64(p + 8));
      v3 = xxh_round(v3, le64(p + 16));
      v4 = xxh_round(v4, le64(p + 24));
      p += 32;
      left -= 32;
    }
    h = rotl64(v1, 1) + rotl64(v2, 7) + rotl64(v3, 12) + rotl64(v4, 18);
    h = xxh_merge(h, v1);
    h = xxh_merge(h, v2);
    h = xxh_merge(h, v3);
    h = xxh_merge(h, v4);
  } else {
    h = seed + P5;
  }

  h += len;

  /* the last len mod 32 bytes: 8-byte words, then one 4-byte word, then bytes */
  while (left >= 8) {
    h ^= xxh_round(0, le64(p));
    h = rotl64(h, 27) * P1 + P4;
    p += 8;
    left -= 8;
  }
  if (left >= 4) {
    h ^= le32(p) * P1;
    h = rotl64(h, 23) * P2 + P3;
    p += 4;
    left -= 4;
  }
  while (left > 0) {
    h ^= (uint64_t)(*p) * P5;
    h = rotl64(h, 11) * P1;
    p += 1;
    left -= 1;
  }

  /* avalanche */
  h ^= h >> 33;
  h *= P2;
  h ^= h >> 29;
  h *= P3;
  h ^= h >> 32;
  return h;
}

/* --------------------------------------------------------------- chunking */
/* Buffer i is cut into n_i = ceil(nbytes_i / chunk) chunks; chunk j of buffer
 * i covers bytes [j*chunk, min((j+1)*chunk, nbytes_i)).  A chunk never spans
 * two buffers.  Global chunk ids run over the buffers in list order. */

static uint64_t chunks_of(uint64_t nbytes, uint64_t chunk) {
  return nbytes / chunk + (nbytes % chunk != 0);
}

static uint64_t pad16(uint64_t x) { return (x + 15) & ~(uint64_t)15; }

uint64_t ora_nchunks(const ora_buf_t *bufs, uint64_t nbufs, uint64_t chunk) {
  uint64_t n = 0;
  for (uint64_t i = 0; i < nbufs; ++i) n += chunks_of(bufs[i].nbytes, chunk);
  return n;
}

/* Length of every chunk in global order (lens has ora_nchunks entries). */
void ora_chunk_lens(const ora_buf_t *bufs, uint64_t nbufs, uint64_t chunk, uint32_t *lens) {
  uint64_t k = 0;
  for (uint64_t i = 0; i < nbufs; ++i) {
    uint64_t n = chunks_of(bufs[i].nbytes, chunk);
    for (uint64_t j = 0; j < n; ++j) {
      uint64_t off = j * chunk;
      uint64_t len = bufs[i].nbytes - off;
      if (len > chunk) len = chunk;
      lens[k++] = (uint32_t)len;
    }
  }
}

/* ------------------------------------------------------------ fingerprint */
/* dig[k] = XXH64(bytes of chunk k, seed 0)  (sec. 5.2.1: a content checksum
 * of each live buffer; here one per chunk). */

typedef struct {
  const ora_buf_t *bufs;
  uint64_t nbufs, chunk;
  uint64_t k_lo, k_hi; /* this worker hashes global chunk ids [k_lo, k_hi) */
  uint64_t *dig;
} fp_job_t;

static void *fp_worker(void *arg) {
  fp_job_t *job = (fp_job_t *)arg;
  uint64_t k = 0;
  for (uint64_t i = 0; i < job->nbufs; ++i) {
    uint64_t n = chunks_of(job->bufs[i].nbytes, job->chunk);
    if (k + n <= job->k_lo) { /* whole buffer before this worker's range */
      k += n;
      continue;
    }
    if (k >= job->k_hi) break;
    const uint8_t *base = (const uint8_t *)job->bufs[i].ptr;
    for (uint64_t j = 0; j < n; ++j, ++k) {
      if (k < job->k_lo || k >= job->k_hi) continue;
      uint64_t off = j * job->chunk;
      uint64_t len = job->bufs[i].nbytes - off;
      if (len > job->chunk) len = job->chunk;
      job->dig[k] = ora_xxh64(base + off, len, 0);
    }
  }
  return NULL;
}

/* nthreads <= 1: one plain loop.  Otherwise the chunk id range is split into
 * nthreads equal contiguous parts, one pthread each.  Returns 0, or -1 if a
 * thread could not be started. */
int ora_fingerprint(const ora_buf_t *bufs, uint64_t nbufs, uint64_t chunk, uint64_t *dig,
                    int nthreads) {
  uint64_t N = ora_nchunks(bufs, nbufs, chunk);
  if (nthreads <= 1 || N < 2) {
    fp_job_t job = {bufs, nbufs, chunk, 0, N, dig};
    fp_worker(&job);
    return 0;
  }
  if ((uint64_t)nthreads > N) nthreads = (int)N;
  pthread_t *tid = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nthreads);
  fp_job_t *jobs = (fp_job_t *)malloc(sizeof(fp_job_t) * (size_t)nthreads);
  if (!tid || !jobs) {
    free(tid);
    free(jobs);
    return -1;
  }
  int started = 0, rc = 0;
  for (int t = 0; t < nthreads; ++t) {
    fp_job_t job = {bufs, nbufs, chunk, N * (uint64_t)t / (uint64_t)nthreads,
                    N * (uint64_t)(t + 1) / (uint64_t)nthreads, dig};
    jobs[t] = job;
    if (pthread_create(&tid[t], NULL, fp_worker, &jobs[t]) != 0) {
      rc = -1;
      break;
    }
    ++started;
  }
  for (int t = 0; t < started; ++t) pthread_join(tid[t], NULL);
  free(tid);
  free(jobs);
  return rc;
}

/* ------------------------------------------------------------------- diff */
/* mask[k] = 1 when chunk k must be moved: no reference at all (the first
 * rank really swaps out, sec. 5.2.1) or its checksum differs from the
 * reference's checksum at the same position; else 0.  counts gets the number
 * of such chunks and the staging bytes they need.  overflow is set to 0. */
void ora_diff(const ora_buf_t *bufs, uint64_t nbufs, uint64_t chunk, const uint64_t *dig,
              const uint64_t *ref, uint8_t *mask, ora_counts_t *counts) {
  uint64_t k = 0, ndirty = 0, bytes = 0;
  for (uint64_t i = 0; i < nbufs; ++i) {
    uint64_t n = chunks_of(bufs[i].nbytes, chunk);
    for (uint64_t j = 0; j < n; ++j, ++k) {
      uint64_t len = bufs[i].nbytes - j * chunk;
      if (len > chunk) len = chunk;
      uint8_t m = (ref == NULL || dig[k] != ref[k]) ? 1 : 0;
      mask[k] = m;
      if (m) {
        ndirty += 1;
        bytes += pad16(len);
      }
    }
  }
  counts->ndirty = ndirty;
  counts->staged_bytes = bytes;
  counts->overflow = 0;
}

/* ---------------------------------------------------------------- compact */
/* Walk the chunks in ascending global id.  Every chunk with mask 1 gets the
 * next manifest entry and the next pad16(len) bytes of staging: its bytes,
 * then zeros up to the 16-byte boundary.  Offsets are therefore the exclusive
 * prefix sum of pad16(len) over the dirty chunks.
 *
 * Capacities: entry e is written to the manifest only if e < manifest_cap;
 * its bytes are written to staging only if, in addition, they end at or
 * before staging_cap.  Each dirty chunk that misses either test adds one to
 * counts->overflow.  ndirty and staged_bytes always report the full need. */
void ora_compact(const ora_buf_t *bufs, uint64_t nbufs, uint64_t chunk, const uint8_t *mask,
                 const uint64_t *dig, void *staging, uint64_t staging_cap,
                 ora_entry_t *manifest, uint64_t manifest_cap, ora_counts_t *counts) {
  uint8_t *out = (uint8_t *)staging;
  uint64_t k = 0, e = 0, soff = 0, overflow = 0;
  for (uint64_t i = 0; i < nbufs; ++i) {
    uint64_t n = chunks_of(bufs[i].nbytes, chunk);
    const uint8_t *base = (const uint8_t *)bufs[i].ptr;
    for (uint64_t j = 0; j < n; ++j, ++k) {
      if (!mask[k]) continue;
      uint64_t off = j * chunk;
      uint64_t len = bufs[i].nbytes - off;
      if (len > chunk) len = chunk;
      uint64_t padded = pad16(len);
      int fits_manifest = e < manifest_cap;
      int fits_staging = fits_manifest && soff + padded <= staging_cap;
      if (fits_manifest) {
        manifest[e].buf = (uint32_t)i;
        manifest[e].len = (uint32_t)len;
        manifest[e].buf_off = off;
        manifest[e].stage_off = soff;
        manifest[e].digest = dig[k];
      }
      if (fits_staging) {
        memcpy(out + soff, base + off, len);
        memset(out + soff + len, 0, padded - len);
      }
      if (!fits_staging) overflow += 1;
      e += 1;
      soff += padded;
    }
  }
  counts->ndirty = e;
  counts->staged_bytes = soff;
  counts->overflow = overflow;
}

/* ---------------------------------------------------------------- restore */
/* For each manifest entry, in order, copy len bytes from staging back to the
 * place in the destination buffer list the entry names (sec. 4.5: tensors go
 * back to the addresses they had).  Nothing else is written.  An entry that
 * compact could not have produced for this destination -- a buffer outside the
 * list, a range outside its buffer or outside staging, an offset that is not a
 * multiple of 16, a length above the chunk size -- is skipped; the return value is the number of entries
 * skipped (0 = everything applied). */
uint64_t ora_restore(const ora_buf_t *dst, uint64_t nbufs, uint64_t chunk, const void *staging,
                     uint64_t staging_bytes, const ora_entry_t *manifest,
                     uint64_t nentries) {
  const uint8_t *in = (const uint8_t *)staging;
  uint64_t rejected = 0;
  for (uint64_t e = 0; e < nentries; ++e) {
    const ora_entry_t *m = &manifest[e];
    int ok = m->buf < nbufs && m->buf_off % 16 == 0 && m->stage_off % 16 == 0 && m->len <= chunk;
    if (ok) ok = m->buf_off <= dst[m->buf].nbytes && m->len <= dst[m->buf].nbytes - m->buf_off;
    if (ok) ok = m->stage_off <= staging_bytes && m->len <= staging_bytes - m->stage_off;
    if (!ok) {
      rejected += 1;
      continue;
    }
    memcpy((uint8_t *)dst[m->buf].ptr + m->buf_off, in + m->stage_off, m->len);
  }
  return rejected;
}

/* ---------------------------------------------------------- restore chain */
/* Restore from a chain of incremental snapshots (sec. 4.6: successive
 * checkpoints of one process mostly coincide, so each later one holds only
 * what changed since the one before).  Link 0 is the oldest.  The links are
 * applied one after the other, each entry in manifest order, so where two
 * links hold the same chunk the later link's bytes stay.  Every link was taken
 * with the destination's chunk geometry, so an entry is applied only if it is a
 * whole chunk of the destination: besides what ora_restore asks, buf_off is a
 * multiple of the chunk size and len is that chunk's length (the chunk size,
 * or what is left of the buffer).  Other entries are skipped and counted.
 * only (may be NULL) restricts the restore to some chunks: with only[k] == 0
 * chunk k keeps its bytes whatever the links hold, and the entries that name it
 * are not counted anywhere.  (At a context switch between time-sliced ranks,
 * sec. 5.2.1, only the chunks whose checksum differs between the resident and
 * the incoming rank have to come in.)
 *   stats[0] = chunks of the destination written at least once
 *   stats[1] = applied entries whose chunk a later entry wrote again
 *   stats[2] = entries skipped
 * Returns 0, or -1 when the table of written chunks cannot be allocated. */
typedef struct {
  const void *staging;
  uint64_t staging_bytes;
  const ora_entry_t *manifest;
  uint64_t nentries;
} ora_link_t;

int ora_restore_chain(const ora_buf_t *dst, uint64_t nbufs, uint64_t chunk, const ora_link_t *links,
                      uint64_t nlinks, const uint8_t *only, uint64_t *stats) {
  uint64_t n = 0;
  uint64_t *base = (uint64_t *)malloc((nbufs + 1) * sizeof(uint64_t));
  if (!base) return -1;
  for (uint64_t i = 0; i < nbufs; ++i) {
    base[i] = n;
    n += (dst[i].nbytes + chunk - 1) / chunk;
  }
  uint8_t *written = (uint8_t *)calloc(n + 1, 1);
  if (!written) {
    free(base);
    return -1;
  }
  uint64_t applied = 0, distinct = 0, skipped = 0;
  for (uint64_t l = 0; l < nlinks; ++l) {
    const uint8_t *from = (const uint8_t *)links[l].staging;
    for (uint64_t e = 0; e < links[l].nentries; ++e) {
      const ora_entry_t *t = &links[l].manifest[e];
      int ok = t->buf < nbufs && t->stage_off % 16 == 0 && t->buf_off % chunk == 0;
      if (ok) ok = t->buf_off < dst[t->buf].nbytes;
      if (ok) {
        uint64_t left = dst[t->buf].nbytes - t->buf_off;
        ok = t->len == (left < chunk ? left : chunk);
      }
      if (ok) ok = t->stage_off <= links[l].staging_bytes &&
                   t->len <= links[l].staging_bytes - t->stage_off;
      if (!ok) {
        skipped += 1;
        continue;
      }
      uint64_t k = base[t->buf] + t->buf_off / chunk;
      if (only && !only[k]) continue;
      memcpy((uint8_t *)dst[t->buf].ptr + t->buf_off, from + t->stage_off, t->len);
      applied += 1;
      if (!written[k]) {
        written[k] = 1;
        distinct += 1;
      }
    }
  }
  stats[0] = distinct;
  stats[1] = applied - distinct;
  stats[2] = skipped;
  free(written);
  free(base);
  return 0;
}

/* ------------------------------------------------------------ merge chain */
/* Fold a chain of incremental snapshots into ONE link that restores to the same
 * result (sec. 4.6: a long chain of increments is shortened by merging them;
 * what a later increment replaced need not be kept).  The destination's bytes
 * are not needed, only its geometry: sizes[i] is the length of buffer i.
 * Pass one takes the links oldest first and their entries in manifest order;
 * every entry that ora_restore_chain would apply becomes the holder of its
 * chunk, replacing an earlier holder.  Pass two walks the chunks in ascending
 * id: a chunk with a holder gets the next manifest entry and the next
 * pad16(len) bytes of staging, laid out as ora_compact lays out a snapshot
 * (bytes, then zeros to the 16-byte boundary; offsets = exclusive prefix sum),
 * and the entry carries the holder's digest.  Capacities and counts as
 * ora_compact; stats as ora_restore_chain.  Returns 0, or -1 without memory. */
int ora_merge_chain(const uint64_t *sizes, uint64_t nbufs, uint64_t chunk, const ora_link_t *links,
                    uint64_t nlinks, void *staging, uint64_t staging_cap, ora_entry_t *manifest,
                    uint64_t manifest_cap, ora_counts_t *counts, uint64_t *stats) {
  uint64_t n = 0;
  uint64_t *first_chunk = (uint64_t *)malloc((nbufs + 1) * sizeof(uint64_t));
  if (!first_chunk) return -1;
  for (uint64_t i = 0; i < nbufs; ++i) {
    first_chunk[i] = n;
    n += (sizes[i] + chunk - 1) / chunk;
  }
  const ora_entry_t **holder = (const ora_entry_t **)calloc(n + 1, sizeof(*holder));
  const uint8_t **bytes_of = (const uint8_t **)calloc(n + 1, sizeof(*bytes_of));
  if (!holder || !bytes_of) {
    free(first_chunk);
    free(holder);
    free(bytes_of);
    return -1;
  }
  uint64_t taken = 0, held = 0, skipped = 0;
  for (uint64_t l = 0; l < nlinks; ++l) {
    for (uint64_t e = 0; e < links[l].nentries; ++e) {
      const ora_entry_t *c = &links[l].manifest[e];
      int ok = c->buf < nbufs && c->stage_off % 16 == 0 && c->buf_off % chunk == 0;
      if (ok) ok = c->buf_off < sizes[c->buf];
      if (ok) {
        uint64_t rest = sizes[c->buf] - c->buf_off;
        ok = c->len == (rest < chunk ? rest : chunk);
      }
      if (ok) ok = c->stage_off <= links[l].staging_bytes &&
                   c->len <= links[l].staging_bytes - c->stage_off;
      if (!ok) {
        skipped += 1;
        continue;
      }
      uint64_t k = first_chunk[c->buf] + c->buf_off / chunk;
      taken += 1;
      if (!holder[k]) held += 1;
      holder[k] = c;
      bytes_of[k] = (const uint8_t *)links[l].staging + c->stage_off;
    }
  }
  uint8_t *merged = (uint8_t *)staging;
  uint64_t made = 0, at = 0, missed = 0;
  for (uint64_t k = 0; k < n; ++k) {
    if (!holder[k]) continue;
    uint64_t width = holder[k]->len, slot = pad16(width);
    int entry_fits = made < manifest_cap;
    int bytes_fit = entry_fits && at + slot <= staging_cap;
    if (entry_fits) {
      manifest[made] = *holder[k];
      manifest[made].stage_off = at;
    }
    if (bytes_fit) {
      memcpy(merged + at, bytes_of[k], width);
      memset(merged + at + width, 0, slot - width);
    } else {
      missed += 1;
    }
    made += 1;
    at += slot;
  }
  counts->ndirty = made;
  counts->staged_bytes = at;
  counts->overflow = missed;
  stats[0] = held;
  stats[1] = taken - held;
  stats[2] = skipped;
  free(first_chunk);
  free(holder);
  free(bytes_of);
  return 0;
}

/* ------------------------------------------------- content-addressed match */
/* The paper's own rule (sec. 5.2.1) looks a checksum up by content, wherever
 * the buffer with that content lives; a hit at another address becomes a
 * device-to-device move instead of a swap.  For every snapshot chunk k:
 *   src[k] =  k            if the reference chunk at the same position has the
 *                          same checksum (nothing to do),
 *             j            else the lowest reference position j whose checksum
 *                          equals dig[k] (content present elsewhere: move),
 *             -2 - k0      else, if an earlier snapshot chunk has the same
 *                          checksum, k0 being the first such chunk (a duplicate
 *                          of a chunk that is itself new),
 *             -1           else (new content: must be staged).
 * mask[k] = 1 exactly for src[k] == -1.  The reference may have any number of
 * chunks.  The lookup is done the plain way: sort (checksum, position) pairs,
 * then binary-search the first pair with the wanted checksum. */

typedef struct {
  uint64_t nsame, nmoved, ndup, nnew, staged_bytes, table_full;
} ora_match_counts_t;

typedef struct {
  uint64_t dig, pos;
} ora_pair_t;

static int pair_cmp(const void *a, const void *b) {
  const ora_pair_t *x = (const ora_pair_t *)a, *y = (const ora_pair_t *)b;
  if (x->dig != y->dig) return x->dig < y->dig ? -1 : 1;
  if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;
  return 0;
}

/* lowest position with checksum d in a sorted pair array, or -1 */
static int64_t first_pos(const ora_pair_t *pairs, uint64_t n, uint64_t d) {
  uint64_t lo = 0, hi = n;
  while (lo < hi) {
    uint64_t mid = lo + (hi - lo) / 2;
    if (pairs[mid].dig < d) lo = mid + 1; else hi = mid;
  }
  return (lo < n && pairs[lo].dig == d) ? (int64_t)pairs[lo].pos : -1;
}

int ora_match(const ora_buf_t *bufs, uint64_t nbufs, uint64_t chunk, const uint64_t *dig,
              const uint64_t *ref, uint64_t n_ref, int64_t *src, uint8_t *mask,
              ora_match_counts_t *counts) {
  uint64_t N = ora_nchunks(bufs, nbufs, chunk);
  ora_pair_t *rp = (ora_pair_t *)malloc(sizeof(ora_pair_t) * (size_t)(n_ref ? n_ref : 1));
  ora_pair_t *sp = (ora_pair_t *)malloc(sizeof(ora_pair_t) * (size_t)(N ? N : 1));
  uint32_t *lens = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)(N ? N : 1));
  if (!rp || !sp || !lens) {
    free(rp); free(sp); free(lens);
    return -1;
  }
  for (uint64_t j = 0; j < n_ref; ++j) { rp[j].dig = ref[j]; rp[j].pos = j; }
  for (uint64_t k = 0; k < N; ++k) { sp[k].dig = dig[k]; sp[k].pos = k; }
  qsort(rp, (size_t)n_ref, sizeof(ora_pair_t), pair_cmp);
  qsort(sp, (size_t)N, sizeof(ora_pair_t), pair_cmp);
  ora_chunk_lens(bufs, nbufs, chunk, lens);
  memset(counts, 0, sizeof(*counts));
  for (uint64_t k = 0; k < N; ++k) {
    int64_t s;
    if (k < n_ref && ref[k] == dig[k]) {
      s = (int64_t)k;
      counts->nsame += 1;
    } else {
      int64_t j = first_pos(rp, n_ref, dig[k]);
      if (j >= 0) {
        s = j;
        counts->nmoved += 1;
      } else {
        int64_t k0 = first_pos(sp, N, dig[k]); /* always found: at worst k itself */
        if ((uint64_t)k0 < k) {
          s = -2 - k0;
          counts->ndup += 1;
        } else {
          s = -1;
          counts->nnew += 1;
          counts->staged_bytes += pad16(lens[k]);
        }
      }
    }
    src[k] = s;
    mask[k] = (s == -1) ? 1 : 0;
  }
  free(rp); free(sp); free(lens);
  return 0;
}

/* Rebuilds the snapshot's content in dst from what the match found, after the
 * new chunks have been restored from staging: a matched chunk (src >= 0) is
 * copied from chunk src[k] of the reference buffer list, a duplicate
 * (src <= -2) from chunk -2 - src[k] of dst itself.  New chunks (src == -1)
 * are left alone.  A chunk whose source does not exist or has another length
 * is skipped and counted in the return value.  ref and dst must not overlap
 * in memory unless every match is in place. */
static int chunk_addr(const ora_buf_t *bufs, uint64_t nbufs, uint64_t chunk, uint64_t k,
                      uint8_t **ptr, uint64_t *len) {
  for (uint64_t i = 0; i < nbufs; ++i) {
    uint64_t n = chunks_of(bufs[i].nbytes, chunk);
    if (k < n) {
      uint64_t off = k * chunk, l = bufs[i].nbytes - off;
      *ptr = (uint8_t *)bufs[i].ptr + off;
      *len = l > chunk ? chunk : l;
      return 1;
    }
    k -= n;
  }
  return 0;
}

uint64_t ora_apply_matches(const ora_buf_t *dst, uint64_t ndst, const ora_buf_t *ref,
                           uint64_t nref, uint64_t chunk, const int64_t *src) {
  uint64_t N = ora_nchunks(dst, ndst, chunk), rejected = 0;
  for (int pass = 0; pass < 2; ++pass) { /* pass 0: from the reference, pass 1: duplicates */
    for (uint64_t k = 0; k < N; ++k) {
      int64_t s = src[k];
      if (s == -1 || (pass == 0) != (s >= 0)) continue;
      uint8_t *to, *from;
      uint64_t tlen, flen;
      chunk_addr(dst, ndst, chunk, k, &to, &tlen);
      int ok = pass == 0 ? chunk_addr(ref, nref, chunk, (uint64_t)s, &from, &flen)
                         : ((uint64_t)(-2 - s) < k &&
                            chunk_addr(dst, ndst, chunk, (uint64_t)(-2 - s), &from, &flen));
      if (!ok || flen != tlen) {
        rejected += 1;
        continue;
      }
      if (from != to) memmove(to, from, tlen);
    }
  }
  return rejected;
}

/* -------------------------------------------------------- buffer verdicts */
/* The paper compares checksums per buffer (sec. 5.2.1): a buffer is swapped as
 * a whole if its content differs.  At chunk granularity the same verdict is:
 * buffer i differs if any of its chunks is marked.  dirty[i] = 1 for such a
 * buffer, else 0 (a buffer without bytes has no chunk and never differs).
 *   result[0] = buffers that differ
 *   result[1] = their total size in bytes: what a swap at buffer granularity
 *               would have to move, to set against the marked chunks' bytes */
void ora_buffer_verdicts(const uint64_t *sizes, uint64_t nbufs, uint64_t chunk, const uint8_t *mask,
                         uint8_t *dirty, uint64_t *result) {
  uint64_t k = 0, differing = 0, bytes = 0;
  for (uint64_t i = 0; i < nbufs; ++i) {
    uint64_t n = (sizes[i] + chunk - 1) / chunk;
    uint8_t any = 0;
    for (uint64_t j = 0; j < n; ++j, ++k)
      if (mask[k]) any = 1;
    dirty[i] = any;
    if (any) {
      differing += 1;
      bytes += sizes[i];
    }
  }
  result[0] = differing;
  result[1] = bytes;
}

/* --------------------------------------------------- marks from buffers */
/* The reverse of ora_buffer_verdicts: every chunk of a flagged buffer is marked.
 * Which buffers hold per-replica state (gradients, activations, sec. 5.2.1) is
 * stable from switch to switch and known per buffer, so a prediction of the
 * chunk marks -- the hint of the single-pass snapshot -- can be kept as one
 * byte per buffer. */
void ora_marks_from_buffers(const uint64_t *sizes, uint64_t nbufs, uint64_t chunk,
                            const uint8_t *flags, uint8_t *marks) {
  uint64_t k = 0;
  for (uint64_t i = 0; i < nbufs; ++i) {
    uint64_t n = (sizes[i] + chunk - 1) / chunk;
    for (uint64_t j = 0; j < n; ++j) marks[k++] = flags[i] ? 1 : 0;
  }
}

/* ---------------------------------------------------------- mask and-not */
/* out[k] = 1 where mask[k] is set and without[k] is not, else 0.  At a context
 * switch (sec. 5.2.1) with mask = the chunks in which the outgoing rank differs
 * from the common base and without = those of the incoming rank, these are the
 * chunks the incoming rank's own delta does not bring back: the outgoing rank
 * changed them, the incoming one never did, so the base's bytes have to return. */
void ora_mask_andnot(uint64_t n, const uint8_t *mask, const uint8_t *without, uint8_t *out) {
  for (uint64_t k = 0; k < n; ++k) out[k] = (mask[k] != 0 && without[k] == 0) ? 1 : 0;
}

/* ----------------------------------------------------- mutation validation */
/* Squashing validation (sec. 5.2.3): the mutations a rank performed between
 * two points are the chunks whose checksum changed; two ranks sharing a GPU
 * may be squashed only if their mutations are identical in address, checksum
 * and size.  With one chunk geometry for both ranks (same addresses by the
 * consistent allocation of sec. 5.2.2, hence same sizes) that is, for every
 * chunk k:  changed_a(k) == changed_b(k), and where changed, the new checksums
 * are equal.  result = { chunks rank a changed, chunks rank b changed, chunks
 * that break the rule, lowest such chunk or all-ones }. */
void ora_validate_mutations(uint64_t nchunks, const uint64_t *before_a, const uint64_t *after_a,
                            const uint64_t *before_b, const uint64_t *after_b,
                            uint64_t result[4]) {
  uint64_t na = 0, nb = 0, bad = 0, first = ~(uint64_t)0;
  for (uint64_t k = 0; k < nchunks; ++k) {
    int ca = before_a[k] != after_a[k];
    int cb = before_b[k] != after_b[k];
    na += (uint64_t)ca;
    nb += (uint64_t)cb;
    if (ca != cb || (ca && after_a[k] != after_b[k])) {
      bad += 1;
      if (first == ~(uint64_t)0) first = k;
    }
  }
  result[0] = na;
  result[1] = nb;
  result[2] = bad;
  result[3] = first;
}

/* ------------------------------------------------- cross-worker upload owner */
/* Checkpoint de-duplication across workers (sec. 4.6): a worker uploads a
 * piece of device state only if no other worker uploads the same content.
 * With the checksums of all `world` workers gathered (gathered[r*N + k] is
 * worker r's checksum of chunk k; one chunk geometry for all, the replicas
 * being consistent by sec. 5.2.2), the decision is taken per chunk position
 * and without further communication: the workers whose checksum at k equals
 * this worker's form a group, listed by ascending rank; the group's member
 * number (k mod group size) uploads that content, the others skip it.  Every
 * distinct content at every position is thus uploaded exactly once, and the
 * content all replicas share is spread evenly over them.
 * mask[k] = 1 when worker `rank` uploads chunk k; counts as ora_diff. */
int ora_upload_owners(const ora_buf_t *bufs, uint64_t nbufs, uint64_t chunk,
                      const uint64_t *gathered, uint32_t world, uint32_t rank, uint8_t *mask,
                      ora_counts_t *counts) {
  if (world == 0 || rank >= world) return -1;
  uint64_t N = ora_nchunks(bufs, nbufs, chunk);
  uint64_t k = 0, nup = 0, bytes = 0;
  for (uint64_t i = 0; i < nbufs; ++i) {
    uint64_t n = chunks_of(bufs[i].nbytes, chunk);
    for (uint64_t j = 0; j < n; ++j, ++k) {
      uint64_t len = bufs[i].nbytes - j * chunk;
      if (len > chunk) len = chunk;
      uint64_t mine = gathered[(uint64_t)rank * N + k];
      uint32_t size = 0, my_place = 0;
      for (uint32_t r = 0; r < world; ++r) {
        if (gathered[(uint64_t)r * N + k] != mine) continue;
        if (r == rank) my_place = size;
        size += 1;
      }
      uint8_t m = (k % size == my_place) ? 1 : 0;
      mask[k] = m;
      if (m) {
        nup += 1;
        bytes += pad16(len);
      }
    }
  }
  counts->ndirty = nup;
  counts->staged_bytes = bytes;
  counts->overflow = 0;
  return 0;
}
