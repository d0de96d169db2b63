// Restore from a chain of incremental snapshots as ONE pass over the destination
// (Singularity paper sec. 4.6: successive checkpoints of one process mostly
// coincide, so a later one holds only what changed since the one before; a
// restore therefore starts from an early snapshot and applies the later ones).
//
// Applying the links one after the other writes a chunk once per link that
// holds it.  Gradients and activations change at every step, so in a chain of m
// snapshots of a training job the same third of the state would be written m
// times.  Here every chunk is written once, from the last link that holds it:
//   k_chain_clear  last[k] = 0
//   k_chain_mark   every whole-chunk entry e of link l raises last[k] to
//                  (l + 1, e) with a 64-bit atomic maximum, k being the chunk the
//                  entry names; the entry that finds 0 there is the first for its
//                  chunk, which gives the number of chunks written
//   k_chain_list   the keys that are left, one per chunk that any link holds, as a
//                  dense list (one atomic add per 16 384 chunks)
//   k_chain_move   every listed key copies its entry's bytes
// The maximum over (link, entry index) is the entry a one-by-one restore would
// apply last, so the result is the same for any manifests, including ones that
// hold a chunk twice.
#include "ckpt_internal.h"
#include "stream_copy.h"

namespace ckpt {

namespace {

constexpr int CHAIN_ENTRY_BITS = 40;   // key = (link + 1) << 40 | entry index

__device__ __forceinline__ uint64_t link_entries(const ChainArgs &a, uint32_t l) {
  uint64_t n = a.cap[l];
  if (a.counts[l] != nullptr) {
    const uint64_t c = a.counts[l]->ndirty;
    if (c < n) n = c;
  }
  return n;
}

// Is t a whole chunk of the destination whose bytes lie inside the link's staging area?
// Sets *k to the chunk's global id.  Written so that no sum can wrap.
__device__ __forceinline__ bool whole_chunk(const PlanDev &p, const ckpt_entry_t &t,
                                            uint64_t staging_bytes, uint64_t *k) {
  const uint64_t c = 1ull << p.chunk_log2;
  if (t.buf >= p.nbufs || (t.stage_off & 15) != 0 || (t.buf_off & (c - 1)) != 0) return false;
  const uint64_t nb = p.list_nbytes[t.buf];
  if (t.buf_off >= nb) return false;
  const uint64_t left = nb - t.buf_off;
  if (t.len != (left < c ? left : c)) return false;
  if (t.stage_off > staging_bytes || t.len > staging_bytes - t.stage_off) return false;
  *k = p.list_base[t.buf] + (t.buf_off >> p.chunk_log2);
  return true;
}

__global__ __launch_bounds__(256) void k_chain_clear(unsigned long long *__restrict__ last,
                                                     uint64_t n, unsigned long long *count,
                                                     unsigned long long *stats) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  for (uint64_t k = (uint64_t)blockIdx.x * 256 + threadIdx.x; k < n; k += stride) last[k] = 0;
  if (blockIdx.x == 0 && threadIdx.x == 3) *count = 0;
  if (stats != nullptr && blockIdx.x == 0 && threadIdx.x < 3) stats[threadIdx.x] = 0;
}

// grid = (workgroups per link, links)
__global__ __launch_bounds__(256) void k_chain_mark(PlanDev p, ChainArgs a,
                                                    const uint8_t *__restrict__ only,
                                                    unsigned long long *__restrict__ last,
                                                    unsigned long long *stats) {
  const uint32_t l = blockIdx.y;
  const uint64_t n = link_entries(a, l);
  const ckpt_entry_t *manifest = a.manifest[l];
  const uint64_t staging_bytes = a.staging_bytes[l];
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  uint32_t applied = 0, first = 0, skipped = 0;
  for (uint64_t e = (uint64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += stride) {
    const ckpt_entry_t t = manifest[e];
    uint64_t k;
    if (!whole_chunk(p, t, staging_bytes, &k)) {
      ++skipped;
      continue;
    }
    if (only != nullptr && only[k] == 0) continue;          // the caller keeps this chunk as it is
    const unsigned long long key = ((unsigned long long)(l + 1) << CHAIN_ENTRY_BITS) | e;
    const unsigned long long old = atomicMax(&last[k], key);
    ++applied;
    first += old == 0;
  }
  if (stats == nullptr) return;                 // uniform: a kernel argument
  // one atomic per counter and workgroup: all workgroups add to the same three words
  __shared__ uint32_t s_sum[3][256 / 64];
  uint32_t again = applied - first;
  for (int o = 32; o > 0; o >>= 1) {
    first += __shfl_down(first, o, 64);
    again += __shfl_down(again, o, 64);
    skipped += __shfl_down(skipped, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    s_sum[0][threadIdx.x >> 6] = first;
    s_sum[1][threadIdx.x >> 6] = again;
    s_sum[2][threadIdx.x >> 6] = skipped;
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    unsigned long long v = 0;
    for (int wv = 0; wv < 256 / 64; ++wv) v += s_sum[threadIdx.x][wv];
    if (v != 0) atomicAdd(&stats[threadIdx.x], v);
  }
}

// The keys of the chunks that have one, gathered into list[0 .. *count).  A workgroup owns
// LIST_SPAN consecutive chunk ids: it counts its keys, reserves that many list slots with ONE
// atomic add (every wave of a large plan adding to the same word costs a millisecond at six
// million chunks), and then writes its keys in chunk order.  The list is therefore in ascending
// chunk order inside every span; which span lands where decides nothing but which waves of
// k_chain_move run side by side.
constexpr int LIST_SPAN = 16384;
__global__ __launch_bounds__(256) void k_chain_list(const unsigned long long *__restrict__ last,
                                                    uint64_t n, unsigned long long *__restrict__ list,
                                                    unsigned long long *count) {
  __shared__ uint32_t s_wave[256 / 64];
  __shared__ unsigned long long s_base;
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t lo = (uint64_t)blockIdx.x * LIST_SPAN;
  const uint64_t hi = lo + LIST_SPAN < n ? lo + LIST_SPAN : n;

  uint32_t mine = 0;
  for (uint64_t k = lo + threadIdx.x; k < hi; k += 256) mine += last[k] != 0;
  for (int o = 32; o > 0; o >>= 1) mine += __shfl_down(mine, o, 64);
  if (lane == 0) s_wave[wave] = mine;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t total = 0;
    for (int v = 0; v < 256 / 64; ++v) total += s_wave[v];
    s_base = total != 0 ? atomicAdd(count, (unsigned long long)total) : 0;
  }
  __syncthreads();
  unsigned long long at = s_base;
  __syncthreads();                               // s_wave is reused below

  for (uint64_t row = lo; row < hi; row += 256) {          // uniform trip count for the workgroup
    const uint64_t k = row + threadIdx.x;
    const unsigned long long key = k < hi ? last[k] : 0;
    const uint64_t holders = __ballot(key != 0);
    if (lane == 0) s_wave[wave] = (uint32_t)__popcll(holders);
    __syncthreads();
    uint32_t before = 0, all = 0;
    for (uint32_t v = 0; v < 256 / 64; ++v) {
      if (v < wave) before += s_wave[v];
      all += s_wave[v];
    }
    if (key != 0) list[at + before + __popcll(holders & ((1ull << lane) - 1))] = key;
    at += all;
    __syncthreads();
  }
}

// Work item = one piece (min(C, 16 KiB)) of one listed chunk, dealt round-robin over a fixed
// grid like the plain scatter; the key names the link and the entry that holds the bytes.
__global__ __launch_bounds__(COPY_THREADS) void k_chain_move(
    PlanDev p, ChainArgs a, const unsigned long long *__restrict__ list,
    const unsigned long long *__restrict__ count) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t wave_in_group = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t nwaves = (uint64_t)gridDim.x * (COPY_THREADS / 64);
  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint32_t ppc_log2 = p.chunk_log2 - piece_log2;
  const uint64_t nitems = *count << ppc_log2;

  for (uint64_t item = (uint64_t)blockIdx.x * (COPY_THREADS / 64) + wave_in_group; item < nitems;
       item += nwaves) {
    const unsigned long long key = list[item >> ppc_log2];
    const uint32_t piece = (uint32_t)(item & ((1ull << ppc_log2) - 1));
    const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)(key >> CHAIN_ENTRY_BITS)) - 1;
    if (l >= a.nlinks) continue;                             // cannot happen: keys come from k_chain_mark
    const ckpt_entry_t t = a.manifest[l][key & ((1ull << CHAIN_ENTRY_BITS) - 1)];
    uint64_t k;
    if (!whole_chunk(p, t, a.staging_bytes[l], &k)) continue;   // the same test as in k_chain_mark
    const uint32_t lo = piece << piece_log2;
    uint32_t hi = lo + (1u << piece_log2);
    const uint32_t padded = (uint32_t)pad16(t.len);
    if (hi > padded) hi = padded;
    move_piece<false>(a.staging[l] + t.stage_off,
                      reinterpret_cast<uint8_t *>(p.list_ptr[t.buf]) + t.buf_off, lo, hi, t.len,
                      lane);
  }
}

// Merge, step one: mask[k] = chunk k has a holder; dig[k] = the holder's digest.  These two feed
// the compaction scan, which lays the merged link out like a snapshot.
__global__ __launch_bounds__(256) void k_chain_mask(ChainArgs a,
                                                    const unsigned long long *__restrict__ last,
                                                    uint64_t n, uint8_t *__restrict__ mask,
                                                    uint64_t *__restrict__ dig) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  for (uint64_t k = (uint64_t)blockIdx.x * 256 + threadIdx.x; k < n; k += stride) {
    const unsigned long long key = last[k];
    uint64_t d = 0;
    if (key != 0) {
      const uint32_t l = (uint32_t)(key >> CHAIN_ENTRY_BITS) - 1;
      if (l < a.nlinks) d = a.manifest[l][key & ((1ull << CHAIN_ENTRY_BITS) - 1)].digest;
    }
    mask[k] = key != 0;
    dig[k] = d;
  }
}

// Merge, step two: the bytes.  Work item = one piece of one entry of the merged manifest (written
// by the scan just before); the chunk's key names the link and entry that hold its bytes, which
// go to the merged staging area zero padded to 16, if they fit below staging_cap.
__global__ __launch_bounds__(COPY_THREADS) void k_chain_gather(
    PlanDev p, ChainArgs a, const unsigned long long *__restrict__ last,
    const ckpt_entry_t *__restrict__ merged, uint64_t manifest_cap,
    const ckpt_counts_t *__restrict__ counts, uint8_t *__restrict__ staging, uint64_t staging_cap) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t wave_in_group = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t nwaves = (uint64_t)gridDim.x * (COPY_THREADS / 64);
  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint32_t ppc_log2 = p.chunk_log2 - piece_log2;
  uint64_t nentries = counts->ndirty;
  if (nentries > manifest_cap) nentries = manifest_cap;
  const uint64_t nitems = nentries << ppc_log2;

  for (uint64_t item = (uint64_t)blockIdx.x * (COPY_THREADS / 64) + wave_in_group; item < nitems;
       item += nwaves) {
    const ckpt_entry_t m = merged[item >> ppc_log2];
    const uint32_t piece = (uint32_t)(item & ((1ull << ppc_log2) - 1));
    const uint64_t padded = pad16(m.len);
    if (m.buf >= p.nbufs || m.stage_off > staging_cap || padded > staging_cap - m.stage_off)
      continue;                                              // does not fit: counted as overflow
    const unsigned long long key = last[p.list_base[m.buf] + (m.buf_off >> p.chunk_log2)];
    const uint32_t l = __builtin_amdgcn_readfirstlane((uint32_t)(key >> CHAIN_ENTRY_BITS)) - 1;
    if (l >= a.nlinks) continue;                             // cannot happen: the mask came from the keys
    const ckpt_entry_t t = a.manifest[l][key & ((1ull << CHAIN_ENTRY_BITS) - 1)];
    uint64_t k;
    if (!whole_chunk(p, t, a.staging_bytes[l], &k)) continue;   // the same test as in k_chain_mark
    const uint32_t lo = piece << piece_log2;
    uint32_t hi = lo + (1u << piece_log2);
    if (hi > padded) hi = (uint32_t)padded;
    move_piece<true>(a.staging[l] + t.stage_off, staging + m.stage_off, lo, hi, t.len, lane);
  }
}

}  // namespace

namespace {

uint32_t groups_for(uint64_t n, uint64_t per_group, uint64_t most) {
  const uint64_t g = (n + per_group - 1) / per_group;
  return (uint32_t)(g > most ? most : (g == 0 ? 1 : g));
}

// clear + mark.  *entries receives the host bound on the entries of all links together; zero
// means no link can hold anything.
hipError_t launch_chain_keys(const PlanDev &p, const ChainArgs &a, const uint8_t *only,
                             unsigned long long *last, unsigned long long *count,
                             unsigned long long *stats, uint64_t *entries, hipStream_t s) {
  hipLaunchKernelGGL(k_chain_clear, dim3(groups_for(p.nchunks, 256 * 8, 4096)), dim3(256), 0, s,
                     last, p.nchunks, count, stats);
  hipError_t e = hipGetLastError();
  uint64_t most = 0, sum = 0;
  for (uint32_t l = 0; l < a.nlinks; ++l) {
    most = a.cap[l] > most ? a.cap[l] : most;
    sum += a.cap[l];
  }
  *entries = sum;
  if (e != hipSuccess || most == 0) return e;
  // with an empty destination this still counts every entry as skipped
  hipLaunchKernelGGL(k_chain_mark, dim3(groups_for(most, 256, 2048), a.nlinks), dim3(256), 0, s, p,
                     a, only, last, stats);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_restore_chain(const PlanDev &p, const ChainArgs &a, const uint8_t *d_only,
                                uint64_t *d_workspace, uint64_t *d_stats, hipStream_t s) {
  // workspace: last[N], list[N], one counter
  unsigned long long *last = reinterpret_cast<unsigned long long *>(d_workspace);
  unsigned long long *list = last + p.nchunks;
  unsigned long long *count = list + p.nchunks;
  uint64_t entries = 0;
  hipError_t e = launch_chain_keys(p, a, d_only, last, count,
                                   reinterpret_cast<unsigned long long *>(d_stats), &entries, s);
  if (e != hipSuccess || entries == 0 || p.nchunks == 0) return e;

  const uint64_t spans = (p.nchunks + LIST_SPAN - 1) / LIST_SPAN;
  if (spans > 0x7FFFFFFFull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_chain_list, dim3((uint32_t)spans), dim3(256), 0, s, last, p.nchunks, list,
                     count);
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint64_t chunks = entries < p.nchunks ? entries : p.nchunks;   // at most this many are listed
  const uint64_t items = chunks << (p.chunk_log2 - piece_log2);
  hipLaunchKernelGGL(k_chain_move,
                     dim3(groups_for(items, COPY_THREADS / 64, COPY_MAX_GROUPS)),
                     dim3(COPY_THREADS), 0, s, p, a, list, count);
  return hipGetLastError();
}

hipError_t launch_merge_chain(const PlanDev &p, const ChainArgs &a, void *d_staging,
                              uint64_t staging_cap, ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                              ckpt_counts_t *d_counts, uint64_t *d_workspace, uint64_t *d_pairs,
                              uint64_t *d_stats, hipStream_t s) {
  // workspace: last[N], dig[N], one spare word, mask[N]
  unsigned long long *last = reinterpret_cast<unsigned long long *>(d_workspace);
  uint64_t *dig = d_workspace + p.nchunks;
  unsigned long long *spare = last + 2 * p.nchunks;
  uint8_t *mask = reinterpret_cast<uint8_t *>(spare + 2);
  uint64_t entries = 0;
  hipError_t e = launch_chain_keys(p, a, nullptr, last, spare,
                                   reinterpret_cast<unsigned long long *>(d_stats), &entries, s);
  if (e != hipSuccess) return e;
  if (p.nchunks != 0)
    hipLaunchKernelGGL(k_chain_mask, dim3(groups_for(p.nchunks, 256, 4096)), dim3(256), 0, s, a,
                       last, p.nchunks, mask, dig);
  e = launch_compact_scan(p, mask, dig, staging_cap, d_manifest, manifest_cap, d_pairs, d_counts,
                          nullptr, nullptr, false, s);
  if (e != hipSuccess || entries == 0 || p.nchunks == 0) return e;

  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  uint64_t chunks = entries < p.nchunks ? entries : p.nchunks;
  if (chunks > manifest_cap) chunks = manifest_cap;
  if (chunks == 0) return hipSuccess;
  const uint64_t items = chunks << (p.chunk_log2 - piece_log2);
  hipLaunchKernelGGL(k_chain_gather,
                     dim3(groups_for(items, COPY_THREADS / 64, COPY_MAX_GROUPS)),
                     dim3(COPY_THREADS), 0, s, p, a, last, d_manifest, manifest_cap, d_counts,
                     reinterpret_cast<uint8_t *>(d_staging), staging_cap);
  return hipGetLastError();
}

}  // namespace ckpt
