// Content-addressed comparison of checksums and the moves it implies.
//
// The Singularity paper looks a checksum up by content (sec. 5.2.1): a buffer
// whose checksum is already present is not swapped, and if the content sits at
// another device address it is moved device-to-device, which costs less than
// bringing it in from the host.  Here the lookup is a hash join on the device: the reference's
// digests go into an open-addressing table (key = digest, value = lowest
// position that carries it), so do the snapshot's own digests (value = first
// occurrence), and one probe per snapshot chunk classifies it as same place /
// moved / duplicate of an earlier new chunk / new.
//
// The tables live in a caller-supplied workspace.  Capacity is a power of two
// >= 2 x entries, so a linear probe always meets an empty slot; every loop is
// bounded by the capacity besides.  Results are deterministic although the
// slot a key lands in is not: the value is an atomic minimum.
#include "ckpt_internal.h"
#include "stream_copy.h"

namespace ckpt {

namespace {

constexpr uint64_t EMPTY = ~0ull;   // also a possible digest: that one key gets a slot of its own

struct Table {
  unsigned long long *keys;   // [cap]
  unsigned long long *vals;   // [cap]
  unsigned long long *lone;   // lowest position whose digest equals EMPTY
  uint64_t cap_mask;          // cap - 1
};

struct MatchSpace {
  Table ref, self;
};

__device__ __forceinline__ uint64_t slot_of(uint64_t d, uint64_t cap_mask) {
  return (d ^ (d >> 32) ^ (d >> 17)) & cap_mask;
}

__global__ __launch_bounds__(256) void k_match_init(MatchSpace m, ckpt_match_counts_t *counts) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  const uint64_t i0 = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  for (uint64_t i = i0; i <= m.ref.cap_mask; i += stride) {
    m.ref.keys[i] = EMPTY;
    m.ref.vals[i] = EMPTY;
  }
  for (uint64_t i = i0; i <= m.self.cap_mask; i += stride) {
    m.self.keys[i] = EMPTY;
    m.self.vals[i] = EMPTY;
  }
  if (i0 == 0) {
    *m.ref.lone = EMPTY;
    *m.self.lone = EMPTY;
    counts->nsame = counts->nmoved = counts->ndup = counts->nnew = 0;
    counts->staged_bytes = counts->table_full = 0;
  }
}

__global__ __launch_bounds__(256) void k_match_insert(Table t, const uint64_t *__restrict__ dig,
                                                      uint64_t n, ckpt_match_counts_t *counts) {
  const uint64_t j = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (j >= n) return;
  const uint64_t d = dig[j];
  if (d == EMPTY) {
    atomicMin(t.lone, (unsigned long long)j);
    return;
  }
  // Heavily repeated digests (all-zero chunks: one key for a fifth of a fragmented
  // heap) would serialise on one slot, so look before touching it: values only
  // ever decrease, hence a value already <= j, however stale, proves there is
  // nothing left for this thread to do.  Loads go to L2 (agent scope).
  uint64_t s = slot_of(d, t.cap_mask);
  for (uint64_t tries = 0; tries <= t.cap_mask; ++tries) {
    unsigned long long key = __hip_atomic_load(&t.keys[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (key == EMPTY)
      key = atomicCAS(&t.keys[s], (unsigned long long)EMPTY, (unsigned long long)d);
    if (key == EMPTY || key == d) {
      if (__hip_atomic_load(&t.vals[s], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > j)
        atomicMin(&t.vals[s], (unsigned long long)j);
      return;
    }
    s = (s + 1) & t.cap_mask;
  }
  atomicAdd(reinterpret_cast<unsigned long long *>(&counts->table_full), 1ull);
}

// lowest position carrying digest d, or EMPTY
__device__ __forceinline__ uint64_t table_find(const Table &t, uint64_t d) {
  if (d == EMPTY) return *t.lone;
  uint64_t s = slot_of(d, t.cap_mask);
  for (uint64_t tries = 0; tries <= t.cap_mask; ++tries) {
    const uint64_t key = t.keys[s];
    if (key == d) return t.vals[s];
    if (key == EMPTY) return EMPTY;
    s = (s + 1) & t.cap_mask;
  }
  return EMPTY;
}

__global__ __launch_bounds__(256) void k_match_probe(PlanDev p, MatchSpace m,
                                                     const uint64_t *__restrict__ dig,
                                                     const uint64_t *__restrict__ ref, uint64_t n_ref,
                                                     int64_t *__restrict__ src,
                                                     uint8_t *__restrict__ mask,
                                                     ckpt_match_counts_t *counts) {
  const uint64_t k = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  uint32_t same = 0, moved = 0, dup = 0, fresh = 0;
  uint64_t bytes = 0;
  if (k < p.nchunks) {
    const uint64_t d = dig[k];
    int64_t s;
    if (k < n_ref && ref[k] == d) {
      s = (int64_t)k;
      same = 1;
    } else {
      const uint64_t j = table_find(m.ref, d);
      if (j != EMPTY) {
        s = (int64_t)j;
        moved = 1;
      } else {
        const uint64_t k0 = table_find(m.self, d);   // first occurrence in the snapshot (<= k)
        if (k0 < k) {
          s = -2 - (int64_t)k0;
          dup = 1;
        } else {
          s = -1;
          fresh = 1;
          bytes = pad16(locate_chunk(p, k).len);
        }
      }
    }
    src[k] = s;
    mask[k] = s == -1 ? 1 : 0;
  }
  // workgroup totals, then one atomic per counter
  __shared__ unsigned long long s_sum[5];
  if (threadIdx.x < 5) s_sum[threadIdx.x] = 0;
  __syncthreads();
  const uint64_t v[5] = {same, moved, dup, fresh, bytes};
#pragma unroll
  for (int i = 0; i < 5; ++i) {
    uint64_t x = v[i];
    for (int o = 32; o > 0; o >>= 1) x += __shfl_down(x, o, 64);
    if ((threadIdx.x & 63) == 0 && x) atomicAdd(&s_sum[i], (unsigned long long)x);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long *c = reinterpret_cast<unsigned long long *>(counts);
    for (int i = 0; i < 5; ++i)
      if (s_sum[i]) atomicAdd(&c[i], s_sum[i]);
  }
}

// Copies matched chunks into the destination: FROM_REF handles src >= 0 (bytes
// of chunk src[k] of the reference plan), !FROM_REF handles src <= -2 (bytes
// of the earlier destination chunk -2 - src[k]).  One 16 KiB piece per wave.
template <bool FROM_REF>
__global__ __launch_bounds__(COPY_THREADS) void k_apply_matches(PlanDev dstp, PlanDev refp,
                                                                const int64_t *__restrict__ src,
                                                                unsigned long long *rejected) {
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t wave_in_group = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t nwaves = (uint64_t)gridDim.x * (COPY_THREADS / 64);
  const uint32_t piece_log2 = dstp.chunk_log2 < COPY_PIECE_LOG2 ? dstp.chunk_log2 : COPY_PIECE_LOG2;
  const uint32_t ppc_log2 = dstp.chunk_log2 - piece_log2;
  const uint64_t nitems = dstp.nchunks << ppc_log2;
  for (uint64_t item = (uint64_t)blockIdx.x * (COPY_THREADS / 64) + wave_in_group; item < nitems;
       item += nwaves) {
    const uint64_t k = item >> ppc_log2;
    const uint32_t piece = (uint32_t)(item & ((1ull << ppc_log2) - 1));
    const int64_t s = src[k];
    if (s == -1 || FROM_REF != (s >= 0)) continue;
    const ChunkRef to = locate_chunk(dstp, k);
    const PlanDev &fromp = FROM_REF ? refp : dstp;
    const uint64_t j = FROM_REF ? (uint64_t)s : (uint64_t)(-2 - s);
    bool ok = FROM_REF ? j < refp.nchunks : j < k;
    ChunkRef from = to;
    if (ok) {
      from = locate_chunk(fromp, j);
      ok = from.len == to.len;
    }
    if (!ok) {
      if (rejected != nullptr && piece == 0 && lane == 0) atomicAdd(rejected, 1ull);
      continue;
    }
    const uint8_t *sp = reinterpret_cast<const uint8_t *>(fromp.dense_ptr[from.row]) + from.off;
    uint8_t *dp = reinterpret_cast<uint8_t *>(dstp.dense_ptr[to.row]) + to.off;
    if (sp == dp) continue;                      // already in place
    const uint32_t lo = piece << piece_log2;
    uint32_t hi = lo + (1u << piece_log2);
    const uint32_t padded = (uint32_t)pad16(to.len);
    if (hi > padded) hi = padded;
    move_piece<false>(sp, dp, lo, hi, to.len, lane);
  }
}

// ---- moves inside one memory image ------------------------------------------
// When the destination already holds the reference (the paper's case: the next
// rank's data is assembled in the memory the previous rank left), chunk k must
// receive what chunk src[k] held *before* anything was overwritten, and moves
// can form cycles (a -> b -> a).  Two phases through a temporary buffer break
// every cycle: first all sources are gathered, then all destinations written.

__global__ __launch_bounds__(256) void k_mark_moves(const int64_t *__restrict__ src, uint64_t n,
                                                    uint8_t *__restrict__ moved) {
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  for (uint64_t k = (uint64_t)blockIdx.x * 256 + threadIdx.x; k < n; k += stride) {
    const int64_t s = src[k];
    moved[k] = (s >= 0 && (uint64_t)s != k) ? 1 : 0;
  }
}

// moves[e] (written by the manifest scan with the src array in place of the digests) names
// destination chunk (buf, buf_off), its place in temp (stage_off) and, in `digest`, the source
// chunk id.  SCATTER = false: source chunk -> temp.  SCATTER = true: temp -> destination chunk.
// Nothing is done unless every move fits temp (counts->overflow == 0): half a permutation
// would destroy sources that have not been read yet.
template <bool SCATTER>
__global__ __launch_bounds__(COPY_THREADS) void k_moves(PlanDev p,
                                                        const ckpt_entry_t *__restrict__ moves,
                                                        const ckpt_counts_t *__restrict__ counts,
                                                        uint8_t *__restrict__ temp,
                                                        unsigned long long *rejected) {
  if (counts->overflow != 0) return;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t wave_in_group = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t nwaves = (uint64_t)gridDim.x * (COPY_THREADS / 64);
  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint32_t ppc_log2 = p.chunk_log2 - piece_log2;
  const uint64_t nitems = counts->ndirty << ppc_log2;
  for (uint64_t item = (uint64_t)blockIdx.x * (COPY_THREADS / 64) + wave_in_group; item < nitems;
       item += nwaves) {
    const ckpt_entry_t ent = moves[item >> ppc_log2];
    const uint32_t piece = (uint32_t)(item & ((1ull << ppc_log2) - 1));
    const uint32_t lo = piece << piece_log2;
    uint32_t hi = lo + (1u << piece_log2);
    const uint32_t padded = (uint32_t)pad16(ent.len);
    if (hi > padded) hi = padded;
    uint8_t *slot = temp + ent.stage_off;
    // a move whose source is no chunk of the plan, or a chunk of another length, is rejected in
    // both phases alike: its temp slot is never filled and its destination never written
    const uint64_t j = ent.digest;                        // source chunk id
    bool ok = j < p.nchunks;
    ChunkRef from = {0, 0, 0};
    if (ok) {
      from = locate_chunk(p, j);
      ok = from.len == ent.len;
    }
    if (!ok) {
      if (!SCATTER && rejected != nullptr && piece == 0 && lane == 0) atomicAdd(rejected, 1ull);
      continue;
    }
    if (SCATTER) {
      uint8_t *to = reinterpret_cast<uint8_t *>(p.list_ptr[ent.buf]) + ent.buf_off;
      move_piece<false>(slot, to, lo, hi, ent.len, lane);
    } else {
      const uint8_t *sp = reinterpret_cast<const uint8_t *>(p.dense_ptr[from.row]) + from.off;
      move_piece<true>(sp, slot, lo, hi, ent.len, lane);
    }
  }
}

__global__ void k_zero_rejected(unsigned long long *p) { *p = 0; }

inline uint64_t pow2_at_least(uint64_t x) {
  uint64_t c = 1;
  while (c < x) c <<= 1;
  return c;
}

}  // namespace

uint64_t match_table_capacity(uint64_t n) { return pow2_at_least(2 * n + 2); }

uint64_t match_workspace_bytes(uint64_t n_ref, uint64_t n) {
  return 16 * (match_table_capacity(n_ref) + match_table_capacity(n)) + 64;
}

hipError_t launch_match(const PlanDev &p, const uint64_t *d_dig, const uint64_t *d_ref,
                        uint64_t n_ref, void *d_workspace, int64_t *d_src, uint8_t *d_mask,
                        ckpt_match_counts_t *d_counts, hipStream_t s) {
  const uint64_t cap_ref = match_table_capacity(n_ref), cap_self = match_table_capacity(p.nchunks);
  unsigned long long *w = reinterpret_cast<unsigned long long *>(d_workspace);
  MatchSpace m;
  m.ref.keys = w;
  m.ref.vals = w + cap_ref;
  m.self.keys = w + 2 * cap_ref;
  m.self.vals = w + 2 * cap_ref + cap_self;
  m.ref.lone = w + 2 * cap_ref + 2 * cap_self;
  m.self.lone = m.ref.lone + 1;
  m.ref.cap_mask = cap_ref - 1;
  m.self.cap_mask = cap_self - 1;
  const uint64_t biggest = cap_ref > cap_self ? cap_ref : cap_self;
  uint64_t init_groups = (biggest + 255) / 256;
  if (init_groups > 8192) init_groups = 8192;
  hipLaunchKernelGGL(k_match_init, dim3((uint32_t)init_groups), dim3(256), 0, s, m, d_counts);
  if (n_ref)
    hipLaunchKernelGGL(k_match_insert, dim3((uint32_t)((n_ref + 255) / 256)), dim3(256), 0, s, m.ref,
                       d_ref, n_ref, d_counts);
  if (p.nchunks) {
    const uint32_t groups = (uint32_t)((p.nchunks + 255) / 256);
    hipLaunchKernelGGL(k_match_insert, dim3(groups), dim3(256), 0, s, m.self, d_dig, p.nchunks,
                       d_counts);
    hipLaunchKernelGGL(k_match_probe, dim3(groups), dim3(256), 0, s, p, m, d_dig, d_ref, n_ref,
                       d_src, d_mask, d_counts);
  }
  return hipGetLastError();
}

uint64_t moves_workspace_bytes(uint64_t n) { return ((n + 15) & ~15ull) + 32 * n + 64; }

hipError_t launch_moves_inplace(const PlanDev &p, const int64_t *d_src, void *d_temp,
                                uint64_t temp_cap, void *d_workspace, uint64_t *d_blocksums,
                                ckpt_counts_t *d_counts, uint64_t *d_rejected, hipStream_t s) {
  unsigned long long *rej = reinterpret_cast<unsigned long long *>(d_rejected);
  if (rej) hipLaunchKernelGGL(k_zero_rejected, dim3(1), dim3(1), 0, s, rej);
  const uint64_t n = p.nchunks;
  uint8_t *moved = static_cast<uint8_t *>(d_workspace);
  ckpt_entry_t *moves = reinterpret_cast<ckpt_entry_t *>(moved + ((n + 15) & ~15ull));
  uint32_t groups = (uint32_t)((n + 255) / 256);
  if (groups > 4096) groups = 4096;
  if (groups) hipLaunchKernelGGL(k_mark_moves, dim3(groups), dim3(256), 0, s, d_src, n, moved);
  // the manifest scan, with src[k] travelling in the digest field of each entry
  hipError_t e = launch_compact_scan(p, moved, reinterpret_cast<const uint64_t *>(d_src), temp_cap,
                                     moves, n, d_blocksums, d_counts, nullptr, nullptr, false, s);
  if (e != hipSuccess || n == 0) return e;
  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint64_t items = n << (p.chunk_log2 - piece_log2);
  uint64_t cgroups = (items + COPY_THREADS / 64 - 1) / (COPY_THREADS / 64);
  if (cgroups > COPY_MAX_GROUPS) cgroups = COPY_MAX_GROUPS;
  hipLaunchKernelGGL(k_moves<false>, dim3((uint32_t)cgroups), dim3(COPY_THREADS), 0, s, p, moves,
                     d_counts, static_cast<uint8_t *>(d_temp), rej);
  hipLaunchKernelGGL(k_moves<true>, dim3((uint32_t)cgroups), dim3(COPY_THREADS), 0, s, p, moves,
                     d_counts, static_cast<uint8_t *>(d_temp), rej);
  return hipGetLastError();
}

hipError_t launch_apply_matches(const PlanDev &dstp, const PlanDev *refp, const int64_t *d_src,
                                uint64_t *d_rejected, hipStream_t s) {
  unsigned long long *rej = reinterpret_cast<unsigned long long *>(d_rejected);
  if (rej) hipLaunchKernelGGL(k_zero_rejected, dim3(1), dim3(1), 0, s, rej);
  if (dstp.nchunks == 0) return hipGetLastError();
  const uint32_t piece_log2 = dstp.chunk_log2 < COPY_PIECE_LOG2 ? dstp.chunk_log2 : COPY_PIECE_LOG2;
  const uint64_t items = dstp.nchunks << (dstp.chunk_log2 - piece_log2);
  uint64_t groups = (items + COPY_THREADS / 64 - 1) / (COPY_THREADS / 64);
  if (groups > COPY_MAX_GROUPS) groups = COPY_MAX_GROUPS;
  // first everything that comes from the reference, then the duplicates, which may
  // read destination chunks the first pass (or an earlier restore) has written
  if (refp != nullptr)
    hipLaunchKernelGGL(k_apply_matches<true>, dim3((uint32_t)groups), dim3(COPY_THREADS), 0, s, dstp,
                       *refp, d_src, rej);
  hipLaunchKernelGGL(k_apply_matches<false>, dim3((uint32_t)groups), dim3(COPY_THREADS), 0, s, dstp,
                     dstp, d_src, rej);
  return hipGetLastError();
}

}  // namespace ckpt
