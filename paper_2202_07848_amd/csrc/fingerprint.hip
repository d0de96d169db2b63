// Fingerprint kernel: one XXH64 (seed 0) per chunk of every live buffer -- the
// per-buffer content checksums of the Singularity paper (sec. 5.2.1, sec. 6),
// at chunk granularity.
//
// Mapping.  XXH64 offers four independent chains per chunk and nothing more, so
// a wavefront takes GROUP = 16 chunks of equal (or, for short last chunks,
// similar) length and gives each chunk a quad of lanes: lane 4c+t owns
// accumulator t of chunk c.  That lane needs the t-th 8-byte word of every
// 32-byte stripe -- 8 bytes at stride 32 -- which is the opposite of what
// coalesces.  So the wave loads in a different role: each global_load_dwordx4
// instruction fetches 256 contiguous bytes (one TILE) from each of four chunks,
// 16 lanes x 16 B per chunk, the tile goes through LDS, and the hashing lanes
// read their words back with ds_read2_b64.  Tiles are prefetched DEPTH deep in
// registers, so LDS only ever holds the tile being hashed (4.5 KiB per wave).
// Loads are never inside a branch: a loader lane with nothing left to fetch
// reads a 256-byte spare block owned by the plan.  The workgroup is a single
// wavefront: LDS traffic of one wave is executed in order, so only
// compiler-level (wavefront-scope) fences are needed between the write and
// read phases, never s_barrier and never a wait on outstanding global loads.
//
// A chunk of length len is split as  full tiles | up to 7 stripes | < 32 bytes.
// The tile loop is wave-uniform up to the longest chunk in the group; lanes of
// shorter chunks are masked.  Residual stripes and the tail are read straight
// from global memory (they are < 256 bytes per chunk).
//
// The same kernel is the single pass of ckpt_snapshot: there the loader lanes
// also write each tile of a hinted chunk to its place in the staging buffer from
// the registers they loaded it into.  That pass runs as two launches, first the
// groups that stage something, then the rest, each over a device-built list of
// its groups.  Measured on MI355X (3 B state, 1 MiB chunks, 36 % staged): with
// both kinds of group in one launch the wavefronts that also write take twice
// as long as the others and the pass needs 18.0 ms; read/write traffic and pure
// reads in separate phases, the working workgroups of each launch numbered
// densely, need 16.3 ms (a copy with the same per-wavefront stream structure
// runs at 5.2 TB/s, a read at 6.7 TB/s: 14.9 ms).
#include "ckpt_internal.h"
#include "stream_copy.h"
#include "xxh64_device.h"

namespace ckpt {

namespace {

constexpr int TILE = 256;              // bytes of one chunk staged per step
constexpr int TILE_LOG2 = 8;
constexpr int LDS_PITCH = TILE + 32;   // per-chunk pitch; the 32-byte skew spreads chunks over banks
constexpr int LOADS = GROUP * TILE / (64 * 16);   // dwordx4 loads per lane per step (= 4)
// Tiles in flight per lane.  2, 3 and 4 measure the same within noise on MI355X;
// 2 keeps the kernel at 95 VGPRs (five waves per SIMD).
constexpr int DEPTH = 2;

__device__ __forceinline__ void lds_phase_fence() {
  // Orders this wave's LDS writes and reads in the compiler; the hardware
  // executes one wave's LDS instructions in issue order.
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// 16-byte load through a pointer known to be global memory (global_load, which
// only counts on vmcnt, instead of flat_load, which also holds up LDS waits).
// Every byte is read exactly once, so the load is non-temporal: measured on
// MI355X a plain streaming read reaches 7.2 TB/s with the nt hint and 6.4 TB/s
// without it.
__device__ __forceinline__ u32x4 gload16(const uint8_t *p) {
  return __builtin_nontemporal_load((global_load_ptr)(p));
}
__device__ __forceinline__ void gstore16(uint8_t *p, u32x4 v) {
  __builtin_nontemporal_store(v, (global_store_ptr)(p));
}

// One step of the tile pipeline: the prefetched tile in q goes to LDS, the
// slot is refilled with tile `next` (REFILL), the hashing lanes consume it.
// In the non-uniform case a loader lane whose chunk has no tile `next` reads
// the plan's spare block instead, and a hashing lane whose chunk is already
// finished sits the step out; nothing in the step is a branch around a load,
// so the compiler can count outstanding loads exactly.  With STAGE the tile
// is also written to the staging position of its chunk (sptr, null for chunks
// that are not staged) straight from the registers it was loaded into: the
// single-pass snapshot never reads a byte twice.
template <bool UNIFORM, bool REFILL, bool STAGE>
__device__ __forceinline__ uint64_t tile_step(u32x4 (&q)[LOADS], uint8_t *wr, const uint8_t *rd,
                                              const uint8_t *const (&lptr)[LOADS],
                                              uint8_t *const (&sptr)[LOADS],
                                              const uint32_t (&ltiles)[LOADS],
                                              const uint8_t *spare, uint32_t my_tiles, uint32_t tt,
                                              uint32_t next, uint64_t acc) {
#pragma unroll
  for (int i = 0; i < LOADS; ++i) *reinterpret_cast<u32x4 *>(wr + i * 4 * LDS_PITCH) = q[i];
  if (STAGE) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      if (sptr[i] != nullptr && (UNIFORM || tt < ltiles[i]))
        gstore16(sptr[i] + (uint64_t)tt * TILE, q[i]);
    }
  }
  lds_phase_fence();
  if (REFILL) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const uint8_t *a = lptr[i] + (uint64_t)next * TILE;
      if (!UNIFORM) a = next < ltiles[i] ? a : spare;
      q[i] = gload16(a);
    }
  }
  if (UNIFORM || tt < my_tiles) {
#pragma unroll
    for (int s = 0; s < TILE / 32; ++s)
      acc = xxh::round(acc, *reinterpret_cast<const uint64_t *>(rd + 32 * s));
  }
  lds_phase_fence();
  return acc;
}

template <bool UNIFORM, bool STAGE>
__device__ __forceinline__ uint64_t hash_tiles(uint8_t *s_tile, const uint8_t *const (&lptr)[LOADS],
                                               uint8_t *const (&sptr)[LOADS],
                                               const uint32_t (&ltiles)[LOADS],
                                               const uint8_t *spare, uint32_t my_tiles,
                                               uint32_t max_tiles, int lane, uint64_t acc) {
  const int c = lane >> 2, t = lane & 3;
  uint8_t *wr = s_tile + (lane >> 4) * LDS_PITCH + 16 * (lane & 15);
  const uint8_t *rd = s_tile + c * LDS_PITCH + 8 * t;
  spare += 16 * (lane & 15);

  // prologue: tiles 0..DEPTH-1 (those that exist)
  u32x4 q[DEPTH][LOADS];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const uint32_t have = UNIFORM ? max_tiles : ltiles[i];
      q[d][i] = gload16((uint32_t)d < have ? lptr[i] + (uint64_t)d * TILE : spare);
    }
  }

  // steady state: every step refills its slot, DEPTH steps per trip
  const uint32_t steady = max_tiles > DEPTH ? (max_tiles - DEPTH) / DEPTH * DEPTH : 0;
  uint32_t tile = 0;
  for (; tile < steady; tile += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d)
      acc = tile_step<UNIFORM, true, STAGE>(q[d], wr, rd, lptr, sptr, ltiles, spare, my_tiles,
                                            tile + d, tile + d + DEPTH, acc);
  }
  // drain: the last DEPTH..2*DEPTH-1 tiles (or all of them if there are fewer)
#pragma unroll
  for (int d = 0; d < 2 * DEPTH; ++d) {
    const uint32_t tt = steady + d;              // wave-uniform
    if (tt < max_tiles) {
      if (tt + DEPTH < max_tiles)
        acc = tile_step<UNIFORM, true, STAGE>(q[d % DEPTH], wr, rd, lptr, sptr, ltiles, spare,
                                              my_tiles, tt, tt + DEPTH, acc);
      else
        acc = tile_step<UNIFORM, false, STAGE>(q[d % DEPTH], wr, rd, lptr, sptr, ltiles, spare,
                                               my_tiles, tt, 0, acc);
    }
  }
  return acc;
}

// STAGE: the fused snapshot.  A chunk k with hint[k] != 0 is copied, while it is
// hashed, to staging + hoff[k] (zero padded to 16 bytes) provided it ends at or
// before staging_cap -- the same rule ckpt_compact applies.
struct StageArgs {
  const uint8_t *hint;      // [N]
  const uint64_t *hoff;     // [N] staging offset of every hinted chunk
  uint8_t *staging;
  uint64_t staging_cap;
  // groups that stage at least one chunk, list[0 .. counts[0]), and the others, from the back:
  // list[ngroups-1 - i], i in [0, counts[1]) -- written by k_group_lists
  const uint32_t *list;
  const unsigned long long *counts;
  uint32_t ngroups;
  // the comparison of ckpt_diff done on the spot: mask[k] = (ref == null || digest != ref[k]),
  // written by the lane that finishes the digest (mask null: not wanted)
  const uint64_t *ref;
  uint8_t *mask;
  // words the first workgroup clears for the kernels that follow the pass (each may be null)
  unsigned long long *clear_a, *clear_b;
};

// Slot `lane` of group `group`: the chunk's address, global id and length (0: empty slot).
// The groups are the full-chunk groups (longest work first) followed by the groups of short
// chunks, which are sorted by length.
__device__ __forceinline__ void group_slot(const PlanDev &p, uint64_t group, int lane, uint64_t *ptr,
                                           uint64_t *k, uint32_t *len) {
  const uint64_t full_groups = (p.nfull + GROUP - 1) / GROUP;
  *ptr = 0;
  *k = 0;
  *len = 0;
  if (group < full_groups) {
    const uint64_t f = group * GROUP + lane;                    // ordinal among full chunks
    if (f < p.nfull) {
      uint32_t row = p.full_group_first[group];
      while (f >= p.full_base[row + 1]) ++row;                  // ends: full_base[nf] = nfull > f
      const uint64_t j = f - p.full_base[row];
      *ptr = p.full_ptr[row] + (j << p.chunk_log2);
      *k = p.full_chunk0[row] + j;
      *len = 1u << p.chunk_log2;
    }
  } else {
    const uint64_t s = (group - full_groups) * GROUP + lane;
    if (s < p.nshort) {
      *ptr = p.short_ptr[s];
      *k = p.short_chunk[s];
      *len = p.short_len[s];
    }
  }
}

// Where chunk k (of length len != 0) is staged, or 0 if it is not: hinted, and ending at or
// before staging_cap -- the same rule ckpt_compact applies.
__device__ __forceinline__ uint64_t stage_address(const StageArgs &st, uint64_t k, uint32_t len) {
  if (st.hint[k] == 0) return 0;
  const uint64_t off = st.hoff[k];
  if (off <= st.staging_cap && pad16(len) <= st.staging_cap - off)
    return reinterpret_cast<uint64_t>(st.staging) + off;
  return 0;
}

// Sorting the groups into those that stage something and the rest (see StageArgs), in two
// kernels.  k_group_flags: does group g stage a chunk?  GROUP lanes per group, one per slot,
// because each lookup is a chain of dependent loads.
__global__ __launch_bounds__(256) void k_group_flags(PlanDev p, StageArgs st,
                                                     uint8_t *__restrict__ flags) {
  const uint64_t gid = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  const uint64_t g = gid / GROUP;
  const int lane = threadIdx.x & 63;
  bool staged = false;
  if (g < st.ngroups) {
    uint64_t ptr, k;
    uint32_t len;
    group_slot(p, g, (int)(gid % GROUP), &ptr, &k, &len);
    staged = len != 0 && stage_address(st, k, len) != 0;
  }
  const uint64_t staged_lanes = __ballot(staged);
  if (g < st.ngroups && gid % GROUP == 0)
    flags[g] = ((staged_lanes >> (lane & ~(GROUP - 1))) & ((1ull << GROUP) - 1)) != 0;
}

// k_group_lists: a workgroup takes LIST_RUN consecutive groups and appends its share to each
// list as one run, in group order, with one atomic per list.  The lists stay sorted in long
// runs, which keeps the pass a forward sweep through memory: with 4 KiB chunks a list
// shuffled in runs of 4 costs 30 %; runs of 64, 256 and 1024 measure alike within 3 %.
// Which run lands where only decides which workgroup runs which group, never a result.
// counts[0..1] are zero on entry.
template <int LIST_RUN>
__global__ __launch_bounds__(LIST_RUN) void k_group_lists(const uint8_t *__restrict__ flags,
                                                          uint32_t ngroups, uint32_t *list,
                                                          unsigned long long *counts) {
  __shared__ uint32_t s_wave_stage[LIST_RUN / 64], s_wave_rest[LIST_RUN / 64];
  __shared__ unsigned long long s_base[2];
  const uint64_t g = (uint64_t)blockIdx.x * LIST_RUN + threadIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool valid = g < ngroups;
  const bool any = valid && flags[valid ? g : 0] != 0;
  // rank of this group among the workgroup's groups of the same kind
  const uint64_t lanes_below = (1ull << lane) - 1;
  const uint64_t m_stage = __ballot(any), m_rest = __ballot(valid && !any);
  if (lane == 0) {
    s_wave_stage[wave] = (uint32_t)__popcll(m_stage);
    s_wave_rest[wave] = (uint32_t)__popcll(m_rest);
  }
  __syncthreads();
  uint32_t before_stage = 0, before_rest = 0, all_stage = 0, all_rest = 0;
#pragma unroll
  for (int v = 0; v < LIST_RUN / 64; ++v) {
    if (v < wave) {
      before_stage += s_wave_stage[v];
      before_rest += s_wave_rest[v];
    }
    all_stage += s_wave_stage[v];
    all_rest += s_wave_rest[v];
  }
  if (threadIdx.x == 0) {
    s_base[0] = all_stage ? atomicAdd(&counts[0], (unsigned long long)all_stage) : 0;
    s_base[1] = all_rest ? atomicAdd(&counts[1], (unsigned long long)all_rest) : 0;
  }
  __syncthreads();
  if (any)
    list[s_base[0] + before_stage + __popcll(m_stage & lanes_below)] = (uint32_t)g;
  else if (valid)
    list[ngroups - 1 - (s_base[1] + before_rest + __popcll(m_rest & lanes_below))] = (uint32_t)g;
}

// MODE_PLAIN: ckpt_fingerprint, workgroup b takes group b.  The fused snapshot runs
// MODE_STAGING over the list of groups that stage at least one chunk and then MODE_REST over
// the list of the others; workgroups beyond a list's length exit at once, so the working ones
// have the lowest numbers and spread evenly over the chip.
// MODE_MIXED is the same pass as one launch, workgroup b taking group b and staging whatever
// its chunks need: for small states, where two more launches cost more than the split gains.
constexpr int MODE_PLAIN = 0, MODE_STAGING = 1, MODE_REST = 2, MODE_MIXED = 3;

template <int MODE>
__global__ __launch_bounds__(64) void k_fingerprint(PlanDev p, uint64_t *__restrict__ dig,
                                                    StageArgs st) {
  constexpr bool STAGE = MODE == MODE_STAGING || MODE == MODE_MIXED;   // writes to staging
  __shared__ __align__(16) uint8_t s_tile[GROUP * LDS_PITCH];
  __shared__ uint64_t s_ptr[GROUP];
  __shared__ uint64_t s_chunk[GROUP];
  __shared__ uint64_t s_stage[STAGE ? GROUP : 1];
  __shared__ uint32_t s_len[GROUP];

  const int lane = threadIdx.x;
  uint64_t group = blockIdx.x;
  if (blockIdx.x == 0 && lane == 0) {
    if (st.clear_a != nullptr) *st.clear_a = 0;
    if (st.clear_b != nullptr) *st.clear_b = 0;
  }
  if (MODE == MODE_STAGING) {
    if (group >= st.counts[0]) return;                   // one wavefront: uniform for the workgroup
    group = st.list[group];
  } else if (MODE == MODE_REST) {
    if (group >= st.counts[1]) return;
    group = st.list[st.ngroups - 1 - group];
  }

  if (lane < GROUP) {
    uint64_t ptr, k;
    uint32_t len;
    group_slot(p, group, lane, &ptr, &k, &len);
    s_ptr[lane] = ptr;
    s_chunk[lane] = k;
    s_len[lane] = len;
    if (STAGE) s_stage[lane] = len != 0 ? stage_address(st, k, len) : 0;
  }
  __syncthreads();

  const int c = lane >> 2, t = lane & 3;
  const uint32_t my_len = s_len[c];
  const uint8_t *my_ptr = reinterpret_cast<const uint8_t *>(s_ptr[c]);
  const uint32_t my_tiles = my_len >> TILE_LOG2;
  const uint64_t my_stage = STAGE ? s_stage[STAGE ? c : 0] : 0;

  // loader role: load i of this lane serves chunk 4*i + lane/16, bytes 16*(lane%16)..+15 of a tile
  const uint8_t *lptr[LOADS];
  uint8_t *sptr[LOADS];
  uint32_t ltiles[LOADS];
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int lc = 4 * i + (lane >> 4);
    lptr[i] = reinterpret_cast<const uint8_t *>(s_ptr[lc]) + 16 * (lane & 15);
    ltiles[i] = s_len[lc] >> TILE_LOG2;
    sptr[i] = nullptr;
    if (STAGE && s_stage[STAGE ? lc : 0] != 0)
      sptr[i] = reinterpret_cast<uint8_t *>(s_stage[STAGE ? lc : 0]) + 16 * (lane & 15);
  }
  uint32_t max_tiles = 0, min_tiles = 0xFFFFFFFFu;
#pragma unroll
  for (int i = 0; i < GROUP; ++i) {
    const uint32_t n = s_len[i] >> TILE_LOG2;
    max_tiles = n > max_tiles ? n : max_tiles;
    min_tiles = n < min_tiles ? n : min_tiles;
  }
  max_tiles = __builtin_amdgcn_readfirstlane(max_tiles);
  min_tiles = __builtin_amdgcn_readfirstlane(min_tiles);

  uint64_t acc = xxh::acc_init(t);
  if (max_tiles == min_tiles)
    acc = hash_tiles<true, STAGE>(s_tile, lptr, sptr, ltiles, p.spare, my_tiles, max_tiles, lane,
                                  acc);
  else
    acc = hash_tiles<false, STAGE>(s_tile, lptr, sptr, ltiles, p.spare, my_tiles, max_tiles, lane,
                                   acc);

  // up to 7 stripes between the last full tile and the tail
  const uint32_t rem = my_len & (TILE - 1);
  const uint32_t rstripes = rem >> 5;
  const uint8_t *rp = my_ptr + ((uint64_t)my_tiles << TILE_LOG2);
#pragma unroll
  for (int s = 0; s < TILE / 32 - 1; ++s) {
    if ((uint32_t)s < rstripes)
      acc = xxh::round(acc, *reinterpret_cast<const uint64_t *>(rp + 32 * s + 8 * t));
  }

  // staged copy of what follows the last full tile (< 256 bytes), zero padded to 16:
  // the quad's four lanes take the 16-byte units round-robin
  if (STAGE && my_stage != 0) {
    uint8_t *sp = reinterpret_cast<uint8_t *>(my_stage);
    const uint32_t done = my_tiles << TILE_LOG2, padded = (uint32_t)pad16(my_len);
#pragma unroll
    for (int j = 0; j < TILE / 64; ++j) {
      const uint32_t o = done + 16 * (t + 4 * j);
      if (o < padded) {
        const uint4 v = o + 16 <= my_len ? stream_load16(my_ptr + o)
                                         : load_partial16(my_ptr + o, my_len - o);
        stream_store16(sp + o, v);
      }
    }
  }

  // gather the quad's four accumulators (every lane of the quad gets all four)
  const int qbase = lane & ~3;
  const uint64_t v1 = __shfl(acc, qbase + 0, 64);
  const uint64_t v2 = __shfl(acc, qbase + 1, 64);
  const uint64_t v3 = __shfl(acc, qbase + 2, 64);
  const uint64_t v4 = __shfl(acc, qbase + 3, 64);

  if (t == 0 && my_len != 0) {
    uint64_t h = my_len >= 32 ? xxh::converge(v1, v2, v3, v4) : xxh::PRIME5;
    h += my_len;
    const uint8_t *tp = rp + 32 * rstripes;
    uint32_t left = my_len & 31;
    while (left >= 8) {
      h = xxh::tail8(h, *reinterpret_cast<const uint64_t *>(tp));
      tp += 8;
      left -= 8;
    }
    if (left >= 4) {
      h = xxh::tail4(h, *reinterpret_cast<const uint32_t *>(tp));
      tp += 4;
      left -= 4;
    }
    while (left > 0) {
      h = xxh::tail1(h, *tp);
      tp += 1;
      left -= 1;
    }
    h = xxh::avalanche(h);
    const uint64_t k = s_chunk[c];
    dig[k] = h;
    if (st.mask != nullptr) st.mask[k] = (st.ref == nullptr || h != st.ref[k]) ? 1 : 0;
  }
}

}  // namespace

constexpr int LIST_RUN = 1024;   // groups per run of the fused pass's group lists

uint64_t fingerprint_groups(const PlanDev &p) {
  return (p.nfull + GROUP - 1) / GROUP + (p.nshort + GROUP - 1) / GROUP;
}

hipError_t launch_fingerprint(const PlanDev &p, uint64_t *d_digests, hipStream_t s) {
  if (p.nchunks == 0) return hipSuccess;
  const uint64_t groups = fingerprint_groups(p);
  if (groups > 0x7FFFFFFFull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_fingerprint<MODE_PLAIN>, dim3((uint32_t)groups), dim3(64), 0, s, p,
                     d_digests,
                     StageArgs{nullptr, nullptr, nullptr, 0, nullptr, nullptr, 0, nullptr, nullptr,
                               nullptr, nullptr});
  return hipGetLastError();
}

hipError_t launch_fingerprint_diff(const PlanDev &p, uint64_t *d_digests, const uint64_t *d_ref,
                                   uint8_t *d_mask, ckpt_counts_t *d_counts, uint64_t *d_misses_out,
                                   hipStream_t s) {
  if (p.nchunks == 0) return hipSuccess;
  const uint64_t groups = fingerprint_groups(p);
  if (groups > 0x7FFFFFFFull) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_fingerprint<MODE_PLAIN>, dim3((uint32_t)groups), dim3(64), 0, s, p,
                     d_digests,
                     StageArgs{nullptr, nullptr, nullptr, 0, nullptr, nullptr, 0, d_ref, d_mask,
                               reinterpret_cast<unsigned long long *>(&d_counts->overflow),
                               reinterpret_cast<unsigned long long *>(d_misses_out)});
  return hipGetLastError();
}

// split: the group lists, then two launches: first the groups that stage at least one chunk,
// then the others.  d_list holds one uint32 and d_flags one byte per group; d_list_counts two
// uint64 that are zero when the first kernel here starts.  !split: one launch over all groups.
hipError_t launch_fingerprint_staging(const PlanDev &p, uint64_t *d_digests, const uint64_t *d_ref,
                                      uint8_t *d_mask, const uint8_t *d_hint,
                                      const uint64_t *d_hint_off, void *d_staging,
                                      uint64_t staging_cap, uint32_t *d_list, uint8_t *d_flags,
                                      uint64_t *d_list_counts, bool split, hipStream_t s) {
  if (p.nchunks == 0) return hipSuccess;
  const uint64_t groups = fingerprint_groups(p);
  if (groups > 0x7FFFFFFFull) return hipErrorInvalidValue;
  unsigned long long *counts = reinterpret_cast<unsigned long long *>(d_list_counts);
  const StageArgs st{d_hint, d_hint_off, reinterpret_cast<uint8_t *>(d_staging), staging_cap,
                     d_list,  counts,    (uint32_t)groups, d_ref, d_mask, nullptr, nullptr};
  if (!split) {
    hipLaunchKernelGGL(k_fingerprint<MODE_MIXED>, dim3((uint32_t)groups), dim3(64), 0, s, p,
                       d_digests, st);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(k_group_flags, dim3((uint32_t)((groups * GROUP + 255) / 256)), dim3(256), 0, s,
                     p, st, d_flags);
  hipLaunchKernelGGL(k_group_lists<LIST_RUN>, dim3((uint32_t)((groups + LIST_RUN - 1) / LIST_RUN)),
                     dim3(LIST_RUN), 0, s, d_flags, (uint32_t)groups, d_list, counts);
  hipLaunchKernelGGL(k_fingerprint<MODE_STAGING>, dim3((uint32_t)groups), dim3(64), 0, s, p,
                     d_digests, st);
  hipLaunchKernelGGL(k_fingerprint<MODE_REST>, dim3((uint32_t)groups), dim3(64), 0, s, p, d_digests,
                     st);
  return hipGetLastError();
}

}  // namespace ckpt
