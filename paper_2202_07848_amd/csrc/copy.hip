// Data movement of the snapshot path: gather of the marked chunks into the
// contiguous staging buffer (the swap-out of what was not de-duplicated,
// Singularity paper sec. 5.2.1) and the inverse scatter (swap-in / restore to
// the original addresses, sec. 4.5).  Also two plain streaming kernels used to
// calibrate bandwidth and HBM counters.
//
// Work item = one piece (min(C, 16 KiB)) of one manifest entry, handled by one
// wavefront: 64 lanes x 16 B = 1 KiB per instruction, all sixteen loads of a
// piece issued before its stores, non-temporal both ways.  Items are dealt to wavefronts round-robin (item = wave id + i * number
// of waves), so neighbouring waves stream neighbouring 16 KiB pieces of source
// and staging.  The gather does not know the entry count on the host (it sits
// in device memory right after the scan), so the grid is fixed and every wave
// loops until its item index passes the device-side count: every wave reaches
// the exit, nothing waits on another wave.
#include "ckpt_internal.h"
#include "stream_copy.h"
#include "xxh64_device.h"

namespace ckpt {

namespace {

constexpr int UNROLL = 8;        // streaming yardsticks: 16-byte units per lane in flight

// GATHER: buffers -> staging (zero padded to 16).  !GATHER: staging -> buffers
// (exactly len bytes).  `count_dev`, when not null, supplies the entry count
// (its ndirty, clipped to entry_cap); otherwise entry_cap is the count.
template <bool GATHER>
__global__ __launch_bounds__(COPY_THREADS) void k_move(PlanDev p,
                                                       const ckpt_entry_t *__restrict__ manifest,
                                                       uint64_t entry_cap,
                                                       const ckpt_counts_t *__restrict__ count_dev,
                                                       uint8_t *__restrict__ staging,
                                                       uint64_t staging_limit,
                                                       unsigned long long *__restrict__ rejected,
                                                       const unsigned long long *only_if_nonzero,
                                                       const uint8_t *__restrict__ need) {
  // the fused snapshot has already staged everything when its hint was exact; when it was not,
  // `need` marks the entries that are not yet where they belong
  if (only_if_nonzero != nullptr && *only_if_nonzero == 0) return;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t wave_in_group = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t nwaves = (uint64_t)gridDim.x * (COPY_THREADS / 64);
  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint32_t ppc_log2 = p.chunk_log2 - piece_log2;     // pieces per chunk

  uint64_t nentries = entry_cap;
  if (count_dev != nullptr) {
    const uint64_t n = count_dev->ndirty;
    nentries = n < entry_cap ? n : entry_cap;
  }
  const uint64_t nitems = nentries << ppc_log2;

  for (uint64_t item = (uint64_t)blockIdx.x * (COPY_THREADS / 64) + wave_in_group; item < nitems;
       item += nwaves) {
    const uint64_t e = item >> ppc_log2;
    const uint32_t piece = (uint32_t)(item & ((1ull << ppc_log2) - 1));
    if (need != nullptr && need[e] == 0) continue;
    const ckpt_entry_t ent = manifest[e];
    const uint64_t padded = pad16(ent.len);

    // validity (always true for a manifest this library wrote with enough capacity);
    // written so that no sum can wrap
    bool ok = ent.buf < p.nbufs && ((ent.buf_off | ent.stage_off) & 15) == 0 &&
              ent.len <= (1ull << p.chunk_log2);
    if (ok) {
      const uint64_t nb = p.list_nbytes[ent.buf];
      ok = ent.buf_off <= nb && ent.len <= nb - ent.buf_off;
    }
    const uint64_t need = GATHER ? padded : (uint64_t)ent.len;
    ok = ok && ent.stage_off <= staging_limit && need <= staging_limit - ent.stage_off;
    if (!ok) {
      if (!GATHER && rejected != nullptr && piece == 0 && lane == 0) atomicAdd(rejected, 1ull);
      continue;
    }

    uint8_t *buf = reinterpret_cast<uint8_t *>(p.list_ptr[ent.buf]) + ent.buf_off;
    uint8_t *stg = staging + ent.stage_off;
    const uint8_t *src = GATHER ? buf : stg;
    uint8_t *dst = GATHER ? stg : buf;

    const uint32_t lo = piece << piece_log2;
    uint32_t hi = lo + (1u << piece_log2);
    if (hi > padded) hi = (uint32_t)padded;
    const uint32_t len = ent.len;

    move_piece<GATHER>(src, dst, lo, hi, len, lane);
  }
}

__global__ void k_zero_u64(unsigned long long *p) { *p = 0; }

__global__ __launch_bounds__(256) void k_bw_copy(uint4 *__restrict__ dst,
                                                 const uint4 *__restrict__ src, uint64_t n16) {
  // non-temporal both ways, like every streaming access of the path
  const uint8_t *s8 = reinterpret_cast<const uint8_t *>(src);
  uint8_t *d8 = reinterpret_cast<uint8_t *>(dst);
  const uint64_t stride = (uint64_t)gridDim.x * 256 * UNROLL;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 * UNROLL + threadIdx.x; i < n16; i += stride) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (i + u * 256 < n16) v[u] = stream_load16(s8 + 16 * (i + u * 256));
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
      if (i + u * 256 < n16) stream_store16(d8 + 16 * (i + u * 256), v[u]);
  }
}

__global__ __launch_bounds__(256) void k_bw_read(const uint4 *__restrict__ src, uint64_t n16,
                                                 uint64_t *__restrict__ sink) {
  const uint64_t stride = (uint64_t)gridDim.x * 256 * UNROLL;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (uint64_t i = (uint64_t)blockIdx.x * 256 * UNROLL + threadIdx.x; i < n16; i += stride) {
    uint4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      v[u] = make_uint4(0, 0, 0, 0);
      if (i + u * 256 < n16)
        v[u] = stream_load16(reinterpret_cast<const uint8_t *>(src) + 16 * (i + u * 256));
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      acc.x ^= v[u].x;
      acc.y ^= v[u].y;
      acc.z ^= v[u].z;
      acc.w ^= v[u].w;
    }
  }
  __shared__ uint64_t s_x[256];
  s_x[threadIdx.x] = ((uint64_t)(acc.x ^ acc.z) << 32) | (acc.y ^ acc.w);
  __syncthreads();
  for (int d = 128; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) s_x[threadIdx.x] ^= s_x[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0) sink[blockIdx.x] = s_x[0];
}

// The fingerprint kernel's memory access pattern without its arithmetic: single-wavefront
// workgroups, 16 streams per wavefront (stream i = bytes [i, i+1) * stream_bytes of src), two
// tiles per stream prefetched in registers.  TILE = bytes of one stream fetched per step: with
// 256 (the fingerprint kernel's tile) each load instruction takes 256 bytes from each of four
// streams, with 1024 one kibibyte of a single stream.  COPY: every tile is stored to the same
// offset of dst (what the fused snapshot pass does with staged chunks); otherwise the tiles are
// XOR-ed into one word per wavefront.  Its rate is the ceiling this access pattern leaves the
// fingerprint pass.
template <int TILE, bool COPY>
__global__ __launch_bounds__(64) void k_bw_streams(const uint8_t *__restrict__ src,
                                                   uint8_t *__restrict__ dst,
                                                   uint64_t stream_bytes,
                                                   uint64_t *__restrict__ sink) {
  constexpr int LANES = TILE / 16;        // lanes that share one stream in a load instruction
  constexpr int PER_LOAD = 64 / LANES;    // streams one load instruction serves
  constexpr int NLOADS = 16 / PER_LOAD;   // load instructions per step
  const uint32_t lane = threadIdx.x;
  const uint64_t first = (uint64_t)blockIdx.x * 16;
  const uint8_t *lp[NLOADS];
  uint8_t *sp[NLOADS];
#pragma unroll
  for (int i = 0; i < NLOADS; ++i) {
    const uint64_t off = (first + PER_LOAD * i + lane / LANES) * stream_bytes + 16 * (lane % LANES);
    lp[i] = src + off;
    sp[i] = dst + off;
  }
  const uint64_t tiles = stream_bytes / TILE;      // even and >= 2 (checked on the host)
  uint4 q0[NLOADS], q1[NLOADS], acc = make_uint4(0, 0, 0, 0);
#pragma unroll
  for (int i = 0; i < NLOADS; ++i) {
    q0[i] = stream_load16(lp[i]);
    q1[i] = stream_load16(lp[i] + TILE);
  }
  for (uint64_t t = 0; t < tiles; t += 2) {
#pragma unroll
    for (int i = 0; i < NLOADS; ++i) {
      if (COPY) {
        stream_store16(sp[i] + t * TILE, q0[i]);
      } else {
        acc.x ^= q0[i].x; acc.y ^= q0[i].y; acc.z ^= q0[i].z; acc.w ^= q0[i].w;
      }
      if (t + 2 < tiles) q0[i] = stream_load16(lp[i] + (t + 2) * TILE);
    }
#pragma unroll
    for (int i = 0; i < NLOADS; ++i) {
      if (COPY) {
        stream_store16(sp[i] + (t + 1) * TILE, q1[i]);
      } else {
        acc.x ^= q1[i].x; acc.y ^= q1[i].y; acc.z ^= q1[i].z; acc.w ^= q1[i].w;
      }
      if (t + 3 < tiles) q1[i] = stream_load16(lp[i] + (t + 3) * TILE);
    }
  }
  if (!COPY) {
    uint64_t v = ((uint64_t)(acc.x ^ acc.z) << 32) | (acc.y ^ acc.w);
    for (int o = 32; o > 0; o >>= 1) v ^= __shfl_down(v, o, 64);
    if (lane == 0) sink[blockIdx.x % 2048] = v;      // keeps the loads alive; value unused
  }
}

// The hash arithmetic alone: every lane runs `rounds` XXH64 accumulator steps on words it
// makes up in registers (one 64-bit add per word), no memory traffic.  Its rate, times 8 bytes
// per step, is the ceiling the integer units set for the fingerprint kernel.
__global__ __launch_bounds__(256) void k_alu_xxh64(uint64_t rounds, uint64_t *__restrict__ sink) {
  uint64_t acc = xxh::acc_init(threadIdx.x & 3) + blockIdx.x;
  uint64_t w = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  for (uint64_t i = 0; i < rounds; i += 8) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      acc = xxh::round(acc, w);
      w += 0x9E3779B97F4A7C15ull;
    }
  }
  // keeps the loop alive; one word per workgroup, as k_bw_read
  __shared__ uint64_t s_x[256];
  s_x[threadIdx.x] = acc;
  __syncthreads();
  for (int d = 128; d > 0; d >>= 1) {
    if ((int)threadIdx.x < d) s_x[threadIdx.x] ^= s_x[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0) sink[blockIdx.x] = s_x[0];
}

inline uint32_t move_groups(const PlanDev &p, uint64_t max_entries) {
  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint32_t ppc_log2 = p.chunk_log2 - piece_log2;
  const uint64_t items = max_entries << ppc_log2;
  uint64_t groups = (items + COPY_THREADS / 64 - 1) / (COPY_THREADS / 64);
  if (groups > COPY_MAX_GROUPS) groups = COPY_MAX_GROUPS;
  return (uint32_t)groups;
}

}  // namespace

hipError_t launch_gather(const PlanDev &p, const ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                         const ckpt_counts_t *d_counts, void *d_staging, uint64_t staging_cap,
                         const uint64_t *d_only_if_nonzero, const uint8_t *d_need, hipStream_t s) {
  const uint64_t most = p.nchunks < manifest_cap ? p.nchunks : manifest_cap;
  const uint32_t groups = move_groups(p, most);
  if (groups == 0) return hipSuccess;
  hipLaunchKernelGGL(k_move<true>, dim3(groups), dim3(COPY_THREADS), 0, s, p, d_manifest, most,
                     d_counts, reinterpret_cast<uint8_t *>(d_staging), staging_cap,
                     (unsigned long long *)nullptr,
                     reinterpret_cast<const unsigned long long *>(d_only_if_nonzero), d_need);
  return hipGetLastError();
}

hipError_t launch_scatter(const PlanDev &p, const ckpt_entry_t *d_manifest, uint64_t nentries,
                          const ckpt_counts_t *d_counts, const void *d_staging,
                          uint64_t staging_bytes, uint64_t *d_rejected, hipStream_t s) {
  if (d_rejected)
    hipLaunchKernelGGL(k_zero_u64, dim3(1), dim3(1), 0, s,
                       reinterpret_cast<unsigned long long *>(d_rejected));
  const uint32_t groups = move_groups(p, nentries);
  if (groups == 0) return hipGetLastError();
  hipLaunchKernelGGL(k_move<false>, dim3(groups), dim3(COPY_THREADS), 0, s, p, d_manifest, nentries,
                     d_counts,
                     const_cast<uint8_t *>(reinterpret_cast<const uint8_t *>(d_staging)),
                     staging_bytes, reinterpret_cast<unsigned long long *>(d_rejected),
                     (const unsigned long long *)nullptr, (const uint8_t *)nullptr);
  return hipGetLastError();
}

hipError_t launch_scatter_gated(const PlanDev &p, const ckpt_entry_t *d_manifest, uint64_t nentries,
                                const ckpt_counts_t *d_counts, const void *d_staging,
                                uint64_t staging_bytes, uint64_t *d_rejected,
                                const uint64_t *d_only_if_nonzero, hipStream_t s) {
  const uint64_t most = p.nchunks < nentries ? p.nchunks : nentries;
  const uint32_t groups = move_groups(p, most);
  if (groups == 0) return hipSuccess;
  hipLaunchKernelGGL(k_move<false>, dim3(groups), dim3(COPY_THREADS), 0, s, p, d_manifest, most,
                     d_counts,
                     const_cast<uint8_t *>(reinterpret_cast<const uint8_t *>(d_staging)),
                     staging_bytes, reinterpret_cast<unsigned long long *>(d_rejected),
                     reinterpret_cast<const unsigned long long *>(d_only_if_nonzero),
                     (const uint8_t *)nullptr);
  return hipGetLastError();
}

hipError_t launch_bw_copy(void *d_dst, const void *d_src, uint64_t nbytes, hipStream_t s) {
  const uint64_t n16 = nbytes / 16;
  if (n16 == 0) return hipSuccess;
  uint64_t groups = (n16 + 256 * UNROLL - 1) / (256 * UNROLL);
  if (groups > 65536) groups = 65536;   // short-lived workgroups: the copy sweeps memory front to back
  hipLaunchKernelGGL(k_bw_copy, dim3((uint32_t)groups), dim3(256), 0, s,
                     reinterpret_cast<uint4 *>(d_dst), reinterpret_cast<const uint4 *>(d_src), n16);
  return hipGetLastError();
}

hipError_t launch_bw_streams(void *d_dst, const void *d_src, uint64_t nstreams,
                             uint64_t stream_bytes, uint32_t tile_bytes, uint64_t *d_sink,
                             hipStream_t s) {
  const uint32_t groups = (uint32_t)(nstreams / 16);
  if (groups == 0) return hipSuccess;
  const uint8_t *src = reinterpret_cast<const uint8_t *>(d_src);
  uint8_t *dst = reinterpret_cast<uint8_t *>(d_dst);
  const bool copy = d_dst != nullptr;
  if (tile_bytes == 256 && copy)
    hipLaunchKernelGGL((k_bw_streams<256, true>), dim3(groups), dim3(64), 0, s, src, dst,
                       stream_bytes, d_sink);
  else if (tile_bytes == 256)
    hipLaunchKernelGGL((k_bw_streams<256, false>), dim3(groups), dim3(64), 0, s, src, dst,
                       stream_bytes, d_sink);
  else if (tile_bytes == 1024 && copy)
    hipLaunchKernelGGL((k_bw_streams<1024, true>), dim3(groups), dim3(64), 0, s, src, dst,
                       stream_bytes, d_sink);
  else if (tile_bytes == 1024)
    hipLaunchKernelGGL((k_bw_streams<1024, false>), dim3(groups), dim3(64), 0, s, src, dst,
                       stream_bytes, d_sink);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_alu_xxh64(uint64_t rounds_per_lane, uint64_t *d_sink, hipStream_t s) {
  hipLaunchKernelGGL(k_alu_xxh64, dim3(ALU_PROBE_GROUPS), dim3(256), 0, s, rounds_per_lane, d_sink);
  return hipGetLastError();
}

hipError_t launch_bw_read(const void *d_src, uint64_t nbytes, uint64_t *d_sink, hipStream_t s) {
  const uint64_t n16 = nbytes / 16;
  uint64_t groups = (n16 + 256 * UNROLL - 1) / (256 * UNROLL);
  if (groups > 2048) groups = 2048;
  if (groups == 0) groups = 1;
  hipLaunchKernelGGL(k_bw_read, dim3((uint32_t)groups), dim3(256), 0, s,
                     reinterpret_cast<const uint4 *>(d_src), n16, d_sink);
  return hipGetLastError();
}

}  // namespace ckpt
