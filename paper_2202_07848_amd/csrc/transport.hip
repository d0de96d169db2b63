// Swap-out to / swap-in from host memory (Singularity paper sec. 5.1, 5.2.1:
// the state that is not de-duplicated is copied to host memory at a context
// switch and copied back when the rank gets its next time slice).
//
// The staged bytes never exist in full on the device.  The manifest fixes where
// every dirty chunk lives in staging coordinates; the staging range is cut into
// slices, each slice is gathered into one half of a small device ring and DMA'd
// to pinned host memory on a second stream while the next slice is gathered
// into the other half (and the reverse for swap-in).  Events order the two
// streams; both have the default priority.
//
// Slice kernels work in staging coordinates: a wavefront owns a 64 KiB window
// of the slice, finds the manifest entry that covers the window's first byte by
// binary search (staging is covered by the entries without gaps) and walks
// forward entry by entry, copying each overlap.  A chunk may span many windows
// and many slices; a window may span many small chunks.
#include "ckpt_internal.h"
#include "stream_copy.h"

namespace ckpt {

namespace {

constexpr uint32_t WINDOW = 64 * 1024;

// GATHER: plan buffers -> ring.  !GATHER: ring -> plan buffers.
// The ring holds staging bytes [b0, b1) at ring[0 .. b1-b0).
template <bool GATHER>
__global__ __launch_bounds__(COPY_THREADS) void k_slice(PlanDev p,
                                                        const ckpt_entry_t *__restrict__ manifest,
                                                        uint64_t nentries, uint8_t *__restrict__ ring,
                                                        uint64_t b0, uint64_t b1,
                                                        unsigned long long *rejected) {
  const uint32_t lane = threadIdx.x & 63;
  const uint64_t wave = (uint64_t)blockIdx.x * (COPY_THREADS / 64) +
                        __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t w_lo = b0 + wave * WINDOW;
  if (w_lo >= b1 || nentries == 0) return;
  const uint64_t w_hi = w_lo + WINDOW < b1 ? w_lo + WINDOW : b1;

  // last entry whose stage_off <= w_lo  (entry 0 starts at 0, so one exists)
  uint64_t lo = 0, hi = nentries;
  while (hi - lo > 1) {
    const uint64_t mid = lo + (hi - lo) / 2;
    if (manifest[mid].stage_off <= w_lo) lo = mid; else hi = mid;
  }

  uint64_t pos = w_lo;
  for (uint64_t e = lo; e < nentries && pos < w_hi; ++e) {
    const ckpt_entry_t ent = manifest[e];
    const uint64_t padded = pad16(ent.len);
    // the walk needs gap-free coverage; anything else ends this window
    bool ok = ent.stage_off <= pos && pos < ent.stage_off + padded && (ent.stage_off & 15) == 0 &&
              (ent.buf_off & 15) == 0 && ent.buf < p.nbufs && ent.len <= (1ull << p.chunk_log2);
    if (ok) {
      const uint64_t nb = p.list_nbytes[ent.buf];
      ok = ent.buf_off <= nb && ent.len <= nb - ent.buf_off;
    }
    if (!ok) {
      if (rejected != nullptr && lane == 0) atomicAdd(rejected, 1ull);
      return;
    }
    const uint64_t seg_hi = ent.stage_off + padded < w_hi ? ent.stage_off + padded : w_hi;
    uint8_t *buf = reinterpret_cast<uint8_t *>(p.list_ptr[ent.buf]) + ent.buf_off;
    // address of the chunk's byte 0 inside the ring (may lie before the ring's start;
    // only offsets inside [pos, seg_hi) are touched)
    uint8_t *stg = ring + (ent.stage_off - b0);
    const uint32_t c_lo = (uint32_t)(pos - ent.stage_off), c_hi = (uint32_t)(seg_hi - ent.stage_off);
    if (GATHER)
      move_piece<true>(buf, stg, c_lo, c_hi, ent.len, lane);
    else
      move_piece<false>(stg, buf, c_lo, c_hi, ent.len, lane);
    pos = seg_hi;
  }
}

__global__ void k_zero_one(unsigned long long *p) { *p = 0; }

}  // namespace

hipError_t launch_slice(bool gather, const PlanDev &p, const ckpt_entry_t *d_manifest,
                        uint64_t nentries, void *d_ring, uint64_t b0, uint64_t b1,
                        uint64_t *d_rejected, hipStream_t s) {
  if (b1 <= b0 || nentries == 0) return hipSuccess;
  const uint64_t windows = (b1 - b0 + WINDOW - 1) / WINDOW;
  const uint32_t groups = (uint32_t)((windows + COPY_THREADS / 64 - 1) / (COPY_THREADS / 64));
  unsigned long long *rej = reinterpret_cast<unsigned long long *>(d_rejected);
  if (gather)
    hipLaunchKernelGGL(k_slice<true>, dim3(groups), dim3(COPY_THREADS), 0, s, p, d_manifest, nentries,
                       reinterpret_cast<uint8_t *>(d_ring), b0, b1, rej);
  else
    hipLaunchKernelGGL(k_slice<false>, dim3(groups), dim3(COPY_THREADS), 0, s, p, d_manifest,
                       nentries, reinterpret_cast<uint8_t *>(d_ring), b0, b1, rej);
  return hipGetLastError();
}

hipError_t launch_zero_u64(uint64_t *d_value, hipStream_t s) {
  hipLaunchKernelGGL(k_zero_one, dim3(1), dim3(1), 0, s,
                     reinterpret_cast<unsigned long long *>(d_value));
  return hipGetLastError();
}

}  // namespace ckpt
