// Swap-out of one rank's delta and swap-in of another's as ONE pass over the
// chunks they share (Singularity paper sec. 5.1, 5.2.1: at a context switch the
// outgoing rank's buffers that are not de-duplicated go to host memory and the
// incoming rank's come back, to the same addresses).
//
// Time-sliced data-parallel ranks differ from their common base in the same
// chunks (their gradients and activations; consistent allocation, sec. 5.2.2),
// so the two manifests describe the same places: entry e of both names the same
// buffer range and the same staging offset.  Then a wavefront can take a piece of
// entry e, read the outgoing bytes from the buffer and the incoming bytes from
// the incoming staging area, and write each where the other came from.  With the
// staging areas in pinned host memory the two directions of the host link carry
// data at the same time, which halves the switch against swap-out followed by
// swap-in.
//
// Whether the manifests do line up is decided on the device (k_compare_layouts),
// so the whole switch stays one enqueue: if they do not, the exchange kernel
// returns at once and the ordinary gather and scatter kernels, launched behind
// it, do the work one after the other.
#include "ckpt_internal.h"
#include "stream_copy.h"

namespace ckpt {

namespace {

constexpr int XCHG_UNROLL = 8;   // 2 x 8 x 16 bytes in flight per lane: 8 KiB of each direction per wave

// *differs = number of places where the two manifests disagree (entry count, or an entry's
// buffer, offset, length or staging offset); zero on entry.
__global__ __launch_bounds__(256) void k_compare_layouts(const ckpt_entry_t *__restrict__ a,
                                                         const ckpt_counts_t *__restrict__ na,
                                                         const ckpt_entry_t *__restrict__ b,
                                                         const ckpt_counts_t *__restrict__ nb,
                                                         uint64_t cap, unsigned long long *differs) {
  const uint64_t n_a = na->ndirty, n_b = nb->ndirty;
  uint32_t bad = 0;
  if (blockIdx.x == 0 && threadIdx.x == 0 && (n_a != n_b || n_a > cap)) bad = 1;
  const uint64_t n = n_a < cap ? n_a : cap;
  const uint64_t stride = (uint64_t)gridDim.x * 256;
  for (uint64_t e = (uint64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += stride) {
    const ckpt_entry_t x = a[e], y = b[e];
    bad += x.buf != y.buf || x.len != y.len || x.buf_off != y.buf_off || x.stage_off != y.stage_off;
  }
  for (int o = 32; o > 0; o >>= 1) bad += __shfl_down(bad, o, 64);
  if ((threadIdx.x & 63) == 0 && bad) atomicAdd(differs, (unsigned long long)bad);
}

// Runs only if *differs == 0.  Work item = one piece (min(C, 16 KiB)) of one entry, dealt
// round-robin over a fixed grid like the gather.  Per 16-byte unit: outgoing = buffer bytes
// (zero padded to 16 in staging), incoming = staging bytes (exactly len bytes reach the buffer).
__global__ __launch_bounds__(COPY_THREADS) void k_exchange(
    PlanDev p, const ckpt_entry_t *__restrict__ manifest, uint64_t entry_cap,
    const ckpt_counts_t *__restrict__ count_dev, uint8_t *__restrict__ stage_out, uint64_t out_cap,
    const uint8_t *__restrict__ stage_in, uint64_t in_bytes, const unsigned long long *differs,
    unsigned long long *__restrict__ rejected) {
  if (*differs != 0) return;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t wave_in_group = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t nwaves = (uint64_t)gridDim.x * (COPY_THREADS / 64);
  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint32_t ppc_log2 = p.chunk_log2 - piece_log2;
  const uint64_t n = count_dev->ndirty;
  const uint64_t nitems = (n < entry_cap ? n : entry_cap) << ppc_log2;

  for (uint64_t item = (uint64_t)blockIdx.x * (COPY_THREADS / 64) + wave_in_group; item < nitems;
       item += nwaves) {
    const uint64_t e = item >> ppc_log2;
    const uint32_t piece = (uint32_t)(item & ((1ull << ppc_log2) - 1));
    const ckpt_entry_t ent = manifest[e];
    const uint64_t padded = pad16(ent.len);
    // the entry must fit the plan and both staging areas (written so that no sum can wrap);
    // one that does not is left alone in both directions
    bool ok = ent.buf < p.nbufs && ((ent.buf_off | ent.stage_off) & 15) == 0 &&
              ent.len <= (1ull << p.chunk_log2);
    if (ok) {
      const uint64_t nb = p.list_nbytes[ent.buf];
      ok = ent.buf_off <= nb && ent.len <= nb - ent.buf_off;
    }
    ok = ok && ent.stage_off <= out_cap && padded <= out_cap - ent.stage_off &&
         ent.stage_off <= in_bytes && padded <= in_bytes - ent.stage_off;
    if (!ok) {
      if (rejected != nullptr && piece == 0 && lane == 0) atomicAdd(rejected, 1ull);
      continue;
    }
    uint8_t *buf = reinterpret_cast<uint8_t *>(p.list_ptr[ent.buf]) + ent.buf_off;
    uint8_t *out = stage_out + ent.stage_off;
    const uint8_t *in = stage_in + ent.stage_off;
    const uint32_t len = ent.len;
    const uint32_t lo = piece << piece_log2;
    uint32_t hi = lo + (1u << piece_log2);
    if (hi > padded) hi = (uint32_t)padded;

    for (uint32_t base = lo + lane * 16; base < hi; base += 64 * 16 * XCHG_UNROLL) {
      uint4 going[XCHG_UNROLL], coming[XCHG_UNROLL];
#pragma unroll
      for (int u = 0; u < XCHG_UNROLL; ++u) {
        const uint32_t o = base + u * 64 * 16;
        if (o >= hi) continue;                   // every unit below hi starts below len
        if (o + 16 <= len) {
          going[u] = stream_load16(buf + o);
          coming[u] = stream_load16(in + o);
        } else {
          going[u] = load_partial16(buf + o, len - o);     // zero padded
          coming[u] = stream_load16(in + o);               // staging holds the padded unit
        }
      }
#pragma unroll
      for (int u = 0; u < XCHG_UNROLL; ++u) {
        const uint32_t o = base + u * 64 * 16;
        if (o >= hi) continue;
        stream_store16(out + o, going[u]);
        if (o + 16 <= len)
          stream_store16(buf + o, coming[u]);
        else
          store_partial16(buf + o, coming[u], len - o);
      }
    }
  }
}

__global__ void k_clear_words(unsigned long long *a, unsigned long long *b) {
  *a = 0;
  if (b != nullptr) *b = 0;
}

__global__ void k_publish_word(const unsigned long long *src, unsigned long long *dst) { *dst = *src; }

}  // namespace

hipError_t launch_exchange(const PlanDev &p, const ckpt_entry_t *d_manifest_out,
                           const ckpt_counts_t *d_counts_out, void *d_stage_out, uint64_t out_cap,
                           const ckpt_entry_t *d_manifest_in, const ckpt_counts_t *d_counts_in,
                           const void *d_stage_in, uint64_t in_bytes, uint64_t manifest_cap,
                           uint64_t *d_differs, uint64_t *d_serial, uint64_t *d_rejected,
                           hipStream_t s) {
  unsigned long long *differs = reinterpret_cast<unsigned long long *>(d_differs);
  unsigned long long *rej = reinterpret_cast<unsigned long long *>(d_rejected);
  hipLaunchKernelGGL(k_clear_words, dim3(1), dim3(1), 0, s, differs, rej);
  const uint64_t most = p.nchunks < manifest_cap ? p.nchunks : manifest_cap;
  uint64_t cgroups = (most + 255) / 256;
  if (cgroups > 1024) cgroups = 1024;
  if (cgroups == 0) cgroups = 1;
  hipLaunchKernelGGL(k_compare_layouts, dim3((uint32_t)cgroups), dim3(256), 0, s, d_manifest_out,
                     d_counts_out, d_manifest_in, d_counts_in, most, differs);
  if (d_serial != nullptr)
    hipLaunchKernelGGL(k_publish_word, dim3(1), dim3(1), 0, s, differs,
                       reinterpret_cast<unsigned long long *>(d_serial));
  const uint32_t piece_log2 = p.chunk_log2 < COPY_PIECE_LOG2 ? p.chunk_log2 : COPY_PIECE_LOG2;
  const uint64_t items = most << (p.chunk_log2 - piece_log2);
  uint64_t groups = (items + COPY_THREADS / 64 - 1) / (COPY_THREADS / 64);
  if (groups > COPY_MAX_GROUPS) groups = COPY_MAX_GROUPS;
  if (groups != 0)
    hipLaunchKernelGGL(k_exchange, dim3((uint32_t)groups), dim3(COPY_THREADS), 0, s, p,
                       d_manifest_out, most, d_counts_out, reinterpret_cast<uint8_t *>(d_stage_out),
                       out_cap, reinterpret_cast<const uint8_t *>(d_stage_in), in_bytes,
                       (const unsigned long long *)differs, rej);
  // the manifests do not line up: swap-out, then swap-in, each skipped when *differs == 0
  hipError_t e = hipGetLastError();
  if (e == hipSuccess)
    e = launch_gather(p, d_manifest_out, manifest_cap, d_counts_out, d_stage_out, out_cap, d_differs,
                      nullptr, s);
  if (e == hipSuccess)
    e = launch_scatter_gated(p, d_manifest_in, manifest_cap, d_counts_in, d_stage_in, in_bytes,
                             d_rejected, d_differs, s);
  return e;
}

}  // namespace ckpt
