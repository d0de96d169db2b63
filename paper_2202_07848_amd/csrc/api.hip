// C ABI of libckpt.so: argument checks, the plan object, kernel launches.
// Semantics and citations are in include/ckpt.h.
#include <algorithm>
#include <cstring>
#include <new>
#include <numeric>
#include <vector>

#include <atomic>

#include "ckpt_internal.h"

namespace {

thread_local int g_last_hip_error = 0;

int device_error(hipError_t e) {
  g_last_hip_error = (int)e;
  (void)hipGetLastError();   // clear the sticky launch error, it has been recorded
  return CKPT_ERR_DEVICE;
}

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

struct ckpt_plan {
  ckpt::PlanDev dev{};
  uint64_t nbytes = 0;
  uint64_t chunk = 0;
  void *d_tables = nullptr;        // one allocation holding every table
  uint64_t *d_blocksums = nullptr; // scan scratch: 2 x uint64 per SCAN_BLOCK chunks (+2)
  int device = -1;
  // Below this much state the fused pass stays one launch (measured: at 64 MiB two more launches
  // cost 20 us of 58; at 3 GB the split saves 7 %).
  uint64_t split_pass_bytes = 256ull << 20;
};

namespace ckpt {
const PlanDev *plan_dev(const ckpt_plan_t *plan) { return &plan->dev; }
uint64_t *plan_scratch(const ckpt_plan_t *plan) { return plan->d_blocksums; }
void set_last_device_error(hipError_t e) {
  g_last_hip_error = (int)e;
  (void)hipGetLastError();
}
}  // namespace ckpt

namespace {

constexpr uint64_t snapshot_ws_bytes(uint64_t nchunks) {
  // hint offsets, counter block, private copy of the hint, one byte per manifest entry (already
  // staged or not), one uint32 and one byte per group of 16 chunks (full and short chunks are
  // grouped separately, hence at most N/16 + 2 groups)
  return 8 * nchunks + 64 + 2 * ((nchunks + 15) & ~15ull) + 5 * (nchunks / 16 + 2);
}

// ckpt_snapshot_static: the scan scratch (as a plan owns it) followed by the snapshot workspace
// (as ckpt_snapshot takes it), for plans of at most STATIC_MAX_CHUNKS chunks.
constexpr uint64_t STATIC_MAX_CHUNKS = 1ull << 18;
constexpr uint64_t STATIC_SCAN_BYTES =
    (16 * (STATIC_MAX_CHUNKS / ckpt::SCAN_BLOCK + 1) + 255) & ~255ull;
constexpr uint64_t STATIC_BYTES =
    STATIC_SCAN_BYTES + ((snapshot_ws_bytes(STATIC_MAX_CHUNKS) + 255) & ~255ull);
constexpr int STATIC_MAX_DEVICES = 64;

}  // namespace

// Scratch of ckpt_snapshot_static.  In host code this name is only a handle for
// hipGetSymbolAddress; kernels get the device address that call returns.
static __device__ __align__(256) unsigned char scratch[STATIC_BYTES];
static std::atomic<void *> g_static_scratch[STATIC_MAX_DEVICES];

extern "C" {

int ckpt_plan_create(const ckpt_buf_t *bufs, uint64_t nbufs, uint64_t chunk_bytes,
                     ckpt_plan_t **out) {
  if (out == nullptr) return CKPT_ERR_INVALID_ARG;
  *out = nullptr;
  if (bufs == nullptr && nbufs != 0) return CKPT_ERR_INVALID_ARG;
  if (nbufs >= 0xFFFFFFFFull) return CKPT_ERR_INVALID_ARG;
  if (chunk_bytes < 256 || chunk_bytes > (1ull << 30) || (chunk_bytes & (chunk_bytes - 1)) != 0)
    return CKPT_ERR_CHUNK;
  uint32_t chunk_log2 = 0;
  while ((1ull << chunk_log2) < chunk_bytes) ++chunk_log2;

  std::vector<uint64_t> dense_ptr, dense_nbytes, dense_base, list_ptr, list_nbytes, list_base;
  std::vector<uint32_t> dense_orig, group_first;
  std::vector<uint64_t> full_ptr, full_chunk0, full_base, short_ptr, short_chunk;
  std::vector<uint32_t> full_group_first, short_len;
  uint64_t nchunks = 0, total = 0, nfull = 0;
  try {
    list_ptr.reserve(nbufs);
    list_nbytes.reserve(nbufs);
    list_base.reserve(nbufs);
    for (uint64_t i = 0; i < nbufs; ++i) {
      const uint64_t n = bufs[i].nbytes;
      if (n != 0) {
        if (bufs[i].ptr == nullptr) return CKPT_ERR_INVALID_ARG;
        if (!aligned(bufs[i].ptr, 16)) return CKPT_ERR_ALIGNMENT;
        if (total + n < total) return CKPT_ERR_INVALID_ARG;
        if (reinterpret_cast<uintptr_t>(bufs[i].ptr) + n < n) return CKPT_ERR_INVALID_ARG;
      }
      list_ptr.push_back(reinterpret_cast<uint64_t>(n ? bufs[i].ptr : nullptr));
      list_nbytes.push_back(n);
      list_base.push_back(nchunks);
      if (n == 0) continue;
      dense_ptr.push_back(reinterpret_cast<uint64_t>(bufs[i].ptr));
      dense_nbytes.push_back(n);
      dense_base.push_back(nchunks);
      dense_orig.push_back((uint32_t)i);
      const uint64_t whole = n >> chunk_log2, rest = n & (chunk_bytes - 1);
      if (whole != 0) {
        full_ptr.push_back(reinterpret_cast<uint64_t>(bufs[i].ptr));
        full_chunk0.push_back(nchunks);
        full_base.push_back(nfull);
        nfull += whole;
      }
      if (rest != 0) {
        short_ptr.push_back(reinterpret_cast<uint64_t>(bufs[i].ptr) + (whole << chunk_log2));
        short_chunk.push_back(nchunks + whole);
        short_len.push_back((uint32_t)rest);
      }
      nchunks += whole + (rest != 0);
      total += n;
    }
    dense_base.push_back(nchunks);
    full_base.push_back(nfull);
    {
      // short chunks, longest first (stable, so equal lengths keep list order)
      std::vector<uint32_t> order(short_len.size());
      std::iota(order.begin(), order.end(), 0u);
      std::stable_sort(order.begin(), order.end(),
                       [&](uint32_t a, uint32_t b) { return short_len[a] > short_len[b]; });
      std::vector<uint64_t> sp(order.size()), sc(order.size());
      std::vector<uint32_t> sl(order.size());
      for (size_t j = 0; j < order.size(); ++j) {
        sp[j] = short_ptr[order[j]];
        sc[j] = short_chunk[order[j]];
        sl[j] = short_len[order[j]];
      }
      short_ptr.swap(sp);
      short_chunk.swap(sc);
      short_len.swap(sl);
    }
    {
      const uint64_t nfg = (nfull + ckpt::GROUP - 1) / ckpt::GROUP;
      full_group_first.resize(nfg);
      uint32_t frow = 0;
      for (uint64_t g = 0; g < nfg; ++g) {
        const uint64_t f = g * ckpt::GROUP;
        while (f >= full_base[frow + 1]) ++frow;
        full_group_first[g] = frow;
      }
    }
    const uint64_t ngroups = (nchunks + ckpt::GROUP - 1) / ckpt::GROUP;
    if (ngroups > 0x7FFFFFFFull) return CKPT_ERR_INVALID_ARG;
    group_first.resize(ngroups);
    uint32_t row = 0;
    for (uint64_t g = 0; g < ngroups; ++g) {
      const uint64_t k = g * ckpt::GROUP;
      while (k >= dense_base[row + 1]) ++row;
      group_first[g] = row;
    }
    // two buffers of one list may not share a byte: a restore into such a list has no defined
    // result.  Sorted by address, each non-empty buffer must end before the next one starts.
    std::vector<uint32_t> by_addr(dense_ptr.size());
    std::iota(by_addr.begin(), by_addr.end(), 0u);
    std::sort(by_addr.begin(), by_addr.end(),
              [&](uint32_t a, uint32_t b) { return dense_ptr[a] < dense_ptr[b]; });
    for (size_t j = 1; j < by_addr.size(); ++j) {
      const uint32_t a = by_addr[j - 1], b = by_addr[j];
      if (dense_ptr[a] + dense_nbytes[a] > dense_ptr[b]) return CKPT_ERR_INVALID_ARG;
    }
  } catch (const std::bad_alloc &) {
    return CKPT_ERR_NOMEM;
  }

  ckpt_plan *plan = new (std::nothrow) ckpt_plan();
  if (plan == nullptr) return CKPT_ERR_NOMEM;
  plan->nbytes = total;
  plan->chunk = chunk_bytes;
  if (hipGetDevice(&plan->device) != hipSuccess) {
    delete plan;
    return device_error(hipGetLastError());
  }

  // one device allocation, every table 16-byte aligned inside it
  const size_t nb = dense_ptr.size();
  auto up16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
  const size_t o_dptr = 0;
  const size_t o_dnb = o_dptr + up16(8 * nb);
  const size_t o_dbase = o_dnb + up16(8 * nb);
  const size_t o_dorig = o_dbase + up16(8 * (nb + 1));
  const size_t o_gfirst = o_dorig + up16(4 * nb);
  const size_t o_lptr = o_gfirst + up16(4 * group_first.size());
  const size_t o_lnb = o_lptr + up16(8 * (size_t)nbufs);
  const size_t nf = full_ptr.size(), ns = short_ptr.size();
  const size_t o_lbase = o_lnb + up16(8 * (size_t)nbufs);
  const size_t o_fptr = o_lbase + up16(8 * (size_t)nbufs);
  const size_t o_fc0 = o_fptr + up16(8 * nf);
  const size_t o_fbase = o_fc0 + up16(8 * nf);
  const size_t o_fgf = o_fbase + up16(8 * (nf + 1));
  const size_t o_sptr = o_fgf + up16(4 * full_group_first.size());
  const size_t o_sck = o_sptr + up16(8 * ns);
  const size_t o_slen = o_sck + up16(8 * ns);
  const size_t o_spare = (o_slen + up16(4 * ns) + 255) & ~(size_t)255;
  const size_t bytes = o_spare + 256;

  hipError_t e = hipMalloc(&plan->d_tables, bytes);
  if (e != hipSuccess) {
    delete plan;
    (void)hipGetLastError();
    g_last_hip_error = (int)e;
    return e == hipErrorOutOfMemory ? CKPT_ERR_NOMEM : CKPT_ERR_DEVICE;
  }
  const uint64_t nscan = (nchunks + ckpt::SCAN_BLOCK - 1) / ckpt::SCAN_BLOCK;
  e = hipMalloc(reinterpret_cast<void **>(&plan->d_blocksums), 16 * (nscan + 1));
  if (e != hipSuccess) {
    (void)hipFree(plan->d_tables);
    delete plan;
    (void)hipGetLastError();
    g_last_hip_error = (int)e;
    return e == hipErrorOutOfMemory ? CKPT_ERR_NOMEM : CKPT_ERR_DEVICE;
  }

  // one host image of all tables, one copy to the device
  char *base = static_cast<char *>(plan->d_tables);
  std::vector<char> image;
  try {
    image.assign(bytes, 0);          // zeros: the spare block, and the gaps between tables
  } catch (const std::bad_alloc &) {
    (void)hipFree(plan->d_tables);
    (void)hipFree(plan->d_blocksums);
    delete plan;
    return CKPT_ERR_NOMEM;
  }
  auto put = [&](size_t off, const void *src, size_t n) {
    if (n != 0) std::memcpy(image.data() + off, src, n);
  };
  put(o_dptr, dense_ptr.data(), 8 * nb);
  put(o_dnb, dense_nbytes.data(), 8 * nb);
  put(o_dbase, dense_base.data(), 8 * (nb + 1));
  put(o_dorig, dense_orig.data(), 4 * nb);
  put(o_gfirst, group_first.data(), 4 * group_first.size());
  put(o_lptr, list_ptr.data(), 8 * (size_t)nbufs);
  put(o_lnb, list_nbytes.data(), 8 * (size_t)nbufs);
  put(o_lbase, list_base.data(), 8 * (size_t)nbufs);
  put(o_fptr, full_ptr.data(), 8 * nf);
  put(o_fc0, full_chunk0.data(), 8 * nf);
  put(o_fbase, full_base.data(), 8 * (nf + 1));
  put(o_fgf, full_group_first.data(), 4 * full_group_first.size());
  put(o_sptr, short_ptr.data(), 8 * ns);
  put(o_sck, short_chunk.data(), 8 * ns);
  put(o_slen, short_len.data(), 4 * ns);
  e = hipMemcpy(base, image.data(), bytes, hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(plan->d_tables);
    (void)hipFree(plan->d_blocksums);
    delete plan;
    return device_error(e);
  }

  ckpt::PlanDev &d = plan->dev;
  d.dense_ptr = reinterpret_cast<const uint64_t *>(base + o_dptr);
  d.dense_nbytes = reinterpret_cast<const uint64_t *>(base + o_dnb);
  d.dense_base = reinterpret_cast<const uint64_t *>(base + o_dbase);
  d.dense_orig = reinterpret_cast<const uint32_t *>(base + o_dorig);
  d.group_first = reinterpret_cast<const uint32_t *>(base + o_gfirst);
  d.list_ptr = reinterpret_cast<const uint64_t *>(base + o_lptr);
  d.list_nbytes = reinterpret_cast<const uint64_t *>(base + o_lnb);
  d.list_base = reinterpret_cast<const uint64_t *>(base + o_lbase);
  d.spare = reinterpret_cast<const uint8_t *>(base + o_spare);
  d.full_ptr = reinterpret_cast<const uint64_t *>(base + o_fptr);
  d.full_chunk0 = reinterpret_cast<const uint64_t *>(base + o_fc0);
  d.full_base = reinterpret_cast<const uint64_t *>(base + o_fbase);
  d.full_group_first = reinterpret_cast<const uint32_t *>(base + o_fgf);
  d.short_ptr = reinterpret_cast<const uint64_t *>(base + o_sptr);
  d.short_chunk = reinterpret_cast<const uint64_t *>(base + o_sck);
  d.short_len = reinterpret_cast<const uint32_t *>(base + o_slen);
  d.nfull = nfull;
  d.nshort = ns;
  d.nchunks = nchunks;
  d.nbufs = nbufs;
  d.nb = (uint32_t)nb;
  d.chunk_log2 = chunk_log2;
  *out = plan;
  return CKPT_OK;
}

int ckpt_plan_destroy(ckpt_plan_t *plan) {
  if (plan == nullptr) return CKPT_OK;
  hipError_t e1 = hipFree(plan->d_tables);
  hipError_t e2 = hipFree(plan->d_blocksums);
  delete plan;
  if (e1 != hipSuccess) return device_error(e1);
  if (e2 != hipSuccess) return device_error(e2);
  return CKPT_OK;
}

uint64_t ckpt_plan_nchunks(const ckpt_plan_t *plan) { return plan ? plan->dev.nchunks : 0; }
uint64_t ckpt_plan_nbytes(const ckpt_plan_t *plan) { return plan ? plan->nbytes : 0; }
uint64_t ckpt_plan_nbufs(const ckpt_plan_t *plan) { return plan ? plan->dev.nbufs : 0; }
uint64_t ckpt_plan_chunk_bytes(const ckpt_plan_t *plan) { return plan ? plan->chunk : 0; }

uint64_t ckpt_plan_split_threshold(const ckpt_plan_t *plan) {
  return plan ? plan->split_pass_bytes : 0;
}
int ckpt_plan_set_split_threshold(ckpt_plan_t *plan, uint64_t nbytes) {
  if (plan == nullptr) return CKPT_ERR_INVALID_ARG;
  plan->split_pass_bytes = nbytes;
  return CKPT_OK;
}

int ckpt_fingerprint(const ckpt_plan_t *plan, uint64_t *d_digests, void *stream) {
  if (plan == nullptr) return CKPT_ERR_INVALID_ARG;
  if (plan->dev.nchunks == 0) return CKPT_OK;
  if (d_digests == nullptr) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_digests, 8)) return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_fingerprint(plan->dev, d_digests, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_diff(const ckpt_plan_t *plan, const uint64_t *d_digests, const uint64_t *d_ref,
              uint64_t n_ref, uint8_t *d_mask, ckpt_counts_t *d_counts, void *stream) {
  if (plan == nullptr || d_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  const uint64_t n = plan->dev.nchunks;
  if (d_ref != nullptr && n_ref != n) return CKPT_ERR_GEOMETRY;
  if (n != 0 && (d_digests == nullptr || d_mask == nullptr)) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_digests, 8) || !aligned(d_ref, 8) || !aligned(d_counts, 8))
    return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_diff(plan->dev, d_digests, d_ref, d_mask, plan->d_blocksums, d_counts,
                                   static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_upload_owners(const ckpt_plan_t *plan, const uint64_t *d_gathered, uint32_t world,
                       uint32_t rank, uint8_t *d_mask, ckpt_counts_t *d_counts, void *stream) {
  if (plan == nullptr || d_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  if (world == 0 || rank >= world) return CKPT_ERR_INVALID_ARG;
  const uint64_t n = plan->dev.nchunks;
  if (n != 0 && (d_gathered == nullptr || d_mask == nullptr)) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_gathered, 8) || !aligned(d_counts, 8)) return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_upload_owners(plan->dev, d_gathered, world, rank, d_mask,
                                            plan->d_blocksums, d_counts,
                                            static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_compact(const ckpt_plan_t *plan, const uint8_t *d_mask, const uint64_t *d_digests,
                 void *d_staging, uint64_t staging_cap, ckpt_entry_t *d_manifest,
                 uint64_t manifest_cap, ckpt_counts_t *d_counts, void *stream) {
  if (plan == nullptr || d_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  const uint64_t n = plan->dev.nchunks;
  if (n != 0 && (d_mask == nullptr || d_digests == nullptr)) return CKPT_ERR_INVALID_ARG;
  if (staging_cap != 0 && d_staging == nullptr) return CKPT_ERR_INVALID_ARG;
  if (manifest_cap != 0 && d_manifest == nullptr) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_staging, 16) || !aligned(d_manifest, 8) || !aligned(d_digests, 8) ||
      !aligned(d_counts, 8))
    return CKPT_ERR_ALIGNMENT;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = ckpt::launch_compact_scan(plan->dev, d_mask, d_digests, staging_cap, d_manifest,
                                           manifest_cap, plan->d_blocksums, d_counts, nullptr,
                                           nullptr, false, s);
  if (e == hipSuccess)
    e = ckpt::launch_gather(plan->dev, d_manifest, manifest_cap, d_counts, d_staging, staging_cap,
                            nullptr, nullptr, s);
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

uint64_t ckpt_snapshot_workspace_bytes(uint64_t nchunks) { return snapshot_ws_bytes(nchunks); }
uint64_t ckpt_snapshot_stats_offset(uint64_t nchunks) { return 8 * nchunks; }

int ckpt_manifest(const ckpt_plan_t *plan, const uint8_t *d_mask, const uint64_t *d_digests,
                  uint64_t staging_cap, ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                  ckpt_counts_t *d_counts, void *stream) {
  if (plan == nullptr || d_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  const uint64_t n = plan->dev.nchunks;
  if (n != 0 && (d_mask == nullptr || d_digests == nullptr)) return CKPT_ERR_INVALID_ARG;
  if (manifest_cap != 0 && d_manifest == nullptr) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_manifest, 8) || !aligned(d_digests, 8) || !aligned(d_counts, 8))
    return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_compact_scan(plan->dev, d_mask, d_digests, staging_cap, d_manifest,
                                           manifest_cap, plan->d_blocksums, d_counts, nullptr,
                                           nullptr, false, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_exchange(const ckpt_plan_t *plan, const ckpt_entry_t *d_manifest_out,
                  const ckpt_counts_t *d_counts_out, void *d_staging_out, uint64_t staging_out_cap,
                  const ckpt_entry_t *d_manifest_in, const ckpt_counts_t *d_counts_in,
                  const void *d_staging_in, uint64_t staging_in_bytes, uint64_t manifest_cap,
                  uint64_t *d_serial, uint64_t *d_rejected, void *stream) {
  if (plan == nullptr || d_counts_out == nullptr || d_counts_in == nullptr)
    return CKPT_ERR_INVALID_ARG;
  if (manifest_cap != 0 && (d_manifest_out == nullptr || d_manifest_in == nullptr))
    return CKPT_ERR_INVALID_ARG;
  if (staging_out_cap != 0 && d_staging_out == nullptr) return CKPT_ERR_INVALID_ARG;
  if (staging_in_bytes != 0 && d_staging_in == nullptr) return CKPT_ERR_INVALID_ARG;
  if (manifest_cap > (1ull << 40)) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_staging_out, 16) || !aligned(d_staging_in, 16) || !aligned(d_manifest_out, 8) ||
      !aligned(d_manifest_in, 8) || !aligned(d_counts_out, 8) || !aligned(d_counts_in, 8) ||
      !aligned(d_serial, 8) || !aligned(d_rejected, 8))
    return CKPT_ERR_ALIGNMENT;
  // the word that says whether the manifests line up: the spare pair behind the scan scratch
  const uint64_t nscan = (plan->dev.nchunks + ckpt::SCAN_BLOCK - 1) / ckpt::SCAN_BLOCK;
  uint64_t *differs = plan->d_blocksums + 2 * nscan;
  hipError_t e = ckpt::launch_exchange(plan->dev, d_manifest_out, d_counts_out, d_staging_out,
                                       staging_out_cap, d_manifest_in, d_counts_in, d_staging_in,
                                       staging_in_bytes, manifest_cap, differs, d_serial, d_rejected,
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

// Argument checks and launches of ckpt_snapshot; d_blocksums is the scan scratch to use (the
// plan's own, or the library's static block).
static int snapshot_impl(const ckpt_plan_t *plan, const uint64_t *d_ref, uint64_t n_ref,
                         const uint8_t *d_hint, uint64_t *d_digests, uint8_t *d_mask,
                         void *d_staging, uint64_t staging_cap, ckpt_entry_t *d_manifest,
                         uint64_t manifest_cap, ckpt_counts_t *d_counts, uint64_t *d_hint_misses,
                         void *d_workspace, uint64_t workspace_bytes, uint64_t *d_blocksums,
                         void *stream) {
  if (plan == nullptr || d_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  const uint64_t n = plan->dev.nchunks;
  if (d_ref != nullptr && n_ref != n) return CKPT_ERR_GEOMETRY;
  if (n != 0 && (d_digests == nullptr || d_mask == nullptr)) return CKPT_ERR_INVALID_ARG;
  if (staging_cap != 0 && d_staging == nullptr) return CKPT_ERR_INVALID_ARG;
  if (manifest_cap != 0 && d_manifest == nullptr) return CKPT_ERR_INVALID_ARG;
  if (d_hint != nullptr && d_workspace == nullptr) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_staging, 16) || !aligned(d_manifest, 8) || !aligned(d_digests, 8) ||
      !aligned(d_ref, 8) || !aligned(d_counts, 8) || !aligned(d_workspace, 16) ||
      !aligned(d_hint_misses, 8))
    return CKPT_ERR_ALIGNMENT;
  if (d_hint != nullptr && workspace_bytes < snapshot_ws_bytes(n)) return CKPT_ERR_CAPACITY;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const ckpt::PlanDev &p = plan->dev;
  hipError_t e = hipSuccess;
  ckpt::HintState h{};
  if (d_hint != nullptr) {
    // workspace: [hint offsets: N x u64][counter block: 8 x u64][hint copy: N bytes, padded to
    // 16][already-staged flags: N bytes, padded to 16][group list: uint32 per group][group
    // flags: byte per group]
    const uint64_t npad = (n + 15) & ~15ull;
    h.hoff = static_cast<uint64_t *>(d_workspace);
    h.misses = h.hoff + n;
    ckpt_counts_t *tmp = reinterpret_cast<ckpt_counts_t *>(h.misses + 1);
    uint64_t *list_counts = h.misses + 4;
    h.copy = reinterpret_cast<uint8_t *>(h.misses + 8);
    h.need = h.copy + npad;
    uint32_t *list = reinterpret_cast<uint32_t *>(h.need + npad);
    uint8_t *flags = reinterpret_cast<uint8_t *>(list + (n / 16 + 2));
    e = ckpt::launch_hint_offsets(p, d_hint, h, d_blocksums, tmp, manifest_cap, d_counts,
                                  d_hint_misses, s);
    if (e == hipSuccess)
      e = ckpt::launch_fingerprint_staging(p, d_digests, d_ref, d_mask, h.copy, h.hoff, d_staging,
                                           staging_cap, list, flags, list_counts,
                                           plan->nbytes >= plan->split_pass_bytes, s);
  } else {
    e = ckpt::launch_fingerprint_diff(p, d_digests, d_ref, d_mask, d_counts, d_hint_misses, s);
  }
  // Kernels up to SMALL_SCAN_CHUNKS chunks: with a hint 4 (its offsets, the pass, the manifest,
  // the conditional gather; 7 when the pass is split), 3 without.  Above: 8 (11) and 5.
  // Either first kernel has cleared what the one-kernel manifest path adds to.
  const ckpt::HintState *hp = d_hint != nullptr ? &h : nullptr;
  if (e == hipSuccess)
    e = ckpt::launch_compact_scan(p, d_mask, d_digests, staging_cap, d_manifest, manifest_cap,
                                  d_blocksums, d_counts, hp, d_hint_misses, n != 0, s);
  if (e == hipSuccess)
    e = ckpt::launch_gather(p, d_manifest, manifest_cap, d_counts, d_staging, staging_cap,
                            hp ? h.misses : nullptr, hp ? h.need : nullptr, s);
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_snapshot(const ckpt_plan_t *plan, const uint64_t *d_ref, uint64_t n_ref,
                  const uint8_t *d_hint, uint64_t *d_digests, uint8_t *d_mask, void *d_staging,
                  uint64_t staging_cap, ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                  ckpt_counts_t *d_counts, uint64_t *d_hint_misses, void *d_workspace,
                  uint64_t workspace_bytes, void *stream) {
  return snapshot_impl(plan, d_ref, n_ref, d_hint, d_digests, d_mask, d_staging, staging_cap,
                       d_manifest, manifest_cap, d_counts, d_hint_misses, d_workspace,
                       workspace_bytes, plan ? plan->d_blocksums : nullptr, stream);
}

uint64_t ckpt_snapshot_static_max_chunks(void) { return STATIC_MAX_CHUNKS; }

int ckpt_snapshot_static(const ckpt_plan_t *plan, const uint64_t *d_ref, uint64_t n_ref,
                         const uint8_t *d_hint, uint64_t *d_digests, uint8_t *d_mask,
                         void *d_staging, uint64_t staging_cap, ckpt_entry_t *d_manifest,
                         uint64_t manifest_cap, ckpt_counts_t *d_counts, uint64_t *d_hint_misses,
                         void *stream) {
  if (plan == nullptr) return CKPT_ERR_INVALID_ARG;
  if (plan->dev.nchunks > STATIC_MAX_CHUNKS) return CKPT_ERR_CAPACITY;
  int device = -1;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return device_error(e);
  if (device != plan->device || device < 0 || device >= STATIC_MAX_DEVICES)
    return CKPT_ERR_INVALID_ARG;
  // each GPU holds its own copy of the array at its own address: looked up once per device,
  // with that device current (two threads racing here store the same value)
  void *block = g_static_scratch[device].load(std::memory_order_acquire);
  if (block == nullptr) {
    e = hipGetSymbolAddress(&block, HIP_SYMBOL(scratch));
    if (e != hipSuccess || block == nullptr) return device_error(e);
    g_static_scratch[device].store(block, std::memory_order_release);
  }
  uint8_t *base = static_cast<uint8_t *>(block);
  return snapshot_impl(plan, d_ref, n_ref, d_hint, d_digests, d_mask, d_staging, staging_cap,
                       d_manifest, manifest_cap, d_counts, d_hint_misses, base + STATIC_SCAN_BYTES,
                       STATIC_BYTES - STATIC_SCAN_BYTES, reinterpret_cast<uint64_t *>(base), stream);
}

int ckpt_restore(const ckpt_plan_t *dst_plan, const void *d_staging, uint64_t staging_bytes,
                 const ckpt_entry_t *d_manifest, uint64_t nentries, uint64_t *d_rejected,
                 void *stream) {
  if (dst_plan == nullptr) return CKPT_ERR_INVALID_ARG;
  if (nentries != 0 && d_manifest == nullptr) return CKPT_ERR_INVALID_ARG;
  if (staging_bytes != 0 && d_staging == nullptr) return CKPT_ERR_INVALID_ARG;
  if (nentries > (1ull << 40)) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_staging, 16) || !aligned(d_manifest, 8) || !aligned(d_rejected, 8))
    return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_scatter(dst_plan->dev, d_manifest, nentries, nullptr, d_staging,
                                      staging_bytes, d_rejected, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_restore_counted(const ckpt_plan_t *dst_plan, const void *d_staging, uint64_t staging_bytes,
                         const ckpt_entry_t *d_manifest, uint64_t manifest_cap,
                         const ckpt_counts_t *d_counts, uint64_t *d_rejected, void *stream) {
  if (dst_plan == nullptr || d_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  if (manifest_cap != 0 && d_manifest == nullptr) return CKPT_ERR_INVALID_ARG;
  if (staging_bytes != 0 && d_staging == nullptr) return CKPT_ERR_INVALID_ARG;
  if (manifest_cap > (1ull << 40)) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_staging, 16) || !aligned(d_manifest, 8) || !aligned(d_rejected, 8) ||
      !aligned(d_counts, 8))
    return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_scatter(dst_plan->dev, d_manifest, manifest_cap, d_counts, d_staging,
                                      staging_bytes, d_rejected, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

uint64_t ckpt_restore_chain_workspace_bytes(uint64_t nchunks) { return 16 * nchunks + 16; }

}  // extern "C"

namespace {

// Host checks of a chain and its translation into kernel arguments.
int chain_args(const ckpt_link_t *links, uint64_t nlinks, ckpt::ChainArgs *a) {
  if (nlinks > CKPT_CHAIN_MAX || (nlinks != 0 && links == nullptr)) return CKPT_ERR_INVALID_ARG;
  *a = ckpt::ChainArgs{};
  a->nlinks = (uint32_t)nlinks;
  for (uint64_t l = 0; l < nlinks; ++l) {
    const ckpt_link_t &k = links[l];
    if (k.manifest_cap != 0 && k.d_manifest == nullptr) return CKPT_ERR_INVALID_ARG;
    if (k.staging_bytes != 0 && k.d_staging == nullptr) return CKPT_ERR_INVALID_ARG;
    if (k.manifest_cap >= (1ull << 40)) return CKPT_ERR_INVALID_ARG;
    if (!aligned(k.d_staging, 16) || !aligned(k.d_manifest, 8) || !aligned(k.d_counts, 8))
      return CKPT_ERR_ALIGNMENT;
    a->staging[l] = static_cast<const uint8_t *>(k.d_staging);
    a->staging_bytes[l] = k.staging_bytes;
    a->manifest[l] = k.d_manifest;
    a->cap[l] = k.manifest_cap;
    a->counts[l] = k.d_counts;
  }
  return CKPT_OK;
}

}  // namespace

extern "C" {

int ckpt_restore_chain(const ckpt_plan_t *dst_plan, const ckpt_link_t *links, uint64_t nlinks,
                       const uint8_t *d_only, void *d_workspace, uint64_t workspace_bytes,
                       ckpt_chain_stats_t *d_stats, void *stream) {
  if (dst_plan == nullptr || d_workspace == nullptr) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_workspace, 16) || !aligned(d_stats, 8)) return CKPT_ERR_ALIGNMENT;
  ckpt::ChainArgs a;
  const int rc = chain_args(links, nlinks, &a);
  if (rc != CKPT_OK) return rc;
  if (workspace_bytes < ckpt_restore_chain_workspace_bytes(dst_plan->dev.nchunks))
    return CKPT_ERR_CAPACITY;
  hipError_t e = ckpt::launch_restore_chain(dst_plan->dev, a, d_only,
                                            static_cast<uint64_t *>(d_workspace),
                                            reinterpret_cast<uint64_t *>(d_stats),
                                            static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

uint64_t ckpt_merge_chain_workspace_bytes(uint64_t nchunks) {
  return 16 * nchunks + 16 + ((nchunks + 15) & ~15ull);
}

int ckpt_merge_chain(const ckpt_plan_t *plan, const ckpt_link_t *links, uint64_t nlinks,
                     void *d_staging, uint64_t staging_cap, ckpt_entry_t *d_manifest,
                     uint64_t manifest_cap, ckpt_counts_t *d_counts, void *d_workspace,
                     uint64_t workspace_bytes, ckpt_chain_stats_t *d_stats, void *stream) {
  if (plan == nullptr || d_workspace == nullptr || d_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  if (staging_cap != 0 && d_staging == nullptr) return CKPT_ERR_INVALID_ARG;
  if (manifest_cap != 0 && d_manifest == nullptr) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_workspace, 16) || !aligned(d_stats, 8) || !aligned(d_staging, 16) ||
      !aligned(d_manifest, 8) || !aligned(d_counts, 8))
    return CKPT_ERR_ALIGNMENT;
  ckpt::ChainArgs a;
  const int rc = chain_args(links, nlinks, &a);
  if (rc != CKPT_OK) return rc;
  if (workspace_bytes < ckpt_merge_chain_workspace_bytes(plan->dev.nchunks))
    return CKPT_ERR_CAPACITY;
  hipError_t e = ckpt::launch_merge_chain(plan->dev, a, d_staging, staging_cap, d_manifest,
                                          manifest_cap, d_counts,
                                          static_cast<uint64_t *>(d_workspace), plan->d_blocksums,
                                          reinterpret_cast<uint64_t *>(d_stats),
                                          static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

uint64_t ckpt_match_workspace_bytes(uint64_t n_ref, uint64_t nchunks) {
  return ckpt::match_workspace_bytes(n_ref, nchunks);
}

int ckpt_match(const ckpt_plan_t *plan, const uint64_t *d_digests, const uint64_t *d_ref,
               uint64_t n_ref, void *d_workspace, uint64_t workspace_bytes, int64_t *d_src,
               uint8_t *d_mask, ckpt_match_counts_t *d_counts, void *stream) {
  if (plan == nullptr || d_counts == nullptr || d_workspace == nullptr) return CKPT_ERR_INVALID_ARG;
  const uint64_t n = plan->dev.nchunks;
  if (n != 0 && (d_digests == nullptr || d_src == nullptr || d_mask == nullptr))
    return CKPT_ERR_INVALID_ARG;
  if (n_ref != 0 && d_ref == nullptr) return CKPT_ERR_INVALID_ARG;
  if (n_ref > (1ull << 40)) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_digests, 8) || !aligned(d_ref, 8) || !aligned(d_workspace, 16) ||
      !aligned(d_src, 8) || !aligned(d_counts, 8))
    return CKPT_ERR_ALIGNMENT;
  if (workspace_bytes < ckpt::match_workspace_bytes(n_ref, n)) return CKPT_ERR_CAPACITY;
  hipError_t e = ckpt::launch_match(plan->dev, d_digests, d_ref, n_ref, d_workspace, d_src, d_mask,
                                    d_counts, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_apply_matches(const ckpt_plan_t *dst_plan, const ckpt_plan_t *ref_plan,
                       const int64_t *d_src, uint64_t *d_rejected, void *stream) {
  if (dst_plan == nullptr) return CKPT_ERR_INVALID_ARG;
  if (dst_plan->dev.nchunks != 0 && d_src == nullptr) return CKPT_ERR_INVALID_ARG;
  if (ref_plan != nullptr && dst_plan->chunk != ref_plan->chunk) return CKPT_ERR_CHUNK;
  if (!aligned(d_src, 8) || !aligned(d_rejected, 8)) return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_apply_matches(dst_plan->dev, ref_plan ? &ref_plan->dev : nullptr,
                                            d_src, d_rejected, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

uint64_t ckpt_moves_workspace_bytes(uint64_t nchunks) { return ckpt::moves_workspace_bytes(nchunks); }

int ckpt_apply_moves_inplace(const ckpt_plan_t *plan, const int64_t *d_src, void *d_temp,
                             uint64_t temp_cap, void *d_workspace, uint64_t workspace_bytes,
                             ckpt_counts_t *d_counts, uint64_t *d_rejected, void *stream) {
  if (plan == nullptr || d_counts == nullptr || d_workspace == nullptr) return CKPT_ERR_INVALID_ARG;
  const uint64_t n = plan->dev.nchunks;
  if (n != 0 && d_src == nullptr) return CKPT_ERR_INVALID_ARG;
  if (temp_cap != 0 && d_temp == nullptr) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_src, 8) || !aligned(d_temp, 16) || !aligned(d_workspace, 16) ||
      !aligned(d_counts, 8) || !aligned(d_rejected, 8))
    return CKPT_ERR_ALIGNMENT;
  if (workspace_bytes < ckpt::moves_workspace_bytes(n)) return CKPT_ERR_CAPACITY;
  hipError_t e = ckpt::launch_moves_inplace(plan->dev, d_src, d_temp, temp_cap, d_workspace,
                                            plan->d_blocksums, d_counts, d_rejected,
                                            static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_marks_from_buffers(const ckpt_plan_t *plan, const uint8_t *d_buf_flags, uint8_t *d_marks,
                            void *stream) {
  if (plan == nullptr) return CKPT_ERR_INVALID_ARG;
  if (plan->dev.nchunks != 0 && (d_buf_flags == nullptr || d_marks == nullptr))
    return CKPT_ERR_INVALID_ARG;
  hipError_t e = ckpt::launch_marks_from_buffers(plan->dev, d_buf_flags, d_marks,
                                                 static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_mask_andnot(const ckpt_plan_t *plan, const uint8_t *d_mask, const uint8_t *d_without,
                     uint8_t *d_out, void *stream) {
  if (plan == nullptr) return CKPT_ERR_INVALID_ARG;
  if (plan->dev.nchunks != 0 && (d_mask == nullptr || d_without == nullptr || d_out == nullptr))
    return CKPT_ERR_INVALID_ARG;
  hipError_t e = ckpt::launch_mask_andnot(plan->dev.nchunks, d_mask, d_without, d_out,
                                          static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_buffer_verdicts(const ckpt_plan_t *plan, const uint8_t *d_mask, uint8_t *d_buf_dirty,
                         ckpt_buffer_counts_t *d_counts, void *stream) {
  if (plan == nullptr || d_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  if (plan->dev.nchunks != 0 && d_mask == nullptr) return CKPT_ERR_INVALID_ARG;
  if (plan->dev.nbufs != 0 && d_buf_dirty == nullptr) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_counts, 8)) return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_buffer_verdicts(plan->dev, d_mask, d_buf_dirty,
                                              reinterpret_cast<uint64_t *>(d_counts),
                                              static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_validate_mutations(const ckpt_plan_t *plan, const uint64_t *d_before_a,
                            const uint64_t *d_after_a, const uint64_t *d_before_b,
                            const uint64_t *d_after_b, ckpt_validation_t *d_result, void *stream) {
  if (plan == nullptr || d_result == nullptr) return CKPT_ERR_INVALID_ARG;
  const uint64_t n = plan->dev.nchunks;
  if (n != 0 && (d_before_a == nullptr || d_after_a == nullptr || d_before_b == nullptr ||
                 d_after_b == nullptr))
    return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_before_a, 8) || !aligned(d_after_a, 8) || !aligned(d_before_b, 8) ||
      !aligned(d_after_b, 8) || !aligned(d_result, 8))
    return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_validate(n, d_before_a, d_after_a, d_before_b, d_after_b, d_result,
                                       static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_bw_copy(void *d_dst, const void *d_src, uint64_t nbytes, void *stream) {
  if (nbytes == 0) return CKPT_OK;
  if (d_dst == nullptr || d_src == nullptr || (nbytes & 15) != 0) return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_dst, 16) || !aligned(d_src, 16)) return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_bw_copy(d_dst, d_src, nbytes, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_bw_read(const void *d_src, uint64_t nbytes, uint64_t *d_sink, void *stream) {
  if (d_sink == nullptr || (nbytes != 0 && d_src == nullptr) || (nbytes & 15) != 0)
    return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_src, 16) || !aligned(d_sink, 8)) return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_bw_read(d_src, nbytes, d_sink, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

int ckpt_bw_streams(void *d_dst, const void *d_src, uint64_t nstreams, uint64_t stream_bytes,
                    uint64_t tile_bytes, uint64_t *d_sink, void *stream) {
  if (tile_bytes != 256 && tile_bytes != 1024) return CKPT_ERR_INVALID_ARG;
  if (nstreams == 0) return CKPT_OK;
  if (d_src == nullptr || d_sink == nullptr) return CKPT_ERR_INVALID_ARG;
  if ((nstreams & 15) != 0 || stream_bytes % (2 * tile_bytes) != 0 || stream_bytes == 0 ||
      nstreams / 16 > 0x7FFFFFFFull || stream_bytes > (1ull << 40) ||
      nstreams > (~0ull) / stream_bytes)
    return CKPT_ERR_INVALID_ARG;
  if (!aligned(d_dst, 16) || !aligned(d_src, 16) || !aligned(d_sink, 8)) return CKPT_ERR_ALIGNMENT;
  hipError_t e = ckpt::launch_bw_streams(d_dst, d_src, nstreams, stream_bytes,
                                         (uint32_t)tile_bytes, d_sink,
                                         static_cast<hipStream_t>(stream));
  return e == hipSuccess ? CKPT_OK : device_error(e);
}

uint64_t ckpt_alu_xxh64(uint64_t rounds_per_lane, uint64_t *d_sink, void *stream) {
  if (d_sink == nullptr || !aligned(d_sink, 8) || rounds_per_lane == 0 ||
      rounds_per_lane > (1ull << 32))
    return 0;
  rounds_per_lane = (rounds_per_lane + 7) & ~7ull;
  hipError_t e = ckpt::launch_alu_xxh64(rounds_per_lane, d_sink, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) {
    (void)device_error(e);
    return 0;
  }
  return 8ull * rounds_per_lane * 256 * ckpt::ALU_PROBE_GROUPS;
}

const char *ckpt_strerror(int status) {
  switch (status) {
    case CKPT_OK: return "ok";
    case CKPT_ERR_INVALID_ARG: return "invalid argument";
    case CKPT_ERR_ALIGNMENT: return "pointer not aligned as required";
    case CKPT_ERR_CHUNK: return "chunk size must be a power of two in [256, 2^30] (and equal between plans)";
    case CKPT_ERR_GEOMETRY: return "reference digests have a different chunk geometry";
    case CKPT_ERR_CAPACITY: return "staging or manifest capacity exceeded";
    case CKPT_ERR_DEVICE: return "HIP call failed";
    case CKPT_ERR_NOMEM: return "out of memory";
    default: return "unknown status";
  }
}

int ckpt_last_device_error(void) { return g_last_hip_error; }

int ckpt_version(void) { return 1000 * 0 + 2; }

}  // extern "C"
