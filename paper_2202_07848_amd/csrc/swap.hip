// Host side of ckpt_swap_out / ckpt_swap_in: slices, the two-slot device ring,
// the copy stream and the events that order it against the caller's stream.
// Semantics are in include/ckpt.h.
#include <new>

#include "ckpt_internal.h"

struct ckpt_swapper {
  void *ring[2] = {nullptr, nullptr};
  uint64_t slice = 0;
  hipStream_t copy = nullptr;
  hipEvent_t filled[2] = {nullptr, nullptr};    // ring slot holds a complete slice
  hipEvent_t drained[2] = {nullptr, nullptr};   // ring slot may be overwritten
  ckpt_counts_t *d_counts = nullptr;            // device scratch for the scan's totals
  uint64_t *d_rejected = nullptr;
};

namespace {

int fail(hipError_t e) {
  ckpt::set_last_device_error(e);
  return CKPT_ERR_DEVICE;
}

void destroy(ckpt_swapper *s) {
  for (int i = 0; i < 2; ++i) {
    if (s->ring[i]) (void)hipFree(s->ring[i]);
    if (s->filled[i]) (void)hipEventDestroy(s->filled[i]);
    if (s->drained[i]) (void)hipEventDestroy(s->drained[i]);
  }
  if (s->copy) (void)hipStreamDestroy(s->copy);
  if (s->d_counts) (void)hipFree(s->d_counts);
  if (s->d_rejected) (void)hipFree(s->d_rejected);
  delete s;
}

}  // namespace

extern "C" {

int ckpt_swapper_create(uint64_t slice_bytes, ckpt_swapper_t **out) {
  if (out == nullptr) return CKPT_ERR_INVALID_ARG;
  *out = nullptr;
  if (slice_bytes < 65536 || (slice_bytes & 65535) != 0 || slice_bytes > (1ull << 34))
    return CKPT_ERR_INVALID_ARG;
  ckpt_swapper *s = new (std::nothrow) ckpt_swapper();
  if (s == nullptr) return CKPT_ERR_NOMEM;
  s->slice = slice_bytes;
  hipError_t e = hipSuccess;
  for (int i = 0; i < 2 && e == hipSuccess; ++i) {
    e = hipMalloc(&s->ring[i], slice_bytes);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->filled[i], hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&s->drained[i], hipEventDisableTiming);
  }
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&s->copy, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s->d_counts), sizeof(ckpt_counts_t));
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&s->d_rejected), sizeof(uint64_t));
  if (e != hipSuccess) {
    destroy(s);
    (void)hipGetLastError();
    ckpt::set_last_device_error(e);
    return e == hipErrorOutOfMemory ? CKPT_ERR_NOMEM : CKPT_ERR_DEVICE;
  }
  *out = s;
  return CKPT_OK;
}

int ckpt_swapper_destroy(ckpt_swapper_t *s) {
  if (s != nullptr) destroy(s);
  return CKPT_OK;
}

int ckpt_swap_out(ckpt_swapper_t *sw, const ckpt_plan_t *plan, const uint8_t *d_mask,
                  const uint64_t *d_digests, void *h_staging, uint64_t h_staging_cap,
                  ckpt_entry_t *d_manifest, uint64_t manifest_cap, ckpt_counts_t *h_counts,
                  void *stream) {
  if (sw == nullptr || plan == nullptr || h_counts == nullptr) return CKPT_ERR_INVALID_ARG;
  const ckpt::PlanDev &p = *ckpt::plan_dev(plan);
  if (p.nchunks != 0 && (d_mask == nullptr || d_digests == nullptr)) return CKPT_ERR_INVALID_ARG;
  if (manifest_cap != 0 && d_manifest == nullptr) return CKPT_ERR_INVALID_ARG;
  if (h_staging_cap != 0 && h_staging == nullptr) return CKPT_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(d_manifest) & 7) || (reinterpret_cast<uintptr_t>(d_digests) & 7))
    return CKPT_ERR_ALIGNMENT;
  hipStream_t s = static_cast<hipStream_t>(stream);

  // metadata: offsets and manifest; no staging capacity applies on the device
  hipError_t e = ckpt::launch_compact_scan(p, d_mask, d_digests, ~0ull, d_manifest, manifest_cap,
                                           ckpt::plan_scratch(plan), sw->d_counts, nullptr, nullptr,
                                           false, s);
  if (e == hipSuccess)
    e = hipMemcpyAsync(h_counts, sw->d_counts, sizeof(ckpt_counts_t), hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail(e);
  if (h_counts->overflow != 0 || h_counts->staged_bytes > h_staging_cap) {
    // report what does not fit the same way ckpt_compact counts it, copy nothing
    if (h_counts->overflow == 0) h_counts->overflow = 1;
    return CKPT_ERR_CAPACITY;
  }

  const uint64_t staged = h_counts->staged_bytes, nentries = h_counts->ndirty;
  uint64_t slice_no = 0;
  for (uint64_t b0 = 0; b0 < staged; b0 += sw->slice, ++slice_no) {
    const uint64_t b1 = b0 + sw->slice < staged ? b0 + sw->slice : staged;
    const int r = (int)(slice_no & 1);
    if (slice_no >= 2) e = hipStreamWaitEvent(s, sw->drained[r], 0);
    if (e == hipSuccess)
      e = ckpt::launch_slice(true, p, d_manifest, nentries, sw->ring[r], b0, b1, nullptr, s);
    if (e == hipSuccess) e = hipEventRecord(sw->filled[r], s);
    if (e == hipSuccess) e = hipStreamWaitEvent(sw->copy, sw->filled[r], 0);
    if (e == hipSuccess)
      e = hipMemcpyAsync(static_cast<char *>(h_staging) + b0, sw->ring[r], b1 - b0,
                         hipMemcpyDeviceToHost, sw->copy);
    if (e == hipSuccess) e = hipEventRecord(sw->drained[r], sw->copy);
    if (e != hipSuccess) break;
  }
  hipError_t e2 = hipStreamSynchronize(sw->copy);
  if (e != hipSuccess) return fail(e);
  if (e2 != hipSuccess) return fail(e2);
  return CKPT_OK;
}

int ckpt_swap_in(ckpt_swapper_t *sw, const ckpt_plan_t *dst_plan, const void *h_staging,
                 uint64_t staged_bytes, const ckpt_entry_t *d_manifest, uint64_t nentries,
                 uint64_t *h_rejected, void *stream) {
  if (sw == nullptr || dst_plan == nullptr) return CKPT_ERR_INVALID_ARG;
  if (staged_bytes != 0 && (h_staging == nullptr || d_manifest == nullptr || nentries == 0))
    return CKPT_ERR_INVALID_ARG;
  if ((staged_bytes & 15) != 0 || (reinterpret_cast<uintptr_t>(d_manifest) & 7))
    return CKPT_ERR_ALIGNMENT;
  const ckpt::PlanDev &p = *ckpt::plan_dev(dst_plan);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = ckpt::launch_zero_u64(sw->d_rejected, s);
  uint64_t slice_no = 0;
  for (uint64_t b0 = 0; b0 < staged_bytes && e == hipSuccess; b0 += sw->slice, ++slice_no) {
    const uint64_t b1 = b0 + sw->slice < staged_bytes ? b0 + sw->slice : staged_bytes;
    const int r = (int)(slice_no & 1);
    if (slice_no >= 2) e = hipStreamWaitEvent(sw->copy, sw->drained[r], 0);
    if (e == hipSuccess)
      e = hipMemcpyAsync(sw->ring[r], static_cast<const char *>(h_staging) + b0, b1 - b0,
                         hipMemcpyHostToDevice, sw->copy);
    if (e == hipSuccess) e = hipEventRecord(sw->filled[r], sw->copy);
    if (e == hipSuccess) e = hipStreamWaitEvent(s, sw->filled[r], 0);
    if (e == hipSuccess)
      e = ckpt::launch_slice(false, p, d_manifest, nentries, sw->ring[r], b0, b1, sw->d_rejected, s);
    if (e == hipSuccess) e = hipEventRecord(sw->drained[r], s);
  }
  uint64_t rejected = 0;
  if (e == hipSuccess)
    e = hipMemcpyAsync(&rejected, sw->d_rejected, sizeof(uint64_t), hipMemcpyDeviceToHost, s);
  hipError_t e2 = hipStreamSynchronize(s);
  hipError_t e3 = hipStreamSynchronize(sw->copy);
  if (e != hipSuccess) return fail(e);
  if (e2 != hipSuccess) return fail(e2);
  if (e3 != hipSuccess) return fail(e3);
  if (h_rejected != nullptr) *h_rejected = rejected;
  return CKPT_OK;
}

}  // extern "C"
