// Measurement aid: optional per-kernel timing with HIP events on the caller's stream.
// Off by default; when on, every kernel launch made through the handle is bracketed by two
// events and recorded with its algorithmic work, for roofline reports.
#include <hip/hip_runtime.h>

#include <cstring>

#include "ntp_internal.h"

namespace ntp {

void timing_begin(ntp_handle* h, void* stream, const char* name, double flops, double bytes) {
  if (!h->timing_on) return;
  std::lock_guard<std::mutex> lk(h->timing_mu);
  ntp_handle::Pending p{};
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return;
  if (hipEventCreate(&b) != hipSuccess) {
    (void)hipEventDestroy(a);
    return;
  }
  p.start = a;
  p.stop = b;
  std::strncpy(p.rec.name, name, sizeof(p.rec.name) - 1);
  p.rec.flops = flops;
  p.rec.bytes = bytes;
  (void)hipEventRecord(a, static_cast<hipStream_t>(stream));
  h->timing_pending.push_back(p);
}

void timing_end(ntp_handle* h, void* stream) {
  if (!h->timing_on) return;
  std::lock_guard<std::mutex> lk(h->timing_mu);
  if (h->timing_pending.empty()) return;
  (void)hipEventRecord(static_cast<hipEvent_t>(h->timing_pending.back().stop), static_cast<hipStream_t>(stream));
}

}  // namespace ntp

extern "C" int ntp_kernel_timing_enable(ntp_handle_t* h, int32_t on) {
  if (!h) return NTP_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(h->timing_mu);
  h->timing_on = on != 0;
  return NTP_OK;
}

extern "C" int ntp_kernel_timing_read(ntp_handle_t* h, ntp_kernel_time_t* out, int64_t max_records, int64_t* count) {
  if (!h || !count || max_records < 0 || (max_records > 0 && !out)) return NTP_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(h->timing_mu);
  int64_t n = 0;
  for (ntp_handle::Pending& p : h->timing_pending) {
    hipEvent_t a = static_cast<hipEvent_t>(p.start), b = static_cast<hipEvent_t>(p.stop);
    float ms = 0.0f;
    if (hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(&ms, a, b) == hipSuccess) {
      p.rec.ms = ms;
      if (n < max_records) out[n] = p.rec;
      ++n;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
  }
  h->timing_pending.clear();
  *count = n;
  return NTP_OK;
}
