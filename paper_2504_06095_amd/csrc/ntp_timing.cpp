// Measurement aid: optional per-kernel timing with HIP events on the caller's stream.
// Off by default; when on, every kernel launch of the library is bracketed by two
// events and recorded with its algorithmic work, for roofline reports.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <vector>

#include "ntp_internal.h"

namespace {
struct Pending {
  hipEvent_t start, stop;
  ntp_kernel_time_t rec;
};
std::mutex g_mu;
bool g_on = false;
std::vector<Pending> g_pending;
}  // namespace

namespace ntp {

bool timing_on() { return g_on; }

void timing_begin(void* stream, const char* name, double flops, double bytes) {
  if (!g_on) return;
  std::lock_guard<std::mutex> lk(g_mu);
  Pending p{};
  if (hipEventCreate(&p.start) != hipSuccess || hipEventCreate(&p.stop) != hipSuccess) return;
  std::strncpy(p.rec.name, name, sizeof(p.rec.name) - 1);
  p.rec.flops = flops;
  p.rec.bytes = bytes;
  (void)hipEventRecord(p.start, static_cast<hipStream_t>(stream));
  g_pending.push_back(p);
}

void timing_end(void* stream) {
  if (!g_on) return;
  std::lock_guard<std::mutex> lk(g_mu);
  if (g_pending.empty()) return;
  (void)hipEventRecord(g_pending.back().stop, static_cast<hipStream_t>(stream));
}

}  // namespace ntp

extern "C" int ntp_kernel_timing_enable(int32_t on) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_on = on != 0;
  return NTP_OK;
}

extern "C" int ntp_kernel_timing_read(ntp_kernel_time_t* out, int64_t max_records, int64_t* count) {
  if (!count || max_records < 0 || (max_records > 0 && !out)) return NTP_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lk(g_mu);
  int64_t n = 0;
  for (Pending& p : g_pending) {
    float ms = 0.0f;
    if (hipEventSynchronize(p.stop) == hipSuccess && hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
      p.rec.ms = ms;
      if (n < max_records) out[n] = p.rec;
      ++n;
    }
    (void)hipEventDestroy(p.start);
    (void)hipEventDestroy(p.stop);
  }
  g_pending.clear();
  *count = n;
  return NTP_OK;
}
