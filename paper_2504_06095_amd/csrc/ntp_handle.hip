// The library handle: device query, the caller's workspace, tuning overrides; and the static device scratch
// array that serves callers who cannot allocate a workspace.
#include <hip/hip_runtime.h>

#include "ntp_internal.h"

// Device memory that belongs to the library's code object: every GPU the library runs on holds one copy of it
// from the moment the code object is loaded there until the process ends.  In host code this name is only a
// stand-in for the symbol; the memory's device address is looked up once per handle (ntp_create, with the
// handle's device current) and only that address is ever passed to a kernel.
static __device__ __align__(256) unsigned char scratch[NTP_STATIC_SCRATCH_BYTES];

extern "C" int ntp_create(ntp_handle_t** out) {
  if (!out) return NTP_ERR_INVALID_ARG;
  ntp_handle* h = new ntp_handle;
  int dev = -1, cus = 0;
  if (hipGetDevice(&dev) == hipSuccess && dev >= 0 &&
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) {
    h->device = dev;
    h->compute_units = cus;
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      delete h;
      return NTP_ERR_LAUNCH;
    }
    h->static_scratch = ptr;  // this device's copy of the array
  } else {
    (void)hipGetLastError();  // no device visible: a handle for the host-only calls
  }
  *out = h;
  return NTP_OK;
}

extern "C" int ntp_destroy(ntp_handle_t* h) {
  if (!h) return NTP_OK;
  int64_t n = 0;
  (void)ntp_kernel_timing_read(h, nullptr, 0, &n);  // releases the events of launches that were never read
  delete h;
  return NTP_OK;
}

extern "C" int ntp_device_info(const ntp_handle_t* h, int32_t* device, int32_t* compute_units) {
  if (!h) return NTP_ERR_INVALID_ARG;
  if (device) *device = h->device;
  if (compute_units) *compute_units = h->compute_units;
  return NTP_OK;
}

extern "C" int ntp_set_workspace(ntp_handle_t* h, void* workspace, int64_t bytes) {
  if (!h || bytes < 0 || (bytes > 0 && !workspace) || (reinterpret_cast<uintptr_t>(workspace) & 255)) return NTP_ERR_INVALID_ARG;
  h->workspace = bytes > 0 ? workspace : nullptr;
  h->workspace_bytes = bytes > 0 ? bytes : 0;
  return NTP_OK;
}

extern "C" int ntp_set_option(ntp_handle_t* h, int32_t option, int64_t value) {
  if (!h || option < 0 || option >= NTP_OPT_COUNT_) return NTP_ERR_INVALID_ARG;
  switch (option) {
    case NTP_OPT_GEMM_TILE:
      if (value < 0 || value > 10) return NTP_ERR_INVALID_ARG;
      break;
    case NTP_OPT_GEMM_SPLIT:
      if (value < 0 || value > 8) return NTP_ERR_INVALID_ARG;
      break;
    case NTP_OPT_ATTN_PARTS:
      if (value < 0 || value > 16) return NTP_ERR_INVALID_ARG;
      break;
    case NTP_OPT_GEMM_SCHEDULE:
      if (value < 0 || value > 2) return NTP_ERR_INVALID_ARG;
      break;
    case NTP_OPT_ATTN_COPY:
    case NTP_OPT_ATTN_BWD_LAUNCHES:
      if (value < 0 || value > 2) return NTP_ERR_INVALID_ARG;
      break;
    case NTP_OPT_GEMM_WORKGROUPS:
      if (value < 0 || value > 65536) return NTP_ERR_INVALID_ARG;
      break;
    case NTP_OPT_GEMM_NO_RING_TAIL:
    case NTP_OPT_RESHARD_NO_FLAT:
    case NTP_OPT_RESHARD_NO_TABLE:
      if (value != 0 && value != 1) return NTP_ERR_INVALID_ARG;
      break;
    default:  // block sizes in bytes
      if (value < 0 || value > (int64_t(1) << 30)) return NTP_ERR_INVALID_ARG;
  }
  h->opt[option] = value;
  return NTP_OK;
}
