// Measurement aid (not part of the method): small loops that measure what this GPU sustains on the two
// resources the GEMM kernel leans on, the matrix pipe and LDS reads, each alone and both together in the
// GEMM kernel's own proportions, with no global memory traffic.  The results bound what any schedule of the
// GEMM's inner loop can reach on this device at its power limit; the benchmark prints them beside the kernels.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "ntp_gemm_kernels.h"
#include "ntp_internal.h"

namespace {

using ntp_gemm::bf16x8;
using ntp_gemm::f32x4;
using ntp_gemm::s16x4;

constexpr int kProbeThreads = 512;  // 8 wavefronts, two per SIMD, like the GEMM kernel
constexpr int kAcc = 32;            // independent 16 x 16 accumulator blocks per wavefront (128 registers)

// MFMAS matrix instructions and READS LDS reads per loop turn; TR: the reads are transposing 64-bit reads
// (8 bytes per lane) instead of 128-bit reads (16 bytes per lane).  Operands of the matrix instructions are
// pseudo-random bf16 values (the chip's power draw, and so its clock, depends on the data).
template <int MFMAS, int READS, bool TR>
__global__ __launch_bounds__(kProbeThreads) void probe_kernel(float* out, int turns, uint32_t seed) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[64 * 1024];  // 128 KiB
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // fill LDS with pseudo-random bf16 bit patterns of moderate magnitude
  uint32_t x = seed ^ (uint32_t(blockIdx.x) * 9781u + uint32_t(tid) * 6271u);
  for (int i = tid; i < 64 * 1024; i += kProbeThreads) {
    x = x * 1664525u + 1013904223u;
    lds[i] = uint16_t(0x3c00u | ((x >> 9) & 0x83ffu));  // +-(0.0078 .. 0.0156) * mantissa: finite, mixed signs
  }
  __syncthreads();
  f32x4 acc[kAcc];
#pragma unroll
  for (int i = 0; i < kAcc; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  // each wavefront reads its own 16 KiB region; a 128-bit read takes 64 consecutive 16-byte chunks (no bank
  // conflicts), a transposing read 64 consecutive 8-byte chunks
  const uint16_t* base = lds + wave * 8192;
  bf16x8 fa[8], fb[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    fa[i] = *reinterpret_cast<const bf16x8*>(base + ((i * 64 + lane) * 8) % 8192);
    fb[i] = *reinterpret_cast<const bf16x8*>(base + ((i * 64 + lane) * 8 + 4096) % 8192);
  }
  // The loop's reads are written as inline assembly so that the compiler neither drops nor merges them (one wait
  // per turn bounds what is in flight).  The matrix instructions run on the fragments loaded above.
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  const uint32_t lds_addr = uint32_t(reinterpret_cast<uintptr_t>(base)) + uint32_t(lane) * (TR ? 8u : 16u);
  for (int t = 0; t < turns; ++t) {
    constexpr int STEPS = MFMAS > READS ? MFMAS : (READS > 0 ? READS : 1);
    u32x4 wide;    // (each read's destination is dead at once: the statement itself keeps the read)
    u32x2 narrow;
    const uint32_t addr = lds_addr + uint32_t(t & 7) * 1024u;
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      if (READS > 0 && s * READS / STEPS != (s + 1) * READS / STEPS) {
        const int r = s * READS / STEPS;
        if constexpr (TR) asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(narrow) : "v"(addr), "n"((r & 7) * 512));
        else asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(wide) : "v"(addr), "n"((r & 7) * 1024));
      }
      if (MFMAS > 0 && s * MFMAS / STEPS != (s + 1) * MFMAS / STEPS) {
        const int m = s * MFMAS / STEPS;
        acc[m % kAcc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[m & 7], fa[(m >> 3) & 7], acc[m % kAcc], 0, 0, 0);
      }
    }
    if (READS > 0) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  f32x4 sum = acc[0];
#pragma unroll
  for (int i = 1; i < kAcc; ++i) sum = sum + acc[i];
  float extra = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) extra += float(fa[i][0]) + float(fb[i][1]);
  out[int64_t(blockIdx.x) * kProbeThreads + tid] = sum[0] + sum[1] + sum[2] + sum[3] + extra;
}

// Wavefronts 0-3 (one per SIMD) run 32 matrix instructions per turn when mode & 1; wavefronts 4-7 (one per SIMD) run,
// when mode & 2, the vector arithmetic an attention kernel spends on 16 scores per lane: running maximum, scale and
// subtract, hardware exponential, sum.  With both bits set each SIMD holds one wavefront of each kind; the time
// against the two alone says how much of the vector work hides behind the matrix instructions.
__global__ __launch_bounds__(kProbeThreads) void probe_overlap_kernel(float* out, int turns, int mode) {
  const int tid = threadIdx.x, wave = tid >> 6;
  float r = 0.f;
  if (wave < 4) {
    if (!(mode & 1)) return;
    f32x4 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      a[i] = static_cast<__bf16>(0.01f * float((tid * 7 + i) % 13 - 6));
      b[i] = static_cast<__bf16>(0.02f * float((tid * 5 + i) % 11 - 5));
    }
    for (int t = 0; t < turns; ++t) {
#pragma unroll
      for (int i = 0; i < 32; ++i) acc[i % 16] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i % 16], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) r += acc[i][0] + acc[i][3];
  } else {
    if (!(mode & 2)) return;
    float x[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = 0.001f * float(tid + i);
    float m = 0.f, l = 0.f;
    for (int t = 0; t < turns; ++t) {
      float mx = m;
#pragma unroll
      for (int i = 0; i < 16; i += 2) mx = fmaxf(mx, fmaxf(x[i], x[i + 1]));
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const float p = __builtin_amdgcn_exp2f(fmaf(x[i], 0.125f, -mx));
        s += p;
        x[i] = fmaf(p, 0.5f, 0.001f * float(i));
      }
      l = fmaf(l, 0.5f, s);
      m = mx * 0.999f;
    }
    r = l + m;
  }
  out[int64_t(blockIdx.x) * kProbeThreads + tid] = r;
}

int run_overlap_probe(ntp_handle* h, float* scratch, int mode, int turns, int reps, double* ms_out) {
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return NTP_ERR_LAUNCH;
  if (hipEventCreate(&b) != hipSuccess) {
    (void)hipEventDestroy(a);
    return NTP_ERR_LAUNCH;
  }
  const dim3 grid(uint32_t(h->compute_units)), block(kProbeThreads);
  hipLaunchKernelGGL(probe_overlap_kernel, grid, block, 0, nullptr, scratch, turns / 8, mode);  // warm-up
  (void)hipEventRecord(a, nullptr);
  for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(probe_overlap_kernel, grid, block, 0, nullptr, scratch, turns, mode);
  (void)hipEventRecord(b, nullptr);
  float ms = 0.f;
  const bool ok = hipGetLastError() == hipSuccess && hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(&ms, a, b) == hipSuccess;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  *ms_out = double(ms) / reps;
  return ok ? NTP_OK : NTP_ERR_LAUNCH;
}

template <int MFMAS, int READS, bool TR>
int run_probe(ntp_handle* h, float* scratch, int turns, int reps, double* ms_out) {
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess) return NTP_ERR_LAUNCH;
  if (hipEventCreate(&b) != hipSuccess) {
    (void)hipEventDestroy(a);
    return NTP_ERR_LAUNCH;
  }
  const dim3 grid(uint32_t(h->compute_units)), block(kProbeThreads);
  hipLaunchKernelGGL((probe_kernel<MFMAS, READS, TR>), grid, block, 0, nullptr, scratch, turns / 8, 1u);  // warm-up
  (void)hipEventRecord(a, nullptr);
  for (int r = 0; r < reps; ++r) hipLaunchKernelGGL((probe_kernel<MFMAS, READS, TR>), grid, block, 0, nullptr, scratch, turns, uint32_t(r + 2));
  (void)hipEventRecord(b, nullptr);
  float ms = 0.f;
  const bool ok = hipGetLastError() == hipSuccess && hipEventSynchronize(b) == hipSuccess && hipEventElapsedTime(&ms, a, b) == hipSuccess;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  *ms_out = double(ms) / reps;
  return ok ? NTP_OK : NTP_ERR_LAUNCH;
}

}  // namespace

extern "C" int ntp_probe_rates(ntp_handle_t* h, int32_t which, void* scratch, int64_t scratch_bytes, ntp_probe_result_t* out) {
  if (!h || !out || !scratch) return NTP_ERR_INVALID_ARG;
  if (h->device < 0) return NTP_ERR_NO_DEVICE;
  if (scratch_bytes < int64_t(h->compute_units) * kProbeThreads * 4 || (reinterpret_cast<uintptr_t>(scratch) & 3)) return NTP_ERR_INVALID_ARG;
  float* s = static_cast<float*>(scratch);
  const int turns = 4000, reps = 5;
  int mfmas = 0, reads = 0, read_bytes = 0, st;
  double ms = 0.0;
  if (which >= NTP_PROBE_MFMA_1WAVE && which <= NTP_PROBE_MFMA_AND_SOFTMAX) {
    const int mode = which == NTP_PROBE_MFMA_1WAVE ? 1 : which == NTP_PROBE_SOFTMAX_1WAVE ? 2 : 3;
    st = run_overlap_probe(h, s, mode, 4 * turns, reps, &ms);
    if (st != NTP_OK) return st;
    out->ms = ms;
    out->tflops = mode & 1 ? double(h->compute_units) * 4 * (4.0 * turns) * 32 * 16384.0 / (ms * 1e-3) / 1e12 : 0.0;
    out->lds_gbps_per_cu = 0.0;
    out->mfma_per_turn = mode & 1 ? 32 : 0;
    out->reads_per_turn = 0;
    return NTP_OK;
  }
  switch (which) {
    case NTP_PROBE_MFMA: mfmas = 64; st = run_probe<64, 0, false>(h, s, turns, reps, &ms); break;
    case NTP_PROBE_LDS_B128: reads = 24; read_bytes = 1024; st = run_probe<0, 24, false>(h, s, turns, reps, &ms); break;
    case NTP_PROBE_LDS_TR_B64: reads = 44; read_bytes = 512; st = run_probe<0, 44, true>(h, s, turns, reps, &ms); break;
    case NTP_PROBE_MFMA_LDS_B128: mfmas = 64; reads = 24; read_bytes = 1024; st = run_probe<64, 24, false>(h, s, turns, reps, &ms); break;
    case NTP_PROBE_MFMA_LDS_TR_B64: mfmas = 56; reads = 44; read_bytes = 512; st = run_probe<56, 44, true>(h, s, turns, reps, &ms); break;
    default: return NTP_ERR_INVALID_ARG;
  }
  if (st != NTP_OK) return st;
  const double waves = double(h->compute_units) * (kProbeThreads / 64);
  out->ms = ms;
  out->tflops = mfmas ? waves * turns * mfmas * 16384.0 / (ms * 1e-3) / 1e12 : 0.0;  // 2 x 16 x 16 x 32 flops per instruction
  out->lds_gbps_per_cu = reads ? double(kProbeThreads / 64) * turns * reads * read_bytes / (ms * 1e-3) / 1e9 : 0.0;
  out->mfma_per_turn = mfmas;
  out->reads_per_turn = reads;
  return NTP_OK;
}
