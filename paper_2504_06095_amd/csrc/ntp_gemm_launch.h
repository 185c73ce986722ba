// Launch side of the ring GEMM kernel: one translation unit per operand layout instantiates the
// tile variants it needs (they compile in parallel); ntp_gemm.hip picks a variant and calls in.
#ifndef NTP_GEMM_LAUNCH_H_
#define NTP_GEMM_LAUNCH_H_

#include <hip/hip_runtime.h>

#include <type_traits>

#include "ntp_gemm_pp.h"
#include "ntp_gemm_ring.h"
#include "ntp_internal.h"

namespace ntp_gemm {

// Tile shapes of the ring kernel.  Wavefront grids are chosen so that a wavefront's tile is
// 64..128 rows by 48..112 columns (LDS fragment reads per MFMA stay low).
struct TileShape {
  int bm, bn, waves;
};
constexpr TileShape kTileShapes[] = {
    {256, 256, 8}, {256, 224, 8}, {224, 256, 8}, {256, 192, 8}, {192, 256, 8}, {256, 128, 8}, {128, 256, 8}, {128, 128, 4},
    {128, 128, 8},  // the same tile on 8 wavefronts: one workgroup per compute unit, for at most 256 tiles
};
constexpr int kNumTileShapes = int(sizeof(kTileShapes) / sizeof(kTileShapes[0]));

// Enqueue the ring kernel for tile shape `tile` (index into kTileShapes).  A is K-contiguous in
// the "n*" layouts, B in the "*t" layouts.  Returns an NTP_* status; NTP_ERR_UNSUPPORTED if the
// (layout, epilogue) pair has no ring instantiation.
int launch_ring_nt(GemmArgs g, int epilogue, int tile, hipStream_t s);  // A [M x K], B [N x K]
int launch_ring_nn(GemmArgs g, int epilogue, int tile, hipStream_t s);  // A [M x K], B [K x N]
int launch_ring_tn(GemmArgs g, int epilogue, int tile, hipStream_t s);  // A [K x M], B [K x N]
// Non-persistent form (tile shapes with kSplitTile set).  g.k_splits > 1: split-K, g.C is the fp32
// workspace, g.ldc its row length, g.k_chunk / g.split_stride describe the chunks; partial sums only, no
// epilogue.  g.k_splits == 1 (weight-gradient layout only): the whole GEMM with its fp32 epilogue; the
// accumulating epilogue exists for the 256 x 256 tile only.
// The same with the ping-pong schedule of the K loop (tile shapes 0-6, persistent form).
int launch_pp_nt(GemmArgs g, int epilogue, int tile, hipStream_t s);
int launch_pp_nn(GemmArgs g, int epilogue, int tile, hipStream_t s);
int launch_pp_tn(GemmArgs g, int epilogue, int tile, hipStream_t s);
int launch_ring_split_nt(GemmArgs g, int tile, hipStream_t s);
int launch_ring_split_nn(GemmArgs g, int tile, hipStream_t s);
int launch_ring_split_tn(GemmArgs g, int epilogue, int tile, hipStream_t s);
// tile shapes that have a split-K instantiation
constexpr bool kSplitTile[] = {true, true, true, true, true, true, true, false, false};

template <bool AKC, bool BKC, int EPI, int BM_, int BN_, int WGM, int WGN, bool PP = false>
int launch_ring_one(GemmArgs g, hipStream_t s) {
  g.tiles_m = (g.M + BM_ - 1) / BM_;
  g.tiles_n = (g.n_store + BN_ - 1) / BN_;
  if (int64_t(g.tiles_m) * g.tiles_n > 0x7fffffff) return NTP_ERR_UNSUPPORTED;
  // persistent workgroups: one per compute unit (two for the 4-wavefront tile, whose LDS ring is half
  // as large), each walking over its share of the output tiles
  // (a grid of several blocks per workgroup has to be a multiple of 8, the tile walk's XCD stride)
  const uint32_t resident = uint32_t(g.resident > 8 ? g.resident & ~7 : 8) * (WGM * WGN == 4 ? 2 : 1);
  const uint32_t nblk = uint32_t(g.tiles_m) * uint32_t(g.tiles_n);
  const dim3 grid(nblk < resident ? nblk : resident), block(64 * WGM * WGN);
  if constexpr (PP) hipLaunchKernelGGL((gemm_pp_kernel<AKC, BKC, EPI, BM_, BN_, WGM, WGN>), grid, block, 0, s, g);
  else hipLaunchKernelGGL((gemm_ring_kernel<AKC, BKC, EPI, BM_, BN_, WGM, WGN>), grid, block, 0, s, g);
  return hipGetLastError() == hipSuccess ? NTP_OK : NTP_ERR_LAUNCH;
}

template <bool AKC, bool BKC, int BM_, int BN_, int WGM, int WGN, int EPI = ntp::EPI_F32>
int launch_ring_split_one(GemmArgs g, hipStream_t s) {
  g.tiles_m = (g.M + BM_ - 1) / BM_;
  g.tiles_n = (g.n_store + BN_ - 1) / BN_;
  const int64_t per_split = (int64_t(g.tiles_m) * g.tiles_n + 7) / 8 * 8;
  if (g.k_splits < 1 || g.k_chunk < 64 || g.k_chunk % 64 || int64_t(g.k_splits - 1) * g.k_chunk >= g.K ||
      per_split * g.k_splits > 0x7fffffff)
    return NTP_ERR_INVALID_ARG;
  const dim3 grid(uint32_t(per_split * g.k_splits)), block(64 * WGM * WGN);
  hipLaunchKernelGGL((gemm_ring_kernel<AKC, BKC, EPI, BM_, BN_, WGM, WGN, true>), grid, block, 0, s, g);
  return hipGetLastError() == hipSuccess ? NTP_OK : NTP_ERR_LAUNCH;
}

template <bool AKC, bool BKC>
int launch_ring_split_tile(const GemmArgs& g, int tile, hipStream_t s) {
  switch (tile) {
    case 0: return launch_ring_split_one<AKC, BKC, 256, 256, 2, 4>(g, s);
    case 1: return launch_ring_split_one<AKC, BKC, 256, 224, 4, 2>(g, s);
    case 2: return launch_ring_split_one<AKC, BKC, 224, 256, 2, 4>(g, s);
    case 3: return launch_ring_split_one<AKC, BKC, 256, 192, 4, 2>(g, s);
    case 4: return launch_ring_split_one<AKC, BKC, 192, 256, 2, 4>(g, s);
    case 5: return launch_ring_split_one<AKC, BKC, 256, 128, 4, 2>(g, s);
    case 6: return launch_ring_split_one<AKC, BKC, 128, 256, 2, 4>(g, s);
    default: return NTP_ERR_INVALID_ARG;
  }
}

// Ping-pong schedule (8-wavefront tile shapes 0-6).
template <bool AKC, bool BKC, int EPI>
int launch_pp_tile(const GemmArgs& g, int tile, hipStream_t s) {
  switch (tile) {
    case 0: return launch_ring_one<AKC, BKC, EPI, 256, 256, 2, 4, true>(g, s);
    case 1: return launch_ring_one<AKC, BKC, EPI, 256, 224, 4, 2, true>(g, s);
    case 2: return launch_ring_one<AKC, BKC, EPI, 224, 256, 2, 4, true>(g, s);
    case 3: return launch_ring_one<AKC, BKC, EPI, 256, 192, 4, 2, true>(g, s);
    case 4: return launch_ring_one<AKC, BKC, EPI, 192, 256, 2, 4, true>(g, s);
    case 5: return launch_ring_one<AKC, BKC, EPI, 256, 128, 4, 2, true>(g, s);
    case 6: return launch_ring_one<AKC, BKC, EPI, 128, 256, 2, 4, true>(g, s);
    default: return NTP_ERR_INVALID_ARG;
  }
}

template <bool AKC, bool BKC, int EPI>
int launch_ring_tile(const GemmArgs& g, int tile, hipStream_t s) {
  switch (tile) {
    case 0:
      // (the weight-gradient layout has this tile in the non-persistent form only)
      if constexpr (AKC || BKC) return launch_ring_one<AKC, BKC, EPI, 256, 256, 2, 4>(g, s);
      else return NTP_ERR_INVALID_ARG;
    case 1: return launch_ring_one<AKC, BKC, EPI, 256, 224, 4, 2>(g, s);
    case 2: return launch_ring_one<AKC, BKC, EPI, 224, 256, 2, 4>(g, s);
    case 3: return launch_ring_one<AKC, BKC, EPI, 256, 192, 4, 2>(g, s);
    case 4: return launch_ring_one<AKC, BKC, EPI, 192, 256, 2, 4>(g, s);
    case 5: return launch_ring_one<AKC, BKC, EPI, 256, 128, 4, 2>(g, s);
    case 6: return launch_ring_one<AKC, BKC, EPI, 128, 256, 2, 4>(g, s);
    case 7: return launch_ring_one<AKC, BKC, EPI, 128, 128, 2, 2>(g, s);
    case 8: return launch_ring_one<AKC, BKC, EPI, 128, 128, 2, 4>(g, s);
    default: return NTP_ERR_INVALID_ARG;
  }
}

}  // namespace ntp_gemm

// Explicit instantiation of every tile shape for one (layout, epilogue) pair; each translation unit
// lists the pairs it owns (implicit instantiation alone does not emit all host-side launch stubs).
#define NTP_RING_INSTANTIATE(AKC, BKC, EPI)                                                        \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 256, 256, 2, 4>(const GemmArgs);        \
  NTP_RING_INSTANTIATE_BELOW_256(AKC, BKC, EPI)
#define NTP_RING_INSTANTIATE_BELOW_256(AKC, BKC, EPI)                                              \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 256, 224, 4, 2>(const GemmArgs);        \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 224, 256, 2, 4>(const GemmArgs);        \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 256, 192, 4, 2>(const GemmArgs);        \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 192, 256, 2, 4>(const GemmArgs);        \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 256, 128, 4, 2>(const GemmArgs);        \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 128, 256, 2, 4>(const GemmArgs);        \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 128, 128, 2, 2>(const GemmArgs);        \
  template __global__ void gemm_ring_kernel<AKC, BKC, EPI, 128, 128, 2, 4>(const GemmArgs);

#define NTP_PP_INSTANTIATE(AKC, BKC, EPI)                                                   \
  template __global__ void gemm_pp_kernel<AKC, BKC, EPI, 256, 256, 2, 4>(const GemmArgs);   \
  template __global__ void gemm_pp_kernel<AKC, BKC, EPI, 256, 224, 4, 2>(const GemmArgs);   \
  template __global__ void gemm_pp_kernel<AKC, BKC, EPI, 224, 256, 2, 4>(const GemmArgs);   \
  template __global__ void gemm_pp_kernel<AKC, BKC, EPI, 256, 192, 4, 2>(const GemmArgs);   \
  template __global__ void gemm_pp_kernel<AKC, BKC, EPI, 192, 256, 2, 4>(const GemmArgs);   \
  template __global__ void gemm_pp_kernel<AKC, BKC, EPI, 256, 128, 4, 2>(const GemmArgs);   \
  template __global__ void gemm_pp_kernel<AKC, BKC, EPI, 128, 256, 2, 4>(const GemmArgs);

#define NTP_RING_INSTANTIATE_SPLIT(AKC, BKC)                                                                   \
  template __global__ void gemm_ring_kernel<AKC, BKC, ntp::EPI_F32, 256, 256, 2, 4, true>(const GemmArgs);     \
  template __global__ void gemm_ring_kernel<AKC, BKC, ntp::EPI_F32, 256, 224, 4, 2, true>(const GemmArgs);     \
  template __global__ void gemm_ring_kernel<AKC, BKC, ntp::EPI_F32, 224, 256, 2, 4, true>(const GemmArgs);     \
  template __global__ void gemm_ring_kernel<AKC, BKC, ntp::EPI_F32, 256, 192, 4, 2, true>(const GemmArgs);     \
  template __global__ void gemm_ring_kernel<AKC, BKC, ntp::EPI_F32, 192, 256, 2, 4, true>(const GemmArgs);     \
  template __global__ void gemm_ring_kernel<AKC, BKC, ntp::EPI_F32, 256, 128, 4, 2, true>(const GemmArgs);     \
  template __global__ void gemm_ring_kernel<AKC, BKC, ntp::EPI_F32, 128, 256, 2, 4, true>(const GemmArgs);

#endif  // NTP_GEMM_LAUNCH_H_
