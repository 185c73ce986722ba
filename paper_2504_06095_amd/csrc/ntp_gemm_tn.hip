// Ring GEMM instantiations, both operands K-strided: the weight gradients (Y_i^T dZ, dP_i^T X,
// C_i^T dZ, dQKV_i^T X), contraction over tokens, fp32 store or accumulate.
#include "ntp_gemm_launch.h"

namespace ntp_gemm {

NTP_RING_INSTANTIATE_BELOW_256(false, false, ntp::EPI_F32)
NTP_RING_INSTANTIATE_BELOW_256(false, false, ntp::EPI_F32_ACCUM)
NTP_RING_INSTANTIATE_SPLIT(false, false)

template __global__ void gemm_ring_kernel<false, false, ntp::EPI_F32_ACCUM, 256, 256, 2, 4, true>(const GemmArgs);

int launch_ring_split_tn(GemmArgs g, int epilogue, int tile, hipStream_t s) {
  if (epilogue == ntp::EPI_F32) return launch_ring_split_tile<false, false>(g, tile, s);
  if (epilogue == ntp::EPI_F32_ACCUM && tile == 0 && g.k_splits == 1)
    return launch_ring_split_one<false, false, 256, 256, 2, 4, ntp::EPI_F32_ACCUM>(g, s);
  return NTP_ERR_UNSUPPORTED;
}

int launch_ring_tn(GemmArgs g, int epilogue, int tile, hipStream_t s) {
  switch (epilogue) {
    case ntp::EPI_F32: return launch_ring_tile<false, false, ntp::EPI_F32>(g, tile, s);
    case ntp::EPI_F32_ACCUM: return launch_ring_tile<false, false, ntp::EPI_F32_ACCUM>(g, tile, s);
    default: return NTP_ERR_UNSUPPORTED;
  }
}

}  // namespace ntp_gemm
