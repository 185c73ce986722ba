// Ring GEMM instantiations with the ping-pong schedule, both operands K-strided: the weight gradients.
#include "ntp_gemm_launch.h"

namespace ntp_gemm {

NTP_PP_INSTANTIATE(false, false, ntp::EPI_F32)
NTP_PP_INSTANTIATE(false, false, ntp::EPI_F32_ACCUM)

int launch_pp_tn(GemmArgs g, int epilogue, int tile, hipStream_t s) {
  switch (epilogue) {
    case ntp::EPI_F32: return launch_pp_tile<false, false, ntp::EPI_F32>(g, tile, s);
    case ntp::EPI_F32_ACCUM: return launch_pp_tile<false, false, ntp::EPI_F32_ACCUM>(g, tile, s);
    default: return NTP_ERR_UNSUPPORTED;
  }
}

}  // namespace ntp_gemm
