// Ring GEMM instantiations with the ping-pong schedule, A K-contiguous and B K-strided (Y_i B_i, C_i W_O,i and the
// partial input gradients dP_i A_i^T, dQKV_i W_qkv,i^T).
#include "ntp_gemm_launch.h"

namespace ntp_gemm {

NTP_PP_INSTANTIATE(true, false, ntp::EPI_BF16)

int launch_pp_nn(GemmArgs g, int epilogue, int tile, hipStream_t s) {
  if (epilogue != ntp::EPI_BF16) return NTP_ERR_UNSUPPORTED;
  return launch_pp_tile<true, false, ntp::EPI_BF16>(g, tile, s);
}

}  // namespace ntp_gemm
