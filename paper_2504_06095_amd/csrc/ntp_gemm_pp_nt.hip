// Ring GEMM instantiations with the ping-pong schedule, both operands K-contiguous (X A_i, X W_qkv,i, dZ B_i^T,
// dZ W_O,i^T and their bf16 / GeLU / GeLU' epilogues).
#include "ntp_gemm_launch.h"

namespace ntp_gemm {

NTP_PP_INSTANTIATE(true, true, ntp::EPI_BF16)
NTP_PP_INSTANTIATE(true, true, ntp::EPI_GELU)
NTP_PP_INSTANTIATE(true, true, ntp::EPI_DGELU)

int launch_pp_nt(GemmArgs g, int epilogue, int tile, hipStream_t s) {
  switch (epilogue) {
    case ntp::EPI_BF16: return launch_pp_tile<true, true, ntp::EPI_BF16>(g, tile, s);
    case ntp::EPI_GELU: return launch_pp_tile<true, true, ntp::EPI_GELU>(g, tile, s);
    case ntp::EPI_DGELU: return launch_pp_tile<true, true, ntp::EPI_DGELU>(g, tile, s);
    default: return NTP_ERR_UNSUPPORTED;
  }
}

}  // namespace ntp_gemm
