// Ring GEMM instantiations, both operands K-contiguous: the column-parallel forward GEMMs
// (Eq. 3 and Eq. 6: X A_i, X W_qkv,i) and the activation gradients of the row-parallel ones
// (dZ B_i^T, dZ W_O,i^T), with their bf16 / GeLU / GeLU' epilogues.
#include "ntp_gemm_launch.h"

namespace ntp_gemm {

NTP_RING_INSTANTIATE(true, true, ntp::EPI_BF16)
NTP_RING_INSTANTIATE(true, true, ntp::EPI_GELU)
NTP_RING_INSTANTIATE(true, true, ntp::EPI_DGELU)
NTP_RING_INSTANTIATE_SPLIT(true, true)

int launch_ring_split_nt(GemmArgs g, int tile, hipStream_t s) { return launch_ring_split_tile<true, true>(g, tile, s); }

int launch_ring_nt(GemmArgs g, int epilogue, int tile, hipStream_t s) {
  switch (epilogue) {
    case ntp::EPI_BF16: return launch_ring_tile<true, true, ntp::EPI_BF16>(g, tile, s);
    case ntp::EPI_GELU: return launch_ring_tile<true, true, ntp::EPI_GELU>(g, tile, s);
    case ntp::EPI_DGELU: return launch_ring_tile<true, true, ntp::EPI_DGELU>(g, tile, s);
    default: return NTP_ERR_UNSUPPORTED;
  }
}

}  // namespace ntp_gemm
