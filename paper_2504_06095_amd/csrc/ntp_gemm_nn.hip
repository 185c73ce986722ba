// Ring GEMM instantiations, A K-contiguous and B K-strided: the row-parallel forward GEMMs
// (Eq. 2 and Eq. 4: Y_i B_i, C_i W_O,i) and the partial input gradients (dP_i A_i^T, dQKV_i W_qkv,i^T),
// whose contraction runs over the ragged shard width.
#include "ntp_gemm_launch.h"

namespace ntp_gemm {

NTP_RING_INSTANTIATE(true, false, ntp::EPI_BF16)
NTP_RING_INSTANTIATE_SPLIT(true, false)

int launch_ring_split_nn(GemmArgs g, int tile, hipStream_t s) { return launch_ring_split_tile<true, false>(g, tile, s); }

int launch_ring_nn(GemmArgs g, int epilogue, int tile, hipStream_t s) {
  switch (epilogue) {
    case ntp::EPI_BF16: return launch_ring_tile<true, false, ntp::EPI_BF16>(g, tile, s);
    default: return NTP_ERR_UNSUPPORTED;
  }
}

}  // namespace ntp_gemm
