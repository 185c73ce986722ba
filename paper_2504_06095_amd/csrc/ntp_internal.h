// Declarations shared by the translation units of the NTP library (not part of the ABI).
#ifndef NTP_INTERNAL_H_
#define NTP_INTERNAL_H_

#include <stdint.h>

#include <mutex>
#include <vector>

#include "ntp.h"

// The library's per-caller state.  Everything a device call reads besides its arguments lives here: the
// device it was created on and its size, the caller's workspace, the tuning overrides and the timing list.
// The library has no file-scope mutable state; two handles never share anything.
struct ntp_handle {
  int device = -1;          // HIP device ordinal the handle was created on (-1: no device was visible)
  int compute_units = 256;  // of that device (an MI355X has 256; the value used when none was visible)
  void* workspace = nullptr;
  int64_t workspace_bytes = 0;
  void* static_scratch = nullptr;  // device address of the library's static scratch array on `device`
  int64_t opt[NTP_OPT_COUNT_] = {};  // ntp_set_option values; 0 everywhere = the library's own choices
  // measurement aid (ntp_kernel_timing_*)
  struct Pending {
    void* start;
    void* stop;
    ntp_kernel_time_t rec;
  };
  std::mutex timing_mu;
  bool timing_on = false;
  std::vector<Pending> timing_pending;
};

namespace ntp {

// `count` consecutive logical units starting at `first`, stored from local unit `local` of a shard.
struct Run {
  int64_t first, count, local;
};

int check_spec(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp, int64_t* n_units);
int rank_runs(const ntp_tensor_spec_t* spec, int64_t n_units, int32_t tp, int32_t rank,
              std::vector<Run>* runs);
int shard_units(const ntp_tensor_spec_t* spec, int64_t n_units, int32_t tp, int32_t rank,
                int64_t* units);
int build_segments(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp,
                   std::vector<ntp_segment_t>* segs);
// Sub-shards between two layouts given by unit -> rank maps (each rank holds its units in ascending
// unit order), in destination order; also the number of units per rank of either layout.
int build_segments_mapped(int64_t n_units, int32_t src_tp, const int32_t* src_rank_of_unit, int32_t dst_tp,
                          const int32_t* dst_rank_of_unit, std::vector<ntp_segment_t>* segs,
                          std::vector<int64_t>* src_units, std::vector<int64_t>* dst_units);
// Shape, alignment and aliasing checks of the shards of a reshard.
int check_shards(const ntp_tensor_spec_t* spec, const std::vector<int64_t>& src_units,
                 const std::vector<int64_t>& dst_units, const void* const* src_shards, const int64_t* src_ld,
                 void* const* dst_shards, const int64_t* dst_ld);
// Device side of a reshard: checks the shards (shape, alignment, aliasing) and enqueues the copies
// of `segs` (destination order).  src_units / dst_units: partition units held by each rank.
int reshard_launch(ntp_handle* h, const ntp_tensor_spec_t* spec, const std::vector<ntp_segment_t>& segs,
                   const std::vector<int64_t>& src_units, const std::vector<int64_t>& dst_units,
                   const void* const* src_shards, const int64_t* src_ld, void* const* dst_shards,
                   const int64_t* dst_ld, void* stream);

// ---- optional per-kernel timing (measurement aid) ------------------------------
inline bool timing_on(const ntp_handle* h) { return h->timing_on; }
void timing_begin(ntp_handle* h, void* stream, const char* name, double flops, double bytes);
void timing_end(ntp_handle* h, void* stream);

// ---- GEMM family -------------------------------------------------------------
// C[M x N] = op(A) op(B), bf16 operands, fp32 accumulation on the matrix cores.
// An operand is "K-contiguous" when consecutive k sit next to each other in memory:
//   a_kc: A stored [M x K] (row m, ld lda)   else stored [K x M]
//   b_kc: B stored [N x K] (row n, ld ldb)   else stored [K x N]
enum Epilogue : int32_t {
  EPI_BF16 = 0,        // C = bf16(acc)
  EPI_GELU = 1,        // C = bf16(acc), C2 = bf16(gelu(acc))
  EPI_DGELU = 2,       // C = bf16(acc * gelu'(AUX))
  EPI_F32 = 3,         // C = acc            (fp32)
  EPI_F32_ACCUM = 4,   // C += acc           (fp32)
};

struct GemmDesc {
  const void* A;
  int64_t lda;
  const void* B;
  int64_t ldb;
  int64_t M, N, K;
  bool a_kc, b_kc;
  int32_t epilogue;
  void* C;
  int64_t ldc;
  void* C2;  // EPI_GELU second output
  int64_t ldc2;
  const void* AUX;  // EPI_DGELU pre-activation, bf16 [M x N]
  int64_t ldaux;
  int32_t gelu_mode;
  bool zero_pad_n;  // bf16 outputs: also write zeros to columns [N, round_up(N, 8))
  bool pad_n_64;    // ... up to round_up(N, 64) (every leading dimension of an output must reach that far)
  // A is K-contiguous, lda >= round_up(K, 64), and every row of A holds zeros in columns [K, round_up(K, 64)):
  // with B K-strided, the K tail can then go through the ring like a whole K tile
  bool a_k_pad_64;
  // fp32 epilogues: when n_segs > 0 the output rows go to these destinations instead of C
  // (host array; a row that no segment lists is not stored)
  const ntp_row_segment_t* segs;
  int32_t n_segs;
  // when set, the split-K partial sums go here instead of to the handle's workspace
  void* ws_override;
  int64_t ws_override_bytes;
};

// Validates and enqueues one GEMM on `stream`.  Returns an NTP_* status.
int gemm_launch(ntp_handle* h, const GemmDesc& d, void* stream);
// Largest workspace (bytes) a GEMM of this shape could use, i.e. what the split-K choice would take if the
// workspace were unlimited (0: it would not split).  layout as for ntp_gemm_choice; n_store: columns stored.
// The same for the three attention core kernels of a shape (checked like the calls check it).
int attn_core_workspace_wish(const ntp_handle* h, const ntp_attn_core_shape_t* shape, int64_t* bytes);
int64_t gemm_workspace_wish(const ntp_handle* h, int layout, int64_t M, int64_t N, int64_t n_store, int64_t K);

}  // namespace ntp

#endif  // NTP_INTERNAL_H_
