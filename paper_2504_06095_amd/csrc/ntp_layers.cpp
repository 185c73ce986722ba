// ABI entry points of the shard layers: argument checks and the sequence of GEMMs.
// Every step runs in the GEMM kernels; nothing is computed on the host.
#include <algorithm>

#include "ntp_internal.h"

using ntp::GemmDesc;

namespace {

GemmDesc gemm(const void* A, int64_t lda, bool a_kc, const void* B, int64_t ldb, bool b_kc, int64_t M,
              int64_t N, int64_t K, int32_t epilogue, void* C, int64_t ldc) {
  GemmDesc d{};
  d.A = A;
  d.lda = lda;
  d.a_kc = a_kc;
  d.B = B;
  d.ldb = ldb;
  d.b_kc = b_kc;
  d.M = M;
  d.N = N;
  d.K = K;
  d.epilogue = epilogue;
  d.C = C;
  d.ldc = ldc;
  return d;
}

bool bad_mlp_shape(const ntp_mlp_shape_t* s) {
  return !s || s->M < 0 || s->H < 0 || s->n_r < 0 ||
         (s->gelu_mode != NTP_GELU_ERF && s->gelu_mode != NTP_GELU_TANH);
}

}  // namespace

// Eq. 3 then Eq. 2 for this rank's shard.
extern "C" int ntp_mlp_shard_fwd(ntp_handle_t* h, const ntp_mlp_shape_t* s, const void* X, int64_t ldx, const void* A_t,
                                 int64_t lda, const void* B, int64_t ldb, void* P, int64_t ldp, void* Y,
                                 int64_t ldy, void* Zpart, int64_t ldz, void* stream) {
  if (!h || bad_mlp_shape(s)) return NTP_ERR_INVALID_ARG;
  if (s->H % 8) return NTP_ERR_ALIGNMENT;
  if (s->M == 0 || s->H == 0) return NTP_OK;
  if (!X || !Zpart || (s->n_r > 0 && (!A_t || !B || !P || !Y))) return NTP_ERR_INVALID_ARG;
  int st = NTP_OK;
  // rows long enough: the pad columns are zeroed up to the next multiple of 64 (a whole K tile of the second GEMM)
  const int64_t n64 = (s->n_r + 63) / 64 * 64;
  const bool pad64 = s->n_r > 0 && ldp >= n64 && ldy >= n64;
  if (s->n_r > 0) {
    // P = X A_i (A_t holds A_i's columns as rows), Y = GeLU(P); pad columns zeroed
    GemmDesc d = gemm(X, ldx, true, A_t, lda, true, s->M, s->n_r, s->H, ntp::EPI_GELU, P, ldp);
    d.C2 = Y;
    d.ldc2 = ldy;
    d.gelu_mode = s->gelu_mode;
    d.zero_pad_n = true;
    d.pad_n_64 = pad64;
    if ((st = ntp::gemm_launch(h, d, stream)) != NTP_OK) return st;
  }
  // Zpart = Y B_i, contraction over the ragged shard width
  GemmDesc d2 = gemm(Y, ldy, true, B, ldb, false, s->M, s->H, s->n_r, ntp::EPI_BF16, Zpart, ldz);
  d2.a_k_pad_64 = pad64;  // Y's pad columns were zeroed just above
  return ntp::gemm_launch(h, d2, stream);
}

namespace {

// Backward of the MLP shard; the two weight gradients go to row segments.
int mlp_bwd(ntp_handle_t* h, const ntp_mlp_shape_t* s, const void* dZ, int64_t lddz, const void* X, int64_t ldx, const void* A_t,
            int64_t lda, const void* B, int64_t ldb, const void* P, int64_t ldp, const void* Y, int64_t ldy, void* dP,
            int64_t lddp, void* dXpart, int64_t lddx, const ntp_row_segment_t* dA_segs, int32_t n_dA,
            const ntp_row_segment_t* dB_segs, int32_t n_dB, int32_t accumulate, void* stream) {
  if (!h || bad_mlp_shape(s)) return NTP_ERR_INVALID_ARG;
  if (s->H % 8) return NTP_ERR_ALIGNMENT;
  if (s->H == 0) return NTP_OK;
  if (s->n_r > 0 && (!A_t || !B || !dA_segs || !dB_segs || n_dA < 1 || n_dB < 1)) return NTP_ERR_INVALID_ARG;
  if (s->M > 0 && (!dZ || !X || !dXpart || (s->n_r > 0 && (!P || !Y || !dP)))) return NTP_ERR_INVALID_ARG;
  const int32_t wepi = accumulate ? ntp::EPI_F32_ACCUM : ntp::EPI_F32;
  int st = NTP_OK;
  const int64_t n64 = (s->n_r + 63) / 64 * 64;
  const bool pad64 = s->n_r > 0 && s->M > 0 && lddp >= n64 && ldp >= n64;  // as in the forward call, for dP
  if (s->n_r > 0 && s->M > 0) {
    // dP = (dZ B_i^T) .* GeLU'(P)
    GemmDesc d = gemm(dZ, lddz, true, B, ldb, true, s->M, s->n_r, s->H, ntp::EPI_DGELU, dP, lddp);
    d.AUX = P;
    d.ldaux = ldp;
    d.gelu_mode = s->gelu_mode;
    d.zero_pad_n = true;
    d.pad_n_64 = pad64;
    if ((st = ntp::gemm_launch(h, d, stream)) != NTP_OK) return st;
  }
  if (s->n_r > 0) {
    // dB = Y^T dZ and dA_t = dP^T X: contraction over tokens, both operands token-major
    GemmDesc db = gemm(Y, ldy, false, dZ, lddz, false, s->n_r, s->H, s->M, wepi, nullptr, 0);
    db.segs = dB_segs;
    db.n_segs = n_dB;
    if ((st = ntp::gemm_launch(h, db, stream)) != NTP_OK) return st;
    GemmDesc da = gemm(dP, lddp, false, X, ldx, false, s->n_r, s->H, s->M, wepi, nullptr, 0);
    da.segs = dA_segs;
    da.n_segs = n_dA;
    if ((st = ntp::gemm_launch(h, da, stream)) != NTP_OK) return st;
  }
  if (s->M == 0) return NTP_OK;
  // dXpart = dP A_i^T, contraction over the ragged shard width
  GemmDesc dx = gemm(dP, lddp, true, A_t, lda, false, s->M, s->H, s->n_r, ntp::EPI_BF16, dXpart, lddx);
  dx.a_k_pad_64 = pad64;  // dP's pad columns were zeroed above
  return ntp::gemm_launch(h, dx, stream);
}

}  // namespace

extern "C" int ntp_mlp_shard_bwd(ntp_handle_t* h, const ntp_mlp_shape_t* s, const void* dZ, int64_t lddz, const void* X,
                                 int64_t ldx, const void* A_t, int64_t lda, const void* B, int64_t ldb,
                                 const void* P, int64_t ldp, const void* Y, int64_t ldy, void* dP,
                                 int64_t lddp, void* dXpart, int64_t lddx, float* dA_t, int64_t ldda,
                                 float* dB, int64_t lddb, int32_t accumulate, void* stream) {
  if (!h || bad_mlp_shape(s)) return NTP_ERR_INVALID_ARG;
  if (s->n_r > 0 && s->H > 0 && (!dA_t || !dB)) return NTP_ERR_INVALID_ARG;
  // the gradients as one block of rows each
  const ntp_row_segment_t a{0, s->n_r, dA_t, ldda}, b{0, s->n_r, dB, lddb};
  return mlp_bwd(h, s, dZ, lddz, X, ldx, A_t, lda, B, ldb, P, ldp, Y, ldy, dP, lddp, dXpart, lddx, &a, 1, &b, 1, accumulate,
                 stream);
}

extern "C" int ntp_mlp_shard_bwd_resharded(ntp_handle_t* h, const ntp_mlp_shape_t* s, const void* dZ, int64_t lddz, const void* X,
                                           int64_t ldx, const void* A_t, int64_t lda, const void* B, int64_t ldb,
                                           const void* P, int64_t ldp, const void* Y, int64_t ldy, void* dP,
                                           int64_t lddp, void* dXpart, int64_t lddx,
                                           const ntp_row_segment_t* dA_segs, int32_t n_dA_segs,
                                           const ntp_row_segment_t* dB_segs, int32_t n_dB_segs, int32_t accumulate,
                                           void* stream) {
  return mlp_bwd(h, s, dZ, lddz, X, ldx, A_t, lda, B, ldb, P, ldp, Y, ldy, dP, lddp, dXpart, lddx, dA_segs, n_dA_segs, dB_segs,
                 n_dB_segs, accumulate, stream);
}

namespace {
bool bad_attn_shape(const ntp_attn_shape_t* s) {
  return !s || s->M < 0 || s->H < 0 || s->w_qkv < 0 || s->w_o < 0;
}
}  // namespace

namespace {

// Eq. 6 (column-parallel QKV) and Eq. 4 (row-parallel output projection).  ws != NULL: split-K partial sums
// go there instead of to the handle's workspace.
int attn_fwd(ntp_handle_t* h, const ntp_attn_shape_t* s, const void* X, int64_t ldx, const void* Wqkv, int64_t ldwqkv,
             void* QKV, int64_t ldqkv, const void* C, int64_t ldc, const void* Wo, int64_t ldwo, void* Zpart, int64_t ldz,
             void* ws, int64_t ws_bytes, void* stream) {
  if (!h || bad_attn_shape(s)) return NTP_ERR_INVALID_ARG;
  if (s->H % 8 || s->w_qkv % 8 || s->w_o % 8) return NTP_ERR_ALIGNMENT;
  int st = NTP_OK;
  if (QKV) {
    if (s->M > 0 && s->w_qkv > 0 && s->H > 0 && (!X || !Wqkv)) return NTP_ERR_INVALID_ARG;
    GemmDesc d = gemm(X, ldx, true, Wqkv, ldwqkv, true, s->M, s->w_qkv, s->H, ntp::EPI_BF16, QKV, ldqkv);
    d.ws_override = ws;
    d.ws_override_bytes = ws_bytes;
    if ((st = ntp::gemm_launch(h, d, stream)) != NTP_OK) return st;
  }
  if (Zpart) {
    if (s->M > 0 && s->w_o > 0 && s->H > 0 && (!C || !Wo)) return NTP_ERR_INVALID_ARG;
    GemmDesc d = gemm(C, ldc, true, Wo, ldwo, false, s->M, s->H, s->w_o, ntp::EPI_BF16, Zpart, ldz);
    d.ws_override = ws;
    d.ws_override_bytes = ws_bytes;
    if ((st = ntp::gemm_launch(h, d, stream)) != NTP_OK) return st;
  }
  return NTP_OK;
}

}  // namespace

extern "C" int ntp_attn_proj_shard_fwd(ntp_handle_t* h, const ntp_attn_shape_t* s, const void* X, int64_t ldx,
                                       const void* Wqkv, int64_t ldwqkv, void* QKV, int64_t ldqkv,
                                       const void* C, int64_t ldc, const void* Wo, int64_t ldwo,
                                       void* Zpart, int64_t ldz, void* stream) {
  return attn_fwd(h, s, X, ldx, Wqkv, ldwqkv, QKV, ldqkv, C, ldc, Wo, ldwo, Zpart, ldz, nullptr, 0, stream);
}

// The same call for callers that cannot allocate: the split-K partial sums go to the library's static device
// array (this device's copy, whose address ntp_create looked up) instead of a caller-provided workspace.
extern "C" int ntp_attn_proj_shard_fwd_static(ntp_handle_t* h, const ntp_attn_shape_t* s, const void* X, int64_t ldx,
                                              const void* Wqkv, int64_t ldwqkv, void* QKV, int64_t ldqkv,
                                              const void* C, int64_t ldc, const void* Wo, int64_t ldwo,
                                              void* Zpart, int64_t ldz, void* stream) {
  if (!h || bad_attn_shape(s)) return NTP_ERR_INVALID_ARG;
  if (s->H % 8 || s->w_qkv % 8 || s->w_o % 8) return NTP_ERR_ALIGNMENT;
  if (h->device < 0 || !h->static_scratch) return NTP_ERR_NO_DEVICE;
  // a shape whose launches would want more partial-sum room than the array has is refused, not run unsplit
  int64_t wish = 0;
  if (QKV) wish = std::max(wish, ntp::gemm_workspace_wish(h, 0, s->M, s->w_qkv, s->w_qkv, s->H));
  if (Zpart) wish = std::max(wish, ntp::gemm_workspace_wish(h, 1, s->M, s->H, s->H, s->w_o));
  if (wish > int64_t(NTP_STATIC_SCRATCH_BYTES)) return NTP_ERR_SCRATCH_TOO_SMALL;
  return attn_fwd(h, s, X, ldx, Wqkv, ldwqkv, QKV, ldqkv, C, ldc, Wo, ldwo, Zpart, ldz, h->static_scratch,
                  int64_t(NTP_STATIC_SCRATCH_BYTES), stream);
}

namespace {

// Backward of the two projections; the two weight gradients go to row segments.
int attn_bwd(ntp_handle_t* h, const ntp_attn_shape_t* s, const void* dZ, int64_t lddz, const void* dQKV, int64_t lddqkv, const void* X,
             int64_t ldx, const void* C, int64_t ldc, const void* Wqkv, int64_t ldwqkv, const void* Wo, int64_t ldwo,
             void* dC, int64_t lddc, void* dXpart, int64_t lddx, const ntp_row_segment_t* dWqkv_segs, int32_t n_dWqkv,
             const ntp_row_segment_t* dWo_segs, int32_t n_dWo, int32_t accumulate, void* stream) {
  if (!h || bad_attn_shape(s)) return NTP_ERR_INVALID_ARG;
  if (s->H % 8 || s->w_qkv % 8 || s->w_o % 8) return NTP_ERR_ALIGNMENT;
  const int32_t wepi = accumulate ? ntp::EPI_F32_ACCUM : ntp::EPI_F32;
  int st = NTP_OK;
  if (dZ) {
    if (!Wo || !C || !dC || !dWo_segs || n_dWo < 1) return NTP_ERR_INVALID_ARG;
    GemmDesc d = gemm(dZ, lddz, true, Wo, ldwo, true, s->M, s->w_o, s->H, ntp::EPI_BF16, dC, lddc);
    if ((st = ntp::gemm_launch(h, d, stream)) != NTP_OK) return st;
    GemmDesc w = gemm(C, ldc, false, dZ, lddz, false, s->w_o, s->H, s->M, wepi, nullptr, 0);
    w.segs = dWo_segs;
    w.n_segs = n_dWo;
    if ((st = ntp::gemm_launch(h, w, stream)) != NTP_OK) return st;
  }
  if (dQKV) {
    if (!Wqkv || !X || !dXpart || !dWqkv_segs || n_dWqkv < 1) return NTP_ERR_INVALID_ARG;
    GemmDesc d = gemm(dQKV, lddqkv, true, Wqkv, ldwqkv, false, s->M, s->H, s->w_qkv, ntp::EPI_BF16, dXpart, lddx);
    if ((st = ntp::gemm_launch(h, d, stream)) != NTP_OK) return st;
    GemmDesc w = gemm(dQKV, lddqkv, false, X, ldx, false, s->w_qkv, s->H, s->M, wepi, nullptr, 0);
    w.segs = dWqkv_segs;
    w.n_segs = n_dWqkv;
    if ((st = ntp::gemm_launch(h, w, stream)) != NTP_OK) return st;
  }
  return NTP_OK;
}

}  // namespace

extern "C" int ntp_attn_proj_shard_bwd(ntp_handle_t* h, const ntp_attn_shape_t* s, const void* dZ, int64_t lddz,
                                       const void* dQKV, int64_t lddqkv, const void* X, int64_t ldx,
                                       const void* C, int64_t ldc, const void* Wqkv, int64_t ldwqkv,
                                       const void* Wo, int64_t ldwo, void* dC, int64_t lddc, void* dXpart,
                                       int64_t lddx, float* dWqkv, int64_t lddwqkv, float* dWo,
                                       int64_t lddwo, int32_t accumulate, void* stream) {
  if (!h || bad_attn_shape(s)) return NTP_ERR_INVALID_ARG;
  if ((dZ && !dWo) || (dQKV && !dWqkv)) return NTP_ERR_INVALID_ARG;
  // the gradients as one block of rows each
  const ntp_row_segment_t q{0, s->w_qkv, dWqkv, lddwqkv}, o{0, s->w_o, dWo, lddwo};
  return attn_bwd(h, s, dZ, lddz, dQKV, lddqkv, X, ldx, C, ldc, Wqkv, ldwqkv, Wo, ldwo, dC, lddc, dXpart, lddx, &q, 1, &o, 1,
                  accumulate, stream);
}

extern "C" int ntp_attn_proj_shard_bwd_resharded(ntp_handle_t* h, const ntp_attn_shape_t* s, const void* dZ, int64_t lddz,
                                                 const void* dQKV, int64_t lddqkv, const void* X, int64_t ldx,
                                                 const void* C, int64_t ldc, const void* Wqkv, int64_t ldwqkv,
                                                 const void* Wo, int64_t ldwo, void* dC, int64_t lddc, void* dXpart,
                                                 int64_t lddx, const ntp_row_segment_t* dWqkv_segs,
                                                 int32_t n_dWqkv_segs, const ntp_row_segment_t* dWo_segs,
                                                 int32_t n_dWo_segs, int32_t accumulate, void* stream) {
  return attn_bwd(h, s, dZ, lddz, dQKV, lddqkv, X, ldx, C, ldc, Wqkv, ldwqkv, Wo, ldwo, dC, lddc, dXpart, lddx, dWqkv_segs,
                  n_dWqkv_segs, dWo_segs, n_dWo_segs, accumulate, stream);
}

// Largest workspace the GEMMs of a shard call could use: the maximum over its GEMMs (they run one after the
// other on the handle's stream and share the workspace).
extern "C" int ntp_workspace_bytes(const ntp_handle_t* h, int32_t call, const void* shape, int64_t* bytes) {
  if (!h || !shape || !bytes) return NTP_ERR_INVALID_ARG;
  auto up = [](int64_t x, int64_t m) { return (x + m - 1) / m * m; };
  int64_t need = 0;
  auto gemm_wish = [&](int layout, int64_t M, int64_t N, int64_t n_store, int64_t K) {
    if (M > 0 && N > 0 && K > 0) need = std::max(need, ntp::gemm_workspace_wish(h, layout, M, N, n_store, K));
  };
  if (call == NTP_CALL_MLP_SHARD) {
    const ntp_mlp_shape_t* s = static_cast<const ntp_mlp_shape_t*>(shape);
    if (bad_mlp_shape(s) || s->H % 8) return NTP_ERR_INVALID_ARG;
    gemm_wish(0, s->M, s->n_r, up(s->n_r, 64), s->H);  // X A_i and dZ B_i^T (pad columns zeroed up to 64)
    gemm_wish(1, s->M, s->H, s->H, s->n_r);            // Y B_i and dP A_i^T
    gemm_wish(2, s->n_r, s->H, s->H, s->M);            // the two weight gradients
  } else if (call == NTP_CALL_ATTN_PROJ_SHARD) {
    const ntp_attn_shape_t* s = static_cast<const ntp_attn_shape_t*>(shape);
    if (bad_attn_shape(s) || s->H % 8 || s->w_qkv % 8 || s->w_o % 8) return NTP_ERR_INVALID_ARG;
    gemm_wish(0, s->M, s->w_qkv, s->w_qkv, s->H);
    gemm_wish(0, s->M, s->w_o, s->w_o, s->H);
    gemm_wish(1, s->M, s->H, s->H, s->w_o);
    gemm_wish(1, s->M, s->H, s->H, s->w_qkv);
    gemm_wish(2, s->w_qkv, s->H, s->H, s->M);
    gemm_wish(2, s->w_o, s->H, s->H, s->M);
  } else if (call == NTP_CALL_ATTN_CORE_SHARD) {
    const int st = ntp::attn_core_workspace_wish(h, static_cast<const ntp_attn_core_shape_t*>(shape), &need);
    if (st != NTP_OK) return st;
  } else {
    return NTP_ERR_INVALID_ARG;
  }
  *bytes = need;
  return NTP_OK;
}
