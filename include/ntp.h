/*
 * ntp.h -- C ABI of the MI355X (gfx950) shard hot path of Nonuniform Tensor
 * Parallelism (NTP).
 *
 * A data-parallel replica that lost GPUs runs at a reduced tensor-parallel
 * degree t' < t, so each surviving GPU computes an uneven shard of every
 * transformer layer, and weight gradients have to be repacked between the
 * TP = t' and TP = t layouts around the data-parallel sync.  This library is
 * one GPU's part of that: the shard plan, the shard's MLP and attention
 * projection GEMMs (forward and backward), and the gradient reshard.
 *
 * Conventions shared by every call
 *   - "device" pointers are HIP device memory owned by the caller; "host"
 *     pointers are ordinary process memory.  Calls that enqueue work take a
 *     handle (ntp_create), allocate no device memory, keep no pointer after
 *     they return, and never synchronise: kernels are enqueued on `stream` (a
 *     hipStream_t passed as void*, NULL = the default stream) and the call
 *     returns at once.  The three exceptions say so where they are declared:
 *     ntp_reshard_plan_prepare (one device allocation and a blocking upload per
 *     plan), ntp_kernel_timing_* (HIP events, off by default) and the static
 *     scratch entry point at the end of this file.
 *   - The library holds no global state.  What a device call reads besides its
 *     arguments (device size, workspace, tuning overrides) is in the handle;
 *     calls on different handles may run concurrently, on any streams; calls on
 *     ONE handle must come from one thread at a time, and those that may use
 *     its workspace must be ordered on the device (same stream, or events).
 *   - Matrices are row-major with an explicit leading dimension `ld*` counted
 *     in ELEMENTS.  bf16 matrices need a 16-byte aligned base pointer and
 *     ld % 8 == 0; fp32 gradient matrices need a 16-byte aligned base and
 *     ld % 4 == 0.  A violated requirement returns NTP_ERR_ALIGNMENT; nothing
 *     is launched.
 *   - Return value: NTP_OK (0) or a negative NTP_ERR_* code; no C++ exception
 *     crosses the boundary.  ntp_status_string() names a code.
 *   - bf16 = bfloat16 bit patterns (uint16_t storage), rounded to nearest even
 *     on output; all contractions accumulate in fp32 on the matrix cores.
 *
 * Storage of the partitioned weights.  The paper writes the MLP as
 * Z = GeLU(X A) B with A split by columns and B by rows (Sec. 3.1, Eq. 1-3).
 * Both shards are held here with the partitioned dimension OUTERMOST:
 *     A_t  [n_r x H]   row j = column j of A_i      (fc1, column-parallel)
 *     B    [n_r x H]   row j = row    j of B_i      (fc2, row-parallel)
 *     Wqkv [w_qkv x H] row j = column j of W_qkv,i  (Eq. 6, rows ordered
 *                      [Q heads | K heads | V heads] of this rank)
 *     Wo   [w_o x H]   row j = row j of W_O,i       (Eq. 4)
 * so a ragged shard width never lands on a contiguous axis of a weight or of
 * its gradient, and gradients come out shaped exactly like their weights.
 */
#ifndef NTP_H_
#define NTP_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define NTP_OK 0
#define NTP_ERR_INVALID_ARG (-1) /* null pointer, negative size, rank out of range, aliasing ... */
#define NTP_ERR_ALIGNMENT (-2)   /* base pointer or leading dimension not aligned as required   */
#define NTP_ERR_LAUNCH (-3)      /* the HIP runtime refused a kernel launch                      */
#define NTP_ERR_UNSUPPORTED (-4) /* a size beyond what the kernels index (see each call)         */
#define NTP_ERR_NOT_PREPARED (-5) /* ntp_reshard_plan_run before ntp_reshard_plan_prepare        */
#define NTP_ERR_NO_DEVICE (-6)   /* a device call on a handle created with no device visible    */
#define NTP_ERR_SCRATCH_TOO_SMALL (-7) /* the shape needs more than NTP_STATIC_SCRATCH_BYTES      */

#define NTP_GELU_ERF 0  /* x * Phi(x)                                  */
#define NTP_GELU_TANH 1 /* 0.5 x (1 + tanh(sqrt(2/pi)(x + 0.044715 x^3))) */

/* Library version, major * 10000 + minor * 100 + patch. */
int ntp_version(void);

/* Static string naming a status code.  Never NULL. */
const char* ntp_status_string(int status);

/* ---------------------------------------------------------------------------
 * Handle.  ntp_create queries the CURRENT HIP device (its ordinal and number of
 * compute units, which the launchers size their grids by) and returns a handle
 * owned by the caller until ntp_destroy; it allocates host memory only.  With no
 * device visible the handle still serves the host-only calls (ntp_gemm_choice,
 * ntp_attn_core_choice, ntp_workspace_bytes) with an MI355X's 256 compute units.
 * Device calls must be made with the handle's device current.
 * ntp_device_info reports what was found (device -1: none). */
typedef struct ntp_handle ntp_handle_t;
int ntp_create(ntp_handle_t** out);
int ntp_destroy(ntp_handle_t* h); /* NULL is accepted; no call on h may still be running on the host */
int ntp_device_info(const ntp_handle_t* h, int32_t* device, int32_t* compute_units);

/* Tuning overrides of one handle.  Every option is 0 by default = the library's
 * own choice.  They exist so that tests and tuning runs can reach every kernel
 * variant at any size; a forced variant computes the same result to within fp32
 * summation order (bit-identical for the reshard options).
 * Errors: unknown option or value out of range -> INVALID_ARG. */
#define NTP_OPT_GEMM_TILE 0          /* 1: the small generic kernel; 2 + i: ring tile shape i in the order 256x256,
                                        256x224, 224x256, 256x192, 192x256, 256x128, 128x256, 128x128 (4 wavefronts),
                                        128x128 (8 wavefronts)                                                       */
#define NTP_OPT_GEMM_SPLIT 1         /* 1: never cut the contraction axis; 2..8: that many chunks where they fit   */
#define NTP_OPT_GEMM_NO_RING_TAIL 2  /* 1: the K tail of row-parallel GEMMs goes through registers                 */
#define NTP_OPT_ATTN_PARTS 3         /* 1..16: parts per attention-core walk where the workspace holds them        */
#define NTP_OPT_RESHARD_BLOCK 4      /* bytes per workgroup of the row-wise gather kernel                           */
#define NTP_OPT_RESHARD_FLAT_BLOCK 5 /* bytes per workgroup of the flat-destination kernel                          */
#define NTP_OPT_RESHARD_TABLE_BLOCK 6 /* bytes per block of the run-table kernel                                    */
#define NTP_OPT_RESHARD_NO_FLAT 7    /* 1: column-partitioned tensors never take the flat-destination kernel       */
#define NTP_OPT_RESHARD_NO_TABLE 8   /* 1: plans never take the run-table kernel                                   */
#define NTP_OPT_GEMM_SCHEDULE 9      /* schedule of the ring kernel's K loop: 1 the default one everywhere, 2 the
                                        ping-pong one wherever it exists (8-wavefront tiles, persistent form)        */
#define NTP_OPT_GEMM_WORKGROUPS 10   /* persistent GEMM launches use at most this many workgroups (rounded down to a
                                        multiple of 8, at least 8; 0: one per compute unit).  Fewer workgroups make
                                        each walk over more output tiles: tests and tuning                            */
#define NTP_OPT_ATTN_COPY 11         /* how the attention kernels bring their 64-row tiles to LDS where both forms
                                        exist (head dimension 128; forward: 16 query rows per wavefront): 1 through
                                        registers, 2 by DMA into chunk-permuted rows; 0: the library's choice          */
#define NTP_OPT_ATTN_BWD_LAUNCHES 12  /* the attention core's dQ and dK/dV kernels: 1 one launch each, 2 one launch for
                                        both where both copy by DMA (they then share the compute units; a small
                                        kernel stores the rows' delta values first); 0: the library's choice          */
#define NTP_OPT_COUNT_ 13
int ntp_set_option(ntp_handle_t* h, int32_t option, int64_t value);

/* ---------------------------------------------------------------------------
 * Shard plan (Sec. 3.1, closing paragraph of "Attention blocks": the partition
 * dimension need not divide by the TP degree, the shards are then uneven).
 * `dim` units are cut into `tp` contiguous slices whose widths differ by at
 * most one, the `dim % tp` lowest ranks holding the wider ones:
 *     width  = dim / tp + (rank < dim % tp)
 *     offset = rank * (dim / tp) + min(rank, dim % tp)
 * Host-only, pure.  tp > dim is legal (trailing ranks get width 0).
 * Errors: dim < 0, tp < 1, rank outside [0, tp), NULL output -> INVALID_ARG.
 */
int ntp_shard_plan(int64_t dim, int32_t tp, int32_t rank, int64_t* offset, int64_t* width);

/* Head-granular plan for an attention block (Sec. 3.1, Eq. 4-6: the W_Q, W_K,
 * W_V, W_O of a head stay together).  Query heads are the partition unit and
 * are split by ntp_shard_plan(n_q, tp, rank).  With grouped KV heads
 * (n_kv < n_q, n_q % n_kv == 0) a rank holds every KV head one of its query
 * heads reads, so a KV head may be replicated on neighbouring ranks.
 *     w_qkv = (q_cnt + 2 kv_cnt) * head_dim   width of this rank's QKV output
 *     w_o   = q_cnt * head_dim                rows of this rank's W_O,i
 * Host-only.  Errors: n_q % n_kv != 0, non-positive sizes, bad rank, NULL. */
typedef struct ntp_attn_plan {
  int32_t q_off, q_cnt;   /* first query head and number of query heads */
  int32_t kv_off, kv_cnt; /* first KV head and number of KV heads       */
  int32_t head_dim;
  int32_t w_qkv, w_o;
} ntp_attn_plan_t;
int ntp_attn_shard_plan(int32_t n_q, int32_t n_kv, int32_t head_dim, int32_t tp, int32_t rank,
                        ntp_attn_plan_t* out);

/* ---------------------------------------------------------------------------
 * MLP shard (Sec. 3.1, Eq. 2-3).  M tokens, hidden H, this rank's width n_r.
 * H % 8 == 0 is required; M and n_r are arbitrary (n_r = 0 is a no-op that
 * still zero-fills Zpart / dXpart). */
typedef struct ntp_mlp_shape {
  int64_t M, H, n_r;
  int32_t gelu_mode; /* NTP_GELU_ERF or NTP_GELU_TANH */
} ntp_mlp_shape_t;

/* Forward: P_i = X A_i, Y_i = GeLU(P_i) (Eq. 3), Zpart = Y_i B_i (Eq. 2, this
 * rank's partial sum; the TP all-reduce is the caller's).
 *   in   X [M x H] bf16, A_t [n_r x H] bf16, B [n_r x H] bf16        (device)
 *   out  P, Y [M x n_r] bf16 with ldp, ldy >= n_r and % 8 == 0; columns from
 *        n_r up to the next multiple of 8 are written with zeros; if both
 *        ldp and ldy reach the next multiple of 64, up to that one (the second
 *        GEMM then needs no special case for the end of its contraction axis).
 *        Every row, the last one included, must be backed by its pad columns
 *        as far as they are written                                  (device)
 *   out  Zpart [M x H] bf16                                           (device)
 * P and Y are kept for the backward call.  No buffer may alias another. */
int ntp_mlp_shard_fwd(ntp_handle_t* h, const ntp_mlp_shape_t* shape, const void* X, int64_t ldx, const void* A_t,
                      int64_t lda, const void* B, int64_t ldb, void* P, int64_t ldp, void* Y,
                      int64_t ldy, void* Zpart, int64_t ldz, void* stream);

/* Backward (chain rule on Eq. 2-3; gradients are shaped and partitioned like
 * A_i and B_i, Sec. 3.1):
 *   dP_i   = (dZ B_i^T) .* GeLU'(P_i)      [M x n_r] bf16, output / workspace
 *   dB     = Y_i^T dZ                      [n_r x H] fp32
 *   dA_t   = dP_i^T X                      [n_r x H] fp32 (= (X^T dP_i)^T)
 *   dXpart = dP_i A_i^T                    [M x H]  bf16, partial sum
 * in: dZ [M x H] bf16 and X, A_t, B, P, Y as in the forward call (P, Y as it
 * wrote them).  dP's pad columns are zeroed like P's (up to the next multiple
 * of 8, or of 64 if lddp and ldp reach it).  accumulate != 0 adds into dA_t / dB instead of overwriting
 * (gradient accumulation over micro-batches before the reshard, Sec. 4.1). */
int ntp_mlp_shard_bwd(ntp_handle_t* h, const ntp_mlp_shape_t* shape, const void* dZ, int64_t lddz, const void* X,
                      int64_t ldx, const void* A_t, int64_t lda, const void* B, int64_t ldb,
                      const void* P, int64_t ldp, const void* Y, int64_t ldy, void* dP,
                      int64_t lddp, void* dXpart, int64_t lddx, float* dA_t, int64_t ldda,
                      float* dB, int64_t lddb, int32_t accumulate, void* stream);

/* ---------------------------------------------------------------------------
 * Attention projections of one shard (Sec. 3.1, Eq. 4 and 6).  The attention
 * core (Eq. 5) sits between the two halves and is the caller's.  w_qkv and
 * w_o come from ntp_attn_shard_plan and must be multiples of 8; H % 8 == 0. */
typedef struct ntp_attn_shape {
  int64_t M, H;
  int64_t w_qkv, w_o;
} ntp_attn_shape_t;

/* Forward.  Column-parallel half: QKV = X Wqkv^T   [M x w_qkv] bf16 (Eq. 6);
 * row-parallel half: Zpart = C Wo [M x H] bf16 (Eq. 4) with C [M x w_o] the
 * attention output of this rank's heads.  A half is skipped when its output
 * pointer (QKV resp. Zpart) is NULL. */
int ntp_attn_proj_shard_fwd(ntp_handle_t* h, const ntp_attn_shape_t* shape, const void* X, int64_t ldx,
                            const void* Wqkv, int64_t ldwqkv, void* QKV, int64_t ldqkv,
                            const void* C, int64_t ldc, const void* Wo, int64_t ldwo, void* Zpart,
                            int64_t ldz, void* stream);

/* Backward.  Row-parallel half (skipped when dZ is NULL):
 *   dC = dZ Wo^T [M x w_o] bf16,  dWo = C^T dZ [w_o x H] fp32.
 * Column-parallel half (skipped when dQKV is NULL):
 *   dXpart = dQKV Wqkv [M x H] bf16 (partial sum),  dWqkv = dQKV^T X [w_qkv x H] fp32.
 * The dW of a KV head replicated on several ranks is each rank's partial sum
 * (over its own query heads); ntp_replica_sum completes it.
 * accumulate != 0 adds into dWqkv / dWo. */
int ntp_attn_proj_shard_bwd(ntp_handle_t* h, const ntp_attn_shape_t* shape, const void* dZ, int64_t lddz,
                            const void* dQKV, int64_t lddqkv, const void* X, int64_t ldx,
                            const void* C, int64_t ldc, const void* Wqkv, int64_t ldwqkv,
                            const void* Wo, int64_t ldwo, void* dC, int64_t lddc, void* dXpart,
                            int64_t lddx, float* dWqkv, int64_t lddwqkv, float* dWo, int64_t lddwo,
                            int32_t accumulate, void* stream);

/* ---------------------------------------------------------------------------
 * Gradient reshard (Sec. 3.1 "Shard-mapping algorithm"; Appendix, the
 * pre-sync hook and the post-sync reshard): repack a partitioned tensor from
 * the TP = src_tp layout into the TP = dst_tp layout.  Both layouts are views
 * of one logical [rows x cols] tensor cut along `partition_dim` in units of
 * `unit` elements (1 for an MLP weight, head_dim for an attention weight).
 * Pure data movement, bit-exact, element type opaque (elem_size 2 or 4). */
#define NTP_KIND_PLAIN 0   /* contiguous ranges of units per ntp_shard_plan                 */
#define NTP_KIND_QKV_GQA 1 /* units = [n_q Q heads | n_kv K heads | n_kv V heads]; a rank
                              holds [its Q heads | the K heads they read | the same V heads] */
typedef struct ntp_tensor_spec {
  int64_t rows, cols;    /* logical (unsharded) shape                                   */
  int32_t partition_dim; /* 0: shards are row blocks, 1: shards are column blocks       */
  int32_t unit;          /* elements per partition unit along partition_dim             */
  int32_t elem_size;     /* bytes per element: 2 or 4                                   */
  int32_t kind;          /* NTP_KIND_*                                                  */
  int32_t n_q, n_kv;     /* QKV_GQA only; the partitioned extent is (n_q + 2 n_kv)*unit */
} ntp_tensor_spec_t;

/* One sub-shard: `units` consecutive units that sit in source rank `src_rank`
 * starting at its local unit `src_unit` and go to destination rank `dst_rank`
 * at local unit `dst_unit` (the overlap of two shards, Sec. 3.1). */
typedef struct ntp_segment {
  int32_t src_rank, dst_rank;
  int64_t src_unit, dst_unit, units;
} ntp_segment_t;

/* Host-only: list the sub-shards of spec for src_tp -> dst_tp, in destination
 * order.  Writes at most `max_segments` entries to `out` (may be NULL when
 * max_segments is 0) and the full count to *count.  A unit held by several
 * source ranks (replicated KV head) is taken from the lowest such rank. */
int ntp_reshard_segments(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp,
                         ntp_segment_t* out, int64_t max_segments, int64_t* count);

/* Sum of replicated units (grouped KV heads; Sec. 3.1 keeps a head's W_Q, W_K, W_V, W_O together, so a KV
 * head sits on every rank whose query heads read it).  ntp_attn_proj_shard_bwd leaves, on each of those ranks,
 * only the share of the head's gradient that the rank's own query heads contribute; the gradient itself is the
 * sum over the holders.  This call adds the holders' [unit]-blocks of every unit of an NTP_KIND_QKV_GQA tensor
 * that more than one rank of the TP = tp layout holds, in ascending rank order (fp32, fixed order:
 * deterministic), and writes the sum back into every holder's block, in place.  It is the one-GPU form of the
 * all-reduce among the holders, and it must run before ntp_reshard_grad, which copies a replicated unit from
 * one holder only.  NTP_KIND_PLAIN tensors have no replicated units: the call does nothing.
 *   shards / ld   HOST arrays of tp DEVICE pointers (fp32, 4-byte aligned; 16-byte aligned blocks with
 *                 ld % 4 == 0 go fastest) and leading dimensions, as for ntp_reshard_grad; a NULL shard is
 *                 "not on this GPU" and takes no part; shards must not overlap (INVALID_ARG)
 * Errors: elem_size != 4 -> INVALID_ARG; more than 96 holders of one unit -> UNSUPPORTED. */
int ntp_replica_sum(ntp_handle_t* h, const ntp_tensor_spec_t* spec, int32_t tp, void* const* shards,
                    const int64_t* ld, void* stream);

/* Enqueue the copy.  src_shards[src_tp] / dst_shards[dst_tp] are HOST arrays of
 * DEVICE pointers, one per rank, each a row-major matrix shaped like that
 * rank's shard with leading dimension src_ld[r] / dst_ld[s] (host arrays,
 * elements).  A NULL shard pointer means "not on this GPU": every sub-shard
 * that touches it is skipped, which is how one GPU's share of the exchange is
 * expressed; shards of width 0 may be NULL.  src_tp and dst_tp may be in
 * either order.  Source and destination must not overlap (checked: INVALID_ARG).
 * A unit that several source ranks hold is read from the lowest of them: the
 * copies must agree (weights do; gradients after ntp_replica_sum).
 * Only 2-byte alignment (elem_size 2) or 4-byte alignment (elem_size 4) of
 * pointers is required; 16-byte aligned rows copy fastest. */
int ntp_reshard_grad(ntp_handle_t* h, const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp,
                     const void* const* src_shards, const int64_t* src_ld,
                     void* const* dst_shards, const int64_t* dst_ld, void* stream);

/* ---------------------------------------------------------------------------
 * Attention core of the rank's local heads (Sec. 3.1, Eq. 5): for every local
 * query head j and the KV head g(j) it reads,
 *   C_j = softmax(Q_j K_g^T / sqrt(head_dim)) V_g,   one sequence at a time.
 * It sits between the two halves of ntp_attn_proj_shard_fwd: QKV is that
 * call's output [M x (q_cnt + 2 kv_cnt) head_dim] with columns
 * [Q heads | K heads | V heads], C its input [M x q_cnt head_dim].  The M =
 * n_seq * seq_len tokens are n_seq sequences of seq_len rows each.  Local
 * query head j reads local KV head (q_off + j) / group - kv_off (q_off, kv_off,
 * q_cnt, kv_cnt from ntp_attn_shard_plan; group = query heads per KV head); all
 * of them must be local (INVALID_ARG).  causal != 0: query t sees keys 0..t of
 * its sequence (the paper writes the unmasked form; decoder training masks).
 * head_dim 64 or 128 (UNSUPPORTED otherwise).  bf16 in and out (16-byte aligned,
 * leading dimensions multiples of 8), fp32 arithmetic for scores and sums.
 * One sequence's rows of QKV (and of dC in the backward call) must span less
 * than 2 GiB: seq_len * leading dimension * 2 < 2^31 (UNSUPPORTED otherwise).
 * LSE (DEVICE, fp32 [q_cnt x M], may be NULL in the forward call): per head and
 * token the natural logarithm of the sum of exp(score) over the visible keys;
 * the backward call reads it. */
typedef struct ntp_attn_core_shape {
  int32_t n_seq, seq_len;
  int32_t q_cnt, kv_cnt;
  int32_t q_off, kv_off, group;
  int32_t head_dim;
  int32_t causal;
} ntp_attn_core_shape_t;
int ntp_attn_core_shard_fwd(ntp_handle_t* h, const ntp_attn_core_shape_t* shape, const void* QKV, int64_t ldqkv,
                            void* C, int64_t ldc, float* LSE, void* stream);
/* Gradient of the above: given dC [M x q_cnt head_dim] (what ntp_attn_proj_shard_bwd
 * returns), the forward call's QKV, C and LSE, writes dQKV [M x (q_cnt + 2 kv_cnt)
 * head_dim] in QKV's layout (what ntp_attn_proj_shard_bwd takes); the gradient of a
 * KV head is the sum over the local query heads that read it, and zero for a KV head
 * that none reads.  Delta: DEVICE scratch, fp32 [q_cnt x M], overwritten (per head
 * and token the dot product of the rows of dC and C).  All matrices bf16, 16-byte
 * aligned, leading dimensions multiples of 8; QKV and dQKV must not overlap. */
int ntp_attn_core_shard_bwd(ntp_handle_t* h, const ntp_attn_core_shape_t* shape, const void* QKV, int64_t ldqkv,
                            const void* C, int64_t ldc, const void* dC, int64_t lddc,
                            const float* LSE, float* Delta, void* dQKV, int64_t lddqkv,
                            void* stream);

/* ---------------------------------------------------------------------------
 * Weight gradients written straight into the destination layout of the
 * reshard (Sec. 3.1 "Shard-mapping algorithm"; Appendix, the pre-sync hook):
 * the gradient GEMMs of a backward call store each output row where the
 * reshard would have copied it, so the separate pass over HBM is not needed.
 * Gradients are stored with the partitioned dimension as rows, so a sub-shard
 * of this rank's gradient is a block of rows.
 *
 * ntp_row_segment_t: `rows` rows of the rank's gradient starting at local row
 *   row_begin go to dst (DEVICE pointer, fp32, 16-byte aligned) with leading
 *   dimension ld (elements, multiple of 4, >= the gradient's row length).
 *   A row may be listed in several segments (a KV head held by several
 *   destination ranks) and is then stored to each.
 * ntp_reshard_row_segments (host only): the segments of source rank src_rank
 *   of spec (partition_dim 0, elem_size 4) for src_tp -> dst_tp, given the
 *   destination shards (HOST array of dst_tp DEVICE pointers and leading
 *   dimensions, as for ntp_reshard_grad; sub-shards whose destination shard
 *   is NULL, "not on this GPU", are left out).  Writes at most max_segments
 *   entries and the full count.  NTP_KIND_QKV_GQA specs in which a KV head of
 *   src_rank is also held by another source rank return UNSUPPORTED: there each
 *   holder's GEMM yields a partial sum, which ntp_replica_sum has to complete
 *   before a reshard (use the unfused calls).
 * ntp_mlp_shard_bwd_resharded / ntp_attn_proj_shard_bwd_resharded: as
 *   ntp_mlp_shard_bwd / ntp_attn_proj_shard_bwd, with the gradient outputs
 *   given as HOST arrays of segments (at most 16 per gradient: UNSUPPORTED
 *   beyond).  The segments of one gradient must not overlap in memory
 *   (INVALID_ARG); a row that no segment lists is not stored (a KV head whose
 *   destination copies are fed by another rank, a destination on another
 *   GPU).  accumulate != 0 adds into the destinations.  Results are bit-identical to the unfused call followed by
 *   ntp_reshard_grad. */
typedef struct ntp_row_segment {
  int64_t row_begin, rows;
  float* dst;
  int64_t ld;
} ntp_row_segment_t;
int ntp_reshard_row_segments(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t src_rank,
                             int32_t dst_tp, void* const* dst_shards, const int64_t* dst_ld,
                             ntp_row_segment_t* out, int64_t max_segments, int64_t* count);
int ntp_mlp_shard_bwd_resharded(ntp_handle_t* h, const ntp_mlp_shape_t* shape, const void* dZ, int64_t lddz,
                                const void* X, int64_t ldx, const void* A_t, int64_t lda,
                                const void* B, int64_t ldb, const void* P, int64_t ldp,
                                const void* Y, int64_t ldy, void* dP, int64_t lddp, void* dXpart,
                                int64_t lddx, const ntp_row_segment_t* dA_segs, int32_t n_dA_segs,
                                const ntp_row_segment_t* dB_segs, int32_t n_dB_segs,
                                int32_t accumulate, void* stream);
int ntp_attn_proj_shard_bwd_resharded(ntp_handle_t* h, const ntp_attn_shape_t* shape, const void* dZ, int64_t lddz,
                                      const void* dQKV, int64_t lddqkv, const void* X, int64_t ldx,
                                      const void* C, int64_t ldc, const void* Wqkv, int64_t ldwqkv,
                                      const void* Wo, int64_t ldwo, void* dC, int64_t lddc,
                                      void* dXpart, int64_t lddx,
                                      const ntp_row_segment_t* dWqkv_segs, int32_t n_dWqkv_segs,
                                      const ntp_row_segment_t* dWo_segs, int32_t n_dWo_segs,
                                      int32_t accumulate, void* stream);

/* ---------------------------------------------------------------------------
 * Comp and sync rank assignment (Sec. 3.1 "Shard-mapping algorithm", Alg. 1).
 * A healthy replica of TP degree full_tp synchronises gradients with replicas
 * that run at reduced_tp <= full_tp.  For each of the k partition units:
 *   sync_rank[u]: the rank (0 .. reduced_tp-1) that holds unit u when gradients
 *     are synchronised: the contiguous even split of ntp_shard_plan(k, reduced_tp);
 *   comp_rank[u]: the rank (0 .. full_tp-1) that holds and computes unit u.  A
 *     sync rank keeps the first k / full_tp (rounded down) units of its slice;
 *     the others are dealt one by one, in unit order, in turn to the offload
 *     ranks reduced_tp .. full_tp-1, the turn running on from one sync rank's
 *     slice to the next, so that all (offload rank, sync rank) pairs carry the
 *     same number of units to within one.
 * Host only.  comp_rank / sync_rank: HOST arrays of k entries, written.
 * reduced_tp == full_tp gives comp_rank == sync_rank.  INVALID_ARG for k < 0,
 * reduced_tp < 1, full_tp < reduced_tp or a NULL array with k > 0. */
int ntp_comp_sync_plan(int64_t k, int32_t full_tp, int32_t reduced_tp, int32_t* comp_rank,
                       int32_t* sync_rank);

/* ---------------------------------------------------------------------------
 * Reshard between two layouts given unit by unit (Sec. 3.1, Alg. 1; Appendix:
 * the pre-sync hook and post-sync reshard with split sizes precomputed from the
 * rank assignment).  A layout is a map unit -> rank; a rank holds its units in
 * ascending unit order, as one dense-in-units shard shaped like the shards of
 * ntp_reshard_grad.  A plan is built once from the two maps (host work
 * proportional to the number of units) and run every step.
 *
 * ntp_reshard_plan_create: spec as for ntp_reshard_grad, kind NTP_KIND_PLAIN
 *   only; src_rank_of_unit / dst_rank_of_unit: HOST arrays of map_len entries,
 *   one per partition unit (values in [0, src_tp) / [0, dst_tp)), read during
 *   the call only; map_len must equal the spec's number of units (INVALID_ARG).  *plan receives a handle owned by the library until
 *   ntp_reshard_plan_destroy.  Host only, touches no GPU.
 * ntp_reshard_plan_segments: the sub-shards (runs of units that are consecutive
 *   in both a source and a destination shard) in destination order, as for
 *   ntp_reshard_segments.
 * ntp_reshard_plan_splits: units[r * dst_tp + s] = units that source rank r
 *   sends to destination rank s (row r: send splits of r; column s: receive
 *   splits of s).  HOST array of src_tp * dst_tp entries, written.
 * ntp_reshard_plan_table: for every destination unit, destination shards one
 *   after the other, the source rank and the local unit in its shard.
 * ntp_reshard_plan_prepare: makes the plan ready to run on the CURRENT device.
 *   Plans of column-partitioned tensors of 4-byte elements have a run table (2
 *   bytes per unit + 16 bytes per sub-shard) that one of the copy kernels reads
 *   from device memory: this call allocates it (hipMalloc) and waits for its
 *   upload.  It is the only call of the library that allocates device memory or
 *   blocks; every plan needs it once before its first run (for plans without a
 *   table it only records the device).  Calling it again on the same device does
 *   nothing; on another device -> INVALID_ARG.
 * ntp_reshard_plan_run: enqueue the copy; shard arrays, NULL shards, alignment
 *   and aliasing rules as for ntp_reshard_grad.  Allocates nothing and never
 *   waits, so a run can be captured into a HIP graph.  A plan that was not
 *   prepared, or was prepared on another device than the current one ->
 *   NTP_ERR_NOT_PREPARED, nothing is enqueued.  Column-partitioned tensors of
 *   4-byte elements whose shards are all on this GPU, with dense 64-byte aligned
 *   destinations, go through the run-table kernel; everything else is copied
 *   sub-shard by sub-shard.
 * ntp_reshard_plan_destroy: frees the handle and its device table; no run of
 *   the plan may still be in flight.  NULL is accepted. */
typedef struct ntp_reshard_plan ntp_reshard_plan_t;
typedef struct ntp_unit_source {
  int32_t src_rank;
  int32_t src_unit; /* local unit in the source rank's shard */
} ntp_unit_source_t;
int ntp_reshard_plan_create(const ntp_tensor_spec_t* spec, int64_t map_len, int32_t src_tp,
                            const int32_t* src_rank_of_unit, int32_t dst_tp,
                            const int32_t* dst_rank_of_unit, ntp_reshard_plan_t** plan);
int ntp_reshard_plan_segments(const ntp_reshard_plan_t* plan, ntp_segment_t* out,
                              int64_t max_segments, int64_t* count);
int ntp_reshard_plan_splits(const ntp_reshard_plan_t* plan, int64_t* units);
int ntp_reshard_plan_table(const ntp_reshard_plan_t* plan, ntp_unit_source_t* out,
                           int64_t max_units, int64_t* count);
int ntp_reshard_plan_prepare(ntp_reshard_plan_t* plan);
int ntp_reshard_plan_run(ntp_handle_t* h, ntp_reshard_plan_t* plan, const void* const* src_shards,
                         const int64_t* src_ld, void* const* dst_shards, const int64_t* dst_ld,
                         void* stream);
int ntp_reshard_plan_destroy(ntp_reshard_plan_t* plan);

/* ---------------------------------------------------------------------------
 * Measurement aid (not part of the method).  When enabled, every kernel the
 * library enqueues is bracketed by two HIP events on the caller's stream and
 * recorded with its algorithmic work: flops = 2 M N K on the logical GEMM
 * dimensions, bytes = bytes read + bytes written by a reshard launch.  This is
 * the only part of the library that creates HIP objects (events); it is off by
 * default and per handle.  ntp_kernel_timing_read waits for the recorded
 * kernels, writes at most max_records entries (launch order), stores the number
 * of launches recorded in *count and clears the list. */
typedef struct ntp_kernel_time {
  char name[48]; /* kernel family and variant, e.g. "gemm_tn_f32"  */
  double flops;  /* algorithmic flops of this launch (0 for copies)  */
  double bytes;  /* algorithmic bytes of this launch (0 for GEMMs)   */
  float ms;      /* duration between the two events                  */
  int32_t pad_;
} ntp_kernel_time_t;
int ntp_kernel_timing_enable(ntp_handle_t* h, int32_t on);
int ntp_kernel_timing_read(ntp_handle_t* h, ntp_kernel_time_t* out, int64_t max_records, int64_t* count);

/* Workspace for split-K (Sec. 3.1: at a high TP degree a column-parallel shard X A_i or
 * X W_qkv,i is a skinny GEMM with fewer output tiles than the GPU has compute units).
 * With a workspace set on the handle, a shard GEMM whose output tiles would leave most
 * compute units idle is also cut along its contraction axis: fp32 partial sums go to the
 * workspace and a second kernel adds them in a fixed order and applies the epilogue
 * (results stay deterministic; they differ from the unsplit GEMM by fp32 rounding order).
 * The attention core uses it the same way when a rank has few heads (Eq. 5 on 2-3
 * heads of a long sequence is fewer workgroups than compute units): every workgroup's
 * walk over the key (or query) tiles is cut into parts that store fp32 partial results,
 * merged by a second kernel (forward: by running maximum and sum).
 *   workspace  device pointer, 256-byte aligned; NULL with bytes == 0 removes it
 *   bytes      its size; a GEMM is split only if splits * M * round_up(N, 16) * 4 fits,
 *              a walk cut only if workgroups * parts * 64 rows * row bytes fits
 * The caller owns the memory and keeps it alive while it is set.  The workspace belongs
 * to the handle: calls on this handle that may use it must be ordered on the device
 * (one stream, or events between streams); to run shard calls concurrently on several
 * streams (the gradient sync beside the backward pass, Sec. 4.1), give each stream a
 * handle and a workspace of its own.  Without a workspace nothing is ever split.
 * Errors: NTP_ERR_INVALID_ARG (misaligned, negative size, NULL with bytes > 0).
 *
 * ntp_workspace_bytes (host only): the largest workspace that the forward or backward
 * call of a shape can use on this handle's device, i.e. what its launch decisions would
 * take if the workspace were unlimited (0: nothing would be split); a smaller workspace
 * is legal and leaves some launches unsplit.  call / shape:
 *   NTP_CALL_MLP_SHARD        const ntp_mlp_shape_t*        ntp_mlp_shard_fwd, _bwd, _bwd_resharded
 *   NTP_CALL_ATTN_PROJ_SHARD  const ntp_attn_shape_t*       ntp_attn_proj_shard_fwd, _bwd, _bwd_resharded
 *   NTP_CALL_ATTN_CORE_SHARD  const ntp_attn_core_shape_t*  ntp_attn_core_shard_fwd, _bwd
 * Errors: NTP_ERR_INVALID_ARG (NULL, unknown call, a shape the call itself would refuse). */
#define NTP_CALL_MLP_SHARD 0
#define NTP_CALL_ATTN_PROJ_SHARD 1
#define NTP_CALL_ATTN_CORE_SHARD 2
int ntp_workspace_bytes(const ntp_handle_t* h, int32_t call, const void* shape, int64_t* bytes);
int ntp_set_workspace(ntp_handle_t* h, void* workspace, int64_t bytes);

/* Diagnostic aid (host only, touches no device memory): which GEMM kernel a shard GEMM
 * of this shape would run on this handle (its compute units, workspace and options at
 * the time of the call), with tightly packed operands.  layout: 0 both operands K-contiguous (column-parallel
 * forward, activation gradients of row-parallel layers), 1 A K-contiguous and B
 * K-strided (row-parallel forward, partial input gradients), 2 both K-strided (weight
 * gradients).  M, N >= 1, K >= 0.
 *   tile_m, tile_n  output tile of a workgroup
 *   wavefronts      wavefronts per workgroup
 *   ring            1: the LDS-ring kernel; 0: the small generic kernel
 *   k_splits        > 1: split-K with that many chunks, followed by the reduce kernel
 *   persistent      1: one workgroup per compute unit walks over the tiles
 *   pingpong        1: the K loop runs the ping-pong schedule (the two wavefronts of a SIMD alternate between
 *                   matrix instructions and LDS reads / DMA issue), 0: the default schedule
 * Errors: NTP_ERR_INVALID_ARG. */
typedef struct ntp_gemm_choice {
  int32_t tile_m, tile_n, wavefronts, ring, k_splits, persistent, pingpong;
} ntp_gemm_choice_t;
int ntp_gemm_choice(const ntp_handle_t* h, int32_t layout, int64_t M, int64_t N, int64_t K, ntp_gemm_choice_t* out);

/* Diagnostic aid (host only): launch decisions of the attention core kernels for a shape,
 * on this handle (its workspace and options at the time of the call).
 *   fwd_rows_per_wavefront  16 or 32 query rows per wavefront in the forward kernel
 *   fwd_parts, dq_parts, dkv_parts  > 1: every workgroup's walk is cut into that many parts
 *                                   (fp32 partial results in the workspace, merged by a second kernel)
 * Errors: as for ntp_attn_core_shard_fwd's shape checks. */
typedef struct ntp_attn_core_choice {
  int32_t fwd_rows_per_wavefront, fwd_parts, dq_parts, dkv_parts;
} ntp_attn_core_choice_t;
int ntp_attn_core_choice(const ntp_handle_t* h, const ntp_attn_core_shape_t* shape, ntp_attn_core_choice_t* out);

/* Measurement aid: a plain dense device-to-device copy of `bytes` bytes (dst, src:
 * device, 16-byte aligned, bytes % 16 == 0, not overlapping) by a kernel named
 * calibration_copy_kernel.  Its known traffic (bytes read, bytes written) is what
 * the profiler's HBM byte counters are scaled by when a kernel's traffic is reported. */
int ntp_calibration_copy(ntp_handle_t* h, void* dst, const void* src, int64_t bytes, void* stream);

/* Measurement aid (blocking; creates HIP events; launches on the default stream): what this device sustains,
 * at its power limit, on the two resources the GEMM kernels' inner loop uses, with no global memory traffic:
 * one workgroup of 8 wavefronts per compute unit runs a loop of
 *   NTP_PROBE_MFMA              64 bf16 16x16x32 matrix instructions per turn on pseudo-random operands
 *   NTP_PROBE_LDS_B128          24 conflict-free 128-bit LDS reads per turn
 *   NTP_PROBE_LDS_TR_B64        44 transposing 64-bit LDS reads per turn
 *   NTP_PROBE_MFMA_LDS_B128     64 matrix instructions + 24 128-bit reads (the mix of a K tile of the
 *                               K-contiguous GEMM kernels, per wavefront)
 *   NTP_PROBE_MFMA_LDS_TR_B64   56 matrix instructions + 44 transposing reads (weight-gradient kernels)
 * and, for the attention core (does the vector arithmetic of one wavefront's softmax hide behind another wavefront's
 * matrix instructions on the same SIMD?), with ONE wavefront per SIMD and kind:
 *   NTP_PROBE_MFMA_1WAVE        wavefronts 0-3: 32 matrix instructions per turn
 *   NTP_PROBE_SOFTMAX_1WAVE     wavefronts 4-7: per turn the vector work of 16 scores per lane (8 maxima, 16
 *                               multiply-adds, 16 exponentials, 16 additions), the other four idle
 *   NTP_PROBE_MFMA_AND_SOFTMAX  both at once: one wavefront of each kind per SIMD
 * scratch: DEVICE, at least compute_units * 2048 bytes, overwritten.  out (HOST): average milliseconds per
 * launch, matrix TFLOP/s of the whole device, LDS read GB/s per compute unit. */
#define NTP_PROBE_MFMA 0
#define NTP_PROBE_LDS_B128 1
#define NTP_PROBE_LDS_TR_B64 2
#define NTP_PROBE_MFMA_LDS_B128 3
#define NTP_PROBE_MFMA_LDS_TR_B64 4
#define NTP_PROBE_MFMA_1WAVE 5
#define NTP_PROBE_SOFTMAX_1WAVE 6
#define NTP_PROBE_MFMA_AND_SOFTMAX 7
typedef struct ntp_probe_result {
  double ms, tflops, lds_gbps_per_cu;
  int32_t mfma_per_turn, reads_per_turn;
} ntp_probe_result_t;
int ntp_probe_rates(ntp_handle_t* h, int32_t which, void* scratch, int64_t scratch_bytes, ntp_probe_result_t* out);

/* ---------------------------------------------------------------------------
 * For callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc) and so cannot give the
 * handle a workspace: ntp_attn_proj_shard_fwd with the split-K partial sums kept
 * in a static device array of NTP_STATIC_SCRATCH_BYTES that is part of the
 * library's code object (each GPU the library runs on holds it until the process
 * ends).  Arguments, results and errors as for ntp_attn_proj_shard_fwd; the
 * handle's own workspace is ignored.  The call allocates nothing and makes the same
 * launch decisions as ntp_attn_proj_shard_fwd would with a workspace of
 * NTP_STATIC_SCRATCH_BYTES, so results are bit-identical to that.  A shape whose
 * launches could use more room than that (ntp_workspace_bytes restricted to the
 * halves this call runs) returns NTP_ERR_SCRATCH_TOO_SMALL and launches nothing.
 * Every call on one GPU, through any handle, uses that GPU's one array: calls
 * that may overlap in time on a GPU race; order them on one stream or with events.
 * Nothing in the array has to be cleared between calls (every partial sum that is
 * read was written by the same call). */
#define NTP_STATIC_SCRATCH_BYTES (32 << 20)
int ntp_attn_proj_shard_fwd_static(ntp_handle_t* h, const ntp_attn_shape_t* shape, const void* X, int64_t ldx,
                                   const void* Wqkv, int64_t ldwqkv, void* QKV, int64_t ldqkv,
                                   const void* C, int64_t ldc, const void* Wo, int64_t ldwo, void* Zpart,
                                   int64_t ldz, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NTP_H_ */
