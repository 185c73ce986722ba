// bf16 MFMA GEMM family for the NTP shard layers (Sec. 3.1, Eq. 2-3 and 4, 6, and
// their chain-rule gradients): C[M x N] = op(A) op(B) with fp32 accumulation and a
// fused epilogue (bf16 store, GeLU, GeLU', fp32 store / accumulate).
//
// Any M, N, K is accepted: ragged shard widths show up as N (column-parallel
// forward), as K (row-parallel forward, dX) and as M (weight gradients).  Rows and
// columns past the edge are never stored; the K tail is zero-filled in LDS.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdint>
#include <cstring>
#include <type_traits>

#include "ntp_gemm_kernels.h"
#include "ntp_gemm_launch.h"
#include "ntp_internal.h"

namespace {

using namespace ntp_gemm;

template <typename F>
int dispatch_epilogue(int epi, F&& f) {
  switch (epi) {
    case ntp::EPI_BF16: return f(std::integral_constant<int, ntp::EPI_BF16>{});
    case ntp::EPI_GELU: return f(std::integral_constant<int, ntp::EPI_GELU>{});
    case ntp::EPI_DGELU: return f(std::integral_constant<int, ntp::EPI_DGELU>{});
    case ntp::EPI_F32: return f(std::integral_constant<int, ntp::EPI_F32>{});
    case ntp::EPI_F32_ACCUM: return f(std::integral_constant<int, ntp::EPI_F32_ACCUM>{});
    default: return NTP_ERR_INVALID_ARG;
  }
}

template <bool AKC, bool BKC>
int launch_generic(GemmArgs g, int epi, hipStream_t s) {
  g.tiles_m = (g.M + BM - 1) / BM;
  g.tiles_n = (g.n_store + BN - 1) / BN;
  if (int64_t(g.tiles_m) * g.tiles_n > 0x7fffffff) return NTP_ERR_UNSUPPORTED;
  const dim3 grid(uint32_t(g.tiles_m) * uint32_t(g.tiles_n)), block(256);
  return dispatch_epilogue(epi, [&](auto e) {
    hipLaunchKernelGGL((gemm_generic_kernel<AKC, BKC, decltype(e)::value>), grid, block, 0, s, g);
    return hipGetLastError() == hipSuccess ? NTP_OK : NTP_ERR_LAUNCH;
  });
}

// Relative throughput of one workgroup per tile shape at full occupancy, per operand layout (measured
// on large problems with operands streaming from HBM): smaller wavefront tiles read more LDS fragments
// per MFMA, smaller workgroup tiles move more bytes per flop, and the K-strided layouts pay two
// transposing reads per fragment (their 256 x 256 variant is also short of registers).
// The 4-wavefront 128 x 128 variant reaches its rate with two workgroups on a compute unit; alone on one
// (at most 256 tiles) it runs at kLoneSmallTileRate, where the 8-wavefront variant of the same tile is faster.
//                                             256x256 256x224 224x256 256x192 192x256 256x128 128x256 128x128 128x128w8
constexpr double kTileRate[3][kNumTileShapes] = {{1.000, 0.957, 0.969, 0.917, 0.923, 0.761, 0.754, 0.65, 0.53},   // A, B K-contiguous
                                                 {1.000, 0.929, 0.986, 0.908, 0.944, 0.770, 0.749, 0.65, 0.53},   // B K-strided
                                                 {1.100, 0.984, 1.000, 0.956, 0.962, 0.797, 0.779, 0.65, 0.53}};  // both K-strided (256x256: its non-persistent form)
constexpr double kLoneSmallTileRate = 0.43;

// Pick the tile shape with the least estimated time: the busiest compute unit's number of
// workgroups (they are dealt evenly; co-resident ones share its throughput) times tile area over rate.
int choose_tile(int64_t M, int64_t N, int layout, int cus) {
  int best = 0;
  double best_t = 1e300;
  for (int i = 0; i < kNumTileShapes; ++i) {
    const TileShape& ts = kTileShapes[i];
    const int64_t tiles = ((M + ts.bm - 1) / ts.bm) * ((N + ts.bn - 1) / ts.bn);
    const int64_t cu_load = (tiles + cus - 1) / cus;
    const double rate = ts.waves == 4 && tiles <= cus ? kLoneSmallTileRate : kTileRate[layout][i];
    const double t = double(cu_load) * ts.bm * ts.bn / rate;
    if (t < best_t) {
      best_t = t;
      best = i;
    }
  }
  return best;
}

void variant_name(int v, char* out, size_t n) {
  if (v < 0) snprintf(out, n, "generic128");
  else if (kTileShapes[v].bm == 128 && kTileShapes[v].bn == 128 && kTileShapes[v].waves == 8) snprintf(out, n, "128x128w8");
  else snprintf(out, n, "%dx%d", kTileShapes[v].bm, kTileShapes[v].bn);
}

// Variant used for a shape: -1 = generic kernel, else an index into kTileShapes.  The handle's
// NTP_OPT_GEMM_TILE overrides the choice (1: generic, 2 + i: tile shape i).
int choose_variant(const ntp_handle* h, const GemmArgs& g, bool ring_ok, int layout) {
  if (const int64_t f = h->opt[NTP_OPT_GEMM_TILE]) {
    if (!ring_ok || f == 1) return -1;
    if (f - 2 < kNumTileShapes) return int(f - 2);
  }
  // the generic 128x128x32 kernel only below two output tiles or two K tiles: from there on the ring kernel
  // measured faster (512 x 586 x 1024: 15 us against 31 us per GEMM)
  if (int64_t(g.M) * g.N < 128 * 128 * 2 || g.K < 128) return -1;
  if (!ring_ok) return -1;
  return choose_tile(g.M, g.n_store, layout, h->compute_units);
}

// (layout, epilogue) pairs the shard layers use have ring instantiations; anything else runs on
// the generic kernel
bool ring_combo(bool a_kc, bool b_kc, int epi) {
  if (a_kc && b_kc) return epi == ntp::EPI_BF16 || epi == ntp::EPI_GELU || epi == ntp::EPI_DGELU;
  if (a_kc && !b_kc) return epi == ntp::EPI_BF16;
  if (!a_kc && !b_kc) return epi == ntp::EPI_F32 || epi == ntp::EPI_F32_ACCUM;
  return false;
}

// ---- split-K ---------------------------------------------------------------------
// A column-parallel shard at a high TP degree is a skinny GEMM: few output tiles, long K.  With
// fewer tiles than compute units the K axis is cut as well: `splits` workgroups per tile store fp32
// partial sums to a caller-provided workspace, and a second kernel adds the slices in ascending
// order and applies the epilogue.
struct SplitChoice {
  int tile, splits, k_chunk;
};

constexpr double kTileCycles = 2650.0;      // one 256 x 256 x 64 K tile on one compute unit at rate 1
constexpr int kTileOverhead = 4;            // prologue and epilogue of an output tile, in K tiles
constexpr double kReduceBytesPerCycle = 2000.0, kReduceFixedCycles = 6000.0;
constexpr int kMaxSplits = 8, kMinSplitTiles = 8;

double tile_time(int64_t M, int64_t N, int64_t ktiles, int layout, int i, int splits, int cus) {
  const TileShape& ts = kTileShapes[i];
  const int64_t tiles = ((M + ts.bm - 1) / ts.bm) * ((N + ts.bn - 1) / ts.bn);
  const int64_t cu_load = (tiles * splits + cus - 1) / cus;
  const double rate = ts.waves == 4 && tiles <= cus ? kLoneSmallTileRate : kTileRate[layout][i];
  const int64_t kt = (ktiles + splits - 1) / splits + kTileOverhead;
  return double(cu_load) * double(kt) * kTileCycles * (ts.bm * ts.bn / 65536.0) / rate;
}

// Least estimated time over (tile shape, splits); splits == 1 means: leave the GEMM as it is.
// ws_bytes: room for the partial sums (0: never split).
SplitChoice choose_split(const ntp_handle* h, int64_t ws_bytes, int64_t M, int64_t N, int64_t K, int layout, int plain_tile,
                         int64_t ldw) {
  SplitChoice best{plain_tile, 1, 0};
  const int64_t ktiles = (K + 63) / 64;
  const int cus = h->compute_units;
  const int forced = int(h->opt[NTP_OPT_GEMM_SPLIT]);  // 1: never split; n > 1: n chunks if they fit
  const int64_t forced_tile = h->opt[NTP_OPT_GEMM_TILE];
  if (ws_bytes <= 0 || forced == 1) return best;
  // splitting has to beat the plain launch by a margin: the estimate is coarse
  double best_t = plain_tile >= 0 ? 0.85 * tile_time(M, N, ktiles, layout, plain_tile, 1, cus) : 1e300;
  if (forced > 1) best_t = 1e300;
  for (int i = 0; i < kNumTileShapes; ++i) {
    if (!kSplitTile[i]) continue;
    if (forced_tile >= 2 && forced_tile - 2 != i) continue;
    for (int sp = 2; sp <= kMaxSplits; ++sp) {
      if (forced > 1 && sp != forced) continue;
      const int64_t chunk_tiles = (ktiles + sp - 1) / sp;
      if (forced <= 1 && chunk_tiles < kMinSplitTiles) break;
      if ((sp - 1) * chunk_tiles * 64 >= K) continue;  // the last chunk would be empty
      if (int64_t(sp) * M * ldw * 4 > ws_bytes) break;
      const double reduce = kReduceFixedCycles + double(M) * double(N) * (4.0 * sp + 4.0) / kReduceBytesPerCycle;
      const double t = tile_time(M, N, ktiles, layout, i, sp, cus) + reduce;
      if (t < best_t) {
        best_t = t;
        best = SplitChoice{i, sp, int(chunk_tiles * 64)};
      }
    }
  }
  return best;
}

// Adds the partial-sum slices of a split-K launch and applies the GEMM's own epilogue.
template <int EPI>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmArgs g, const float* __restrict__ ws, int64_t slice,
                                                            int64_t ldw, int splits) {
  const int quads = g.n_store >> 2;  // n_store is a multiple of 4
  const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int64_t m = idx / quads;
  if (m >= g.M) return;
  const int n0 = int(idx - m * quads) * 4;
  const float* p = ws + m * ldw + n0;
  f32x4 acc = *reinterpret_cast<const f32x4*>(p);
  for (int s = 1; s < splits; ++s) acc = acc + *reinterpret_cast<const f32x4*>(p + s * slice);
  store4<EPI>(g, int(m), n0, acc);
}

// Kernel variant (-1 generic, else a tile shape) and K chunks for a GEMM (g: M, N, K, n_store).
SplitChoice plan_gemm(const ntp_handle* h, int64_t ws_bytes, const GemmArgs& g, int layout, bool ring_ok, bool split_ok,
                      int64_t ldw) {
  SplitChoice sc{choose_variant(h, g, ring_ok, layout), 1, 0};
  if (split_ok && int64_t(g.M) * g.N >= 128 * 128 * 8) sc = choose_split(h, ws_bytes, g.M, g.n_store, g.K, layout, sc.tile, ldw);
  return sc;
}

// Which schedule of the K loop a persistent ring launch gets (tile shapes 0-6 have both).  Under the board's power
// limit the two run within a few percent of each other (with all-zero operands, which draw little switching power,
// the ping-pong schedule is 6 % faster).  Measured in the GPT-3-shape step: ping-pong +1-4 % where both operands are
// K-contiguous, -1-8 % where one or both are K-strided (their transposing reads make the memory slots longer), with
// two exceptions: the weight-gradient layout on the 224 x 256 and 256 x 224 tiles, +2.5 %, whose ping-pong kernels also
// need no scratch memory (the default schedule spills 10 and 21 registers there), and the row-parallel layout at short
// K (fc2 / dX of a narrow shard: 8192 x 16384 over K = 750 runs 200-207 us against 215-221 us on the 256 x 256 tile).
// NTP_OPT_GEMM_SCHEDULE: 1 forces the default schedule, 2 the ping-pong schedule.
bool use_pingpong(const ntp_handle* h, int layout, int variant, int64_t K) {
  if (variant < 0 || variant > 6) return false;
  const int64_t f = h->opt[NTP_OPT_GEMM_SCHEDULE];
  if (f == 1) return false;
  if (f == 2) return true;
  return layout == 0 || (layout == 2 && (variant == 1 || variant == 2)) || (layout == 1 && K <= 1024);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

namespace ntp {

int64_t gemm_workspace_wish(const ntp_handle* h, int layout, int64_t M, int64_t N, int64_t n_store, int64_t K) {
  if (M < 1 || N < 1 || K < 1 || M > 0x7fffff00 || N > 0x7fffff00 || K > 0x7fffff00) return 0;
  GemmArgs g{};
  g.M = int32_t(M);
  g.N = int32_t(N);
  g.K = int32_t(K);
  g.n_store = int32_t(n_store);
  const int64_t ldw = (n_store + 15) / 16 * 16;
  const SplitChoice sc = plan_gemm(h, INT64_MAX / 2, g, layout, true, true, ldw);
  return sc.splits > 1 ? int64_t(sc.splits) * M * ldw * 4 : 0;
}

int gemm_launch(ntp_handle* h, const GemmDesc& d, void* stream) {
  if (!h || d.M < 0 || d.N < 0 || d.K < 0) return NTP_ERR_INVALID_ARG;
  if (d.M == 0 || d.N == 0) return NTP_OK;
  if (h->device < 0) return NTP_ERR_NO_DEVICE;
  if (d.M > 0x7fffff00 || d.N > 0x7fffff00 || d.K > 0x7fffff00) return NTP_ERR_UNSUPPORTED;
  const bool to_segs = d.n_segs > 0;
  if ((!d.C && !to_segs) || (d.K > 0 && (!d.A || !d.B))) return NTP_ERR_INVALID_ARG;
  const bool f32_out = d.epilogue == EPI_F32 || d.epilogue == EPI_F32_ACCUM;
  if (d.epilogue == EPI_GELU && !d.C2) return NTP_ERR_INVALID_ARG;
  if (d.epilogue == EPI_DGELU && !d.AUX) return NTP_ERR_INVALID_ARG;

  // extents along the contiguous axis of each operand, and alignment of every 16-byte access
  const int64_t a_cols = d.a_kc ? d.K : d.M, b_cols = d.b_kc ? d.K : d.N;
  if (d.K > 0) {
    if (d.lda < a_cols || d.ldb < b_cols) return NTP_ERR_INVALID_ARG;
    if (!aligned16(d.A) || !aligned16(d.B) || d.lda % 8 || d.ldb % 8) return NTP_ERR_ALIGNMENT;
  }
  int64_t n_store = d.N;
  if (f32_out) {
    if (d.N % 4) return NTP_ERR_ALIGNMENT;
    if (!to_segs && (!aligned16(d.C) || d.ldc % 4)) return NTP_ERR_ALIGNMENT;
  } else {
    if (to_segs) return NTP_ERR_INVALID_ARG;
    if (d.zero_pad_n) n_store = d.pad_n_64 ? (d.N + 63) / 64 * 64 : (d.N + 7) / 8 * 8;
    if (n_store % 4) return NTP_ERR_ALIGNMENT;
    if (!aligned16(d.C) || d.ldc % 8) return NTP_ERR_ALIGNMENT;
    if (d.epilogue == EPI_GELU && (!aligned16(d.C2) || d.ldc2 % 8 || d.ldc2 < n_store)) return NTP_ERR_ALIGNMENT;
    if (d.epilogue == EPI_DGELU && (!aligned16(d.AUX) || d.ldaux % 8 || d.ldaux < n_store)) return NTP_ERR_ALIGNMENT;
  }
  if (!to_segs && d.ldc < n_store) return NTP_ERR_INVALID_ARG;

  GemmArgs g{};
  if (to_segs) {
    // destinations of the output rows: inside [0, M), aligned, wide enough, not overlapping in memory
    // (a row that no segment lists is not stored)
    if (!d.segs || d.n_segs < 0) return NTP_ERR_INVALID_ARG;
    if (d.n_segs > kMaxRowSegs) return NTP_ERR_UNSUPPORTED;
    for (int32_t i = 0; i < d.n_segs; ++i) {
      const ntp_row_segment_t& r = d.segs[i];
      if (r.row_begin < 0 || r.rows < 0 || r.row_begin + r.rows > d.M) return NTP_ERR_INVALID_ARG;
      if (r.rows == 0) continue;
      if (!r.dst || r.ld < d.N) return NTP_ERR_INVALID_ARG;
      if (!aligned16(r.dst) || r.ld % 4) return NTP_ERR_ALIGNMENT;
      const uintptr_t lo = reinterpret_cast<uintptr_t>(r.dst), hi = lo + uintptr_t(((r.rows - 1) * r.ld + d.N) * 4);
      for (int32_t j = 0; j < g.n_segs; ++j) {
        const uintptr_t lo2 = reinterpret_cast<uintptr_t>(g.seg[j].ptr);
        const uintptr_t hi2 = lo2 + uintptr_t(((int64_t(g.seg[j].end - g.seg[j].begin) - 1) * g.seg[j].ld + d.N) * 4);
        if (lo < hi2 && lo2 < hi) return NTP_ERR_INVALID_ARG;
      }
      g.seg[g.n_segs].begin = int32_t(r.row_begin);
      g.seg[g.n_segs].end = int32_t(r.row_begin + r.rows);
      g.seg[g.n_segs].ptr = r.dst;
      g.seg[g.n_segs].ld = r.ld;
      ++g.n_segs;
    }
    if (g.n_segs == 0) return NTP_OK;  // no row has a destination: nothing to compute
  }
  g.A = static_cast<const uint16_t*>(d.A);
  g.B = static_cast<const uint16_t*>(d.B);
  g.C = d.C;
  g.C2 = d.C2;
  g.AUX = static_cast<const uint16_t*>(d.AUX);
  g.lda = d.lda;
  g.ldb = d.ldb;
  g.ldc = d.ldc;
  g.ldc2 = d.ldc2;
  g.ldaux = d.ldaux;
  g.M = int32_t(d.M);
  g.N = int32_t(d.N);
  g.K = int32_t(d.K);
  g.n_store = int32_t(n_store);
  g.gelu_mode = d.gelu_mode;
  hipStream_t s = static_cast<hipStream_t>(stream);
  static const char* const kEpiName[] = {"bf16", "gelu", "dgelu", "f32", "f32acc"};
  // the ring kernel addresses each operand with 32-bit byte offsets from its base
  const int64_t a_rows = d.a_kc ? d.M : d.K, b_rows = d.b_kc ? d.N : d.K;
  const bool ring_ok = ring_combo(d.a_kc, d.b_kc, d.epilogue) && a_rows * d.lda * 2 < (int64_t(1) << 32) &&
                       b_rows * d.ldb * 2 < (int64_t(1) << 32);
  const int layout = d.a_kc ? (d.b_kc ? 0 : 1) : 2;
  // K tail through the ring (row-parallel layout; K is the ragged shard width): B's lines past K lie past its
  // extent and read as zeros, A's columns past K are zeros by the caller's word.  NTP_OPT_GEMM_NO_RING_TAIL
  // switches it off (tests, tuning).
  if (layout == 1 && ring_ok && d.a_k_pad_64 && d.K % 64 != 0 && d.K >= 128 && d.lda >= (d.K + 63) / 64 * 64 &&
      !h->opt[NTP_OPT_GEMM_NO_RING_TAIL])
    g.ring_tail = 1;
  // what the DMA loads are range-checked against (< 4 GiB when ring_ok)
  g.a_extent = uint32_t(std::min<int64_t>(0xFFFFFFFFll, operand_extent_bytes(d.a_kc, d.M, d.K, d.lda, g.ring_tail != 0)));
  g.b_extent = uint32_t(std::min<int64_t>(0xFFFFFFFFll, operand_extent_bytes(d.b_kc, d.N, d.K, d.ldb, false)));
  g.resident = h->compute_units;
  if (const int64_t cap = h->opt[NTP_OPT_GEMM_WORKGROUPS]) g.resident = int32_t(std::min<int64_t>(cap, h->compute_units));
  // split-K: any (layout, epilogue) whose operands the ring kernel can address, except B K-contiguous
  // with A K-strided (no ring kernel)
  const bool split_ok = a_rows * d.lda * 2 < (int64_t(1) << 32) && b_rows * d.ldb * 2 < (int64_t(1) << 32) && (d.a_kc || !d.b_kc);
  const int64_t ldw = (n_store + 15) / 16 * 16;
  void* const ws_ptr = d.ws_override ? d.ws_override : h->workspace;
  const int64_t ws_bytes = d.ws_override ? d.ws_override_bytes : (h->workspace ? h->workspace_bytes : 0);
  const SplitChoice sc = plan_gemm(h, ws_ptr ? ws_bytes : 0, g, layout, ring_ok, split_ok, ldw);
  const int variant = sc.tile;
  if (ntp::timing_on(h)) {
    char name[48], vn[16], sn[8] = "";
    variant_name(variant, vn, sizeof(vn));
    if (sc.splits > 1) snprintf(sn, sizeof(sn), "k%d", sc.splits);
    const bool pp = sc.splits == 1 && use_pingpong(h, layout, variant, d.K) && !(layout == 2 && variant == 0 && ring_ok);
    snprintf(name, sizeof(name), "gemm_%c%c_%s_%s%s%s", d.a_kc ? 'n' : 't', d.b_kc ? 't' : 'n', kEpiName[d.epilogue], vn, sn,
             pp ? "pp" : "");
    ntp::timing_begin(h, stream, name, 2.0 * double(d.M) * double(d.N) * double(d.K), 0.0);
  }
  int st;
  if (layout == 2 && variant == 0 && sc.splits == 1 && ring_ok) {
    // The 256 x 256 weight-gradient tile runs one workgroup per output tile: its persistent form is short of
    // registers (27 spilled, some inside the K loop) and measured 17 % slower (307 against 254 us at
    // 5376 x 12288 x 2048), more than the overlap of one tile's stores with the next tile's first loads gains.
    GemmArgs gp = g;
    gp.k_splits = 1;
    gp.k_chunk = int32_t((d.K + 63) / 64 * 64);
    st = launch_ring_split_tn(gp, d.epilogue, variant, s);
  } else if (sc.splits > 1) {
    GemmArgs gp = g;  // the partial-sum launch: fp32 to the workspace, no row segments
    gp.ring_tail = 0;
    gp.a_extent = uint32_t(operand_extent_bytes(d.a_kc, d.M, d.K, d.lda, false));
    gp.C = ws_ptr;
    gp.ldc = ldw;
    gp.n_segs = 0;
    gp.k_splits = sc.splits;
    gp.k_chunk = sc.k_chunk;
    gp.split_stride = int64_t(d.M) * ldw;
    if (d.a_kc && d.b_kc) st = launch_ring_split_nt(gp, variant, s);
    else if (d.a_kc) st = launch_ring_split_nn(gp, variant, s);
    else st = launch_ring_split_tn(gp, EPI_F32, variant, s);
    if (st == NTP_OK) {
      const int64_t threads = int64_t(d.M) * (n_store / 4);
      const dim3 grid(uint32_t((threads + 255) / 256)), block(256);
      const float* ws = static_cast<const float*>(ws_ptr);
      st = dispatch_epilogue(d.epilogue, [&](auto e) {
        hipLaunchKernelGGL((splitk_reduce_kernel<decltype(e)::value>), grid, block, 0, s, g, ws, gp.split_stride, ldw, sc.splits);
        return hipGetLastError() == hipSuccess ? NTP_OK : NTP_ERR_LAUNCH;
      });
    }
  } else if (use_pingpong(h, layout, variant, d.K)) {
    if (d.a_kc && d.b_kc) st = launch_pp_nt(g, d.epilogue, variant, s);
    else if (d.a_kc) st = launch_pp_nn(g, d.epilogue, variant, s);
    else st = launch_pp_tn(g, d.epilogue, variant, s);
  } else if (variant >= 0) {
    if (d.a_kc && d.b_kc) st = launch_ring_nt(g, d.epilogue, variant, s);
    else if (d.a_kc) st = launch_ring_nn(g, d.epilogue, variant, s);
    else st = launch_ring_tn(g, d.epilogue, variant, s);
  } else if (d.a_kc && d.b_kc) st = launch_generic<true, true>(g, d.epilogue, s);
  else if (d.a_kc && !d.b_kc) st = launch_generic<true, false>(g, d.epilogue, s);
  else if (!d.a_kc && !d.b_kc) st = launch_generic<false, false>(g, d.epilogue, s);
  else st = launch_generic<false, true>(g, d.epilogue, s);
  ntp::timing_end(h, stream);
  return st;
}

}  // namespace ntp

extern "C" int ntp_gemm_choice(const ntp_handle_t* h, int32_t layout, int64_t M, int64_t N, int64_t K, ntp_gemm_choice_t* out) {
  if (!h || !out || layout < 0 || layout > 2 || M < 1 || N < 1 || K < 0 || M > 0x7fffff00 || N > 0x7fffff00 || K > 0x7fffff00)
    return NTP_ERR_INVALID_ARG;
  GemmArgs g{};
  g.M = int32_t(M);
  g.N = int32_t(N);
  g.K = int32_t(K);
  g.n_store = int32_t((N + 7) / 8 * 8);
  const SplitChoice sc = plan_gemm(h, h->workspace ? h->workspace_bytes : 0, g, layout, true, true, (g.n_store + 15) / 16 * 16);
  *out = ntp_gemm_choice_t{};
  out->k_splits = sc.splits;
  if (sc.tile < 0) {
    out->tile_m = out->tile_n = 128;
    out->wavefronts = 4;
    out->ring = 0;
  } else {
    out->tile_m = kTileShapes[sc.tile].bm;
    out->tile_n = kTileShapes[sc.tile].bn;
    out->wavefronts = kTileShapes[sc.tile].waves;
    out->ring = 1;
  }
  out->persistent = sc.tile >= 0 && sc.splits == 1 && !(layout == 2 && sc.tile == 0) ? 1 : 0;
  out->pingpong = out->persistent && use_pingpong(h, layout, sc.tile, K) ? 1 : 0;
  return NTP_OK;
}
