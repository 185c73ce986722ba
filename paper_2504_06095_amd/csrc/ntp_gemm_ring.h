// Main bf16 MFMA GEMM kernel of the NTP shard layers.  Included by ntp_gemm.hip.
//
// Tile BM x BN x 64, WGM x WGN wavefronts, each computing (BM/WGM) x (BN/WGN) with
// 16x16x32 bf16 MFMAs and fp32 accumulators.  Operands go global -> LDS by direct
// (DMA) loads, 16 bytes per lane, no staging registers.
//
// LDS is a ring of FIVE operand slots (one operand of one K tile each, 5 x 32 KiB for
// 256-row operands).  K tile t keeps A in slot 2t mod 5 and B in slot 2t+1 mod 5, so
// while tile t is being multiplied, tile t+1 is complete or landing and A of tile t+2
// already streams into the fifth slot.  A DMA instruction is issued only every few
// MFMAs (the vector memory pipeline takes one 1 KiB instruction per ~18 cycles per
// compute unit; a burst stalls the issuing wavefronts, a trickle does not), and each
// has between one and two tile times to land.
//
// LDS layout of one slot (16-byte chunks stay whole; a wavefront's DMA instruction
// fills 64 consecutive chunks, so bank spreading is done by permuting chunks):
//   K-contiguous operand  [R rows][64 k]:  chunk p of row r holds k-chunk  p ^ ((r >> 1) & 7)
//   K-strided operand     [64 k][R rows]:  chunk p of line k holds row-chunk
//                                          p ^ (2 * ((k & 3) | ((k >> 3) & 1) << 2))
// Fragments come out of LDS in MFMA operand layout (lane l: row l & 15, k 8 (l >> 4) + 0..7
// of a K-step of 32) with one ds_read_b128 (K-contiguous) or two transposing 64-bit
// reads (K-strided).
//
// Pipeline: a K tile is two K-steps of 32; each K-step is split in two halves by A rows.
// While the MFMAs of one half issue, the A fragments of the next half (and, every other
// half, the B fragments of the next K-step) are read.  One barrier per K tile, placed in
// the last half: by then every wavefront has read all its fragments of the tile, and has
// waited for its own DMA instructions of the next tile.
#ifndef NTP_GEMM_RING_H_
#define NTP_GEMM_RING_H_

#include <type_traits>

#include "ntp_gemm_addr.h"
#include "ntp_gemm_kernels.h"

namespace ntp_gemm {

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_cvoid;

constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }       // s_waitcnt vmcnt(n) alone
constexpr int vmcnt_lgkm0_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0070; }  // s_waitcnt vmcnt(n) lgkmcnt(0)
constexpr int lgkm0_imm() { return vmcnt_lgkm0_imm(63); }                               // s_waitcnt lgkmcnt(0) alone

// One operand (R rows of the tile, rounded up to a multiple of 64) as seen by the DMA.
template <bool KC, int R, int NW>
struct DmaOperand {
  static_assert(R % 64 == 0, "the DMA moves operands in units of 64 rows");
  static constexpr int SLOT = R * DK;                   // elements per slot
  static constexpr int NINST = R * DK * 2 / 1024 / NW;  // DMA instructions per wavefront per K tile
  static_assert((R * DK * 2 / 1024) % NW == 0, "operand must split evenly over the wavefronts");
  static constexpr int CPL = R / 8;                     // chunks per k line (K-strided layout)
  static_assert(KC || (CPL >= 16 && (CPL & (CPL - 1)) == 0), "K-strided operands: 128 or 256 rows");

  uint32_t off[NINST];  // byte offset (from the operand base at K tile 0) of this lane's chunk per instruction

  // chunk position `pos` of a slot -> (line, chunk) it holds; see the layout above
  __device__ __forceinline__ static void slot_src(int pos, int& line, int& chunk) { ntp_gemm::slot_src<KC, R>(pos, line, chunk); }

  // row0: first row of the tile, lim: extent of the operand's non-K dimension
  __device__ __forceinline__ void init(int64_t ld, int row0, int lim, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NINST; ++i) {
      int line, chunk;
      slot_src((wave * NINST + i) * 64 + lane, line, chunk);
      off[i] = dma_offset<KC>(ld, row0, lim, line, chunk);
    }
  }

  // start DMA instruction i (0 .. NINST-1) of K tile kt into `slot`: a buffer load whose scalar
  // offset walks along K, so that no vector ALU work is spent on addresses
  __device__ __forceinline__ void dma(__amdgpu_buffer_rsrc_t rsrc, uint32_t kstep_bytes, int kt, uint16_t* slot, int wave,
                                      int i) const {
    uint16_t* dst = slot + (wave * NINST + i) * 512;  // 64 chunks of 8 elements, wave-uniform
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)dst, 16, off[i], uint32_t(kt) * kstep_bytes, 0, 0);
  }

  // Byte offset (from the start of a K tile of this operand) of the 128-byte line that `lane` touches
  // when a wavefront pulls quarter `part` (0..3) of the tile's 256 lines toward L2.
  __device__ __forceinline__ static uint32_t prefetch_offset(int64_t ld, int row0, int lim, int part, int lane) {
    if constexpr (KC) {
      const int row = min(row0 + part * 64 + lane, lim - 1);
      return uint32_t(int64_t(row) * ld * 2);
    } else {
      const int line = part * 16 + (lane >> 2);
      const int cb = min(row0 * 2 + (lane & 3) * 128, (lim * 2 - 4) & ~3);
      return uint32_t(int64_t(line) * ld * 2 + cb);
    }
  }

  // K tail tile through registers: everything at k >= K becomes zero
  __device__ __forceinline__ void tail(const uint16_t* base, int64_t kstep, int kt, int K, uint16_t* slot, int wave,
                                       int lane) const {
    const char* tile = reinterpret_cast<const char*>(base + int64_t(kt) * kstep);
#pragma unroll
    for (int i = 0; i < NINST; ++i) {
      const int pos = (wave * NINST + i) * 64 + lane;
      int line, chunk;
      slot_src(pos, line, chunk);
      u16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
      if constexpr (KC) {
        const int k = kt * DK + chunk * 8;
        if (k < K) {
          val = *reinterpret_cast<const u16x8*>(tile + off[i]);
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (k + j >= K) val[j] = 0;
        }
      } else {
        if (kt * DK + line < K) val = *reinterpret_cast<const u16x8*>(tile + off[i]);
      }
      *reinterpret_cast<u16x8*>(slot + pos * 8) = val;
    }
  }
};

// per-lane LDS element offsets of the fragments of one operand (16 rows x 32 k per fragment)
template <bool KC, int R, int NF>
struct FragAddr {
  uint32_t o[KC ? 2 : NF];
  __device__ __forceinline__ void init(int rbase, int lane) {
    if constexpr (KC) {
      // k-chunk of K-step ks is 4 ks + (l >> 4); its position in the row is that ^ ((row >> 1) & 7),
      // the same for rows 16 apart
      const int r = rbase + (lane & 15);
      const int sw = (r >> 1) & 7;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) o[ks] = uint32_t(r * DK + (((ks * 4 + (lane >> 4)) ^ sw) * 8));
    } else {
      // transposing read: in each 16-lane group g, lane s points at 4 consecutive rows of k line
      // 8 g + (s >> 2); the group hands lane L the 4 k-values of row L.  A second read 4 lines
      // further down completes the 8 k-values.
      const int g = lane >> 4, s = lane & 15;
      const int k = 8 * g + (s >> 2);  // + 32 ks (+ 4 for the second read): neither changes kline_swz
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        const int col = rbase + i * 16 + (s & 3) * 4;
        o[i] = uint32_t(k * R + (((col >> 3) ^ kline_swz(k)) * 8) + (col & 7));
      }
    }
  }
  __device__ __forceinline__ bf16x8 read(const uint16_t* slot, int i, int ks) const {
    if constexpr (KC) {
      return *reinterpret_cast<const bf16x8*>(slot + o[ks] + i * 16 * DK);
    } else {
      typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
      const uint16_t* p = slot + o[i] + ks * 32 * R;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * R));
      const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, both);
    }
  }
};

template <int I>
using Int = std::integral_constant<int, I>;

// SPLIT: the non-persistent form, one workgroup per unit of work.  The K axis is cut into g.k_splits
// chunks of g.k_chunk (a multiple of the K tile; the last chunk takes what is left).  The grid holds
// k_splits groups of round_up(tiles, 8) workgroups; group s computes every output tile over chunk s.
// With several chunks the fp32 partial sums go to slice s of a workspace (g.C + s * g.split_stride
// floats, rows of g.ldc); with one chunk the tile gets its normal epilogue.  Without the cross-tile state
// of the persistent loop this form needs about 30 registers less.
template <bool AKC, bool BKC, int EPI, int BM_, int BN_, int WGM, int WGN, bool SPLIT = false>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_ring_kernel(const GemmArgs g) {
  static_assert(!SPLIT || EPI == ntp::EPI_F32 || EPI == ntp::EPI_F32_ACCUM, "partial sums are stored as fp32");
  constexpr int NW = WGM * WGN;
  constexpr int TM = BM_ / WGM, TN = BN_ / WGN;  // wavefront tile
  constexpr int MI = TM / 16, NI = TN / 16;      // 16 x 16 accumulator blocks
  static_assert(TM % 16 == 0 && TN % 16 == 0 && MI >= 2, "wavefront tile: 16 x 16 blocks, at least two block rows");
  constexpr int MH = (MI + 1) / 2;               // block rows in the first half of a K-step
  // rows moved per operand and K tile: whole DMA instructions; a K-strided slot line must hold a
  // power-of-two number of chunks for its chunk permutation (rows past the tile are never read)
  constexpr int RA = slot_rows(AKC, BM_), RB = slot_rows(BKC, BN_);
  static_assert(BM_ <= 256 && BN_ <= 256, "tile sides up to 256");
  using OpA = DmaOperand<AKC, RA, NW>;
  using OpB = DmaOperand<BKC, RB, NW>;
  constexpr int NA = OpA::NINST, NB = OpB::NINST;
  static_assert(NA <= 4 && NB <= 4, "the DMA schedule places at most 4 instructions per operand and tile");
  constexpr int SLOT = (RA > RB ? RA : RB) * DK;
  // distinct objects, so that the compiler can tell which DMA a fragment read depends on
  __shared__ __attribute__((aligned(1024))) uint16_t r0[SLOT];
  __shared__ __attribute__((aligned(1024))) uint16_t r1[SLOT];
  __shared__ __attribute__((aligned(1024))) uint16_t r2[SLOT];
  __shared__ __attribute__((aligned(1024))) uint16_t r3[SLOT];
  __shared__ __attribute__((aligned(1024))) uint16_t r4[SLOT];
  auto slot = [&](auto idx) -> uint16_t* {
    constexpr int i = decltype(idx)::value;
    if constexpr (i == 0) return r0;
    else if constexpr (i == 1) return r1;
    else if constexpr (i == 2) return r2;
    else if constexpr (i == 3) return r3;
    else return r4;
  };

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  // The kernel is persistent: workgroup w works on virtual blocks w, w + gridDim, ...  Workgroups are
  // dealt round-robin to the 8 XCDs (each with its own L2), so virtual block v belongs to XCD v & 7
  // (the grid is a multiple of 8 whenever a workgroup gets more than one block); every XCD walks a
  // contiguous range of tiles in groups of 8 tile rows, so that its workgroups share operands.
  const int nblk = g.tiles_m * g.tiles_n;
  struct TilePos {
    int tile_m, tile_n, row0, col0;
  };
  auto place = [&](int v) {
    const ntp_gemm::TilePos t = place_tile(v, g.tiles_m, g.tiles_n);
    return TilePos{t.tile_m, t.tile_n, t.tile_m * BM_, t.tile_n * BN_};
  };
  int vblk = blockIdx.x;
  int split = 0;
  if constexpr (SPLIT) {
    const int per_split = (nblk + 7) & ~7;  // keeps (workgroup index & 7) == (tile index & 7)
    split = blockIdx.x / per_split;
    vblk = blockIdx.x - split * per_split;
    if (vblk >= nblk) return;  // padding workgroup (the whole workgroup leaves, before any barrier)
  }
  // this workgroup's share of the K axis: everything below addresses the operands from opA / opB
  const int64_t k_first = SPLIT ? int64_t(split) * g.k_chunk : 0;
  const int K = SPLIT ? min(g.k_chunk, g.K - int(k_first)) : g.K;
  const uint16_t* const opA = g.A + (AKC ? k_first : k_first * g.lda);
  const uint16_t* const opB = g.B + (BKC ? k_first : k_first * g.ldb);
  TilePos pos = place(vblk);
  int row0 = pos.row0, col0 = pos.col0;

  f32x4 acc[MI][NI];
  OpA a;
  OpB b;
  const int64_t astep = AKC ? DK : DK * g.lda, bstep = BKC ? DK : DK * g.ldb;  // elements per K tile
  // Buffer views of the operands for the DMA, each ending where the operand ends (the host checks that an
  // operand spans < 4 GiB and passes the bytes from g.A / g.B on; a K chunk's view starts later and is that much
  // shorter).  The range check of a buffer load covers vector + scalar offset, and what lies past the extent
  // reads as zeros: no offset this kernel can form reaches memory outside the operands.
  constexpr bool RT = AKC && !BKC && !SPLIT;
  const uint32_t a_shift = uint32_t((AKC ? k_first : k_first * g.lda) * 2), b_shift = uint32_t((BKC ? k_first : k_first * g.ldb) * 2);
  const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(opA), 0, int(g.a_extent - a_shift), 0x00020000);
  const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(opB), 0, int(g.b_extent - b_shift), 0x00020000);
  const uint32_t astep_b = uint32_t(astep) * 2, bstep_b = uint32_t(bstep) * 2;
  FragAddr<AKC, RA, MI> fra;
  FragAddr<BKC, RB, NI> frb;
  fra.init(wm * TM, lane);
  frb.init(wn * TN, lane);

  const int nfull = K / DK;  // complete K tiles: all go through the ring
  // The K tail goes through the ring as one more tile when the host says that both operands read as zeros
  // past K there (g.ring_tail); otherwise it is loaded through registers after the loop.
  const bool ring_tail = RT && g.ring_tail != 0 && nfull * DK < K;
  const int nk = nfull + (ring_tail ? 1 : 0);

  // L2 prefetch, PFD tiles ahead.  An A tile is shared by the workgroups of this XCD that have the
  // same tile_m (about four, with different tile_n), a B tile by those with the same tile_n (eight
  // tile rows), so they take turns by K tile: wavefronts 0-3 touch the whole A tile when
  // (kt & 3) == (tile_n & 3), wavefronts 4-7 the whole B tile when (kt & 7) == (tile_m & 7): one
  // 4-byte load per 128-byte line.  The DMA instructions issued one to two tiles later then find
  // their lines in L2 instead of waiting for HBM.  Tiles nobody's turn covers are not prefetched.
  // Every wavefront issues the load in every tile (off turn: all lanes read the operand's first
  // word), so that the instruction counts the waits rely on stay static, and the loaded value lands
  // in a register that nothing else ever uses.
  constexpr int PFD = 4;
  constexpr bool PF_ON = NW == 8;
  uint32_t pf_sink = 0;
  const bool pf_is_a = wave < 4;
  const int pf_mask = pf_is_a ? 3 : 7;
  const bool pf_ok = pf_is_a ? (AKC || g.M >= 2) : (BKC || g.N >= 2);
  const char* const pf_base = reinterpret_cast<const char*>(pf_is_a ? opA : opB);
  const int64_t pf_step = (pf_is_a ? astep : bstep) * 2;  // bytes per K tile
  int pf_turn = 0, pf_turn_next = -1;  // -1: there is no next output tile
  uint32_t pf_voff = 0, pf_voff_next = 0;
  auto pf_params = [&](const TilePos& p, int& turn, uint32_t& voff) {
    turn = pf_is_a ? (p.tile_n & 3) : (p.tile_m & 7);
    voff = pf_is_a ? OpA::prefetch_offset(g.lda, p.row0, g.M, wave & 3, lane)
                   : OpB::prefetch_offset(g.ldb, p.col0, g.N, wave & 3, lane);
  };
  // per output tile: DMA offsets and prefetch parameters
  auto setup_tile = [&] {
    a.init(g.lda, row0, g.M, wave, lane);
    b.init(g.ldb, col0, g.N, wave, lane);
    pf_params(pos, pf_turn, pf_voff);
  };
  setup_tile();
  // K tile t + PFD of this output tile, or, past its end, the first K tiles of the next output tile
  auto prefetch = [&](int t) {
    const int tp = t + PFD;
    const bool own = tp < nfull;
    const int kp = own ? tp : tp - nfull;
    const int want = own ? pf_turn : pf_turn_next;
    const bool turn = kp < nfull && ((kp & pf_mask) == want) && pf_ok;
    const char* src = turn ? pf_base + int64_t(kp) * pf_step : pf_base;
    const uint32_t voff = turn ? (own ? pf_voff : pf_voff_next) : 0u;
    asm volatile("global_load_dword %0, %1, %2" : "+v"(pf_sink) : "v"(voff), "s"(src) : "memory");
  };

  constexpr int RDA = AKC ? 1 : 2, RDB = BKC ? 1 : 2;  // LDS read instructions per fragment
  bf16x8 fa[2][MH], fb[2][NI];
  // A fragments of half h (block rows h MH ...) of K-step ks -> fa[h]
  auto read_a = [&](int h, const uint16_t* pa, int ks) {
#pragma unroll
    for (int i = 0; i < (h ? MI - MH : MH); ++i) fa[h][i] = fra.read(pa, h * MH + i, ks);
  };
  auto read_b = [&](int buf, const uint16_t* pb, int ks) {
#pragma unroll
    for (int j = 0; j < NI; ++j) fb[buf][j] = frb.read(pb, j, ks);
  };
  // MFMAs n0 .. n1-1 of half h (row-major over its block rows x NI); operands swapped so that each
  // lane ends up with 4 consecutive columns of one row
  auto mfma_range = [&](int h, int bbuf, int n0, int n1) {
#pragma unroll
    for (int n = n0; n < n1; ++n) {
      const int i = n / NI, j = n % NI;
      acc[h * MH + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[bbuf][j], fa[h][i], acc[h * MH + i][j], 0, 0, 0);
    }
  };
  // One half of a K-step: `reads` (NR LDS instructions) go out under the first MFMA; up to two
  // DMA instructions sit at one third and two thirds of the MFMAs.
  auto half = [&](auto hh, auto bb, auto nr, auto&& reads, auto&& dma0, auto&& dma1) {
    constexpr int h = decltype(hh)::value, bbuf = decltype(bb)::value, NR = decltype(nr)::value;
    constexpr int nm = (h ? MI - MH : MH) * NI;
    constexpr int n1 = nm / 3 > 0 ? nm / 3 : 1, n2 = 2 * nm / 3 > n1 ? 2 * nm / 3 : n1;
    __builtin_amdgcn_sched_barrier(0);
    reads();
    mfma_range(h, bbuf, 0, n1);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, NR, 0);
    if constexpr (n1 > 1) __builtin_amdgcn_sched_group_barrier(0x008, n1 - 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    dma0();
    __builtin_amdgcn_sched_barrier(0);
    mfma_range(h, bbuf, n1, n2);
    __builtin_amdgcn_sched_barrier(0);
    dma1();
    __builtin_amdgcn_sched_barrier(0);
    mfma_range(h, bbuf, n2, nm);
    __builtin_amdgcn_sched_barrier(0);
  };
  constexpr int NRA0 = MH * RDA, NRA1 = (MI - MH) * RDA, NRB = NI * RDB;

  // The two operands play different parts in the DMA schedule: A is requested two tiles ahead ("long",
  // L below), B one tile ahead ("short", S).
  // K tile t, P = t mod 5, slots mod 5: this tile A 2P, B 2P+1; next tile A 2P+2, B 2P+3; A of tile t+2 2P+4.
  // DMA instructions of the period that ends at this tile's barrier (it began at the previous one):
  //   B of tile t+1 -> slot 2P+3 (second part; the first part went out in the previous tile's last
  //   half), then A of tile t+2 -> slot 2P+4, then the L2 prefetch.
  // After the barrier this tile's slots are free: B of tile t+2 -> slot 2P starts.
  constexpr int NL = NA, NS = NB;
  constexpr int NS0 = (NS + 1) / 2, NL0 = (NL + 1) / 2;
  auto dmaL = [&](int kt, uint16_t* sl, int i) { a.dma(ra, astep_b, kt, sl, wave, i); };
  auto dmaS = [&](int kt, uint16_t* sl, int i) { b.dma(rb, bstep_b, kt, sl, wave, i); };
  auto body = [&](auto p, int t) {
    constexpr int P = decltype(p)::value;
    uint16_t* const sl = slot(Int<(2 * P) % 5>{});
    uint16_t* const ss = slot(Int<(2 * P + 1) % 5>{});
    uint16_t* const nsl = slot(Int<(2 * P + 2) % 5>{});
    uint16_t* const nss = slot(Int<(2 * P + 3) % 5>{});
    uint16_t* const fsl = slot(Int<(2 * P + 4) % 5>{});
    uint16_t* const sa = sl;
    uint16_t* const sb = ss;
    uint16_t* const nsa = nsl;
    uint16_t* const nsb = nss;
    // Past the last tile the schedule keeps running on the last tile's data (clamped index): the
    // slots written are free, nobody reads them, and the instruction counts that the waits rely on
    // stay the same in every tile.
    const int t1 = min(t + 1, nk - 1), t2 = min(t + 2, nk - 1);
    auto dmaS1 = [&](int i) { if (i < NS) dmaS(t1, nss, i); };
    auto dmaL2 = [&](int i) { if (i < NL) dmaL(t2, fsl, i); };
    auto dmaS2 = [&](int i) { if (i < NS) dmaS(t2, sl, i); };
    // on entry: fa[0] = A half 0 of K-step 0, fb[0] = B of K-step 0
    half(Int<0>{}, Int<0>{}, Int<NRA1>{}, [&] { read_a(1, sa, 0); }, [&] { dmaS1(NS0); }, [&] { dmaS1(NS0 + 1); });
    half(Int<1>{}, Int<0>{}, Int<NRA0 + NRB>{}, [&] { read_a(0, sa, 1); read_b(1, sb, 1); }, [&] { dmaL2(0); }, [&] { dmaL2(1); });
    half(Int<0>{}, Int<1>{}, Int<NRA1>{}, [&] { read_a(1, sa, 1); }, [&] { dmaL2(NL0); }, [&] { dmaL2(NL0 + 1); });
    // the newest vector memory instruction of the period: the barrier's wait below lets it fly on
    if constexpr (PF_ON) prefetch(t);
    // last half, with the barrier inside
    constexpr int nm = (MI - MH) * NI;
    constexpr int n1 = nm / 3 > 0 ? nm / 3 : 1, n2 = 2 * nm / 3 > n1 ? 2 * nm / 3 : n1;
    __builtin_amdgcn_sched_barrier(0);
    mfma_range(1, 1, 0, n1);
    __builtin_amdgcn_sched_barrier(0);
    // this wavefront's share of tile t+1 has landed (its L instructions of tile t+2 may still fly),
    // and all its fragment reads of tile t are complete
    __builtin_amdgcn_s_waitcnt(vmcnt_lgkm0_imm(NL + (PF_ON ? 1 : 0)));
    __builtin_amdgcn_s_barrier();
    read_a(0, nsa, 0);
    read_b(0, nsb, 0);
    __builtin_amdgcn_sched_barrier(0);
    dmaS2(0);
    __builtin_amdgcn_sched_barrier(0);
    mfma_range(1, 1, n1, n2);
    __builtin_amdgcn_sched_barrier(0);
    dmaS2(1);
    __builtin_amdgcn_sched_barrier(0);
    mfma_range(1, 1, n2, nm);
    __builtin_amdgcn_sched_barrier(0);
  };

  // first DMA instructions of an output tile: K tile 0 whole, A of K tile 1 whole, first part of B of K tile 1
  auto first_dma = [&] {
    if (nk > 0) {
#pragma unroll
      for (int i = 0; i < NL; ++i) dmaL(0, r0, i);
#pragma unroll
      for (int i = 0; i < NS; ++i) dmaS(0, r1, i);
      const int p1 = min(1, nk - 1);
#pragma unroll
      for (int i = 0; i < NL; ++i) dmaL(p1, r2, i);
#pragma unroll
      for (int i = 0; i < NS0; ++i) dmaS(p1, r3, i);
    }
  };
  // vector memory instructions a wavefront issues in the epilogue of an interior tile
  // (bf16 outputs go out two blocks at a time, see store8_pair; an odd last block goes alone)
  constexpr bool PAIRED = !SPLIT && (EPI == ntp::EPI_BF16 || EPI == ntp::EPI_GELU || EPI == ntp::EPI_DGELU);
  constexpr int NPAIR = NI / 2, NODD = NI & 1;
  constexpr int NEPI = EPI == ntp::EPI_BF16    ? MI * (NPAIR + NODD)
                       : EPI == ntp::EPI_GELU  ? MI * 2 * (NPAIR + NODD)
                       : EPI == ntp::EPI_DGELU ? MI * (3 * NPAIR + 2 * NODD)
                       : EPI == ntp::EPI_F32   ? MI * NI
                                               : MI * NI * 2;
  bool stores_in_flight = false;
  first_dma();
  while (true) {
    const int vnext = vblk + int(gridDim.x);
    const bool more = !SPLIT && vnext < nblk;
    const TilePos npos = more ? place(vnext) : pos;
    if (more) pf_params(npos, pf_turn_next, pf_voff_next);
    else pf_turn_next = -1;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (nk > 0) {
      // The first DMA instructions of this output tile have landed.  After the first output tile the
      // previous tile's stores (and the loads of its epilogue) sit in the same in-order counter,
      // issued after those DMA instructions: when that tile was an interior one, every wavefront
      // issued exactly NEPI of them, which may stay in flight and drain while this tile computes.
      if (stores_in_flight) __builtin_amdgcn_s_waitcnt(vmcnt_imm(NEPI <= 63 ? NEPI : 63));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __builtin_amdgcn_s_barrier();
      read_a(0, r0, 0);
      read_b(0, r1, 0);
    }
    for (int t = 0; t < nk; t += 5) {
      body(Int<0>{}, t);
      if (t + 1 < nk) body(Int<1>{}, t + 1);
      if (t + 2 < nk) body(Int<2>{}, t + 2);
      if (t + 3 < nk) body(Int<3>{}, t + 3);
      if (t + 4 < nk) body(Int<4>{}, t + 4);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // the clamped DMA instructions of the last tiles
    // K tail (K % 64 != 0) through registers with element masks, not overlapped
    if (!ring_tail && nfull * DK < K) {
      __syncthreads();
      a.tail(opA, astep, nfull, K, r0, wave, lane);
      b.tail(opB, bstep, nfull, K, r1, wave, lane);
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        read_b(0, r1, ks);
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          read_a(h, r0, ks);
          mfma_range(h, 0, 0, (h ? MI - MH : MH) * NI);
        }
      }
    }
    // The next output tile's first DMA instructions go out before this tile's results are stored, so
    // that their latency hides behind the stores.  The barrier makes sure that no wavefront still
    // reads LDS and that every wavefront's DMA instructions of this tile have landed.
    const int erow0 = row0, ecol0 = col0;
    vblk = vnext;
    // interior tile: no lane is masked in the epilogue, so its instruction count is the static one
    stores_in_flight = NEPI <= 63 && erow0 + BM_ <= g.M && ecol0 + BN_ <= g.N;
    if (more) {
      __builtin_amdgcn_s_waitcnt(vmcnt_lgkm0_imm(0));
      __builtin_amdgcn_s_barrier();
      pos = npos;
      row0 = pos.row0;
      col0 = pos.col0;
      setup_tile();
      first_dma();
    }
    __builtin_amdgcn_sched_barrier(0);  // the epilogue's memory instructions stay behind those DMA instructions
    // lane l of a 16 x 16 block holds row (l & 15) and columns 4 (l >> 4) + {0..3}
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int m = erow0 + wm * TM + i * 16 + (lane & 15);
      if constexpr (PAIRED) {
#pragma unroll
        for (int j = 0; j + 1 < NI; j += 2) store8_pair<EPI>(g, m, ecol0 + wn * TN + j * 16, lane >> 4, acc[i][j], acc[i][j + 1]);
      }
#pragma unroll
      for (int j = PAIRED ? NI - NODD : 0; j < NI; ++j) {
        const int n0 = ecol0 + wn * TN + j * 16 + (lane >> 4) * 4;
        if constexpr (SPLIT) {
          if (g.k_splits > 1) {
            if (m < g.M && n0 < g.n_store)
              *reinterpret_cast<f32x4*>(static_cast<float*>(g.C) + int64_t(split) * g.split_stride + int64_t(m) * g.ldc + n0) = acc[i][j];
          } else {
            store4<EPI>(g, m, n0, acc[i][j]);
          }
        } else {
          store4<EPI>(g, m, n0, acc[i][j]);
        }
      }
    }
    if (!more) break;
  }
  asm volatile("" : "+v"(pf_sink));  // the prefetch register stays reserved up to here
}

}  // namespace ntp_gemm

#endif  // NTP_GEMM_RING_H_
