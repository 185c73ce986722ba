// Main bf16 MFMA GEMM kernel of the NTP shard layers: global -> LDS by direct (DMA)
// loads, no staging registers.  Included by ntp_gemm.hip.
//
// Tile BM x BN x 64, WGM x WGN wavefronts, each computing (BM/WGM) x (BN/WGN) with
// 32x32x16 bf16 MFMAs and fp32 accumulators.  Two LDS stages.
//
// LDS layout of one stage (16-byte chunks stay whole; a wavefront's DMA instruction
// fills 64 consecutive chunks, so bank spreading is done by permuting chunks, not by padding):
//   K-contiguous operand  [R rows][64 k]:   chunk p of row r holds k-chunk  p ^ ((r >> 1) & 7)
//   K-strided operand     [64 k][R rows]:   chunk p of line k holds row-chunk p ^ ((k & 3) << 2)
// Fragments come out of LDS in MFMA operand layout with ds_read_b128 (K-contiguous) or
// with two transposing 64-bit reads (K-strided).
//
// Pipeline per K tile t (stage s = t & 1, four K-steps of 16), one barrier per tile:
//   K-steps 0-2: read the fragments of the next step while the MFMAs of this step issue
//   K-step 3:    a first batch of MFMAs; then wait for this wavefront's DMA of tile t+1, barrier
//                (every wavefront's tile t+1 has landed and nobody reads tile t any more), start
//                the DMA of tile t+2 into stage s, read fragments (t+1, step 0); remaining MFMAs.
// So a DMA has a whole tile time to land.  The K tail tile (K % 64 != 0) goes through
// registers with element masks so that it contributes zeros.
#ifndef NTP_GEMM_DMA_H_
#define NTP_GEMM_DMA_H_

#include <type_traits>

#include "ntp_gemm_kernels.h"

namespace ntp_gemm {

constexpr int DK = 64;        // K extent of a tile

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_cvoid;

template <bool KC, int R, int NW>
struct DmaOperand {
  static constexpr int STAGE = R * DK;            // elements per stage
  static constexpr int NINST = R * DK * 2 / 1024 / NW;  // DMA instructions per wavefront per tile
  static_assert((R * DK * 2 / 1024) % NW == 0, "tile must split evenly over the wavefronts");
  static constexpr int CPL = R / 8;               // chunks per k line (K-strided layout)

  uint32_t off[NINST];  // byte offset (from the operand base at K tile 0) of this lane's chunk per instruction

  // chunk slot `slot` of a stage -> (line, chunk) it holds; see the layout above
  __device__ __forceinline__ static void slot_src(int slot, int& line, int& chunk) {
    if constexpr (KC) {
      line = slot >> 3;
      chunk = (slot & 7) ^ ((line >> 1) & 7);
    } else {
      line = slot / CPL;
      chunk = (slot % CPL) ^ ((line & 3) << 2);
    }
  }

  __device__ __forceinline__ void init(int64_t ld, int row0, int lim, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < NINST; ++i) {
      int line, chunk;
      slot_src((wave * NINST + i) * 64 + lane, line, chunk);
      if constexpr (KC) {
        const int row = min(row0 + line, lim - 1);  // rows past the edge repeat the last one
        off[i] = uint32_t((int64_t(row) * ld + chunk * 8) * 2);
      } else {
        const int col = min(row0 + chunk * 8, ((lim - 1) >> 3) << 3);
        off[i] = uint32_t((int64_t(line) * ld + col) * 2);
      }
    }
  }

  // start the DMA of K tile `kt` into `stage`
  __device__ __forceinline__ void dma(const uint16_t* base, int64_t kstep, int kt, uint16_t* stage, int wave) const {
    const uint16_t* tile = base + int64_t(kt) * kstep;
#pragma unroll
    for (int i = 0; i < NINST; ++i) {
      uint16_t* dst = stage + (wave * NINST + i) * 512;  // 64 chunks of 8 elements, wave-uniform
      __builtin_amdgcn_global_load_lds((global_cvoid*)(reinterpret_cast<const char*>(tile) + off[i]), (lds_void*)dst, 16, 0, 0);
    }
  }

  // K tail tile through registers: everything at k >= K becomes zero
  __device__ __forceinline__ void tail(const uint16_t* base, int64_t kstep, int kt, int K, uint16_t* stage, int wave,
                                       int lane) const {
    const uint16_t* tile = base + int64_t(kt) * kstep;
#pragma unroll
    for (int i = 0; i < NINST; ++i) {
      const int slot = (wave * NINST + i) * 64 + lane;
      int line, chunk;
      slot_src(slot, line, chunk);
      u16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
      if constexpr (KC) {
        const int k = kt * DK + chunk * 8;
        if (k < K) {
          val = *reinterpret_cast<const u16x8*>(reinterpret_cast<const char*>(tile) + off[i]);
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (k + j >= K) val[j] = 0;
        }
      } else {
        if (kt * DK + line < K) val = *reinterpret_cast<const u16x8*>(reinterpret_cast<const char*>(tile) + off[i]);
      }
      *reinterpret_cast<u16x8*>(stage + slot * 8) = val;
    }
  }
};

// per-lane LDS element offsets of the fragments of one operand (32 rows x 16 k per fragment,
// MFMA operand layout: lane l holds row (l & 31), k = 8 (l >> 5) + 0..7 of the K-step)
template <bool KC, int R, int NF>
struct FragAddr {
  uint32_t o[KC ? 4 : NF];
  __device__ __forceinline__ void init(int rbase, int lane) {
    if constexpr (KC) {
      // k-chunk of step ks is (2 ks + (l >> 5)); its position in the row is that ^ ((row >> 1) & 7)
      const int r = rbase + (lane & 31);
      const int sw = (r >> 1) & 7;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) o[ks] = uint32_t(r * DK + (((ks * 2 + (lane >> 5)) ^ sw) * 8));
    } else {
      // transposing read: in each 16-lane group, lane s points at 4 consecutive rows of k line
      // (s >> 2); the group hands lane L the 4 k-values of row L.  Groups 0/1 take k 0-7 of the
      // step for rows 0-15 / 16-31, groups 2/3 take k 8-15.
      const int g = lane >> 4, s = lane & 15;
      const int k = 8 * (g >> 1) + (s >> 2);  // + 16 * step (+ 4 for the second read): both keep k & 3
#pragma unroll
      for (int i = 0; i < NF; ++i) {
        const int col = rbase + i * 32 + (g & 1) * 16 + (s & 3) * 4;
        o[i] = uint32_t(k * R + (((col >> 3) ^ ((k & 3) << 2)) * 8) + (col & 7));
      }
    }
  }
  __device__ __forceinline__ bf16x8 read(const uint16_t* stage, int i, int ks) const {
    if constexpr (KC) {
      return *reinterpret_cast<const bf16x8*>(stage + o[ks] + i * 32 * DK);
    } else {
      typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
      const uint16_t* p = stage + o[i] + ks * 16 * R;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * R));
      const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, both);
    }
  }
};

template <bool AKC, bool BKC, int EPI, int BM_, int BN_, int WGM, int WGN>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_dma_kernel(const GemmArgs g) {
  constexpr int NW = WGM * WGN;
  constexpr int TM = BM_ / WGM, TN = BN_ / WGN;  // wavefront tile
  constexpr int MI = TM / 32, NI = TN / 32;      // 32 x 32 accumulator blocks
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wavefront tile must be made of 32x32 blocks");
  using OpA = DmaOperand<AKC, BM_, NW>;
  using OpB = DmaOperand<BKC, BN_, NW>;
  // one array per stage and operand: distinct objects, so that the compiler can tell that a DMA in
  // flight into one stage does not alias the fragment reads of the other (no forced wait)
  __shared__ __attribute__((aligned(1024))) uint16_t sA0[OpA::STAGE];
  __shared__ __attribute__((aligned(1024))) uint16_t sA1[OpA::STAGE];
  __shared__ __attribute__((aligned(1024))) uint16_t sB0[OpB::STAGE];
  __shared__ __attribute__((aligned(1024))) uint16_t sB1[OpB::STAGE];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give every XCD a
  // contiguous range of tiles, walked in groups of 8 tile rows so that neighbours share operands.
  const int nblk = g.tiles_m * g.tiles_n;
  const int xq = nblk >> 3, xr = nblk & 7, xcd = blockIdx.x & 7;
  const int L = xcd * xq + min(xcd, xr) + (blockIdx.x >> 3);
  constexpr int GM = 8;
  const int width = GM * g.tiles_n;
  const int first_m = (L / width) * GM;
  const int gsz = min(g.tiles_m - first_m, GM);
  const int tile_m = first_m + (L % width) % gsz, tile_n = (L % width) / gsz;
  const int row0 = tile_m * BM_, col0 = tile_n * BN_;

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  OpA a;
  OpB b;
  a.init(g.lda, row0, g.M, wave, lane);
  b.init(g.ldb, col0, g.N, wave, lane);
  const int64_t astep = AKC ? DK : DK * g.lda, bstep = BKC ? DK : DK * g.ldb;
  FragAddr<AKC, BM_, MI> fra;
  FragAddr<BKC, BN_, NI> frb;
  fra.init(wm * TM, lane);
  frb.init(wn * TN, lane);

  const int kpipe = (g.K / DK) & ~1;  // an even number of complete K tiles goes through the DMA pipeline

  using S0 = std::integral_constant<int, 0>;
  using S1 = std::integral_constant<int, 1>;
  auto fill = [&](int kt, auto stage) {  // start filling `stage` with (complete) K tile kt
    if constexpr (decltype(stage)::value == 0) {
      a.dma(g.A, astep, kt, sA0, wave);
      b.dma(g.B, bstep, kt, sB0, wave);
    } else {
      a.dma(g.A, astep, kt, sA1, wave);
      b.dma(g.B, bstep, kt, sB1, wave);
    }
  };

  constexpr int NREADS = MI * (AKC ? 1 : 2) + NI * (BKC ? 1 : 2);  // LDS reads per K-step
  bf16x8 fa[2][MI], fb[2][NI];
  auto read_frags = [&](int buf, auto stage, int ks) {
    const uint16_t* pa = decltype(stage)::value == 0 ? sA0 : sA1;
    const uint16_t* pb = decltype(stage)::value == 0 ? sB0 : sB1;
#pragma unroll
    for (int i = 0; i < MI; ++i) fa[buf][i] = fra.read(pa, i, ks);
#pragma unroll
    for (int j = 0; j < NI; ++j) fb[buf][j] = frb.read(pb, j, ks);
  };
  // operands swapped: the product comes out transposed, so that each lane holds 4 consecutive
  // columns of one row (vector stores along N)
  auto mfma_rows = [&](int buf, int i0, int i1) {
#pragma unroll
    for (int i = i0; i < i1; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
  };
  // K-steps 0..2 of the tile in `stage`: read the next step's fragments under this step's MFMAs
  auto steps012 = [&](auto stage) {
#pragma unroll
    for (int ks = 0; ks < 3; ++ks) {
      __builtin_amdgcn_sched_barrier(0);
      read_frags((ks + 1) & 1, stage, ks + 1);
      mfma_rows(ks & 1, 0, MI);
      // issue order: one MFMA, all fragment reads of the next step, the remaining MFMAs
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, NREADS, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // One tile of the pipeline.  The barrier, the first fragment reads of the following tile and the
  // DMA start of the tile after that sit inside the MFMAs of the last K-step.  The body is the same
  // for every tile (after the last one the extra fragment reads fetch stale data that nobody uses).
  auto tile = [&](auto stage, auto other, int kt) {
    steps012(stage);
    mfma_rows(1, 0, MI / 2);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's DMA of tile kt + 1 has landed
    __syncthreads();
    read_frags(0, other, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (kt + 2 < kpipe) fill(kt + 2, stage);
    __builtin_amdgcn_sched_barrier(0);
    mfma_rows(1, MI / 2, MI);
  };

  if (kpipe > 0) {
    fill(0, S0{});
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's DMA has landed
    __syncthreads();
    fill(1, S1{});
    read_frags(0, S0{}, 0);
  }
  for (int kt = 0; kt < kpipe; kt += 2) {  // two tiles per trip so that the stage is static
    tile(S0{}, S1{}, kt);
    tile(S1{}, S0{}, kt + 1);
  }
  // What is left (an odd complete tile and / or the K tail) goes through registers with element
  // masks, one tile at a time without overlap: at most two tiles per GEMM.
  for (int kt = kpipe; kt * DK < g.K; ++kt) {
    __syncthreads();
    a.tail(g.A, astep, kt, g.K, sA0, wave, lane);
    b.tail(g.B, bstep, kt, g.K, sB0, wave, lane);
    __syncthreads();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      read_frags(0, S0{}, ks);
      mfma_rows(0, 0, MI);
    }
  }

  // lane l of a 32 x 32 block holds row (l & 31) and columns 8 q + 4 (l >> 5) + {0..3}, q = 0..3
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int m = row0 + wm * TM + i * 32 + (lane & 31);
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n0 = col0 + wn * TN + j * 32 + q * 8 + (lane >> 5) * 4;
        f32x4 v = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
        store4<EPI>(g, m, n0, v);
      }
  }
}

}  // namespace ntp_gemm

#endif  // NTP_GEMM_DMA_H_
