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
#include <cstdlib>
#include <cstring>
#include <type_traits>

#include "ntp_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

struct GemmArgs {
  const uint16_t* A;
  const uint16_t* B;
  void* C;
  void* C2;
  const uint16_t* AUX;
  int64_t lda, ldb, ldc, ldc2, ldaux;
  int32_t M, N, K;
  int32_t n_store;  // columns stored: N, or N rounded up to 8 with zero fill
  int32_t gelu_mode;
  int32_t tiles_m, tiles_n;
};

__device__ __forceinline__ float gelu_fwd(float x, int mode) {
  if (mode == NTP_GELU_TANH) {
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return 0.5f * x * (1.0f + tanhf(u));
  }
  return 0.5f * x * (1.0f + erff(x * 0.7071067811865476f));
}

__device__ __forceinline__ float gelu_bwd(float x, int mode) {
  if (mode == NTP_GELU_TANH) {
    const float c = 0.7978845608028654f;
    const float u = c * (x + 0.044715f * x * x * x);
    const float th = tanhf(u);
    const float du = c * (1.0f + 3.0f * 0.044715f * x * x);
    return 0.5f * (1.0f + th) + 0.5f * x * (1.0f - th * th) * du;
  }
  const float cdf = 0.5f * (1.0f + erff(x * 0.7071067811865476f));
  const float pdf = 0.3989422804014327f * __expf(-0.5f * x * x);
  return cdf + x * pdf;
}

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(uint16_t, static_cast<__bf16>(f));  // round to nearest even
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __builtin_bit_cast(float, uint32_t(h) << 16);
}

// ------------------------------------------------------------------------------
// Generic kernel: 128 x 128 x 32 tile, 4 wavefronts (2 x 2), each 64 x 64 via
// 2 x 2 MFMA 32x32x16.  Operands go global -> registers -> LDS; LDS always holds
// [row][k] with k contiguous, so K-strided operands are transposed on the LDS write.
constexpr int BM = 128, BN = 128, BK = 32;
constexpr int LDS_LD = BK + 8;  // elements; 80-byte rows keep 16-byte alignment and spread banks

template <bool KC>
struct TileLoader {
  // Two 16-byte chunks per thread per tile.
  u16x8 v[2];

  // rows_lim: extent of the non-K dimension; ld in elements
  __device__ __forceinline__ void load(const uint16_t* __restrict__ base, int64_t ld, int row0, int rows_lim,
                                       int k0, int K, int tid) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * 256;
      u16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
      if constexpr (KC) {
        const int r = c >> 2, kc = (c & 3) * 8;
        const int row = row0 + r, k = k0 + kc;
        if (row < rows_lim && k < K) {
          val = *reinterpret_cast<const u16x8*>(base + int64_t(row) * ld + k);
          if (k + 8 > K) {
#pragma unroll
            for (int j = 0; j < 8; ++j)
              if (k + j >= K) val[j] = 0;
          }
        }
      } else {
        const int kk = c >> 4, rc = (c & 15) * 8;
        const int k = k0 + kk, row = row0 + rc;
        if (k < K && row < rows_lim) {
          // a chunk that straddles rows_lim stays inside the padded leading dimension;
          // its extra lanes feed rows/columns that are never stored
          val = *reinterpret_cast<const u16x8*>(base + int64_t(k) * ld + row);
        }
      }
      v[i] = val;
    }
  }

  __device__ __forceinline__ void store(uint16_t* __restrict__ lds, int tid) const {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int c = tid + i * 256;
      if constexpr (KC) {
        const int r = c >> 2, kc = (c & 3) * 8;
        *reinterpret_cast<u16x8*>(lds + r * LDS_LD + kc) = v[i];
      } else {
        const int kk = c >> 4, rc = (c & 15) * 8;
#pragma unroll
        for (int j = 0; j < 8; ++j) lds[(rc + j) * LDS_LD + kk] = v[i][j];
      }
    }
  }
};

template <int EPI>
__device__ __forceinline__ void store4(const GemmArgs& g, int m, int n0, f32x4 acc) {
  if (m >= g.M || n0 >= g.n_store) return;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (n0 + j >= g.N) acc[j] = 0.0f;
  if constexpr (EPI == ntp::EPI_F32) {
    *reinterpret_cast<f32x4*>(static_cast<float*>(g.C) + int64_t(m) * g.ldc + n0) = acc;
  } else if constexpr (EPI == ntp::EPI_F32_ACCUM) {
    f32x4* p = reinterpret_cast<f32x4*>(static_cast<float*>(g.C) + int64_t(m) * g.ldc + n0);
    *p = *p + acc;
  } else {
    if constexpr (EPI == ntp::EPI_DGELU) {
      const u16x4 pre = *reinterpret_cast<const u16x4*>(g.AUX + int64_t(m) * g.ldaux + n0);
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[j] = (n0 + j < g.N) ? acc[j] * gelu_bwd(bf16_to_f32(pre[j]), g.gelu_mode) : 0.0f;
    }
    u16x4 o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = f32_to_bf16(acc[j]);
    *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(g.C) + int64_t(m) * g.ldc + n0) = o;
    if constexpr (EPI == ntp::EPI_GELU) {
      u16x4 y;
#pragma unroll
      for (int j = 0; j < 4; ++j) y[j] = f32_to_bf16(gelu_fwd(acc[j], g.gelu_mode));
      *reinterpret_cast<u16x4*>(static_cast<uint16_t*>(g.C2) + int64_t(m) * g.ldc2 + n0) = y;
    }
  }
}

template <bool AKC, bool BKC, int EPI>
__global__ __launch_bounds__(256) void gemm_generic_kernel(const GemmArgs g) {
  __shared__ __attribute__((aligned(16))) uint16_t sA[BM * LDS_LD];
  __shared__ __attribute__((aligned(16))) uint16_t sB[BN * LDS_LD];
  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  // N-major tile order: consecutive workgroups share the A tile rows
  const int tile_m = blockIdx.x / g.tiles_n, tile_n = blockIdx.x - tile_m * g.tiles_n;
  const int row0 = tile_m * BM, col0 = tile_n * BN;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  TileLoader<AKC> la;
  TileLoader<BKC> lb;
  const int ktiles = (g.K + BK - 1) / BK;
  if (ktiles > 0) {
    la.load(g.A, g.lda, row0, g.M, 0, g.K, tid);
    lb.load(g.B, g.ldb, col0, g.N, 0, g.K, tid);
  }
  for (int kt = 0; kt < ktiles; ++kt) {
    la.store(sA, tid);
    lb.store(sB, tid);
    __syncthreads();
    if (kt + 1 < ktiles) {
      la.load(g.A, g.lda, row0, g.M, (kt + 1) * BK, g.K, tid);
      lb.load(g.B, g.ldb, col0, g.N, (kt + 1) * BK, g.K, tid);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 fa[2], fb[2];
      const int koff = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = *reinterpret_cast<const bf16x8*>(sA + (wm * 64 + i * 32 + (lane & 31)) * LDS_LD + koff);
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = *reinterpret_cast<const bf16x8*>(sB + (wn * 64 + j * 32 + (lane & 31)) * LDS_LD + koff);
      // operands swapped: the product comes out transposed, so that each lane holds
      // 4 consecutive columns of one row (vector stores along N)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // lane (l) of a 32x32 block holds row l % 32 and columns 8 q + 4 (l / 32) + {0..3}, q = 0..3
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int m = row0 + wm * 64 + i * 32 + (lane & 31);
        const int n0 = col0 + wn * 64 + j * 32 + q * 8 + (lane >> 5) * 4;
        f32x4 v = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
        store4<EPI>(g, m, n0, v);
      }
}

// ------------------------------------------------------------------------------
// Fast kernel: BM x BN x 64 tile, 8 wavefronts (WGM x WGN), register-staged double
// buffering in LDS (one barrier per K tile).
//   K-contiguous operand:  LDS [row][k], 144-byte rows  -> ds_read_b128 fragments
//   K-strided operand:     LDS [k][row], (R + 32)-element rows -> two transposing
//                          64-bit LDS reads per fragment (no register shuffles)
// Row strides are chosen so that the 16 lanes served together hit distinct banks.
// Rows past the edge are clamped to the last valid row (their products are never
// stored); the K tail tile is loaded with element masks so that it contributes zeros.
constexpr int FK = 64;
constexpr int FAST_THREADS = 512;

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

template <bool KC, int R>
struct FastOperand {
  static constexpr int LD = KC ? (FK + 8) : (R + 32);
  static constexpr int STAGE = KC ? R * LD : FK * LD;  // elements per pipeline stage
  static constexpr int CHUNKS = R / 64;                // 16-byte chunks per thread per tile
  static_assert(R % 64 == 0, "tile extent must be a multiple of 64");

  const uint16_t* ptr[CHUNKS];  // this thread's chunk addresses in K tile 0
  u16x8 v[CHUNKS];
  int64_t kstep;                // elements between consecutive K tiles

  __device__ __forceinline__ void init(const uint16_t* base, int64_t ld, int row0, int lim, int tid) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int id = tid + FAST_THREADS * i;
      if constexpr (KC) {
        const int r = id >> 3, c = (id & 7) * 8;
        const int row = min(row0 + r, lim - 1);
        ptr[i] = base + int64_t(row) * ld + c;
      } else {
        constexpr int CPR = R / 8;  // chunks per k row
        const int k = id / CPR, c = (id % CPR) * 8;
        const int col = min(row0 + c, ((lim - 1) >> 3) << 3);
        ptr[i] = base + int64_t(k) * ld + col;
      }
    }
    kstep = KC ? FK : FK * ld;
  }

  __device__ __forceinline__ void load_full(int kt) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) v[i] = *reinterpret_cast<const u16x8*>(ptr[i] + kt * kstep);
  }

  // K tile that crosses the end of K: everything at k >= K reads as zero
  __device__ __forceinline__ void load_tail(int kt, int K, int tid) {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int id = tid + FAST_THREADS * i;
      u16x8 val = {0, 0, 0, 0, 0, 0, 0, 0};
      if constexpr (KC) {
        const int k = kt * FK + (id & 7) * 8;
        if (k < K) {
          val = *reinterpret_cast<const u16x8*>(ptr[i] + kt * kstep);
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (k + j >= K) val[j] = 0;
        }
      } else {
        constexpr int CPR = R / 8;
        const int k = kt * FK + id / CPR;
        if (k < K) val = *reinterpret_cast<const u16x8*>(ptr[i] + kt * kstep);
      }
      v[i] = val;
    }
  }

  __device__ __forceinline__ void store(uint16_t* lds, int tid) const {
#pragma unroll
    for (int i = 0; i < CHUNKS; ++i) {
      const int id = tid + FAST_THREADS * i;
      if constexpr (KC) {
        *reinterpret_cast<u16x8*>(lds + (id >> 3) * LD + (id & 7) * 8) = v[i];
      } else {
        constexpr int CPR = R / 8;
        *reinterpret_cast<u16x8*>(lds + (id / CPR) * LD + (id % CPR) * 8) = v[i];
      }
    }
  }

  // 32 rows x 16 k fragment in MFMA operand layout: lane l holds row (l % 32), k = 8 (l / 32) + 0..7
  __device__ __forceinline__ static bf16x8 frag(const uint16_t* lds, int rbase, int ks, int lane) {
    if constexpr (KC) {
      return *reinterpret_cast<const bf16x8*>(lds + (rbase + (lane & 31)) * LD + ks * 16 + (lane >> 5) * 8);
    } else {
      // Transposing read: in each 16-lane group, lane s points at 4 consecutive rows of
      // k-line (s / 4); the group hands lane L the 4 k-values of row L.
      const int g = lane >> 4, s = lane & 15;
      const int krow = ks * 16 + (g >> 1) * 8 + (s >> 2);
      const int col = rbase + (g & 1) * 16 + (s & 3) * 4;
      typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
      const uint16_t* p = lds + krow * LD + col;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * LD));
      const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8, both);
    }
  }
};

template <bool AKC, bool BKC, int EPI, int BM_, int BN_, int WGM, int WGN>
__global__ __launch_bounds__(FAST_THREADS) void gemm_fast_kernel(const GemmArgs g) {
  static_assert(WGM * WGN == 8, "8 wavefronts");
  constexpr int TM = BM_ / WGM, TN = BN_ / WGN;  // wavefront tile
  constexpr int MI = TM / 32, NI = TN / 32;
  static_assert(TM % 32 == 0 && TN % 32 == 0, "wavefront tile must be made of 32x32 blocks");
  using OpA = FastOperand<AKC, BM_>;
  using OpB = FastOperand<BKC, BN_>;
  __shared__ __attribute__((aligned(16))) uint16_t sA[2][OpA::STAGE];
  __shared__ __attribute__((aligned(16))) uint16_t sB[2][OpB::STAGE];

  const int tid = threadIdx.x;
  const int wave = tid >> 6, lane = tid & 63;
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
  a.init(g.A, g.lda, row0, g.M, tid);
  b.init(g.B, g.ldb, col0, g.N, tid);
  const int ktiles = (g.K + FK - 1) / FK;
  const int kfull = g.K / FK;  // tiles below this index need no masking

  auto load = [&](int kt) {
    if (kt < kfull) {
      a.load_full(kt);
      b.load_full(kt);
    } else {
      a.load_tail(kt, g.K, tid);
      b.load_tail(kt, g.K, tid);
    }
  };

  if (ktiles > 0) {
    load(0);
    a.store(sA[0], tid);
    b.store(sB[0], tid);
    __syncthreads();
    if (ktiles > 1) load(1);
  }
  for (int kt = 0; kt < ktiles; ++kt) {
    const uint16_t* cA = sA[kt & 1];
    const uint16_t* cB = sB[kt & 1];
#pragma unroll
    for (int ks = 0; ks < FK / 16; ++ks) {
      bf16x8 fa[MI], fb[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) fa[i] = OpA::frag(cA, wm * TM + i * 32, ks, lane);
#pragma unroll
      for (int j = 0; j < NI; ++j) fb[j] = OpB::frag(cB, wn * TN + j * 32, ks, lane);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < ktiles) {
      a.store(sA[(kt + 1) & 1], tid);
      b.store(sB[(kt + 1) & 1], tid);
      if (kt + 2 < ktiles) load(kt + 2);
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int m = row0 + wm * TM + i * 32 + (lane & 31);
        const int n0 = col0 + wn * TN + j * 32 + q * 8 + (lane >> 5) * 4;
        f32x4 v = {acc[i][j][q * 4 + 0], acc[i][j][q * 4 + 1], acc[i][j][q * 4 + 2], acc[i][j][q * 4 + 3]};
        store4<EPI>(g, m, n0, v);
      }
}

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

template <bool AKC, bool BKC, int BM_, int BN_, int WGM, int WGN>
int launch_fast(GemmArgs g, int epi, hipStream_t s) {
  g.tiles_m = (g.M + BM_ - 1) / BM_;
  g.tiles_n = (g.n_store + BN_ - 1) / BN_;
  if (int64_t(g.tiles_m) * g.tiles_n > 0x7fffffff) return NTP_ERR_UNSUPPORTED;
  const dim3 grid(uint32_t(g.tiles_m) * uint32_t(g.tiles_n)), block(FAST_THREADS);
  return dispatch_epilogue(epi, [&](auto e) {
    hipLaunchKernelGGL((gemm_fast_kernel<AKC, BKC, decltype(e)::value, BM_, BN_, WGM, WGN>), grid, block, 0, s, g);
    return hipGetLastError() == hipSuccess ? NTP_OK : NTP_ERR_LAUNCH;
  });
}

// Tile shapes of the fast kernel, widest first.
struct TileChoice {
  int bm, bn;
  double rate;  // relative throughput of one tile of this shape at full occupancy
};
constexpr TileChoice kTiles[] = {{256, 256, 1.0}, {128, 256, 0.85}, {256, 128, 0.85}, {128, 128, 0.7}};

// Pick the tile shape with the least estimated time: rounds of 256 workgroups times tile area over rate.
int choose_tile(int64_t M, int64_t N) {
  int best = 0;
  double best_t = 1e300;
  for (int i = 0; i < int(sizeof(kTiles) / sizeof(kTiles[0])); ++i) {
    const int64_t tiles = ((M + kTiles[i].bm - 1) / kTiles[i].bm) * ((N + kTiles[i].bn - 1) / kTiles[i].bn);
    const int64_t rounds = (tiles + 255) / 256;
    const double t = double(rounds) * kTiles[i].bm * kTiles[i].bn / kTiles[i].rate;
    if (t < best_t) {
      best_t = t;
      best = i;
    }
  }
  return best;
}

// Variant used for a shape: -1 = generic kernel, else an index into kTiles.  The environment
// variable NTP_GEMM_TILE (generic | 256x256 | 128x256 | 256x128 | 128x128) overrides the choice;
// it exists so that tests and tuning runs can reach every variant at any size.
int choose_variant(const GemmArgs& g) {
  if (const char* f = getenv("NTP_GEMM_TILE")) {
    if (!strcmp(f, "generic")) return -1;
    if (!strcmp(f, "256x256")) return 0;
    if (!strcmp(f, "128x256")) return 1;
    if (!strcmp(f, "256x128")) return 2;
    if (!strcmp(f, "128x128")) return 3;
  }
  // small problems: the generic 128x128x32 kernel (4 wavefronts) has less fixed cost
  if (int64_t(g.M) * g.N < 128 * 128 * 64 || g.K < 128) return -1;
  return choose_tile(g.M, g.n_store);
}

const char* variant_name(int v) {
  static const char* const kName[] = {"generic128", "256x256", "128x256", "256x128", "128x128"};
  return kName[v + 1];
}

template <bool AKC, bool BKC>
int launch_any(const GemmArgs& g, int epi, hipStream_t s, int variant) {
  switch (variant) {
    case 0: return launch_fast<AKC, BKC, 256, 256, 2, 4>(g, epi, s);
    case 1: return launch_fast<AKC, BKC, 128, 256, 2, 4>(g, epi, s);
    case 2: return launch_fast<AKC, BKC, 256, 128, 4, 2>(g, epi, s);
    case 3: return launch_fast<AKC, BKC, 128, 128, 2, 4>(g, epi, s);
    default: return launch_generic<AKC, BKC>(g, epi, s);
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

}  // namespace

namespace ntp {

int gemm_launch(const GemmDesc& d, void* stream) {
  if (d.M < 0 || d.N < 0 || d.K < 0) return NTP_ERR_INVALID_ARG;
  if (d.M == 0 || d.N == 0) return NTP_OK;
  if (d.M > 0x7fffff00 || d.N > 0x7fffff00 || d.K > 0x7fffff00) return NTP_ERR_UNSUPPORTED;
  if (!d.C || (d.K > 0 && (!d.A || !d.B))) return NTP_ERR_INVALID_ARG;
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
    if (!aligned16(d.C) || d.ldc % 4) return NTP_ERR_ALIGNMENT;
  } else {
    if (d.zero_pad_n) n_store = (d.N + 7) / 8 * 8;
    if (n_store % 4) return NTP_ERR_ALIGNMENT;
    if (!aligned16(d.C) || d.ldc % 8) return NTP_ERR_ALIGNMENT;
    if (d.epilogue == EPI_GELU && (!aligned16(d.C2) || d.ldc2 % 8 || d.ldc2 < n_store)) return NTP_ERR_ALIGNMENT;
    if (d.epilogue == EPI_DGELU && (!aligned16(d.AUX) || d.ldaux % 8 || d.ldaux < n_store)) return NTP_ERR_ALIGNMENT;
  }
  if (d.ldc < n_store) return NTP_ERR_INVALID_ARG;

  GemmArgs g{};
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
  const int variant = choose_variant(g);
  if (ntp::timing_on()) {
    char name[48];
    snprintf(name, sizeof(name), "gemm_%c%c_%s_%s", d.a_kc ? 'n' : 't', d.b_kc ? 't' : 'n', kEpiName[d.epilogue],
             variant_name(variant));
    ntp::timing_begin(stream, name, 2.0 * double(d.M) * double(d.N) * double(d.K), 0.0);
  }
  int st;
  if (d.a_kc && d.b_kc) st = launch_any<true, true>(g, d.epilogue, s, variant);
  else if (d.a_kc && !d.b_kc) st = launch_any<true, false>(g, d.epilogue, s, variant);
  else if (!d.a_kc && !d.b_kc) st = launch_any<false, false>(g, d.epilogue, s, variant);
  else st = launch_any<false, true>(g, d.epilogue, s, variant);
  ntp::timing_end(stream);
  return st;
}

}  // namespace ntp
