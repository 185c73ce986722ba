// Device code of the bf16 MFMA GEMM family (kernels and their helpers); included by
// ntp_gemm.hip, which holds the host-side checks and the launch logic.
#ifndef NTP_GEMM_KERNELS_H_
#define NTP_GEMM_KERNELS_H_

#include <hip/hip_runtime.h>

#include "ntp_internal.h"

namespace ntp_gemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x8 __attribute__((ext_vector_type(8)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

constexpr int kMaxRowSegs = 16;

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
  // fp32 epilogues only: where the output rows go.  n_segs == 0: to C / ldc.  Otherwise every row m
  // is stored to each segment with begin <= m < end, at ptr + (m - begin) * ld.
  int32_t n_segs;
  struct RowSeg {
    int32_t begin, end;
    float* ptr;
    int64_t ld;
  } seg[kMaxRowSegs];
  // split-K launches only: number of K chunks, chunk length (elements, a multiple of 64) and the
  // distance in floats between the partial-sum slices that start at C
  int32_t k_splits, k_chunk;
  int64_t split_stride;
  // ring kernel: bytes of A and of B from their first element to the end of the last chunk the kernel may
  // read (operand_extent_bytes); its DMA loads are range-checked against them
  uint32_t a_extent, b_extent;
  // ring kernel, A K-contiguous and B K-strided: the K tail goes through the ring as one more tile.  A's rows
  // hold zeros from K up to the next multiple of 64 (a_extent reaches that far); the lines of B's tail tile at
  // k >= K lie past b_extent and read as zeros
  int32_t ring_tail;
  // persistent launches: workgroups that are resident at a time (compute units of the device, times two for
  // the 4-wavefront tile)
  int32_t resident;
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
  if constexpr (EPI == ntp::EPI_F32 || EPI == ntp::EPI_F32_ACCUM) {
    if (g.n_segs == 0) {
      f32x4* p = reinterpret_cast<f32x4*>(static_cast<float*>(g.C) + int64_t(m) * g.ldc + n0);
      if constexpr (EPI == ntp::EPI_F32) *p = acc;
      else *p = *p + acc;
    } else {
      for (int s = 0; s < g.n_segs; ++s) {
        if (m < g.seg[s].begin || m >= g.seg[s].end) continue;
        f32x4* p = reinterpret_cast<f32x4*>(g.seg[s].ptr + int64_t(m - g.seg[s].begin) * g.seg[s].ld + n0);
        if constexpr (EPI == ntp::EPI_F32) *p = acc;
        else *p = *p + acc;
      }
    }
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

// bf16 epilogues of the ring kernel, two adjacent 16 x 16 accumulator blocks at once.  Lane l holds row
// l % 16 and columns 4 (l / 16) + {0..3} of both blocks (a0: columns from nb, a1: from nb + 16), 8 bytes of
// bf16 each.  After the element-wise part, the four 16-lane rows trade halves (v_permlane16_swap: odd rows
// of the first register against even rows of the second), so that a lane ends up with 8 consecutive
// columns, 16 bytes: rows 0 / 2 take columns 0-7 / 8-15 of the first block, rows 1 / 3 those of the second.
// A store instruction then writes 64 contiguous bytes per output row instead of 32, and there are half as many.
template <int EPI>
__device__ __forceinline__ void store8_pair(const GemmArgs& g, int m, int nb, int lh, f32x4 a0, f32x4 a1) {
  const int n0 = nb + lh * 4, n1 = n0 + 16;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (n0 + j >= g.N) a0[j] = 0.0f;
    if (n1 + j >= g.N) a1[j] = 0.0f;
  }
  if constexpr (EPI == ntp::EPI_DGELU) {
    u16x4 p0 = {0, 0, 0, 0}, p1 = {0, 0, 0, 0};
    if (m < g.M && n0 < g.n_store) p0 = *reinterpret_cast<const u16x4*>(g.AUX + int64_t(m) * g.ldaux + n0);
    if (m < g.M && n1 < g.n_store) p1 = *reinterpret_cast<const u16x4*>(g.AUX + int64_t(m) * g.ldaux + n1);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      a0[j] = (n0 + j < g.N) ? a0[j] * gelu_bwd(bf16_to_f32(p0[j]), g.gelu_mode) : 0.0f;
      a1[j] = (n1 + j < g.N) ? a1[j] * gelu_bwd(bf16_to_f32(p1[j]), g.gelu_mode) : 0.0f;
    }
  }
  auto pack = [](float lo, float hi) { return uint32_t(f32_to_bf16(lo)) | (uint32_t(f32_to_bf16(hi)) << 16); };
  // the lane's 8 output columns after the trade, and the trade itself
  const int c = nb + (lh & 1) * 16 + (lh >> 1) * 8;
  auto trade_store = [&](void* base, int64_t ld, uint32_t x0, uint32_t x1, uint32_t y0, uint32_t y1) {
    const auto r0 = __builtin_amdgcn_permlane16_swap(x0, y0, false, false);
    const auto r1 = __builtin_amdgcn_permlane16_swap(x1, y1, false, false);
    if (m >= g.M) return;
    uint16_t* dst = static_cast<uint16_t*>(base) + int64_t(m) * ld + c;
    if (c + 8 <= g.n_store) {
      typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
      *reinterpret_cast<u32x4*>(dst) = u32x4{r0[0], r1[0], r0[1], r1[1]};
    } else if (c + 4 <= g.n_store) {
      typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
      *reinterpret_cast<u32x2*>(dst) = u32x2{r0[0], r1[0]};
    }
  };
  trade_store(g.C, g.ldc, pack(a0[0], a0[1]), pack(a0[2], a0[3]), pack(a1[0], a1[1]), pack(a1[2], a1[3]));
  if constexpr (EPI == ntp::EPI_GELU) {
    float y0[4], y1[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      y0[j] = gelu_fwd(a0[j], g.gelu_mode);
      y1[j] = gelu_fwd(a1[j], g.gelu_mode);
    }
    trade_store(g.C2, g.ldc2, pack(y0[0], y0[1]), pack(y0[2], y0[3]), pack(y1[0], y1[1]), pack(y1[2], y1[3]));
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

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

}  // namespace ntp_gemm

#endif  // NTP_GEMM_KERNELS_H_
