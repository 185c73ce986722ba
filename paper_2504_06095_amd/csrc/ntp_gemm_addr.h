// Index arithmetic of the ring GEMM kernel's operand DMA, kept apart from the kernel so that a host
// program can include it too and enumerate every address the kernel can form (the kernel's loads are
// range-checked by the hardware against the operand's extent; the host model checks the same
// arithmetic against the same extent without a GPU).
#ifndef NTP_GEMM_ADDR_H_
#define NTP_GEMM_ADDR_H_

#include <stdint.h>

#if defined(__HIPCC__)
#define NTP_HD __host__ __device__ __forceinline__
#else
#define NTP_HD inline
#endif

namespace ntp_gemm {

constexpr int DK = 64;  // K extent of a tile

NTP_HD int imin(int a, int b) { return a < b ? a : b; }

// chunk permutation of a K-strided slot line
NTP_HD constexpr int kline_swz(int k) { return ((k & 3) | (((k >> 3) & 1) << 2)) << 1; }

// Rows a tile side of `b` occupies in an LDS slot: whole DMA instructions of 64 rows (K-contiguous), or a
// power-of-two number of 8-element chunks per K line (K-strided).
constexpr int slot_rows(bool kc, int b) { return kc ? (b + 63) / 64 * 64 : (b <= 128 ? 128 : 256); }

// chunk position `pos` of a slot -> (line, chunk) it holds.  K-contiguous [R rows][64 k]: chunk p of row r
// holds k-chunk p ^ ((r >> 1) & 7).  K-strided [64 k][R rows]: chunk p of line k holds row-chunk p ^ kline_swz(k).
template <bool KC, int R>
NTP_HD void slot_src(int pos, int& line, int& chunk) {
  if constexpr (KC) {
    line = pos >> 3;
    chunk = (pos & 7) ^ ((line >> 1) & 7);
  } else {
    constexpr int CPL = R / 8;
    line = pos / CPL;
    chunk = (pos % CPL) ^ kline_swz(line);
  }
}

// Byte offset, from the operand's base at K tile 0, of the 16-byte chunk that slot position (line, chunk)
// takes from a tile whose first row (of the non-K dimension) is row0; lim = extent of that dimension.
// Rows past the edge repeat the last one; a K-strided chunk past the edge repeats the last whole chunk.
template <bool KC>
NTP_HD uint32_t dma_offset(int64_t ld, int row0, int lim, int line, int chunk) {
  if constexpr (KC) {
    const int row = imin(row0 + line, lim - 1);
    return uint32_t((int64_t(row) * ld + chunk * 8) * 2);
  } else {
    const int col = imin(row0 + chunk * 8, ((lim - 1) >> 3) << 3);
    return uint32_t((int64_t(line) * ld + col) * 2);
  }
}

// Bytes of an operand that the kernel may touch, counted from its first element: the hardware range check
// of the DMA loads is set to this, so that an offset beyond it reads zeros instead of memory.
//   K-contiguous [rows x K], ld: rows - 1 whole rows and k_reach elements of the last one, k_reach = K, or K
//     rounded up to 64 when the caller vouches for zero-filled pad columns (K tail through the ring);
//   K-strided [K x rows], ld: K - 1 whole lines and the last one up to the end of its last 8-element chunk.
NTP_HD int64_t operand_extent_bytes(bool kc, int64_t rows, int64_t K, int64_t ld, bool k_pad_64) {
  if (rows <= 0 || K <= 0) return 0;
  if (kc) return ((rows - 1) * ld + (k_pad_64 ? (K + 63) / 64 * 64 : K)) * 2;
  return ((K - 1) * ld + (rows + 7) / 8 * 8) * 2;
}

// Virtual block v of nblk = tiles_m * tiles_n -> output tile.  Workgroups are dealt round-robin to the 8
// XCDs (each with its own L2), so virtual block v belongs to XCD v & 7; every XCD walks a contiguous range
// of tiles in groups of 8 tile rows, so that its workgroups share operands.
struct TilePos {
  int tile_m, tile_n;
};
NTP_HD TilePos place_tile(int v, int tiles_m, int tiles_n) {
  const int nblk = tiles_m * tiles_n;
  const int xq = nblk >> 3, xr = nblk & 7, xcd = v & 7;
  const int L = xcd * xq + imin(xcd, xr) + (v >> 3);
  constexpr int GM = 8;
  const int width = GM * tiles_n;
  const int first_m = (L / width) * GM;
  const int gsz = imin(tiles_m - first_m, GM);
  TilePos p;
  p.tile_m = first_m + (L % width) % gsz;
  p.tile_n = (L % width) / gsz;
  return p;
}

// K tiles that go through the ring for a contraction of K elements: the whole ones, plus the tail tile when
// it may go through the ring too.
NTP_HD int ring_k_tiles(int K, bool ring_tail) { return K / DK + ((ring_tail && K % DK) ? 1 : 0); }

}  // namespace ntp_gemm

#endif  // NTP_GEMM_ADDR_H_
