// Host model of the ring GEMM kernel's operand DMA addressing (no GPU).
//
// It includes the kernel's own index arithmetic (csrc/ntp_gemm_addr.h) and enumerates, for every tile
// variant, operand layout, split-K chunk and a list of ragged shapes, every (offset, K tile) pair that the
// kernel's schedule can issue, and checks each 16-byte load against the operand as the caller's contract
// defines it:
//   - a load lies wholly inside the operand, or
//   - (K tail through the ring, B operand only) wholly outside the range-checked extent, where the hardware
//     returns zeros, and then only for K lines >= K.
// It also evaluates the schedule of a K loop padded to a multiple of five K tiles WITHOUT the clamp on the
// tile index (a variant that was tried and faulted) and reports how far past the operand it reads.
//
// Prints "OK <cases> <loads>" and exits 0, or prints the first violation and exits 1.
// With the argument "padded" it prints "OVERRUN <bytes>" for the unclamped padded loop instead.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ntp_gemm_addr.h"

using namespace ntp_gemm;

struct Tile {
  int bm, bn, nw;
};
static const Tile kTiles[] = {{256, 256, 8}, {256, 224, 8}, {224, 256, 8}, {256, 192, 8}, {192, 256, 8},
                              {256, 128, 8}, {128, 256, 8}, {128, 128, 4}, {128, 128, 8}};

// What the caller's contract says an operand's memory holds, in bytes from its first element, derived from
// the element ranges rather than from the library's formula: the largest byte offset + 1 of any element that
// may legitimately be read.  K-contiguous [rows x K] with ld: elements (r, k), k < k_reach.  K-strided
// [K x rows] with ld: elements (k, c), c < rows rounded up to 8 (rows of such operands are padded to 8).
static int64_t contract_bytes(bool kc, int64_t rows, int64_t K, int64_t ld, int64_t k_reach) {
  int64_t last = -1;
  if (kc) {
    if (rows > 0 && k_reach > 0) last = (rows - 1) * ld + (k_reach - 1);
  } else {
    const int64_t c = (rows + 7) / 8 * 8;
    if (K > 0 && c > 0) last = (K - 1) * ld + (c - 1);
  }
  return (last + 1) * 2;
}

template <bool KC, int R>
static void offsets(int64_t ld, int row0, int lim, std::vector<uint32_t>* out, std::vector<int>* lines) {
  out->clear();
  lines->clear();
  for (int pos = 0; pos < R * 8; ++pos) {  // every chunk position of a slot: all wavefronts, instructions, lanes
    int line, chunk;
    slot_src<KC, R>(pos, line, chunk);
    out->push_back(dma_offset<KC>(ld, row0, lim, line, chunk));
    lines->push_back(line);
  }
}

static void offsets_dyn(bool kc, int R, int64_t ld, int row0, int lim, std::vector<uint32_t>* out, std::vector<int>* lines) {
  if (kc) {
    switch (R) {
      case 64: return offsets<true, 64>(ld, row0, lim, out, lines);
      case 128: return offsets<true, 128>(ld, row0, lim, out, lines);
      case 192: return offsets<true, 192>(ld, row0, lim, out, lines);
      case 256: return offsets<true, 256>(ld, row0, lim, out, lines);
    }
  } else {
    switch (R) {
      case 128: return offsets<false, 128>(ld, row0, lim, out, lines);
      case 256: return offsets<false, 256>(ld, row0, lim, out, lines);
    }
  }
  fprintf(stderr, "no slot of %d rows\n", R);
  exit(2);
}

struct Shape {
  int M, N, K;
  int pad_a, pad_b;  // extra elements on the leading dimensions (multiples of 8)
};

static int64_t g_loads = 0, g_cases = 0;
static int64_t g_overrun = 0;

// One operand of one output tile over one K chunk.  first: K index where the chunk starts; Kc: its length;
// ring_tail: the chunk's K tail goes through the ring; zero_tail_ok: loads at K lines >= K may be out of range.
static bool check_operand(const char* what, bool kc, int b, int64_t ld, int row0, int lim, int64_t K_total, int64_t first,
                          int Kc, bool ring_tail, bool zero_tail_ok, int64_t extent, int64_t contract, bool padded_loop) {
  std::vector<uint32_t> off;
  std::vector<int> lines;
  offsets_dyn(kc, slot_rows(kc, b), ld, row0, lim, &off, &lines);
  const int64_t shift = (kc ? first : first * ld) * 2;        // the chunk's base inside the operand
  const int64_t kstep = (kc ? int64_t(DK) : int64_t(DK) * ld) * 2;  // bytes per K tile
  const int nk = ring_k_tiles(Kc, ring_tail);
  if (nk == 0) return true;
  // K tiles the schedule issues: 0 .. nk-1 (it clamps t+1 and t+2 to nk-1).  The padded loop ran on to the
  // next multiple of five tiles, plus the two tiles of look-ahead, unclamped.
  const int last_kt = padded_loop ? (nk + 4) / 5 * 5 + 1 : nk - 1;
  for (int kt = 0; kt <= last_kt; ++kt) {
    for (size_t i = 0; i < off.size(); ++i) {
      const int64_t o = shift + int64_t(off[i]) + int64_t(kt) * kstep;  // from the operand's first element
      ++g_loads;
      if (padded_loop) {
        if (o + 16 > contract && o + 16 - contract > g_overrun) g_overrun = o + 16 - contract;
        continue;
      }
      if (int64_t(off[i]) + int64_t(kt) * kstep > 0xFFFFFFFFll) {
        printf("FAIL %s: 32-bit offset overflow\n", what);
        return false;
      }
      if (o + 16 <= contract && o + 16 <= extent) continue;  // inside the operand and inside the checked range
      // Otherwise the hardware must zero the whole load (it checks each lane's 16 bytes against the extent),
      // and that is only legitimate for K lines at or past K of the tail tile.
      const int64_t kline = first + int64_t(kt) * DK + (kc ? 0 : lines[i]);
      if (zero_tail_ok && o >= extent && !kc && kline >= K_total) continue;
      printf("FAIL %s: kc=%d tile side %d ld=%lld row0=%d lim=%d K=%lld first=%lld Kc=%d kt=%d off=%u -> byte %lld, contract %lld, "
             "extent %lld\n",
             what, int(kc), b, (long long)ld, row0, lim, (long long)K_total, (long long)first, Kc, kt, off[i], (long long)o,
             (long long)contract, (long long)extent);
      return false;
    }
  }
  return true;
}

static bool run_gemm(bool akc, bool bkc, const Tile& t, const Shape& s, int splits, bool a_pad64, bool padded_loop) {
  const int64_t a_cols = akc ? s.K : s.M, b_cols = bkc ? s.K : s.N;
  int64_t lda = (a_cols + 7) / 8 * 8 + s.pad_a, ldb = (b_cols + 7) / 8 * 8 + s.pad_b;
  const bool layout_nn = akc && !bkc;
  // the launcher's rule for sending the K tail through the ring (persistent form, row-parallel layout)
  bool ring_tail = layout_nn && splits == 1 && a_pad64 && s.K % 64 != 0 && s.K >= 128;
  if (ring_tail) lda = (s.K + 63) / 64 * 64 + s.pad_a;
  const int64_t a_ext = operand_extent_bytes(akc, s.M, s.K, lda, ring_tail);
  const int64_t b_ext = operand_extent_bytes(bkc, s.N, s.K, ldb, false);
  const int64_t a_con = contract_bytes(akc, s.M, s.K, lda, ring_tail ? (s.K + 63) / 64 * 64 : s.K);
  const int64_t b_con = contract_bytes(bkc, s.N, s.K, ldb, s.K);
  if (a_ext > a_con || b_ext > b_con) {
    printf("FAIL extent beyond the contract: a %lld > %lld or b %lld > %lld\n", (long long)a_ext, (long long)a_con,
           (long long)b_ext, (long long)b_con);
    return false;
  }
  const int tiles_m = (s.M + t.bm - 1) / t.bm, tiles_n = (s.N + t.bn - 1) / t.bn;
  const int ktiles = (s.K + 63) / 64;
  const int chunk = splits > 1 ? (ktiles + splits - 1) / splits * 64 : (s.K + 63) / 64 * 64;
  if (splits > 1 && int64_t(splits - 1) * chunk >= s.K) return true;  // the launcher never makes an empty chunk
  // An operand's addresses depend on its own tile index only (A on tile_m, B on tile_n), and only the last
  // tile of a side clamps differently from the others: first, middle and last tile of each side cover all cases.
  for (int side = 0; side < 2; ++side) {
    const int n_tiles = side == 0 ? tiles_m : tiles_n;
    int picks[3] = {0, n_tiles / 2, n_tiles - 1};
    for (int pi = 0; pi < 3; ++pi) {
      if (pi > 0 && picks[pi] == picks[pi - 1]) continue;
      for (int sp = 0; sp < splits; ++sp) {
        const int64_t first = int64_t(sp) * chunk;
        const int Kc = int(std::min<int64_t>(chunk, s.K - first));
        ++g_cases;
        if (side == 0) {
          if (!check_operand("A", akc, t.bm, lda, picks[pi] * t.bm, s.M, s.K, first, Kc, ring_tail, false, a_ext, a_con, padded_loop))
            return false;
        } else {
          if (!check_operand("B", bkc, t.bn, ldb, picks[pi] * t.bn, s.N, s.K, first, Kc, ring_tail, ring_tail, b_ext, b_con, padded_loop))
            return false;
        }
      }
    }
  }
  for (int v = 0; v < tiles_m * tiles_n; ++v) {
    const TilePos p = place_tile(v, tiles_m, tiles_n);
    if (p.tile_m < 0 || p.tile_m >= tiles_m || p.tile_n < 0 || p.tile_n >= tiles_n) {
      printf("FAIL tile walk: block %d -> (%d, %d) of %d x %d\n", v, p.tile_m, p.tile_n, tiles_m, tiles_n);
      return false;
    }
  }
  // the tile walk must visit every tile exactly once
  std::vector<int> seen(size_t(tiles_m) * tiles_n, 0);
  for (int v = 0; v < tiles_m * tiles_n; ++v) {
    const TilePos p = place_tile(v, tiles_m, tiles_n);
    ++seen[size_t(p.tile_m) * tiles_n + p.tile_n];
  }
  for (int x : seen)
    if (x != 1) {
      printf("FAIL tile walk: a tile is visited %d times (%d x %d tiles)\n", x, tiles_m, tiles_n);
      return false;
    }
  return true;
}

int main(int argc, char** argv) {
  const bool padded = argc > 1 && !strcmp(argv[1], "padded");
  const Shape shapes[] = {
      {777, 1001, 1096, 0, 0},  {1, 8, 128, 0, 0},        {3, 17, 200, 8, 16},     {65, 64, 64, 0, 0},     {520, 1500, 1032, 0, 0},
      {2048, 7022, 12288, 0, 0}, {2048, 12288, 7022, 0, 40}, {7022, 12288, 2048, 0, 0}, {8192, 750, 16384, 0, 0}, {8192, 16384, 750, 18 * 8, 0},
      {750, 16384, 8192, 0, 0},  {4096, 640, 8192, 0, 0},  {4096, 8192, 384, 0, 0},  {896, 8192, 4096, 0, 0}, {1100, 1171, 1096, 0, 0},
      {257, 255, 321, 0, 0},     {256, 256, 5376, 0, 0},   {300, 513, 5376 + 41, 0, 0},
  };
  const bool layouts[3][2] = {{true, true}, {true, false}, {false, false}};
  for (const auto& lay : layouts)
    for (const Tile& t : kTiles)
      for (const Shape& s : shapes)
        for (int splits : {1, 2, 3, 5, 8})
          for (int pad64 = 0; pad64 < 2; ++pad64) {
            if (pad64 && !(lay[0] && !lay[1])) continue;
            if (padded && splits > 1) continue;
            if (!run_gemm(lay[0], lay[1], t, s, splits, pad64 != 0, padded)) return 1;
          }
  if (padded) printf("OVERRUN %lld\n", (long long)g_overrun);
  else printf("OK %lld %lld\n", (long long)g_cases, (long long)g_loads);
  return 0;
}
