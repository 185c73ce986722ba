// Gradient reshard: repack a partitioned tensor between two TP layouts.
// (Sec. 3.1 "Shard-mapping algorithm"; Appendix: pre-sync hook and post-sync reshard.)
//
// The host turns the two shard plans into sub-shards (segments); each segment is a
// 2-D copy: `rows` rows of `row_bytes` bytes with independent source / destination
// strides.  One kernel launch copies up to kMaxSegs segments.  A wavefront copies a
// row (or an 8 KiB piece of a long row) with 16-byte stores that are always aligned
// on the destination side; source loads are 16 bytes wide at element alignment, so
// the two layouts may be misaligned against each other (odd shard widths).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

#include "ntp_internal.h"

namespace {

constexpr int kMaxSegs = 56;          // per launch; the argument block stays below 4 KiB
constexpr int kThreads = 256;         // 4 wavefronts
constexpr int kWaves = kThreads / 64;
constexpr int64_t kColChunk = 8192;   // bytes of a row handled by one workgroup
constexpr int64_t kBlockBytes = 65536;  // target bytes per workgroup

struct CopySeg {
  const char* src;
  char* dst;
  int64_t src_stride, dst_stride;  // bytes between rows
  int64_t row_bytes, rows;
  uint32_t first_block;     // first workgroup of this segment
  uint32_t col_chunks;      // pieces a row is cut into
  uint32_t rows_per_block;
  uint32_t pad_;
};

struct CopyBatch {
  CopySeg seg[kMaxSegs];
  int32_t nseg;
  int32_t elem_size;
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));

// Copy `n` bytes from s to d with one wavefront.  d and s are aligned to ESZ and
// (s - d) % 4 == 0 when WIDE.  Stores of the body are 16-byte aligned.
template <int ESZ, bool WIDE>
__device__ __forceinline__ void wave_copy(const char* __restrict__ s, char* __restrict__ d, int64_t n,
                                          int lane) {
  if constexpr (WIDE) {
    const int64_t head = std::min<int64_t>(n, (16 - (reinterpret_cast<uintptr_t>(d) & 15)) & 15);
    const int64_t body = (n - head) & ~int64_t(15);
    const int64_t tail = n - head - body;
    if (lane * ESZ < head) {
      if constexpr (ESZ == 4)
        *reinterpret_cast<uint32_t*>(d + lane * 4) = *reinterpret_cast<const uint32_t*>(s + lane * 4);
      else
        *reinterpret_cast<uint16_t*>(d + lane * 2) = *reinterpret_cast<const uint16_t*>(s + lane * 2);
    }
    const char* sb = s + head;
    char* db = d + head;
    int64_t o = int64_t(lane) * 16;
    // two independent 16-byte transfers per lane in flight
    for (; o + 1024 < body; o += 2048) {
      const u32x4 v0 = *reinterpret_cast<const u32x4_a4*>(sb + o);
      const u32x4 v1 = *reinterpret_cast<const u32x4_a4*>(sb + o + 1024);
      __builtin_nontemporal_store(v0, reinterpret_cast<u32x4*>(db + o));
      __builtin_nontemporal_store(v1, reinterpret_cast<u32x4*>(db + o + 1024));
    }
    if (o < body) {
      const u32x4 v0 = *reinterpret_cast<const u32x4_a4*>(sb + o);
      __builtin_nontemporal_store(v0, reinterpret_cast<u32x4*>(db + o));
    }
    if (lane * ESZ < tail) {
      const int64_t t = head + body + lane * ESZ;
      if constexpr (ESZ == 4)
        *reinterpret_cast<uint32_t*>(d + t) = *reinterpret_cast<const uint32_t*>(s + t);
      else
        *reinterpret_cast<uint16_t*>(d + t) = *reinterpret_cast<const uint16_t*>(s + t);
    }
  } else {
    // 2-byte elements whose source and destination differ by an odd number of
    // halfwords: element-wise copy
    for (int64_t o = int64_t(lane) * 2; o < n; o += 128)
      *reinterpret_cast<uint16_t*>(d + o) = *reinterpret_cast<const uint16_t*>(s + o);
  }
}

__global__ __launch_bounds__(kThreads) void reshard_copy_kernel(const CopyBatch batch) {
  // find this workgroup's segment (segments are few; the table sits in scalar registers / kernarg)
  const uint32_t b = blockIdx.x;
  int si = 0;
  for (int i = 1; i < batch.nseg; ++i)
    if (batch.seg[i].first_block <= b) si = i;
  const CopySeg& sg = batch.seg[si];
  const uint32_t lb = b - sg.first_block;
  const uint32_t rg = lb / sg.col_chunks;
  const uint32_t cc = lb - rg * sg.col_chunks;
  const int64_t c0 = int64_t(cc) * kColChunk;
  const int64_t nbytes = std::min<int64_t>(kColChunk, sg.row_bytes - c0);
  const int64_t r0 = int64_t(rg) * sg.rows_per_block;
  const int64_t r1 = std::min<int64_t>(sg.rows, r0 + sg.rows_per_block);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const bool wide =
      batch.elem_size == 4 || (((reinterpret_cast<uintptr_t>(sg.src) - reinterpret_cast<uintptr_t>(sg.dst)) & 3) == 0 &&
                               ((sg.src_stride - sg.dst_stride) & 3) == 0);
  for (int64_t r = r0 + wave; r < r1; r += kWaves) {
    const char* s = sg.src + r * sg.src_stride + c0;
    char* d = sg.dst + r * sg.dst_stride + c0;
    if (batch.elem_size == 4)
      wave_copy<4, true>(s, d, nbytes, lane);
    else if (wide)
      wave_copy<2, true>(s, d, nbytes, lane);
    else
      wave_copy<2, false>(s, d, nbytes, lane);
  }
}

struct Extent {
  uintptr_t lo, hi;
};

}  // namespace

extern "C" int ntp_reshard_grad(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp,
                                const void* const* src_shards, const int64_t* src_ld,
                                void* const* dst_shards, const int64_t* dst_ld, void* stream) {
  if (!src_shards || !dst_shards || !src_ld || !dst_ld) return NTP_ERR_INVALID_ARG;
  std::vector<ntp_segment_t> segs;
  int st = ntp::build_segments(spec, src_tp, dst_tp, &segs);
  if (st != NTP_OK) return st;
  int64_t n_units = 0;
  ntp::check_spec(spec, src_tp, dst_tp, &n_units);
  const int64_t esz = spec->elem_size;
  const bool by_rows = spec->partition_dim == 0;

  // shard extents: shape, leading dimension, alignment and aliasing checks
  auto extents = [&](int32_t tp, const void* const* ptrs, const int64_t* ld, std::vector<Extent>* out) -> int {
    out->assign(tp, Extent{0, 0});
    for (int32_t r = 0; r < tp; ++r) {
      int64_t units = 0;
      const int s2 = ntp::shard_units(spec, n_units, tp, r, &units);
      if (s2 != NTP_OK) return s2;
      if (!ptrs[r] || units == 0) continue;
      const int64_t srows = by_rows ? units * spec->unit : spec->rows;
      const int64_t scols = by_rows ? spec->cols : units * spec->unit;
      if (srows == 0 || scols == 0) continue;
      if (ld[r] < scols) return NTP_ERR_INVALID_ARG;
      const uintptr_t p = reinterpret_cast<uintptr_t>(ptrs[r]);
      if (p % esz != 0) return NTP_ERR_ALIGNMENT;
      (*out)[r] = Extent{p, p + uintptr_t(((srows - 1) * ld[r] + scols) * esz)};
    }
    return NTP_OK;
  };
  std::vector<Extent> se, de;
  if ((st = extents(src_tp, src_shards, src_ld, &se)) != NTP_OK) return st;
  if ((st = extents(dst_tp, reinterpret_cast<const void* const*>(dst_shards), dst_ld, &de)) != NTP_OK) return st;
  for (const Extent& a : se)
    for (const Extent& b : de)
      if (a.hi > a.lo && b.hi > b.lo && a.lo < b.hi && b.lo < a.hi) return NTP_ERR_INVALID_ARG;

  // segments -> 2-D copies
  std::vector<CopySeg> copies;
  for (const ntp_segment_t& g : segs) {
    const char* sp = static_cast<const char*>(src_shards[g.src_rank]);
    char* dp = static_cast<char*>(dst_shards[g.dst_rank]);
    if (!sp || !dp) continue;  // not on this GPU
    const int64_t sld = src_ld[g.src_rank] * esz, dld = dst_ld[g.dst_rank] * esz;
    CopySeg c{};
    if (by_rows) {
      c.src = sp + g.src_unit * spec->unit * sld;
      c.dst = dp + g.dst_unit * spec->unit * dld;
      c.rows = g.units * spec->unit;
      c.row_bytes = spec->cols * esz;
    } else {
      c.src = sp + g.src_unit * spec->unit * esz;
      c.dst = dp + g.dst_unit * spec->unit * esz;
      c.rows = spec->rows;
      c.row_bytes = g.units * spec->unit * esz;
    }
    c.src_stride = sld;
    c.dst_stride = dld;
    if (c.rows == 0 || c.row_bytes == 0) continue;
    if (c.src_stride == c.row_bytes && c.dst_stride == c.row_bytes && c.rows > 1) {
      // dense on both sides: one long run, recut into 4 KiB rows (plus a remainder)
      const int64_t total = c.rows * c.row_bytes;
      const int64_t full = total / 4096;
      if (full > 0) {
        CopySeg d = c;
        d.rows = full;
        d.row_bytes = d.src_stride = d.dst_stride = 4096;
        copies.push_back(d);
      }
      if (total % 4096) {
        CopySeg d = c;
        d.src += full * 4096;
        d.dst += full * 4096;
        d.rows = 1;
        d.row_bytes = total % 4096;
        copies.push_back(d);
      }
    } else {
      copies.push_back(c);
    }
  }

  hipStream_t hs = static_cast<hipStream_t>(stream);
  for (size_t base = 0; base < copies.size(); base += kMaxSegs) {
    CopyBatch batch{};
    batch.nseg = int32_t(std::min<size_t>(kMaxSegs, copies.size() - base));
    batch.elem_size = int32_t(esz);
    uint64_t blocks = 0;
    for (int i = 0; i < batch.nseg; ++i) {
      CopySeg c = copies[base + i];
      c.col_chunks = uint32_t((c.row_bytes + kColChunk - 1) / kColChunk);
      const int64_t per_row = std::min<int64_t>(c.row_bytes, kColChunk);
      int64_t rpb = std::max<int64_t>(kWaves, kBlockBytes / per_row);
      rpb = (rpb + kWaves - 1) / kWaves * kWaves;
      c.rows_per_block = uint32_t(std::min<int64_t>(rpb, std::max<int64_t>(c.rows, 1)));
      const uint64_t row_groups = uint64_t((c.rows + c.rows_per_block - 1) / c.rows_per_block);
      c.first_block = uint32_t(blocks);
      blocks += row_groups * c.col_chunks;
      if (blocks > 0x7fffffffull) return NTP_ERR_UNSUPPORTED;
      batch.seg[i] = c;
    }
    if (blocks == 0) continue;
    if (ntp::timing_on()) {
      double bytes = 0.0;
      for (int i = 0; i < batch.nseg; ++i) bytes += 2.0 * double(batch.seg[i].rows) * double(batch.seg[i].row_bytes);
      ntp::timing_begin(stream, "reshard_copy", 0.0, bytes);
    }
    hipLaunchKernelGGL(reshard_copy_kernel, dim3(uint32_t(blocks)), dim3(kThreads), 0, hs, batch);
    const bool ok = hipGetLastError() == hipSuccess;
    ntp::timing_end(stream);
    if (!ok) return NTP_ERR_LAUNCH;
  }
  return NTP_OK;
}
