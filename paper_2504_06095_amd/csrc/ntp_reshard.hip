// Gradient reshard: repack a partitioned tensor between two TP layouts.
// (Sec. 3.1 "Shard-mapping algorithm"; Appendix: pre-sync hook and post-sync reshard.)
//
// The host turns the two shard plans into sub-shards (segments); each segment is a
// 2-D copy: `rows` rows of `row_bytes` bytes with independent source / destination
// strides.  One kernel launch copies up to kMaxSegs segments.  A workgroup takes about
// 64 KiB of a segment (a block of rows, or 8 KiB pieces of long rows) and deals all
// its 16-byte chunks to the threads as one flat list, so short rows (small sub-shards)
// and long rows use the lanes equally well.  The 16-byte accesses need only 4-byte
// alignment, so the two layouts may be misaligned against each other (odd shard
// widths); loads are non-temporal, stores too when the destination rows are 16-byte
// aligned.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <utility>
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

constexpr int kUnroll = 4;  // independent 16-byte transfers per lane in flight

// Exact n / d by a multiply-high with m = ceil(2^32 / d), valid for d >= 2 and n * d <= 2^32
// (d = 1 would need m = 2^32: fast_div passes n through).
__device__ __forceinline__ uint32_t div_magic(uint32_t d) { return uint32_t(((uint64_t(1) << 32) + d - 1) / d); }
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t d, uint32_t magic) {
  return d == 1 ? n : __umulhi(n, magic);
}

// A workgroup copies `nrows` row pieces of `n` bytes each (row i at s + i * ss -> d + i * ds).
// The pieces are cut into 16-byte chunks counted from the piece start and ALL chunks of all rows
// are dealt to the threads as one flat list (item -> row, chunk by a multiply-high), so that short
// pieces (a few elements per row: the small sub-shards) keep every lane busy just like long ones.
// The 16-byte accesses need only 4-byte alignment, so source and destination may be misaligned
// against each other (odd shard widths).  What is left of each piece (n % 16 bytes) is copied
// element by element from a second flat list.
template <int ESZ, bool NT_STORE>
__device__ __forceinline__ void block_copy(const char* __restrict__ s, int64_t ss, char* __restrict__ d, int64_t ds,
                                           uint32_t nrows, uint32_t n, uint32_t tid) {
  const uint32_t cpr = n >> 4;  // whole chunks per row piece
  if (cpr > 0) {
    const uint32_t magic = div_magic(cpr), nitems = nrows * cpr;
    for (uint32_t base = tid; base < nitems; base += kThreads * kUnroll) {
      u32x4 v[kUnroll];
      uint32_t row[kUnroll], off[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint32_t item = base + u * kThreads;
        row[u] = fast_div(item, cpr, magic);
        off[u] = (item - row[u] * cpr) << 4;
        if (item < nitems)
          v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4*>(s + int64_t(row[u]) * ss + off[u]));
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        if (base + u * kThreads < nitems) {
          char* p = d + int64_t(row[u]) * ds + off[u];
          if constexpr (NT_STORE)
            __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4*>(p));
          else
            *reinterpret_cast<u32x4_a4*>(p) = v[u];
        }
      }
    }
  }
  const uint32_t te = (n & 15) / ESZ;  // leftover elements per row piece
  if (te > 0) {
    const uint32_t magic = div_magic(te), nitems = nrows * te, t0 = cpr << 4;
    for (uint32_t item = tid; item < nitems; item += kThreads) {
      const uint32_t row = fast_div(item, te, magic);
      const uint32_t o = t0 + (item - row * te) * ESZ;
      if constexpr (ESZ == 4)
        *reinterpret_cast<uint32_t*>(d + int64_t(row) * ds + o) = *reinterpret_cast<const uint32_t*>(s + int64_t(row) * ss + o);
      else
        *reinterpret_cast<uint16_t*>(d + int64_t(row) * ds + o) = *reinterpret_cast<const uint16_t*>(s + int64_t(row) * ss + o);
    }
  }
}

// 2-byte elements whose addresses are only 2-byte aligned: element-wise copy
__device__ __forceinline__ void block_copy_halfwords(const char* __restrict__ s, int64_t ss, char* __restrict__ d, int64_t ds,
                                                     uint32_t nrows, uint32_t n, uint32_t tid) {
  const uint32_t epr = n >> 1, magic = div_magic(epr), nitems = nrows * epr;
  for (uint32_t item = tid; item < nitems; item += kThreads) {
    const uint32_t row = fast_div(item, epr, magic);
    const uint32_t o = (item - row * epr) << 1;
    *reinterpret_cast<uint16_t*>(d + int64_t(row) * ds + o) = *reinterpret_cast<const uint16_t*>(s + int64_t(row) * ss + o);
  }
}

__global__ __launch_bounds__(kThreads) void reshard_copy_kernel(const CopyBatch batch) {
  // find this workgroup's segment (segments are few; the table sits in the kernel arguments)
  const uint32_t b = blockIdx.x;
  int si = 0;
  for (int i = 1; i < batch.nseg; ++i)
    if (batch.seg[i].first_block <= b) si = i;
  const CopySeg& sg = batch.seg[si];
  const uint32_t lb = b - sg.first_block;
  const uint32_t rg = lb / sg.col_chunks;
  const uint32_t cc = lb - rg * sg.col_chunks;
  const int64_t c0 = int64_t(cc) * kColChunk;
  const uint32_t nbytes = uint32_t(std::min<int64_t>(kColChunk, sg.row_bytes - c0));
  const int64_t r0 = int64_t(rg) * sg.rows_per_block;
  const uint32_t nrows = uint32_t(std::min<int64_t>(sg.rows - r0, sg.rows_per_block));
  const char* s = sg.src + r0 * sg.src_stride + c0;
  char* d = sg.dst + r0 * sg.dst_stride + c0;
  const uintptr_t sa = reinterpret_cast<uintptr_t>(sg.src), da = reinterpret_cast<uintptr_t>(sg.dst);
  // 16-byte accesses need 4-byte aligned rows on both sides (always true for 4-byte elements)
  const bool wide = batch.elem_size == 4 || (((sa | da | uintptr_t(sg.src_stride) | uintptr_t(sg.dst_stride)) & 3) == 0);
  const bool dst16 = ((da | uintptr_t(sg.dst_stride)) & 15) == 0;
  const uint32_t tid = threadIdx.x;
  if (batch.elem_size == 4) {
    if (dst16)
      block_copy<4, true>(s, sg.src_stride, d, sg.dst_stride, nrows, nbytes, tid);
    else
      block_copy<4, false>(s, sg.src_stride, d, sg.dst_stride, nrows, nbytes, tid);
  } else if (wide) {
    block_copy<2, false>(s, sg.src_stride, d, sg.dst_stride, nrows, nbytes, tid);
  } else {
    block_copy_halfwords(s, sg.src_stride, d, sg.dst_stride, nrows, nbytes, tid);
  }
}


// ---- column-partitioned tensors of 4-byte elements: destination-major gather ------------------
// A job is a block of destination columns of one destination shard together with the pieces
// (sub-shards) that fill it, each from another source shard.  A workgroup takes a block of
// destination rows and copies all pieces of those rows, so destination rows are written whole and
// in order.  Within a piece the 16-byte chunks are aligned on the DESTINATION address (aligned
// non-temporal stores; the loads tolerate any 4-byte alignment); what lies before the first and
// after the last aligned chunk of a row piece is copied word by word.
constexpr int kMaxPieces = 8;
constexpr int kMaxJobs = 14;  // the argument block stays below 4 KiB

struct Piece {
  const char* src;      // byte that goes to column `begin` of destination row 0 of the job
  int64_t src_stride;   // bytes between source rows
  uint32_t begin, end;  // byte range within the job's destination row
};
struct GatherJob {
  char* dst;            // first byte of the job's column block in destination row 0
  int64_t dst_stride;
  uint32_t rows, npieces;
  Piece piece[kMaxPieces];
};
struct GatherBatch {
  GatherJob job[kMaxJobs];  // all with the same number of rows
  int32_t njobs;
  uint32_t rows_per_block;
};

// One piece of `nrows` destination rows, n bytes per row.  HBM is written in 64-byte units, and a
// unit written in two parts costs two transactions, so in every row the copy is cut at the 64-byte
// boundaries of the DESTINATION address: `head` bytes (a multiple of 4 below 64) come before the
// first boundary.  Pass 1 moves the whole units of all rows as one flat list of 16-byte chunks (four
// neighbouring lanes fill one unit with one aligned non-temporal store instruction; the loads take
// any 4-byte alignment); pass 2 moves what is left at the two ends of each row word by word, again as
// one flat list.  Offsets inside the block fit in 32 bits (the host sees to that).
__device__ __forceinline__ void piece_copy_aligned(const char* __restrict__ s, uint32_t ss, char* __restrict__ d, uint32_t ds,
                                                   uint32_t nrows, uint32_t n, uint32_t tid) {
  const uint32_t dlow = uint32_t(reinterpret_cast<uintptr_t>(d)) & 63u;
  const uint32_t cpr = (n >> 6) << 2;  // chunks of the most whole units a row can hold
  if (cpr > 0) {
    const uint32_t magic = div_magic(cpr), nitems = nrows * cpr;
    for (uint32_t base = tid; base < nitems; base += kThreads * kUnroll) {
      u32x4 v[kUnroll];
      uint32_t doff[kUnroll];
      bool ok[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint32_t item = base + u * kThreads;
        const uint32_t row = nrows == 1 ? 0u : fast_div(item, cpr, magic);
        const uint32_t k = item - row * cpr;
        const uint32_t drow = row * ds;
        const uint32_t head = (0u - (dlow + drow)) & 63u;
        const uint32_t st = head + (k << 4);
        ok[u] = item < nitems && head + ((k | 3u) << 4) + 16u <= n;  // the whole unit of this chunk fits
        doff[u] = drow + st;
        if (ok[u]) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4*>(s + (row * ss + st)));
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        if (ok[u]) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4*>(d + doff[u]));
    }
  }
  // the ends, one word per item: item = 32 row + 16 (0: before the first boundary, 1: after the last whole unit) + word
  for (uint32_t item = tid; item < 32 * nrows; item += kThreads) {
    const uint32_t row = item >> 5, drow = row * ds, w = item & 15u;
    const uint32_t head = min(n, (0u - (dlow + drow)) & 63u);
    const uint32_t st = (item & 16u) ? head + ((n - head) & ~63u) : 0u;
    const uint32_t en = (item & 16u) ? n : head;
    if (st + 4u * w < en)
      *reinterpret_cast<uint32_t*>(d + (drow + st + 4u * w)) = *reinterpret_cast<const uint32_t*>(s + (row * ss + st + 4u * w));
  }
}

// Workgroup b takes row block b / njobs of job b % njobs: the workgroups that run at the same time
// cover the same rows of neighbouring destination shards, so the two destination shards that split
// a source row read it close together in time (its lines are fetched from HBM once).
__global__ __launch_bounds__(kThreads) void reshard_gather_kernel(const GatherBatch batch) {
  const uint32_t rbi = blockIdx.x / uint32_t(batch.njobs), ji = blockIdx.x - rbi * uint32_t(batch.njobs);
  const GatherJob& job = batch.job[ji];
  const int64_t r0 = int64_t(rbi) * batch.rows_per_block;
  const uint32_t nrows = uint32_t(std::min<int64_t>(int64_t(job.rows) - r0, batch.rows_per_block));
  for (uint32_t p = 0; p < job.npieces; ++p) {
    const Piece& pc = job.piece[p];
    piece_copy_aligned(pc.src + r0 * pc.src_stride, uint32_t(pc.src_stride), job.dst + r0 * job.dst_stride + pc.begin,
                       uint32_t(job.dst_stride), nrows, pc.end - pc.begin, threadIdx.x);
  }
}

// Dense destination shards: the destination is treated as ONE flat byte range, cut into blocks at
// 64-byte boundaries, and every 16-byte chunk of it is stored whole and aligned no matter where rows
// and pieces begin (odd shard widths).  A chunk that lies inside one piece of one row is read with
// one (unaligned) 16-byte load; a chunk that straddles a row end or a piece boundary is assembled
// from four single words.  Needs: destination 64-byte aligned and dense, (kFlatBlock + W) * W <= 2^32
// for the row width W in bytes (exact multiply-high division), source offsets inside a block < 2^32.
constexpr uint32_t kFlatBlockMax = 65536;

__global__ __launch_bounds__(kThreads) void reshard_flat_kernel(const GatherBatch batch) {
  // consecutive workgroups take consecutive blocks of one job (measured faster than dealing the jobs round)
  const uint32_t nblk = gridDim.x / uint32_t(batch.njobs);
  const uint32_t ji = blockIdx.x / nblk, bi = blockIdx.x - ji * nblk;
  const GatherJob& job = batch.job[ji];
  const uint32_t np = job.npieces;
  const uint32_t W = job.piece[np - 1].end;
  const int64_t T = int64_t(job.rows) * W;
  const uint32_t kFlatBlock = batch.rows_per_block;  // bytes per block here
  const int64_t b0 = int64_t(bi) * kFlatBlock;
  if (b0 >= T) return;
  const uint32_t nb = uint32_t(std::min<int64_t>(kFlatBlock, T - b0));
  const int64_t row0 = b0 / W;
  const uint32_t c0 = uint32_t(b0 - row0 * W);
  const uint32_t magic = div_magic(W);
  char* __restrict__ d = job.dst + b0;
  const uint32_t nchunks = (nb + 15) >> 4;
  for (uint32_t base = threadIdx.x; base < nchunks; base += kThreads * kUnroll) {
    u32x4 v[kUnroll];
    uint32_t len[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t k = base + u * kThreads;
      len[u] = k < nchunks ? min(16u, nb - (k << 4)) : 0u;
      const uint32_t x = c0 + (k << 4);
      const uint32_t rr = fast_div(x, W, magic);
      const uint32_t col = x - rr * W;
      bool got = len[u] == 0;
      if (len[u] == 16 && col + 16u <= W) {
        for (uint32_t p = 0; p < np; ++p) {
          const Piece& pc = job.piece[p];
          if (col >= pc.begin && col + 16u <= pc.end) {
            const char* sb = pc.src + row0 * pc.src_stride;
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4*>(sb + (rr * uint32_t(pc.src_stride) + (col - pc.begin))));
            got = true;
          }
        }
      }
      if (!got) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          if (uint32_t(w) * 4 >= len[u]) continue;
          const uint32_t rw = fast_div(x + 4u * w, W, magic), cw = x + 4u * w - rw * W;  // rows may be shorter than a chunk
          for (uint32_t p = 0; p < np; ++p) {
            const Piece& pc = job.piece[p];
            if (cw >= pc.begin && cw < pc.end) {
              const char* sb = pc.src + row0 * pc.src_stride;
              v[u][w] = *reinterpret_cast<const uint32_t*>(sb + (rw * uint32_t(pc.src_stride) + (cw - pc.begin)));
            }
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      char* dp = d + ((base + u * kThreads) << 4);
      if (len[u] == 16) {
        __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4*>(dp));
      } else {
#pragma unroll
        for (int w = 0; w < 3; ++w)
          if (uint32_t(w) * 4 < len[u]) reinterpret_cast<uint32_t*>(dp)[w] = v[u][w];
      }
    }
  }
}

// ---- dense ranges (row-partitioned tensors whose shards are dense): plain streaming copy --------
constexpr int kMaxRanges = 100;  // 100 x 32 B + header < 4 KiB of kernel arguments
constexpr int64_t kDenseBlock = 16384;  // bytes per workgroup
struct DenseRange {
  const char* src;
  char* dst;
  int64_t bytes;         // multiple of 16; both pointers 16-byte aligned
  uint32_t first_block;
  uint32_t pad_;
};
struct DenseBatch {
  DenseRange r[kMaxRanges];
  int32_t n;
};

__global__ __launch_bounds__(kThreads) void reshard_dense_kernel(const DenseBatch batch) {
  const uint32_t b = blockIdx.x;
  int lo = 0, hi = batch.n - 1;  // last range whose first block is <= b
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (batch.r[mid].first_block <= b) lo = mid;
    else hi = mid - 1;
  }
  const DenseRange& rg = batch.r[lo];
  const int64_t off = int64_t(b - rg.first_block) * kDenseBlock;
  const uint32_t n16 = uint32_t(std::min<int64_t>(kDenseBlock, rg.bytes - off) >> 4);
  const u32x4* s = reinterpret_cast<const u32x4*>(rg.src + off);
  u32x4* d = reinterpret_cast<u32x4*>(rg.dst + off);
  for (uint32_t base = threadIdx.x; base < n16; base += kThreads * kUnroll) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (base + u * kThreads < n16) v[u] = __builtin_nontemporal_load(s + base + u * kThreads);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u)
      if (base + u * kThreads < n16) __builtin_nontemporal_store(v[u], d + base + u * kThreads);
  }
}

// ---- layouts given unit by unit (Sec. 3.1, Alg. 1): gather through a run table -------------------
// The destination shards are dense and are written like the flat kernel writes them: as one flat
// byte range cut into blocks at 64-byte boundaries, every 16-byte chunk stored whole and aligned.
// A destination shard is a sequence of runs (units that follow each other in one source shard too);
// the plan keeps, in device memory, the runs of every destination shard and for every destination
// unit the number of its run.  A workgroup serves one destination shard: it copies both tables into
// LDS (runs joined with this call's source pointers) and then takes one block of the shard, or walks
// over several when the shard is very large.  A chunk that lies inside one run is moved by one
// 16-byte load and store.  The
// other chunks (they straddle a run boundary or a row end, or are the short last chunk of the
// shard) are put on a queue that each wavefront keeps in LDS, and are put together word by word when
// the queue has filled up, so that this slower code runs with most lanes in use even when few
// chunks need it.  Needs: 4-byte elements, dense 64-byte aligned destinations,
// (block + W + 16) * W <= 2^32 for the row width W in bytes, source strides below 2^32 bytes, at
// most kMaxRanks source ranks, at most 65535 runs per shard.
constexpr int kMaxRanks = 96;
constexpr int kUnitDsts = 16;               // destination shards per launch: few write streams at a time measured fastest
constexpr uint32_t kUnitLdsMax = 60 << 10;  // bytes of LDS a workgroup may ask for
constexpr uint32_t kQueueCap = 512;         // queued chunks per wavefront
constexpr uint32_t kUnitBlocksPerCu = 256;  // workgroups per compute unit and launch before they start to walk over several blocks

struct UnitSrc {
  const char* base;  // first byte of the source shard
  uint64_t stride;   // bytes between its rows
};
struct RunDev {      // one run of a destination shard (plan, device memory)
  uint32_t begin, end;  // byte range in a destination row
  uint32_t src_off;     // byte offset in a source row of what goes to `begin`
  uint32_t rank;        // source rank
};
struct RunLds {      // the same, joined with the source pointers of this call
  uint32_t begin, end, stride, pad_;
  uint64_t adj;      // source base + src_off - begin: column c of row r is at adj + r * stride + c
  uint64_t pad2_;
};
struct UnitDst {
  char* dst;
  uint32_t idx_first, n_units;   // this shard's slice of the unit -> run numbers
  uint32_t runs_first, n_runs;   // this shard's slice of the runs
};
struct UnitBatch {
  UnitSrc src[kMaxRanks];
  UnitDst dst[kUnitDsts];
  const RunDev* runs;
  const uint16_t* run_of_unit;
  uint32_t rows, unit_bytes, ndst, block_bytes;
};

__host__ __device__ inline uint32_t unit_tables_bytes(uint32_t n_runs, uint32_t n_units) {
  return n_runs * uint32_t(sizeof(RunLds)) + ((n_units * 2u + 15u) & ~15u);
}
__host__ __device__ inline uint32_t unit_lds_bytes(uint32_t n_runs, uint32_t n_units) {
  return unit_tables_bytes(n_runs, n_units) + kWaves * kQueueCap * uint32_t(sizeof(uint2));
}

__global__ __launch_bounds__(kThreads) void reshard_units_kernel(const UnitBatch batch) {
  extern __shared__ __align__(16) unsigned char unit_lds[];
  // consecutive workgroups take consecutive blocks of one destination shard
  const uint32_t nslots = gridDim.x / batch.ndst;
  const uint32_t di = blockIdx.x / nslots, slot = blockIdx.x - di * nslots;
  const UnitDst& dd = batch.dst[di];
  const uint32_t ub = batch.unit_bytes, blk = batch.block_bytes;
  const uint32_t W = dd.n_units * ub;
  const int64_t T = int64_t(batch.rows) * W;
  int64_t b0 = int64_t(slot) * blk;
  if (b0 >= T) return;  // the whole workgroup leaves: nothing left for it in this shard
  RunLds* const runs = reinterpret_cast<RunLds*>(unit_lds);
  uint16_t* const run_of = reinterpret_cast<uint16_t*>(unit_lds + dd.n_runs * sizeof(RunLds));
  const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63u;
  uint2* const queue = reinterpret_cast<uint2*>(unit_lds + unit_tables_bytes(dd.n_runs, dd.n_units)) + wave * kQueueCap;
  for (uint32_t r = threadIdx.x; r < dd.n_runs; r += kThreads) {
    const RunDev rd = batch.runs[dd.runs_first + r];
    const UnitSrc sr = batch.src[rd.rank];
    RunLds o;
    o.begin = rd.begin;
    o.end = rd.end;
    o.stride = uint32_t(sr.stride);
    o.pad_ = 0;
    o.adj = uint64_t(reinterpret_cast<uintptr_t>(sr.base)) + rd.src_off - rd.begin;
    o.pad2_ = 0;
    runs[r] = o;
  }
  for (uint32_t j = threadIdx.x; j < dd.n_units; j += kThreads) run_of[j] = batch.run_of_unit[dd.idx_first + j];
  __syncthreads();  // the only workgroup-wide wait: from here on the wavefronts run on their own

  // W and the unit size are at least 4: the multiply-high division needs no special case
  const uint32_t magic_w = div_magic(W), magic_u = div_magic(ub);
  const char* const dummy = reinterpret_cast<const char*>(batch.runs);  // 16 readable bytes for lanes with nothing to load
  // queued chunks of this wavefront, word by word
  uint32_t nq = 0;  // chunks on this wavefront's queue (the same value in all lanes)
  auto flush = [&]() {
    // what other lanes have queued becomes visible
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    for (uint32_t i = lane; i < nq; i += 64) {
      const uint2 e = queue[i];  // {row, byte column} of the chunk's first word
      const int64_t at = int64_t(e.x) * W + e.y;
      const uint32_t len = uint32_t(std::min<int64_t>(16, T - at));
      u32x4 v;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const bool have = uint32_t(w) * 4 < len;
        const uint32_t xw = e.y + (have ? 4u * w : 0u);
        const uint32_t rw = __umulhi(xw, magic_w), cw = xw - rw * W;  // rows may be shorter than a chunk
        const RunLds rn = runs[run_of[__umulhi(cw, magic_u)]];
        v[w] = *reinterpret_cast<const uint32_t*>(rn.adj + (uint64_t(e.x + rw) * rn.stride + cw));
      }
      char* dp = dd.dst + at;
      if (len == 16) {
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dp));
      } else {
#pragma unroll
        for (int w = 0; w < 3; ++w)
          if (uint32_t(w) * 4 < len) reinterpret_cast<uint32_t*>(dp)[w] = v[w];
      }
    }
    // the entries have been read before the queue is filled again
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    nq = 0;
  };

  // this workgroup's blocks: slot, slot + nslots, ...; (row0, c0) = position of the block's first byte
  const int64_t step = int64_t(nslots) * blk;
  const uint32_t step_rows = uint32_t(step / W), step_cols = uint32_t(step - int64_t(step_rows) * W);
  uint32_t row0 = uint32_t(b0 / W);
  uint32_t c0 = uint32_t(b0 - int64_t(row0) * W);
  for (; b0 < T; b0 += step) {
    const uint32_t nb = uint32_t(std::min<int64_t>(blk, T - b0));
    char* __restrict__ d = dd.dst + b0;
    const uint32_t nchunks = (nb + 15) >> 4;
    // the loop bounds are the same for all lanes of a wavefront: every lane takes part in flush()
    for (uint32_t wbase = wave << 6; wbase < nchunks; wbase += kThreads * kUnroll) {
      const uint32_t base = wbase + lane;
      u32x4 v[kUnroll];
      bool ok[kUnroll], slow[kUnroll];
      uint32_t rowq[kUnroll], colq[kUnroll];
      // look every chunk up and start its load; lanes with no chunk, or with a chunk for the slow way,
      // go through the same steps on chunk 0 and load the dummy bytes (no branches, four loads in flight)
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint32_t k = base + u * kThreads;
        const bool valid = k < nchunks;
        const uint32_t kb = valid ? k << 4 : 0u;
        const uint32_t x = c0 + kb;
        const uint32_t rr = __umulhi(x, magic_w), col = x - rr * W;
        const RunLds rn = runs[run_of[__umulhi(col, magic_u)]];
        ok[u] = valid && kb + 16u <= nb && col + 16u <= rn.end;
        slow[u] = valid && !ok[u];
        rowq[u] = row0 + rr;
        colq[u] = col;
        const char* p = reinterpret_cast<const char*>(rn.adj + (uint64_t(row0 + rr) * rn.stride + col));
        v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4*>(ok[u] ? p : dummy));
      }
      // the chunks that need the slow way go on the queue, in lane order
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) {
        const uint64_t m = __ballot(slow[u]);
        if (slow[u]) queue[nq + __builtin_amdgcn_mbcnt_hi(uint32_t(m >> 32), __builtin_amdgcn_mbcnt_lo(uint32_t(m), 0u))] = make_uint2(rowq[u], colq[u]);
        nq += uint32_t(__popcll(m));
      }
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        if (ok[u]) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4*>(d + ((base + u * kThreads) << 4)));
      // one pass of the loop queues at most 64 * kUnroll chunks per wavefront
      if (nq > kQueueCap - 64 * kUnroll) flush();
    }
    row0 += step_rows;
    c0 += step_cols;
    if (c0 >= W) {
      c0 -= W;
      ++row0;
    }
  }
  flush();
}

struct Extent {
  uintptr_t lo, hi;
};

int64_t gather_block_bytes(const ntp_handle* h) {
  if (const int64_t e = h->opt[NTP_OPT_RESHARD_BLOCK]) return std::max<int64_t>(1024, e);
  return kBlockBytes;
}

// Plain dense copy of 16-byte words: the yardstick that profiler byte counters are scaled by.
__global__ __launch_bounds__(256) void calibration_copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                               int64_t words) {
  const int64_t stride = int64_t(gridDim.x) * blockDim.x;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < words; i += stride) dst[i] = src[i];
}

}  // namespace

extern "C" int ntp_calibration_copy(ntp_handle_t* h, void* dst, const void* src, int64_t bytes, void* stream) {
  if (!h || !dst || !src || bytes < 0) return NTP_ERR_INVALID_ARG;
  if (h->device < 0) return NTP_ERR_NO_DEVICE;
  if (bytes % 16 || reinterpret_cast<uintptr_t>(dst) % 16 || reinterpret_cast<uintptr_t>(src) % 16) return NTP_ERR_ALIGNMENT;
  if (bytes == 0) return NTP_OK;
  const int64_t words = bytes / 16;
  const uint32_t blocks = uint32_t(std::min<int64_t>((words + 255) / 256, int64_t(h->compute_units) * 32));
  if (ntp::timing_on(h)) ntp::timing_begin(h, stream, "calibration_copy", 0.0, 2.0 * double(bytes));
  hipLaunchKernelGGL(calibration_copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), words);
  const bool ok = hipGetLastError() == hipSuccess;
  ntp::timing_end(h, stream);
  return ok ? NTP_OK : NTP_ERR_LAUNCH;
}

// ---- sum of replicated units over their holders --------------------------------------------------
namespace {

constexpr int kMaxHolders = 96;  // ranks that may hold one unit (kernel argument space)

// One replicated unit: a [rows x cols] fp32 block in each of n holders' shards.
struct ReplicaGroup {
  float* ptr[kMaxHolders];
  int64_t ld[kMaxHolders];
  int32_t n, rows, cols, vec4;  // vec4: every pointer is 16-byte aligned, cols % 4 == 0, every ld % 4 == 0
};

// Every element: the holders' values added in ascending rank order (a fixed order, so the result is
// deterministic), then written back to all of them.  One thread owns an element (or four) in every holder, so
// the update in place is safe.
__global__ __launch_bounds__(256) void replica_sum_kernel(const ReplicaGroup g) {
  const int64_t per_row = g.vec4 ? g.cols / 4 : g.cols;
  const int64_t total = int64_t(g.rows) * per_row, stride = int64_t(gridDim.x) * blockDim.x;
  for (int64_t i = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int64_t r = i / per_row, c = i - r * per_row;
    if (g.vec4) {
      typedef float f4 __attribute__((ext_vector_type(4)));
      f4 sum = *reinterpret_cast<const f4*>(g.ptr[0] + r * g.ld[0] + c * 4);
      for (int k = 1; k < g.n; ++k) sum = sum + *reinterpret_cast<const f4*>(g.ptr[k] + r * g.ld[k] + c * 4);
      for (int k = 0; k < g.n; ++k) *reinterpret_cast<f4*>(g.ptr[k] + r * g.ld[k] + c * 4) = sum;
    } else {
      float sum = g.ptr[0][r * g.ld[0] + c];
      for (int k = 1; k < g.n; ++k) sum += g.ptr[k][r * g.ld[k] + c];
      for (int k = 0; k < g.n; ++k) g.ptr[k][r * g.ld[k] + c] = sum;
    }
  }
}

}  // namespace

extern "C" int ntp_replica_sum(ntp_handle_t* h, const ntp_tensor_spec_t* spec, int32_t tp, void* const* shards,
                               const int64_t* ld, void* stream) {
  if (!h || !shards || !ld) return NTP_ERR_INVALID_ARG;
  int64_t n_units = 0;
  int st = ntp::check_spec(spec, tp, tp, &n_units);
  if (st != NTP_OK) return st;
  if (spec->elem_size != 4) return NTP_ERR_INVALID_ARG;  // the sum is fp32 arithmetic
  if (spec->kind == NTP_KIND_PLAIN) return NTP_OK;       // every unit has one holder
  // shape and alignment of the shards, and: no two shards may overlap
  std::vector<int64_t> units(tp), none;
  for (int32_t r = 0; r < tp; ++r)
    if ((st = ntp::shard_units(spec, n_units, tp, r, &units[r])) != NTP_OK) return st;
  std::vector<void*> no_dst;
  {
    std::vector<Extent> ext(tp, Extent{0, 0});
    const bool by_rows = spec->partition_dim == 0;
    for (int32_t r = 0; r < tp; ++r) {
      if (!shards[r] || units[r] == 0) continue;
      const int64_t srows = by_rows ? units[r] * spec->unit : spec->rows, scols = by_rows ? spec->cols : units[r] * spec->unit;
      if (srows == 0 || scols == 0) continue;
      if (ld[r] < scols) return NTP_ERR_INVALID_ARG;
      const uintptr_t p = reinterpret_cast<uintptr_t>(shards[r]);
      if (p % 4) return NTP_ERR_ALIGNMENT;
      ext[r] = Extent{p, p + uintptr_t(((srows - 1) * ld[r] + scols) * 4)};
    }
    for (int32_t a = 0; a < tp; ++a)
      for (int32_t b = a + 1; b < tp; ++b)
        if (ext[a].hi > ext[a].lo && ext[b].hi > ext[b].lo && ext[a].lo < ext[b].hi && ext[b].lo < ext[a].hi) return NTP_ERR_INVALID_ARG;
  }
  if (h->device < 0) return NTP_ERR_NO_DEVICE;
  // holders of every logical unit, ascending rank order
  std::vector<std::vector<std::pair<int32_t, int64_t>>> holders(static_cast<size_t>(n_units));
  std::vector<ntp::Run> runs;
  for (int32_t r = 0; r < tp; ++r) {
    if ((st = ntp::rank_runs(spec, n_units, tp, r, &runs)) != NTP_OK) return st;
    for (const ntp::Run& run : runs)
      for (int64_t i = 0; i < run.count; ++i) holders[size_t(run.first + i)].push_back({r, run.local + i});
  }
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const bool by_rows = spec->partition_dim == 0;
  for (int64_t u = 0; u < n_units; ++u) {
    const auto& hd = holders[size_t(u)];
    if (hd.size() < 2) continue;
    if (hd.size() > size_t(kMaxHolders)) return NTP_ERR_UNSUPPORTED;
    ReplicaGroup g{};
    g.rows = int32_t(by_rows ? spec->unit : spec->rows);
    g.cols = int32_t(by_rows ? spec->cols : spec->unit);
    if ((by_rows ? spec->cols : spec->rows) > 0x7fffffffll) return NTP_ERR_UNSUPPORTED;
    g.vec4 = g.cols % 4 == 0;
    for (const auto& [r, local] : hd) {
      if (!shards[r]) continue;  // a holder that is not on this GPU takes no part
      float* base = static_cast<float*>(shards[r]);
      g.ptr[g.n] = by_rows ? base + local * spec->unit * ld[r] : base + local * spec->unit;
      g.ld[g.n] = ld[r];
      if ((reinterpret_cast<uintptr_t>(g.ptr[g.n]) & 15) || ld[r] % 4) g.vec4 = 0;
      ++g.n;
    }
    if (g.n < 2 || g.rows == 0 || g.cols == 0) continue;
    const int64_t work = int64_t(g.rows) * (g.vec4 ? g.cols / 4 : g.cols);
    const uint32_t blocks = uint32_t(std::max<int64_t>(1, std::min<int64_t>((work + 255) / 256, int64_t(h->compute_units) * 16)));
    if (ntp::timing_on(h)) ntp::timing_begin(h, stream, "replica_sum", 0.0, 2.0 * 4.0 * double(g.n) * double(g.rows) * double(g.cols));
    hipLaunchKernelGGL(replica_sum_kernel, dim3(blocks), dim3(256), 0, hs, g);
    const bool ok = hipGetLastError() == hipSuccess;
    ntp::timing_end(h, stream);
    if (!ok) return NTP_ERR_LAUNCH;
  }
  return NTP_OK;
}

extern "C" int ntp_reshard_grad(ntp_handle_t* h, const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp,
                                const void* const* src_shards, const int64_t* src_ld,
                                void* const* dst_shards, const int64_t* dst_ld, void* stream) {
  if (!h || !src_shards || !dst_shards || !src_ld || !dst_ld) return NTP_ERR_INVALID_ARG;
  std::vector<ntp_segment_t> segs;
  int st = ntp::build_segments(spec, src_tp, dst_tp, &segs);
  if (st != NTP_OK) return st;
  int64_t n_units = 0;
  ntp::check_spec(spec, src_tp, dst_tp, &n_units);
  std::vector<int64_t> su(src_tp), du(dst_tp);
  for (int32_t r = 0; r < src_tp; ++r)
    if ((st = ntp::shard_units(spec, n_units, src_tp, r, &su[r])) != NTP_OK) return st;
  for (int32_t r = 0; r < dst_tp; ++r)
    if ((st = ntp::shard_units(spec, n_units, dst_tp, r, &du[r])) != NTP_OK) return st;
  return ntp::reshard_launch(h, spec, segs, su, du, src_shards, src_ld, dst_shards, dst_ld, stream);
}

int ntp::check_shards(const ntp_tensor_spec_t* spec, const std::vector<int64_t>& src_units,
                      const std::vector<int64_t>& dst_units, const void* const* src_shards, const int64_t* src_ld,
                      void* const* dst_shards, const int64_t* dst_ld) {
  if (!src_shards || !dst_shards || !src_ld || !dst_ld) return NTP_ERR_INVALID_ARG;
  const int64_t esz = spec->elem_size;
  const bool by_rows = spec->partition_dim == 0;
  auto extents = [&](const std::vector<int64_t>& nunits, const void* const* ptrs, const int64_t* ld,
                     std::vector<Extent>* out) -> int {
    const int32_t tp = int32_t(nunits.size());
    out->assign(tp, Extent{0, 0});
    for (int32_t r = 0; r < tp; ++r) {
      const int64_t units = nunits[r];
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
  int st;
  if ((st = extents(src_units, src_shards, src_ld, &se)) != NTP_OK) return st;
  if ((st = extents(dst_units, reinterpret_cast<const void* const*>(dst_shards), dst_ld, &de)) != NTP_OK) return st;
  for (const Extent& a : se)
    for (const Extent& b : de)
      if (a.hi > a.lo && b.hi > b.lo && a.lo < b.hi && b.lo < a.hi) return NTP_ERR_INVALID_ARG;
  return NTP_OK;
}

int ntp::reshard_launch(ntp_handle* h, const ntp_tensor_spec_t* spec, const std::vector<ntp_segment_t>& segs,
                        const std::vector<int64_t>& src_units, const std::vector<int64_t>& dst_units,
                        const void* const* src_shards, const int64_t* src_ld, void* const* dst_shards,
                        const int64_t* dst_ld, void* stream) {
  const int st = check_shards(spec, src_units, dst_units, src_shards, src_ld, dst_shards, dst_ld);
  if (st != NTP_OK) return st;
  if (h->device < 0) return NTP_ERR_NO_DEVICE;
  const int64_t esz = spec->elem_size;
  const bool by_rows = spec->partition_dim == 0;

  hipStream_t hs = static_cast<hipStream_t>(stream);

  if (!by_rows && esz == 4) {
    // destination-major gather: consecutive sub-shards of one destination shard form a job
    std::vector<GatherJob> jobs;
    int32_t cur_dst = -1;
    int64_t cur_end = 0;  // destination column (bytes) where the current job ends
    int64_t job_col0 = 0;
    for (const ntp_segment_t& g : segs) {
      const char* sp = static_cast<const char*>(src_shards[g.src_rank]);
      char* dp = static_cast<char*>(dst_shards[g.dst_rank]);
      const int64_t c0 = g.dst_unit * spec->unit * esz, c1 = c0 + g.units * spec->unit * esz;
      if (!sp || !dp || c1 == c0 || spec->rows == 0) continue;  // not on this GPU, or empty
      if (spec->rows > 0xffffffffll || c1 - c0 > 0x7fffffffll) return NTP_ERR_UNSUPPORTED;
      const bool fresh = jobs.empty() || g.dst_rank != cur_dst || c0 != cur_end || jobs.back().npieces == kMaxPieces ||
                         c1 - job_col0 > 0x7fffffffll;
      if (fresh) {
        GatherJob j{};
        j.dst = dp + c0;
        j.dst_stride = dst_ld[g.dst_rank] * esz;
        j.rows = uint32_t(spec->rows);
        jobs.push_back(j);
        cur_dst = g.dst_rank;
        job_col0 = c0;
      }
      GatherJob& j = jobs.back();
      Piece& pc = j.piece[j.npieces++];
      pc.src = sp + g.src_unit * spec->unit * esz;
      pc.src_stride = src_ld[g.src_rank] * esz;
      pc.begin = uint32_t(c0 - job_col0);
      pc.end = uint32_t(c1 - job_col0);
      cur_end = c1;
    }
    // jobs whose destination is a dense, 64-byte aligned shard go to the flat kernel
    const int64_t kFlatBlock = h->opt[NTP_OPT_RESHARD_FLAT_BLOCK]
                                   ? std::min<int64_t>(kFlatBlockMax, std::max<int64_t>(1024, h->opt[NTP_OPT_RESHARD_FLAT_BLOCK] & ~63ll))
                                   : 16384;
    std::vector<GatherJob> flat, rowwise;
    for (const GatherJob& j : jobs) {
      const int64_t W = j.piece[j.npieces - 1].end;
      int64_t smax = 0;
      for (uint32_t p = 0; p < j.npieces; ++p) smax = std::max(smax, j.piece[p].src_stride);
      const bool ok = j.dst_stride == W && (reinterpret_cast<uintptr_t>(j.dst) & 63) == 0 &&
                      (int64_t(kFlatBlock) + W + 16) * W <= (int64_t(1) << 32) &&
                      smax * (int64_t(kFlatBlock) / W + 2) < (int64_t(1) << 32) && !h->opt[NTP_OPT_RESHARD_NO_FLAT];
      (ok ? flat : rowwise).push_back(j);
    }
    for (size_t base = 0; base < flat.size(); base += kMaxJobs) {
      GatherBatch batch{};
      batch.njobs = int32_t(std::min<size_t>(kMaxJobs, flat.size() - base));
      int64_t nblk = 0;
      double bytes = 0.0;
      for (int i = 0; i < batch.njobs; ++i) {
        const GatherJob& j = flat[base + i];
        const int64_t total = int64_t(j.rows) * j.piece[j.npieces - 1].end;
        nblk = std::max(nblk, (total + kFlatBlock - 1) / kFlatBlock);
        bytes += 2.0 * double(total);
        batch.job[i] = j;
      }
      batch.rows_per_block = uint32_t(kFlatBlock);
      const uint64_t blocks = uint64_t(nblk) * uint64_t(batch.njobs);
      if (blocks > 0x7fffffffull) return NTP_ERR_UNSUPPORTED;
      if (blocks == 0) continue;
      if (ntp::timing_on(h)) ntp::timing_begin(h, stream, "reshard_flat", 0.0, bytes);
      hipLaunchKernelGGL(reshard_flat_kernel, dim3(uint32_t(blocks)), dim3(kThreads), 0, hs, batch);
      const bool ok = hipGetLastError() == hipSuccess;
      ntp::timing_end(h, stream);
      if (!ok) return NTP_ERR_LAUNCH;
    }
    jobs.swap(rowwise);
    for (size_t base = 0; base < jobs.size(); base += kMaxJobs) {
      GatherBatch batch{};
      batch.njobs = int32_t(std::min<size_t>(kMaxJobs, jobs.size() - base));
      // rows per workgroup: about kBlockBytes of the widest job, and row offsets inside a block that
      // fit in 32 bits
      int64_t rpb = spec->rows;
      double bytes = 0.0;
      for (int i = 0; i < batch.njobs; ++i) {
        const GatherJob& j = jobs[base + i];
        const int64_t row_bytes = j.piece[j.npieces - 1].end;
        int64_t stride = j.dst_stride;
        for (uint32_t p = 0; p < j.npieces; ++p) stride = std::max(stride, j.piece[p].src_stride);
        rpb = std::min(rpb, std::max<int64_t>(1, gather_block_bytes(h) / row_bytes));
        rpb = std::min(rpb, std::max<int64_t>(1, (int64_t(1) << 31) / std::max<int64_t>(stride, 1)));
        bytes += 2.0 * double(j.rows) * double(row_bytes);
        batch.job[i] = j;
      }
      if (rpb > 1 && jobs[base].dst_stride > (int64_t(1) << 31)) return NTP_ERR_UNSUPPORTED;
      batch.rows_per_block = uint32_t(rpb);
      const uint64_t blocks = uint64_t((spec->rows + rpb - 1) / rpb) * uint64_t(batch.njobs);
      if (blocks > 0x7fffffffull) return NTP_ERR_UNSUPPORTED;
      if (blocks == 0) continue;
      if (ntp::timing_on(h)) ntp::timing_begin(h, stream, "reshard_gather", 0.0, bytes);
      hipLaunchKernelGGL(reshard_gather_kernel, dim3(uint32_t(blocks)), dim3(kThreads), 0, hs, batch);
      const bool ok = hipGetLastError() == hipSuccess;
      ntp::timing_end(h, stream);
      if (!ok) return NTP_ERR_LAUNCH;
    }
    return NTP_OK;
  }

  // segments -> dense ranges and 2-D copies
  std::vector<CopySeg> copies;
  std::vector<DenseRange> ranges;
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
    if (c.src_stride == c.row_bytes && c.dst_stride == c.row_bytes) {
      // dense on both sides: one long run.  The 16-byte aligned middle goes to the streaming kernel,
      // what is left (misaligned pointers, a few bytes at the end) to the general one.
      const int64_t total = c.rows * c.row_bytes;
      const bool al = ((reinterpret_cast<uintptr_t>(c.src) | reinterpret_cast<uintptr_t>(c.dst)) & 15) == 0;
      const int64_t body = al ? total & ~int64_t(15) : 0;
      if (body > 0) ranges.push_back(DenseRange{c.src, c.dst, body, 0, 0});
      if (total > body) {
        CopySeg d = c;
        d.src += body;
        d.dst += body;
        d.rows = 1;
        d.row_bytes = d.src_stride = d.dst_stride = total - body;
        if (d.row_bytes > (int64_t(1) << 20)) {  // long misaligned run: recut into 4 KiB rows
          const int64_t full = d.row_bytes / 4096;
          CopySeg e = d;
          e.rows = full;
          e.row_bytes = e.src_stride = e.dst_stride = 4096;
          copies.push_back(e);
          d.src += full * 4096;
          d.dst += full * 4096;
          d.row_bytes = d.src_stride = d.dst_stride = d.row_bytes - full * 4096;
        }
        if (d.row_bytes > 0) copies.push_back(d);
      }
    } else {
      copies.push_back(c);
    }
  }

  for (size_t base = 0; base < ranges.size(); base += kMaxRanges) {
    DenseBatch batch{};
    batch.n = int32_t(std::min<size_t>(kMaxRanges, ranges.size() - base));
    uint64_t blocks = 0;
    double bytes = 0.0;
    for (int i = 0; i < batch.n; ++i) {
      DenseRange r = ranges[base + i];
      r.first_block = uint32_t(blocks);
      blocks += uint64_t((r.bytes + kDenseBlock - 1) / kDenseBlock);
      if (blocks > 0x7fffffffull) return NTP_ERR_UNSUPPORTED;
      bytes += 2.0 * double(r.bytes);
      batch.r[i] = r;
    }
    if (ntp::timing_on(h)) ntp::timing_begin(h, stream, "reshard_dense", 0.0, bytes);
    hipLaunchKernelGGL(reshard_dense_kernel, dim3(uint32_t(blocks)), dim3(kThreads), 0, hs, batch);
    const bool ok = hipGetLastError() == hipSuccess;
    ntp::timing_end(h, stream);
    if (!ok) return NTP_ERR_LAUNCH;
  }
  for (size_t base = 0; base < copies.size(); base += kMaxSegs) {
    CopyBatch batch{};
    batch.nseg = int32_t(std::min<size_t>(kMaxSegs, copies.size() - base));
    batch.elem_size = int32_t(esz);
    uint64_t blocks = 0;
    for (int i = 0; i < batch.nseg; ++i) {
      CopySeg c = copies[base + i];
      c.col_chunks = uint32_t((c.row_bytes + kColChunk - 1) / kColChunk);
      const int64_t per_row = std::min<int64_t>(c.row_bytes, kColChunk);
      // about kBlockBytes per workgroup; rows * elements-per-row stays far below 2^32 (exact multiply-high division)
      int64_t rpb = std::max<int64_t>(1, std::min<int64_t>(kBlockBytes / per_row, 16384));
      c.rows_per_block = uint32_t(std::min<int64_t>(rpb, std::max<int64_t>(c.rows, 1)));
      const uint64_t row_groups = uint64_t((c.rows + c.rows_per_block - 1) / c.rows_per_block);
      c.first_block = uint32_t(blocks);
      blocks += row_groups * c.col_chunks;
      if (blocks > 0x7fffffffull) return NTP_ERR_UNSUPPORTED;
      batch.seg[i] = c;
    }
    if (blocks == 0) continue;
    if (ntp::timing_on(h)) {
      double bytes = 0.0;
      for (int i = 0; i < batch.nseg; ++i) bytes += 2.0 * double(batch.seg[i].rows) * double(batch.seg[i].row_bytes);
      ntp::timing_begin(h, stream, "reshard_copy", 0.0, bytes);
    }
    hipLaunchKernelGGL(reshard_copy_kernel, dim3(uint32_t(blocks)), dim3(kThreads), 0, hs, batch);
    const bool ok = hipGetLastError() == hipSuccess;
    ntp::timing_end(h, stream);
    if (!ok) return NTP_ERR_LAUNCH;
  }
  return NTP_OK;
}

// ---- reshard plan between two unit -> rank maps (Sec. 3.1, Alg. 1; Appendix: precomputed splits) -----
struct ntp_reshard_plan {
  ntp_tensor_spec_t spec;
  int32_t src_tp, dst_tp;
  std::vector<ntp_segment_t> segs;           // destination order
  std::vector<int64_t> src_units, dst_units;  // units per rank
  std::vector<int64_t> splits;                // [src_tp x dst_tp] units from rank r to rank s
  std::vector<ntp_unit_source_t> table;       // per destination unit, destination shards one after the other
  std::vector<int64_t> dst_first;             // first table entry of each destination shard
  // run table of the gather kernel (column-partitioned 4-byte elements only)
  bool runs_ok = false;
  std::vector<RunDev> runs;                   // runs of all destination shards, one shard after the other
  std::vector<int64_t> runs_first;            // first run of each destination shard
  std::vector<uint16_t> run_of_unit;          // per destination unit (indexed like `table`): run number in its shard
  void* dev_table = nullptr;                  // `runs` then `run_of_unit` on device `dev`, made by ntp_reshard_plan_prepare
  int dev = -1;                               // device the plan was prepared on (-1: not prepared)
};

extern "C" int ntp_reshard_plan_create(const ntp_tensor_spec_t* spec, int64_t map_len, int32_t src_tp,
                                       const int32_t* src_rank_of_unit, int32_t dst_tp,
                                       const int32_t* dst_rank_of_unit, ntp_reshard_plan_t** plan) {
  if (!plan) return NTP_ERR_INVALID_ARG;
  *plan = nullptr;
  int64_t n_units = 0;
  int st = ntp::check_spec(spec, 1, 1, &n_units);
  if (st != NTP_OK) return st;
  if (spec->kind != NTP_KIND_PLAIN || n_units > 0x7fffffffll || map_len != n_units) return NTP_ERR_INVALID_ARG;
  ntp_reshard_plan* p = new ntp_reshard_plan;
  p->spec = *spec;
  p->src_tp = src_tp;
  p->dst_tp = dst_tp;
  st = ntp::build_segments_mapped(n_units, src_tp, src_rank_of_unit, dst_tp, dst_rank_of_unit, &p->segs, &p->src_units,
                                  &p->dst_units);
  if (st != NTP_OK) {
    delete p;
    return st;
  }
  p->splits.assign(size_t(src_tp) * size_t(dst_tp), 0);
  p->dst_first.assign(size_t(dst_tp) + 1, 0);
  for (int32_t s = 0; s < dst_tp; ++s) p->dst_first[s + 1] = p->dst_first[s] + p->dst_units[s];
  p->table.resize(size_t(n_units));
  for (const ntp_segment_t& g : p->segs) {
    p->splits[size_t(g.src_rank) * dst_tp + g.dst_rank] += g.units;
    for (int64_t i = 0; i < g.units; ++i)
      p->table[size_t(p->dst_first[g.dst_rank] + g.dst_unit + i)] = ntp_unit_source_t{g.src_rank, int32_t(g.src_unit + i)};
  }
  // run table: the sub-shards are the runs
  if (spec->partition_dim == 1 && spec->elem_size == 4) {
    const int64_t ub = int64_t(spec->unit) * 4;
    p->runs_first.assign(size_t(dst_tp) + 1, 0);
    p->run_of_unit.resize(size_t(n_units));
    p->runs_ok = true;
    int32_t cur = 0;
    for (const ntp_segment_t& g : p->segs) {
      while (cur < g.dst_rank) p->runs_first[size_t(++cur)] = int64_t(p->runs.size());
      const int64_t number = int64_t(p->runs.size()) - p->runs_first[size_t(cur)];
      const int64_t end = (g.dst_unit + g.units) * ub, so = g.src_unit * ub;
      if (number > 0xffff || end > 0xffffffffll || so > 0xffffffffll) p->runs_ok = false;
      p->runs.push_back(RunDev{uint32_t(g.dst_unit * ub), uint32_t(end), uint32_t(so), uint32_t(g.src_rank)});
      for (int64_t i = 0; i < g.units; ++i) p->run_of_unit[size_t(p->dst_first[g.dst_rank] + g.dst_unit + i)] = uint16_t(number);
    }
    while (cur < dst_tp) p->runs_first[size_t(++cur)] = int64_t(p->runs.size());
  }
  *plan = p;
  return NTP_OK;
}

extern "C" int ntp_reshard_plan_destroy(ntp_reshard_plan_t* plan) {
  if (!plan) return NTP_OK;
  if (plan->dev_table) {
    int cur = -1;
    (void)hipGetDevice(&cur);
    if (cur != plan->dev) (void)hipSetDevice(plan->dev);
    (void)hipFree(plan->dev_table);
    if (cur != plan->dev && cur >= 0) (void)hipSetDevice(cur);
  }
  delete plan;
  return NTP_OK;
}

extern "C" int ntp_reshard_plan_segments(const ntp_reshard_plan_t* plan, ntp_segment_t* out, int64_t max_segments,
                                         int64_t* count) {
  if (!plan || !count || max_segments < 0 || (max_segments > 0 && !out)) return NTP_ERR_INVALID_ARG;
  *count = int64_t(plan->segs.size());
  for (int64_t i = 0; i < std::min<int64_t>(max_segments, *count); ++i) out[i] = plan->segs[size_t(i)];
  return NTP_OK;
}

extern "C" int ntp_reshard_plan_splits(const ntp_reshard_plan_t* plan, int64_t* units) {
  if (!plan || !units) return NTP_ERR_INVALID_ARG;
  std::copy(plan->splits.begin(), plan->splits.end(), units);
  return NTP_OK;
}

extern "C" int ntp_reshard_plan_table(const ntp_reshard_plan_t* plan, ntp_unit_source_t* out, int64_t max_units,
                                      int64_t* count) {
  if (!plan || !count || max_units < 0 || (max_units > 0 && !out)) return NTP_ERR_INVALID_ARG;
  *count = int64_t(plan->table.size());
  for (int64_t i = 0; i < std::min<int64_t>(max_units, *count); ++i) out[i] = plan->table[size_t(i)];
  return NTP_OK;
}

namespace {

// Whether the run-table kernel can take this call with blocks of `block` bytes.
bool units_path_ok(const ntp_handle* h, const ntp_reshard_plan* p, const void* const* src_shards, const int64_t* src_ld,
                   void* const* dst_shards, const int64_t* dst_ld, int64_t block) {
  const ntp_tensor_spec_t& sp = p->spec;
  if (!p->runs_ok || !p->dev_table || sp.rows == 0 || h->opt[NTP_OPT_RESHARD_NO_TABLE]) return false;
  if (p->src_tp > kMaxRanks || sp.rows > 0x7fffffffll) return false;
  for (int32_t r = 0; r < p->src_tp; ++r) {
    if (p->src_units[r] == 0) continue;
    if (!src_shards[r] || src_ld[r] * 4 >= (int64_t(1) << 32)) return false;
  }
  bool any = false;
  for (int32_t s = 0; s < p->dst_tp; ++s) {
    if (p->dst_units[s] == 0 || !dst_shards[s]) continue;
    const int64_t W = p->dst_units[s] * sp.unit * 4;
    const int64_t n_runs = p->runs_first[s + 1] - p->runs_first[s];
    if (dst_ld[s] * 4 != W || (reinterpret_cast<uintptr_t>(dst_shards[s]) & 63) != 0 ||
        (block + W + 16) * W > (int64_t(1) << 32) ||
        n_runs * int64_t(sizeof(RunLds)) + p->dst_units[s] * 2 + 16 + int64_t(kWaves * kQueueCap * sizeof(uint2)) > int64_t(kUnitLdsMax))
      return false;
    any = true;
  }
  return any;
}

}  // namespace

namespace {

// The plan's run table goes to the current device (allocates and waits for the copy).
int upload_table(ntp_reshard_plan_t* plan) {
  const size_t runs_bytes = plan->runs.size() * sizeof(RunDev), idx_bytes = plan->run_of_unit.size() * sizeof(uint16_t);
  if (hipMalloc(&plan->dev_table, runs_bytes + idx_bytes) != hipSuccess) {
    plan->dev_table = nullptr;
    return NTP_ERR_LAUNCH;
  }
  if (hipMemcpy(plan->dev_table, plan->runs.data(), runs_bytes, hipMemcpyHostToDevice) != hipSuccess ||
      hipMemcpy(static_cast<char*>(plan->dev_table) + runs_bytes, plan->run_of_unit.data(), idx_bytes,
                hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(plan->dev_table);
    plan->dev_table = nullptr;
    return NTP_ERR_LAUNCH;
  }
  return NTP_OK;
}

}  // namespace

extern "C" int ntp_reshard_plan_prepare(ntp_reshard_plan_t* plan) {
  if (!plan) return NTP_ERR_INVALID_ARG;
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess || cur < 0) {
    (void)hipGetLastError();
    return NTP_ERR_NO_DEVICE;
  }
  if (plan->dev >= 0) return cur == plan->dev ? NTP_OK : NTP_ERR_INVALID_ARG;  // a plan lives on one device
  if (plan->runs_ok && !plan->runs.empty()) {
    const int st = upload_table(plan);
    if (st != NTP_OK) return st;
  }
  plan->dev = cur;
  return NTP_OK;
}

extern "C" int ntp_reshard_plan_run(ntp_handle_t* h, ntp_reshard_plan_t* plan, const void* const* src_shards,
                                    const int64_t* src_ld, void* const* dst_shards, const int64_t* dst_ld, void* stream) {
  if (!h || !plan) return NTP_ERR_INVALID_ARG;
  int st = ntp::check_shards(&plan->spec, plan->src_units, plan->dst_units, src_shards, src_ld, dst_shards, dst_ld);
  if (st != NTP_OK) return st;
  if (h->device < 0) return NTP_ERR_NO_DEVICE;
  if (plan->dev != h->device) return NTP_ERR_NOT_PREPARED;
  int64_t block = 16384;
  if (const int64_t e = h->opt[NTP_OPT_RESHARD_TABLE_BLOCK]) block = std::min<int64_t>(1 << 20, std::max<int64_t>(1024, e & ~63ll));
  if (!units_path_ok(h, plan, src_shards, src_ld, dst_shards, dst_ld, block))
    return ntp::reshard_launch(h, &plan->spec, plan->segs, plan->src_units, plan->dst_units, src_shards, src_ld, dst_shards,
                               dst_ld, stream);

  const ntp_tensor_spec_t& sp = plan->spec;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  UnitBatch batch{};
  batch.runs = static_cast<const RunDev*>(plan->dev_table);
  batch.run_of_unit = reinterpret_cast<const uint16_t*>(static_cast<const char*>(plan->dev_table) + plan->runs.size() * sizeof(RunDev));
  batch.rows = uint32_t(sp.rows);
  batch.unit_bytes = uint32_t(sp.unit) * 4u;
  batch.block_bytes = uint32_t(block);
  for (int32_t r = 0; r < plan->src_tp; ++r)
    batch.src[r] = UnitSrc{static_cast<const char*>(src_shards[r]), uint64_t(src_ld[r]) * 4u};
  int32_t s = 0;
  while (s < plan->dst_tp) {
    batch.ndst = 0;
    int64_t nblk = 0;
    uint32_t lds = 0;
    double bytes = 0.0;
    for (; s < plan->dst_tp && batch.ndst < uint32_t(kUnitDsts); ++s) {
      if (plan->dst_units[s] == 0 || !dst_shards[s]) continue;
      const int64_t total = sp.rows * plan->dst_units[s] * sp.unit * 4;
      const uint32_t n_runs = uint32_t(plan->runs_first[s + 1] - plan->runs_first[s]);
      batch.dst[batch.ndst++] = UnitDst{static_cast<char*>(dst_shards[s]), uint32_t(plan->dst_first[s]), uint32_t(plan->dst_units[s]),
                                        uint32_t(plan->runs_first[s]), n_runs};
      nblk = std::max(nblk, (total + block - 1) / block);
      lds = std::max(lds, unit_lds_bytes(n_runs, uint32_t(plan->dst_units[s])));
      bytes += 2.0 * double(total);
    }
    if (batch.ndst == 0) break;
    // workgroups per destination shard: enough of them to fill the chip, each walking over several blocks
    // workgroups per destination shard: one per block, or fewer that walk over several blocks each when
    // the shards are very large (the tables are copied into LDS once per workgroup)
    const int64_t slots = std::max<int64_t>(1, std::min<int64_t>(nblk, (int64_t(h->compute_units) * int64_t(kUnitBlocksPerCu) + batch.ndst - 1) / batch.ndst));
    const uint64_t blocks = uint64_t(slots) * batch.ndst;
    if (ntp::timing_on(h)) ntp::timing_begin(h, stream, "reshard_table", 0.0, bytes);
    hipLaunchKernelGGL(reshard_units_kernel, dim3(uint32_t(blocks)), dim3(kThreads), lds, hs, batch);
    const bool ok = hipGetLastError() == hipSuccess;
    ntp::timing_end(h, stream);
    if (!ok) return NTP_ERR_LAUNCH;
  }
  return NTP_OK;
}
