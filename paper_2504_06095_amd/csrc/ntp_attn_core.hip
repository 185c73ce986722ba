// Attention core of one rank's local heads (Sec. 3.1, Eq. 5): C_j = softmax(Q_j K_g^T / sqrt(d)) V_g for
// every local query head j and the KV head g it reads, sequence by sequence, forward and backward.
//
// Forward: one workgroup (4 wavefronts) takes 128 query rows of one (sequence, head); a wavefront owns
// 32 of them.  Keys and values stream through LDS in tiles of 64 rows; scores never leave registers
// (running maximum and sum per query row, output rescaled when the maximum moves).  Both products run
// on the 16x16x32 bf16 matrix instruction with the query index on the lane axis:
//   S^T tile = K_tile Q^T  : lane (l % 16) = query row, the lane's 4 values per block = 4 consecutive keys,
//                            so a row's maximum and sum are mostly in-lane (two cross-lane steps);
//   O^T     += V_tile^T P^T: the same lane owns the same query row, P goes from the score registers
//                            straight into the second product (the key order inside a 32-key step is
//                            permuted the same way on the V side, read transposed from LDS).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <type_traits>

#include "ntp_gemm_kernels.h"
#include "ntp_gemm_ring.h"
#include "ntp_internal.h"

namespace {

using ntp_gemm::bf16x8;
using ntp_gemm::f32x4;
using ntp_gemm::s16x4;
using ntp_gemm::s16x8;
using ntp_gemm::u16x4;

constexpr int kBKV = 64;   // keys per tile
constexpr int kThreads = 256;

struct CoreArgs {
  const uint16_t* QKV;  // [M x ld] bf16: [Q heads | K heads | V heads]
  uint16_t* C;          // [M x ldc] bf16
  float* LSE;           // [q_cnt x M] natural-log sum of exponentials of the scaled scores
  int64_t ld, ldc;
  int32_t n_seq, seq_len, q_cnt, kv_cnt, q_off, kv_off, group, causal;
  int32_t q_tiles;      // per sequence
  float scale_log2;     // log2(e) / sqrt(d)
  // n_parts > 1 (16 query rows per wavefront only): each workgroup's walk over the key tiles is cut into
  // n_parts pieces, one workgroup each, which store their unnormalised output rows, running maximum and
  // sum to part_sums ([workgroup][piece][64 rows][D + 4]: D outputs, maximum, sum); a second kernel merges them
  float* part_sums;
  int32_t n_parts;
  // pairs > 0 (causal mask): a workgroup takes two query tiles one after the other, number pairs - 1 - u from the
  // end and number u from the start, so that every workgroup walks over the same number of key tiles
  // (q_tiles + 1, cut into n_parts); pairs = (q_tiles + 1) / 2 workgroups per (sequence, head)
  int32_t pairs;
};

// 2^x by the hardware instruction alone: results below the normal range flush to zero, which is what a
// softmax weight that small is worth
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Maximum / sum over the four lanes l % 16 + {0, 16, 32, 48}, left in all four.  The 16-lane rows trade places in
// registers (v_permlane16_swap: odd rows of the first operand against even rows of the second, then
// v_permlane32_swap: upper half of the first against lower half of the second), no LDS round trips.
// (Each result is copied into a scalar variable before its bits are reinterpreted: a bit cast applied to the vector
// element itself compiled to the first element in both places.)
struct SwapPair {
  float a, b;
};
__device__ __forceinline__ SwapPair rows_swap16(float v) {
  const uint32_t x = __builtin_bit_cast(uint32_t, v);
  const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  return SwapPair{__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1)};
}
__device__ __forceinline__ SwapPair rows_swap32(float v) {
  const uint32_t x = __builtin_bit_cast(uint32_t, v);
  const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  return SwapPair{__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1)};
}
__device__ __forceinline__ float xor_max(float v) {
  const SwapPair p = rows_swap16(v);
  const SwapPair q = rows_swap32(fmaxf(p.a, p.b));
  return fmaxf(q.a, q.b);
}
__device__ __forceinline__ float xor_sum(float v) {
  const SwapPair p = rows_swap16(v);
  const SwapPair q = rows_swap32(p.a + p.b);
  return q.a + q.b;
}

// Workgroups go to the chip's 8 XCDs in turn (workgroup b to XCD b % 8), and each XCD has an L2 of its own.  The
// workgroups of one head read the same key / value (or query / output-gradient) rows, 1 MB per head at 2048 tokens:
// spread over all XCDs every L2 sees every head (14 heads: 15 MB against 4 MB of L2).  So the launch order is
// renumbered: XCD x takes the x-th contiguous eighth of the logical order, in which a head's workgroups are
// neighbours.  (Measured gain at 14 heads x 2048 tokens causal: forward 39.4 -> 38.5 us, backward 80 -> 76 us; the
// tiles that miss L2 come from the 256 MB last-level cache either way.)
__device__ __forceinline__ uint32_t xcd_major(uint32_t b, uint32_t total) {
  const uint32_t x = b & 7, q = total >> 3, r = total & 7;
  return x * q + (x < r ? x : r) + (b >> 3);
}

// Source of the 64-row tiles of a [S x ld] bf16 matrix (D columns from `base` on, the first row of a sequence):
// one 16-byte buffer load per thread and chunk.  A thread's offsets inside a tile never change (tile_offsets); the
// tile is chosen by the instruction's scalar offset, so the loop spends no vector arithmetic on addresses.  The
// view ends with the sequence's last row: rows past it read as zeros.  Needs S * ld * 2 < 2^31 (checked on the host).
template <int D>
struct TileSrc {
  static constexpr int CPR = D / 8, NLD = kBKV * CPR / kThreads;
  __amdgpu_buffer_rsrc_t rs;
  uint32_t step;  // bytes from one tile to the next
  __device__ __forceinline__ void init(const uint16_t* base, int64_t ld, int S) {
    rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0, int((int64_t(S - 1) * ld + D) * 2), 0x00020000);
    step = uint32_t(kBKV * ld * 2);
  }
  static __device__ __forceinline__ void tile_offsets(int64_t ld, uint32_t (&voff)[NLD]) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int c = threadIdx.x + i * kThreads;
      voff[i] = uint32_t(((c / CPR) * ld + (c % CPR) * 8) * 2);
    }
  }
  __device__ __forceinline__ void load(int t, const uint32_t (&voff)[NLD], ntp_gemm::u16x8 (&r)[NLD]) const {
#pragma unroll
    for (int i = 0; i < NLD; ++i) r[i] = __builtin_bit_cast(ntp_gemm::u16x8, __builtin_amdgcn_raw_buffer_load_b128(rs, voff[i], uint32_t(t) * step, 0));
  }
};

// (two or three wavefronts per SIMD: one's softmax arithmetic overlaps the others' matrix instructions)
// (the register budget is pinned to that occupancy: left free, the compiler squeezes the 16-row variant into 128
// registers for a fourth wavefront per SIMD that these launches never have, and the loop runs 10 % slower)
template <int D, int QB, bool PAIRED>
__global__ __attribute__((amdgpu_flat_work_group_size(kThreads, kThreads), amdgpu_waves_per_eu(QB == 1 ? 3 : 2, QB == 1 ? 3 : 2))) void
attn_core_fwd_kernel(const CoreArgs a) {
  constexpr int kRows = 64 * QB;  // query rows per workgroup: 16 QB per wavefront
  // LDS row stride (elements): rows shift by 8 banks, so the 8 rows that a 16-byte fragment read touches per
  // cycle and the 4 rows x 32 bytes that a transposing read touches per cycle land on distinct banks
  constexpr int LDT = D + 16, LDV = D + 16;
  constexpr int KS = D / 32;        // K-steps of the score product
  constexpr int DB = D / 16;        // 16-column blocks of the output
  constexpr int CPR = D / 8;        // 16-byte chunks per tile row
  constexpr int NLD = kBKV * CPR / kThreads;  // chunks per thread and tile
  static_assert(D % 32 == 0 && (kBKV * CPR) % kThreads == 0, "tile copy: whole chunks per thread");
  // The 32-row variant (two workgroups per CU) double-buffers the key / value tiles: the next tile is
  // written to the other buffer while this one is multiplied, one barrier per tile.  The 16-row variant
  // keeps one buffer (a second one would cost it the third workgroup per CU) and two barriers.
  constexpr int NBUF = QB == 2 ? 2 : 1;
  __shared__ __attribute__((aligned(16))) uint16_t sKb[NBUF][kBKV * LDT];
  __shared__ __attribute__((aligned(16))) uint16_t sVb[NBUF][kBKV * LDV];

  // workgroup -> (head, sequence, query tile); consecutive workgroups share a head's keys and values.
  // With the causal mask the late tiles have the most keys: they go first.
  const uint32_t bid = xcd_major(blockIdx.x, gridDim.x);
  const int piece = a.n_parts > 1 ? int(bid % a.n_parts) : 0;
  const int blk = a.n_parts > 1 ? int(bid / a.n_parts) : int(bid);
  const int per_seq = PAIRED ? a.pairs : a.q_tiles;  // workgroups per (sequence, head) and piece
  const int u = blk % per_seq;
  const int sh = blk / per_seq;
  const int seq = sh % a.n_seq, head = sh / a.n_seq;
  const int g = (a.q_off + head) / a.group - a.kv_off;  // local KV head
  const int S = a.seq_len;
  const int64_t tok0 = int64_t(seq) * S;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lq = lane & 15, lh = lane >> 4;
  const uint16_t* Qp = a.QKV + int64_t(head) * D;
  const uint16_t* Kp = a.QKV + int64_t(a.q_cnt + g) * D;
  const uint16_t* Vp = a.QKV + int64_t(a.q_cnt + a.kv_cnt + g) * D;
  ntp_gemm::u16x8 rk[NLD], rv[NLD];
  uint32_t voff[NLD];
  TileSrc<D>::tile_offsets(a.ld, voff);
  TileSrc<D> srcK, srcV;
  srcK.init(Kp + tok0 * a.ld, a.ld, S);
  srcV.init(Vp + tok0 * a.ld, a.ld, S);

  for (int seg = 0; seg < (PAIRED ? 2 : 1); ++seg) {
  // this pass's query tile; without pairing the late tiles of a causal launch (the most keys) go first
  const int qt = PAIRED ? (seg == 0 ? a.q_tiles - 1 - u : u) : (a.causal ? a.q_tiles - 1 - u : u);
  if (seg == 1) {
    if (qt == a.q_tiles - 1 - u) break;  // odd tile count: the middle tile has no partner
    __syncthreads();                     // the first pass's last tile has been read by everyone
  }
  // the tile's number in the order the merge kernel counts them (late tiles first under the causal mask)
  const int64_t tblk = int64_t(sh) * a.q_tiles + (a.causal ? a.q_tiles - 1 - qt : qt);
  const int q0 = qt * kRows + wave * (16 * QB);  // first query row (in the sequence) of this wavefront

  // query fragments: operand B[k][j] with j = query row (lane % 16), k = 8 consecutive columns
  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qr = min(q0 + qb * 16 + lq, S - 1);  // rows past the end repeat the last one (never stored)
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[qb][ks] = *reinterpret_cast<const bf16x8*>(Qp + (tok0 + qr) * a.ld + ks * 32 + lh * 8);
  }

  f32x4 acc[QB][DB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
  }

  // keys this workgroup needs: all of the sequence, or up to its last query row
  const int kv_end = a.causal ? min(S, qt * kRows + kRows) : S;
  const int n_tiles = (kv_end + kBKV - 1) / kBKV;

  // tile copy: global -> registers -> LDS, the next tile's loads in flight during the products
  auto load_tile = [&](int t) {  // rows past the sequence end arrive as zeros (their scores are masked below)
    srcK.load(t, voff, rk);
    srcV.load(t, voff, rv);
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int c = threadIdx.x + i * kThreads;
      *reinterpret_cast<ntp_gemm::u16x8*>(sKb[buf] + (c / CPR) * LDT + (c % CPR) * 8) = rk[i];
      *reinterpret_cast<ntp_gemm::u16x8*>(sVb[buf] + (c / CPR) * LDV + (c % CPR) * 8) = rv[i];
    }
  };

  // this workgroup's share of the key tiles (all of them unless the walk is cut)
  const int t_lo = a.n_parts > 1 ? int(int64_t(piece) * n_tiles / a.n_parts) : 0;
  const int t_hi = a.n_parts > 1 ? int(int64_t(piece + 1) * n_tiles / a.n_parts) : n_tiles;
  if (t_lo < t_hi) load_tile(t_lo);
  if constexpr (NBUF == 2) {
    if (t_lo < t_hi) store_tile(0);
  }
  for (int t = t_lo; t < t_hi; ++t) {
    const uint16_t* sK;
    const uint16_t* sV;
    if constexpr (NBUF == 2) {
      // tile t sits in buffer (t - t_lo) & 1, written before the barrier; tile t + 1 goes from global memory
      // to registers now and to the other buffer at the end of this iteration (its last readers, of tile
      // t - 1, passed this barrier)
      __syncthreads();
      if (t + 1 < t_hi) load_tile(t + 1);
      sK = sKb[(t - t_lo) & 1];
      sV = sVb[(t - t_lo) & 1];
    } else {
      __syncthreads();  // everyone has finished reading the previous tile
      store_tile(0);
      __syncthreads();
      if (t + 1 < t_hi) load_tile(t + 1);
      sK = sKb[0];
      sV = sVb[0];
    }
    const int kv0 = t * kBKV;
    // every key of the tile lies after this wavefront's last query row: nothing to do but pass the tile on
    const bool skip = a.causal && kv0 > q0 + 16 * QB - 1;
    if (skip) {
      if constexpr (NBUF == 2) {
        if (t + 1 < t_hi) store_tile((t + 1 - t_lo) & 1);
      }
      continue;
    }

    // scores, transposed: st[kb][qb][r] = S[query qb*16 + lane%16][key kv0 + kb*16 + (lane/16)*4 + r]
    f32x4 st[4][QB];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) st[kb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + (kb * 16 + lq) * LDT + ks * 32 + lh * 8);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) st[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[qb][ks], st[kb][qb], 0, 0, 0);
      }
    }

    // only tiles that reach past the sequence end or past this wavefront's first query row (causal) need
    // the mask; the test is the same for the whole wavefront
    const bool edge = kv0 + kBKV > S || (a.causal && kv0 + kBKV - 1 > q0);
    bf16x8 pf[QB][2];  // P as operand B of the second product, per query block and 32-key step
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int qrow = q0 + qb * 16 + lq;
      if (edge) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int key = kv0 + kb * 16 + lh * 4 + r;
            if (key >= S || (a.causal && key > qrow)) st[kb][qb][r] = -INFINITY;
          }
      }
      // the scale is positive: the maximum can be taken on the raw scores
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) mx = fmaxf(mx, st[kb][qb][r]);
      mx = xor_max(mx) * a.scale_log2;
      const float m_new = fmaxf(m_run[qb], mx);
      // a row with no visible key so far keeps m = -inf: use 0 there
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = fast_exp2(m_run[qb] - m_use);
      float ls = 0.f;
      float p[4][4];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          p[kb][r] = fast_exp2(fmaf(st[kb][qb][r], a.scale_log2, -m_use));
          ls += p[kb][r];
        }
      l_run[qb] = l_run[qb] * alpha + ls;  // per-lane partial sum; the four lane groups are added at the end
      m_run[qb] = m_new;
      // the running maximum rarely moves after the first tiles: skip the rescale when no lane needs it
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[qb][db] *= alpha;
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        bf16x8 f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          f[r] = static_cast<__bf16>(p[2 * s2][r]);
          f[4 + r] = static_cast<__bf16>(p[2 * s2 + 1][r]);
        }
        pf[qb][s2] = f;
      }
    }

    // O^T += V^T P^T.  Key slot (lane/16)*8 + t of step s2 is key 32 s2 + 4 (lane/16) + t for t < 4 and
    // 32 s2 + 16 + 4 (lane/16) + (t - 4) for t >= 4: the order the scores sit in the registers.
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        // transposing read: in a 16-lane group, lane s points at 4 consecutive columns of key line (s >> 2);
        // the group hands lane L the 4 keys of column L
        const uint16_t* vp = sV + (s2 * 32 + lh * 4 + (lq >> 2)) * LDV + db * 16 + (lq & 3) * 4;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 16 * LDV));
        const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) acc[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, pf[qb][s2], acc[qb][db], 0, 0, 0);
      }
    }
    if constexpr (NBUF == 2) {
      if (t + 1 < t_hi) store_tile((t + 1 - t_lo) & 1);
    }
  }

  if (a.n_parts > 1) {
    // this piece's unnormalised rows, maximum (in log2 units) and sum
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float* pp = a.part_sums + ((tblk * a.n_parts + piece) * kRows + wave * (16 * QB) + qb * 16 + lq) * (D + 4);
#pragma unroll
      for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(pp + db * 16 + lh * 4) = acc[qb][db];
      const float l = xor_sum(l_run[qb]);
      if (lh == 0) {
        pp[D] = m_run[qb];
        pp[D + 1] = l;
      }
    }
    continue;
  }
  // normalise and store: lane holds output columns db*16 + (lane/16)*4 .. +3 of query row lane % 16
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qrow = q0 + qb * 16 + lq;
    const float l = xor_sum(l_run[qb]);
    const float inv = 1.0f / l;
    if (qrow < S) {
      uint16_t* cp = a.C + (tok0 + qrow) * a.ldc + int64_t(head) * D + lh * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        u16x4 o;
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = ntp_gemm::f32_to_bf16(acc[qb][db][r] * inv);
        *reinterpret_cast<u16x4*>(cp + db * 16) = o;
      }
      if (lh == 0 && a.LSE) a.LSE[int64_t(head) * (int64_t(a.n_seq) * S) + tok0 + qrow] = (m_run[qb] + log2f(l)) * 0.6931471805599453f;
    }
  }
  }  // the workgroup's passes
}

// ---- forward kernel with key / value tiles brought to LDS by DMA --------------------------------------------
// Head dimension 128, 16 query rows per wavefront.  The tiles go global -> LDS by direct buffer loads (1 KiB per
// instruction, no staging registers, no LDS stores, no vector address arithmetic), two buffers per matrix: the DMA of
// tile t + 1 flies while tile t is multiplied, one barrier per tile.  A DMA instruction fills 64 consecutive
// 16-byte chunks, so rows cannot be padded; bank conflicts are avoided by permuting the chunks of each 256-byte row
// instead: chunk c of row r sits at slot c ^ swz(r), swz(r) = (r & 7) << 1.  A 128-bit LDS read serves 16 lanes per
// cycle, and not 16 consecutive ones: lanes of one half of the wavefront whose bits 2, 3 and 4 have the same parity
// (0-3, 12-15, 20-23, 24-27 come first; measured with reads that collide only for one pair of lane bits at a time).
// In the fragment reads lane bits 0-3 are the row and bits 4-5 the chunk's low bits, so such a group holds rows
// r0 .. r0 + 3 of four row quadruples with chunk bit 0 = parity of the quadruple's number: slot bits 1-3 (row bits
// 0-2) and slot bit 0 (chunk bit 0, which tells rows r and r + 8 apart) are all distinct, no bank conflicts.  (With
// row bit 3 folded into the permutation as well, rows r and r + 8 of a group met in one slot: 2-way conflicts,
// SQ_LDS_BANK_CONFLICT 0.33-0.40 of the LDS cycles.)  A transposing 64-bit read serves half a wavefront per cycle: 8
// rows x 32 bytes, which land on 8 distinct slot pairs.  LDS reads are inline assembly, all of a product's
// fragments first and one wait: with DMA in flight the compiler would guard every LDS read it schedules itself with a
// wait for all of it.
__device__ __forceinline__ uint32_t row_swz(int r) { return uint32_t((r & 7) << 1); }

constexpr int kDmaTile = kBKV * 128;  // elements of one 64-row tile at head dimension 128

typedef uint32_t attn_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t attn_u32x2 __attribute__((ext_vector_type(2)));

template <int OFF>
__device__ __forceinline__ attn_u32x4 lds_frag_b128(uint32_t addr) {
#if !defined(__HIP_DEVICE_COMPILE__)
  return attn_u32x4{};
#else
  attn_u32x4 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
#endif
}
template <int OFF>
__device__ __forceinline__ attn_u32x2 lds_tr_b64(uint32_t addr) {
#if !defined(__HIP_DEVICE_COMPILE__)
  return attn_u32x2{};
#else
  attn_u32x2 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF) : "memory");
  return v;
#endif
}
// The compiler takes an assembly statement's outputs as valid when the statement ends, but an LDS read only
// requests them.  The wait therefore names the requested registers as operands it rewrites: every use of them
// then depends on the wait and cannot be scheduled ahead of it.  (Eight registers per statement: the operand
// limit; the statements after the first emit nothing and only carry the dependence.)
template <typename V>
__device__ __forceinline__ void lds_reads_done(V (&r)[8]) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
               :
               : "memory");
#endif
}
template <typename V>
__device__ __forceinline__ void lds_reads_tied(V (&r)[8]) {
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7]) : : "memory");
#endif
}
template <int N, typename V>
__device__ __forceinline__ void lds_reads_left(V (&r)[8]) {  // at most N later reads may still be in flight
#if defined(__HIP_DEVICE_COMPILE__)
  asm volatile("s_waitcnt lgkmcnt(%8)"
               : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]), "+v"(r[3]), "+v"(r[4]), "+v"(r[5]), "+v"(r[6]), "+v"(r[7])
               : "n"(N)
               : "memory");
#endif
}
__device__ __forceinline__ void dma_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
__device__ __forceinline__ void dma_16(__amdgpu_buffer_rsrc_t rs, uint16_t* dst, uint32_t voff, uint32_t soff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (ntp_gemm::lds_void*)dst, 16, voff, soff, 0, 0);
}

template <bool PAIRED>
__global__ __attribute__((amdgpu_flat_work_group_size(kThreads, kThreads), amdgpu_waves_per_eu(2, 2))) void
attn_core_fwd_dma_kernel(const CoreArgs a) {
  constexpr int D = 128, KS = D / 32, DB = D / 16, kRows = 64;
  constexpr int TILE = kBKV * D;       // elements of one tile
  constexpr int NI = TILE * 2 / 1024 / 4;  // DMA instructions per wavefront, matrix and tile
  __shared__ __attribute__((aligned(1024))) uint16_t sK[2 * TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t sV[2 * TILE];

  const uint32_t bid = xcd_major(blockIdx.x, gridDim.x);
  const int piece = a.n_parts > 1 ? int(bid % a.n_parts) : 0;
  const int blk = a.n_parts > 1 ? int(bid / a.n_parts) : int(bid);
  const int per_seq = PAIRED ? a.pairs : a.q_tiles;
  const int u = blk % per_seq;
  const int sh = blk / per_seq;
  const int seq = sh % a.n_seq, head = sh / a.n_seq;
  const int g = (a.q_off + head) / a.group - a.kv_off;
  const int S = a.seq_len;
  const int64_t tok0 = int64_t(seq) * S;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lq = lane & 15, lh = lane >> 4;
  const uint16_t* Qp = a.QKV + int64_t(head) * D;
  const uint16_t* Kp = a.QKV + int64_t(a.q_cnt + g) * D;
  const uint16_t* Vp = a.QKV + int64_t(a.q_cnt + a.kv_cnt + g) * D;
  TileSrc<D> srcK, srcV;
  srcK.init(Kp + tok0 * a.ld, a.ld, S);
  srcV.init(Vp + tok0 * a.ld, a.ld, S);
  // instruction j of this wavefront fills LDS chunks (4 wave + j) 64 + lane of a tile: row = chunk / 16, and the
  // chunk of that row which belongs in this slot
  uint32_t voff[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int p = (wave * NI + j) * 64 + lane;
    const int row = p >> 4, slot = p & 15;
    voff[j] = uint32_t((int64_t(row) * a.ld + int64_t(uint32_t(slot) ^ row_swz(row)) * 8) * 2);
  }
  auto dma_tile = [&](int t, int buf) {  // rows past the sequence end lie outside the buffer views: zeros
    const uint32_t soff = uint32_t(t) * srcK.step;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      dma_16(srcK.rs, sK + buf * TILE + (wave * NI + j) * 512, voff[j], soff);
      dma_16(srcV.rs, sV + buf * TILE + (wave * NI + j) * 512, voff[j], soff);
    }
  };
  // this lane's read addresses (buffer 0; the other buffer, the 16-row block and the 32-key step are immediates)
  uint32_t ak[KS], av[DB];
  {
    const uint32_t kbase = uint32_t(reinterpret_cast<uintptr_t>(sK)) + uint32_t(lq) * 256u, xk = row_swz(lq);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ak[ks] = kbase + ((uint32_t(ks * 4 + lh) ^ xk) * 16u);
    const int rv = lh * 4 + (lq >> 2);
    const uint32_t vbase = uint32_t(reinterpret_cast<uintptr_t>(sV)) + uint32_t(rv) * 256u + uint32_t(lq & 1) * 8u, xv = row_swz(rv);
#pragma unroll
    for (int db = 0; db < DB; ++db) av[db] = vbase + ((uint32_t(db * 2 + ((lq & 3) >> 1)) ^ xv) * 16u);
  }

  for (int seg = 0; seg < (PAIRED ? 2 : 1); ++seg) {
  const int qt = PAIRED ? (seg == 0 ? a.q_tiles - 1 - u : u) : (a.causal ? a.q_tiles - 1 - u : u);
  if (seg == 1) {
    if (qt == a.q_tiles - 1 - u) break;  // odd tile count: the middle tile has no partner
    __syncthreads();                     // the first pass's last tile has been read by everyone
  }
  const int64_t tblk = int64_t(sh) * a.q_tiles + (a.causal ? a.q_tiles - 1 - qt : qt);
  const int q0 = qt * kRows + wave * 16;

  bf16x8 qf[KS];
  {
    const int qr = min(q0 + lq, S - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(Qp + (tok0 + qr) * a.ld + ks * 32 + lh * 8);
  }
  f32x4 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;
  const int kv_end = a.causal ? min(S, qt * kRows + kRows) : S;
  const int n_tiles = (kv_end + kBKV - 1) / kBKV;
  const int t_lo = a.n_parts > 1 ? int(int64_t(piece) * n_tiles / a.n_parts) : 0;
  const int t_hi = a.n_parts > 1 ? int(int64_t(piece + 1) * n_tiles / a.n_parts) : n_tiles;

  // one key tile out of buffer BUF (a compile-time constant, so that every LDS offset is an immediate)
  auto tile_step = [&](auto bufc, int t) {
    constexpr int BUF = decltype(bufc)::value;
    constexpr int BO = BUF * TILE * 2;  // byte offset of the buffer
    dma_done();        // this wavefront's share of tile t has landed ...
    __syncthreads();   // ... and everyone's; everyone has finished reading tile t - 1 in the other buffer
    if (t + 1 < t_hi) dma_tile(t + 1, BUF ^ 1);
    const int kv0 = t * kBKV;
    if (a.causal && kv0 > q0 + 15) return;  // every key of the tile lies after this wavefront's last query row
    // scores, transposed: st[kb][r] = S[query lane % 16][key kv0 + kb*16 + (lane/16)*4 + r]
    attn_u32x4 kf[2][8];  // [kb / 2][(kb % 2) * 4 + ks]
    kf[0][0] = lds_frag_b128<BO + 0 * 4096>(ak[0]); kf[0][1] = lds_frag_b128<BO + 0 * 4096>(ak[1]);
    kf[0][2] = lds_frag_b128<BO + 0 * 4096>(ak[2]); kf[0][3] = lds_frag_b128<BO + 0 * 4096>(ak[3]);
    kf[0][4] = lds_frag_b128<BO + 1 * 4096>(ak[0]); kf[0][5] = lds_frag_b128<BO + 1 * 4096>(ak[1]);
    kf[0][6] = lds_frag_b128<BO + 1 * 4096>(ak[2]); kf[0][7] = lds_frag_b128<BO + 1 * 4096>(ak[3]);
    kf[1][0] = lds_frag_b128<BO + 2 * 4096>(ak[0]); kf[1][1] = lds_frag_b128<BO + 2 * 4096>(ak[1]);
    kf[1][2] = lds_frag_b128<BO + 2 * 4096>(ak[2]); kf[1][3] = lds_frag_b128<BO + 2 * 4096>(ak[3]);
    kf[1][4] = lds_frag_b128<BO + 3 * 4096>(ak[0]); kf[1][5] = lds_frag_b128<BO + 3 * 4096>(ak[1]);
    kf[1][6] = lds_frag_b128<BO + 3 * 4096>(ak[2]); kf[1][7] = lds_frag_b128<BO + 3 * 4096>(ak[3]);
    lds_reads_done(kf[0]);
    lds_reads_tied(kf[1]);
    f32x4 st[4];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      st[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) st[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kf[kb >> 1][(kb & 1) * 4 + ks]), qf[ks], st[kb], 0, 0, 0);
    }
    // value fragments of the second product: requested now, needed after the softmax
    attn_u32x2 vf[4][8];  // [db / 2][(db % 2) * 4 + s2 * 2 + half]: keys s2*32 + half*16 .. of the tile
    vf[0][0] = lds_tr_b64<BO + 0>(av[0]); vf[0][1] = lds_tr_b64<BO + 4096>(av[0]); vf[0][2] = lds_tr_b64<BO + 8192>(av[0]); vf[0][3] = lds_tr_b64<BO + 12288>(av[0]);
    vf[0][4] = lds_tr_b64<BO + 0>(av[1]); vf[0][5] = lds_tr_b64<BO + 4096>(av[1]); vf[0][6] = lds_tr_b64<BO + 8192>(av[1]); vf[0][7] = lds_tr_b64<BO + 12288>(av[1]);
    vf[1][0] = lds_tr_b64<BO + 0>(av[2]); vf[1][1] = lds_tr_b64<BO + 4096>(av[2]); vf[1][2] = lds_tr_b64<BO + 8192>(av[2]); vf[1][3] = lds_tr_b64<BO + 12288>(av[2]);
    vf[1][4] = lds_tr_b64<BO + 0>(av[3]); vf[1][5] = lds_tr_b64<BO + 4096>(av[3]); vf[1][6] = lds_tr_b64<BO + 8192>(av[3]); vf[1][7] = lds_tr_b64<BO + 12288>(av[3]);
    vf[2][0] = lds_tr_b64<BO + 0>(av[4]); vf[2][1] = lds_tr_b64<BO + 4096>(av[4]); vf[2][2] = lds_tr_b64<BO + 8192>(av[4]); vf[2][3] = lds_tr_b64<BO + 12288>(av[4]);
    vf[2][4] = lds_tr_b64<BO + 0>(av[5]); vf[2][5] = lds_tr_b64<BO + 4096>(av[5]); vf[2][6] = lds_tr_b64<BO + 8192>(av[5]); vf[2][7] = lds_tr_b64<BO + 12288>(av[5]);
    vf[3][0] = lds_tr_b64<BO + 0>(av[6]); vf[3][1] = lds_tr_b64<BO + 4096>(av[6]); vf[3][2] = lds_tr_b64<BO + 8192>(av[6]); vf[3][3] = lds_tr_b64<BO + 12288>(av[6]);
    vf[3][4] = lds_tr_b64<BO + 0>(av[7]); vf[3][5] = lds_tr_b64<BO + 4096>(av[7]); vf[3][6] = lds_tr_b64<BO + 8192>(av[7]); vf[3][7] = lds_tr_b64<BO + 12288>(av[7]);

    const bool edge = kv0 + kBKV > S || (a.causal && kv0 + kBKV - 1 > q0);
    const int qrow = q0 + lq;
    if (edge) {
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = kv0 + kb * 16 + lh * 4 + r;
          if (key >= S || (a.causal && key > qrow)) st[kb][r] = -INFINITY;
        }
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int r = 0; r < 4; ++r) mx = fmaxf(mx, st[kb][r]);
    mx = xor_max(mx) * a.scale_log2;
    const float m_new = fmaxf(m_run, mx);
    const float m_use = m_new == -INFINITY ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_use);
    float ls = 0.f;
    float p[4][4];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        p[kb][r] = fast_exp2(fmaf(st[kb][r], a.scale_log2, -m_use));
        ls += p[kb][r];
      }
    l_run = l_run * alpha + ls;
    m_run = m_new;
    if (__any(alpha != 1.0f)) {
#pragma unroll
      for (int db = 0; db < DB; ++db) acc[db] *= alpha;
    }
    bf16x8 pf[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      bf16x8 f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        f[r] = static_cast<__bf16>(p[2 * s2][r]);
        f[4 + r] = static_cast<__bf16>(p[2 * s2 + 1][r]);
      }
      pf[s2] = f;
    }
    lds_reads_done(vf[0]);
    lds_reads_tied(vf[1]);
    lds_reads_tied(vf[2]);
    lds_reads_tied(vf[3]);
    // O^T += V^T P^T (key slots of a 32-key step in the order the scores sit in the registers: see attn_core_fwd_kernel)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = vf[db >> 1][(db & 1) * 4 + s2 * 2], hi = vf[db >> 1][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pf[s2], acc[db], 0, 0, 0);
      }
  };

  if (t_lo < t_hi) dma_tile(t_lo, 0);
  for (int t = t_lo; t < t_hi; t += 2) {
    tile_step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < t_hi) tile_step(std::integral_constant<int, 1>{}, t + 1);
  }

  if (a.n_parts > 1) {
    float* pp = a.part_sums + ((tblk * a.n_parts + piece) * kRows + wave * 16 + lq) * (D + 4);
#pragma unroll
    for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(pp + db * 16 + lh * 4) = acc[db];
    const float l = xor_sum(l_run);
    if (lh == 0) {
      pp[D] = m_run;
      pp[D + 1] = l;
    }
    continue;
  }
  {
    const int qrow = q0 + lq;
    const float l = xor_sum(l_run);
    const float inv = 1.0f / l;
    if (qrow < S) {
      uint16_t* cp = a.C + (tok0 + qrow) * a.ldc + int64_t(head) * D + lh * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        u16x4 o;
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = ntp_gemm::f32_to_bf16(acc[db][r] * inv);
        *reinterpret_cast<u16x4*>(cp + db * 16) = o;
      }
      if (lh == 0 && a.LSE) a.LSE[int64_t(head) * (int64_t(a.n_seq) * S) + tok0 + qrow] = (m_run + log2f(l)) * 0.6931471805599453f;
    }
  }
  }  // the workgroup's passes
}

// ---- forward kernel by DMA, 32 query rows per wavefront ---------------------------------------------------------
// The form of attn_core_fwd_dma_kernel for launches with many workgroups: a workgroup takes 128 query rows, a wavefront
// two 16-row blocks, so that every fragment read from LDS feeds two matrix instructions (LDS reads are what a
// compute unit runs out of first with 16 rows per wavefront).  Two workgroups share a compute unit (64 KB of LDS each).
template <bool PAIRED>
__global__ __attribute__((amdgpu_flat_work_group_size(kThreads, kThreads), amdgpu_waves_per_eu(2, 2))) void
attn_core_fwd_dma2_kernel(const CoreArgs a) {
  constexpr int D = 128, KS = D / 32, DB = D / 16, QB = 2, kRows = 64 * QB;
  constexpr int TILE = kDmaTile;
  constexpr int NI = TILE * 2 / 1024 / 4;  // DMA instructions per wavefront, matrix and tile
  __shared__ __attribute__((aligned(1024))) uint16_t sK[2 * TILE];
  __shared__ __attribute__((aligned(1024))) uint16_t sV[2 * TILE];

  const uint32_t bid = xcd_major(blockIdx.x, gridDim.x);
  const int piece = a.n_parts > 1 ? int(bid % a.n_parts) : 0;
  const int blk = a.n_parts > 1 ? int(bid / a.n_parts) : int(bid);
  const int per_seq = PAIRED ? a.pairs : a.q_tiles;
  const int u = blk % per_seq;
  const int sh = blk / per_seq;
  const int seq = sh % a.n_seq, head = sh / a.n_seq;
  const int g = (a.q_off + head) / a.group - a.kv_off;
  const int S = a.seq_len;
  const int64_t tok0 = int64_t(seq) * S;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lq = lane & 15, lh = lane >> 4;
  const uint16_t* Qp = a.QKV + int64_t(head) * D;
  const uint16_t* Kp = a.QKV + int64_t(a.q_cnt + g) * D;
  const uint16_t* Vp = a.QKV + int64_t(a.q_cnt + a.kv_cnt + g) * D;
  TileSrc<D> srcK, srcV;
  srcK.init(Kp + tok0 * a.ld, a.ld, S);
  srcV.init(Vp + tok0 * a.ld, a.ld, S);
  uint32_t voff[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int p = (wave * NI + j) * 64 + lane;
    const int row = p >> 4, slot = p & 15;
    voff[j] = uint32_t((int64_t(row) * a.ld + int64_t(uint32_t(slot) ^ row_swz(row)) * 8) * 2);
  }
  auto dma_tile = [&](int t, int buf) {  // rows past the sequence end lie outside the buffer views: zeros
    const uint32_t soff = uint32_t(t) * srcK.step;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      dma_16(srcK.rs, sK + buf * TILE + (wave * NI + j) * 512, voff[j], soff);
      dma_16(srcV.rs, sV + buf * TILE + (wave * NI + j) * 512, voff[j], soff);
    }
  };
  uint32_t ak[KS], av[DB];
  {
    const uint32_t kbase = uint32_t(reinterpret_cast<uintptr_t>(sK)) + uint32_t(lq) * 256u, xk = row_swz(lq);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ak[ks] = kbase + ((uint32_t(ks * 4 + lh) ^ xk) * 16u);
    const int rv = lh * 4 + (lq >> 2);
    const uint32_t vbase = uint32_t(reinterpret_cast<uintptr_t>(sV)) + uint32_t(rv) * 256u + uint32_t(lq & 1) * 8u, xv = row_swz(rv);
#pragma unroll
    for (int db = 0; db < DB; ++db) av[db] = vbase + ((uint32_t(db * 2 + ((lq & 3) >> 1)) ^ xv) * 16u);
  }

  for (int seg = 0; seg < (PAIRED ? 2 : 1); ++seg) {
  const int qt = PAIRED ? (seg == 0 ? a.q_tiles - 1 - u : u) : (a.causal ? a.q_tiles - 1 - u : u);
  if (seg == 1) {
    if (qt == a.q_tiles - 1 - u) break;  // odd tile count: the middle tile has no partner
    __syncthreads();                     // the first pass's last tile has been read by everyone
  }
  const int64_t tblk = int64_t(sh) * a.q_tiles + (a.causal ? a.q_tiles - 1 - qt : qt);
  const int q0 = qt * kRows + wave * (16 * QB);

  bf16x8 qf[QB][KS];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qr = min(q0 + qb * 16 + lq, S - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *reinterpret_cast<const bf16x8*>(Qp + (tok0 + qr) * a.ld + ks * 32 + lh * 8);
  }
  f32x4 acc[QB][DB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
  }
  const int kv_end = a.causal ? min(S, qt * kRows + kRows) : S;
  const int n_tiles = (kv_end + kBKV - 1) / kBKV;
  const int t_lo = a.n_parts > 1 ? int(int64_t(piece) * n_tiles / a.n_parts) : 0;
  const int t_hi = a.n_parts > 1 ? int(int64_t(piece + 1) * n_tiles / a.n_parts) : n_tiles;

  // one key tile out of buffer BUF (a compile-time constant, so that every LDS offset is an immediate)
  auto tile_step = [&](auto bufc, int t) {
    constexpr int BUF = decltype(bufc)::value;
    constexpr int BO = BUF * TILE * 2;  // byte offset of the buffer
    dma_done();        // this wavefront's share of tile t has landed ...
    __syncthreads();   // ... and everyone's; everyone has finished reading tile t - 1 in the other buffer
    if (t + 1 < t_hi) dma_tile(t + 1, BUF ^ 1);
    const int kv0 = t * kBKV;
    if (a.causal && kv0 > q0 + 16 * QB - 1) return;  // every key of the tile lies after this wavefront's last query row
    // scores, transposed: st[kb][qb][r] = S[query qb*16 + lane%16][key kv0 + kb*16 + (lane/16)*4 + r];
    // key blocks 0-1 first, 2-3 read under their matrix instructions
    attn_u32x4 k01[8], k23[8];  // [(kb % 2) * 4 + ks]
    k01[0] = lds_frag_b128<BO + 0 * 4096>(ak[0]); k01[1] = lds_frag_b128<BO + 0 * 4096>(ak[1]); k01[2] = lds_frag_b128<BO + 0 * 4096>(ak[2]); k01[3] = lds_frag_b128<BO + 0 * 4096>(ak[3]);
    k01[4] = lds_frag_b128<BO + 1 * 4096>(ak[0]); k01[5] = lds_frag_b128<BO + 1 * 4096>(ak[1]); k01[6] = lds_frag_b128<BO + 1 * 4096>(ak[2]); k01[7] = lds_frag_b128<BO + 1 * 4096>(ak[3]);
    lds_reads_done(k01);
    k23[0] = lds_frag_b128<BO + 2 * 4096>(ak[0]); k23[1] = lds_frag_b128<BO + 2 * 4096>(ak[1]); k23[2] = lds_frag_b128<BO + 2 * 4096>(ak[2]); k23[3] = lds_frag_b128<BO + 2 * 4096>(ak[3]);
    k23[4] = lds_frag_b128<BO + 3 * 4096>(ak[0]); k23[5] = lds_frag_b128<BO + 3 * 4096>(ak[1]); k23[6] = lds_frag_b128<BO + 3 * 4096>(ak[2]); k23[7] = lds_frag_b128<BO + 3 * 4096>(ak[3]);
    f32x4 st[4][QB];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        st[kb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          st[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k01[kb * 4 + ks]), qf[qb][ks], st[kb][qb], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
    lds_reads_done(k23);
    // value fragments of the second product, 8 reads (two 16-column blocks) per group: the first two groups are
    // requested now and land under the rest of the score product and the softmax
    attn_u32x2 vf[4][8];  // [db / 2][(db % 2) * 4 + s2 * 2 + half]: keys s2*32 + half*16 .. of the tile
    vf[0][0] = lds_tr_b64<BO + 0>(av[0]); vf[0][1] = lds_tr_b64<BO + 4096>(av[0]); vf[0][2] = lds_tr_b64<BO + 8192>(av[0]); vf[0][3] = lds_tr_b64<BO + 12288>(av[0]);
    vf[0][4] = lds_tr_b64<BO + 0>(av[1]); vf[0][5] = lds_tr_b64<BO + 4096>(av[1]); vf[0][6] = lds_tr_b64<BO + 8192>(av[1]); vf[0][7] = lds_tr_b64<BO + 12288>(av[1]);
    vf[1][0] = lds_tr_b64<BO + 0>(av[2]); vf[1][1] = lds_tr_b64<BO + 4096>(av[2]); vf[1][2] = lds_tr_b64<BO + 8192>(av[2]); vf[1][3] = lds_tr_b64<BO + 12288>(av[2]);
    vf[1][4] = lds_tr_b64<BO + 0>(av[3]); vf[1][5] = lds_tr_b64<BO + 4096>(av[3]); vf[1][6] = lds_tr_b64<BO + 8192>(av[3]); vf[1][7] = lds_tr_b64<BO + 12288>(av[3]);
#pragma unroll
    for (int kb = 2; kb < 4; ++kb)
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        st[kb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
          st[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k23[(kb - 2) * 4 + ks]), qf[qb][ks], st[kb][qb], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);

    const bool edge = kv0 + kBKV > S || (a.causal && kv0 + kBKV - 1 > q0);
    bf16x8 pf[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int qrow = q0 + qb * 16 + lq;
      if (edge) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int key = kv0 + kb * 16 + lh * 4 + r;
            if (key >= S || (a.causal && key > qrow)) st[kb][qb][r] = -INFINITY;
          }
      }
      float mx = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) mx = fmaxf(mx, st[kb][qb][r]);
      mx = xor_max(mx) * a.scale_log2;
      const float m_new = fmaxf(m_run[qb], mx);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = fast_exp2(m_run[qb] - m_use);
      float ls = 0.f;
      float pr[4][4];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          pr[kb][r] = fast_exp2(fmaf(st[kb][qb][r], a.scale_log2, -m_use));
          ls += pr[kb][r];
        }
      l_run[qb] = l_run[qb] * alpha + ls;
      m_run[qb] = m_new;
      if (__any(alpha != 1.0f)) {
#pragma unroll
        for (int db = 0; db < DB; ++db) acc[qb][db] *= alpha;
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        bf16x8 f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          f[r] = static_cast<__bf16>(pr[2 * s2][r]);
          f[4 + r] = static_cast<__bf16>(pr[2 * s2 + 1][r]);
        }
        pf[qb][s2] = f;
      }
    }
    // O^T += V^T P^T (key slots of a 32-key step in the order the scores sit in the registers: see
    // attn_core_fwd_kernel); every group of reads lands under the 8 matrix instructions of the group before it
    auto pv_group = [&](attn_u32x2 (&f)[8], int db0) {
#pragma unroll
      for (int d2 = 0; d2 < 2; ++d2)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const attn_u32x2 lo = f[d2 * 4 + s2 * 2], hi = f[d2 * 4 + s2 * 2 + 1];
          const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
#pragma unroll
          for (int qb = 0; qb < QB; ++qb)
            acc[qb][db0 + d2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pf[qb][s2], acc[qb][db0 + d2], 0, 0, 0);
        }
    };
    lds_reads_done(vf[0]);
    lds_reads_tied(vf[1]);
    __builtin_amdgcn_sched_barrier(0);
    vf[2][0] = lds_tr_b64<BO + 0>(av[4]); vf[2][1] = lds_tr_b64<BO + 4096>(av[4]); vf[2][2] = lds_tr_b64<BO + 8192>(av[4]); vf[2][3] = lds_tr_b64<BO + 12288>(av[4]);
    vf[2][4] = lds_tr_b64<BO + 0>(av[5]); vf[2][5] = lds_tr_b64<BO + 4096>(av[5]); vf[2][6] = lds_tr_b64<BO + 8192>(av[5]); vf[2][7] = lds_tr_b64<BO + 12288>(av[5]);
    pv_group(vf[0], 0);
    __builtin_amdgcn_sched_barrier(0);
    vf[3][0] = lds_tr_b64<BO + 0>(av[6]); vf[3][1] = lds_tr_b64<BO + 4096>(av[6]); vf[3][2] = lds_tr_b64<BO + 8192>(av[6]); vf[3][3] = lds_tr_b64<BO + 12288>(av[6]);
    vf[3][4] = lds_tr_b64<BO + 0>(av[7]); vf[3][5] = lds_tr_b64<BO + 4096>(av[7]); vf[3][6] = lds_tr_b64<BO + 8192>(av[7]); vf[3][7] = lds_tr_b64<BO + 12288>(av[7]);
    pv_group(vf[1], 2);
    __builtin_amdgcn_sched_barrier(0);
    lds_reads_left<8>(vf[2]);
    pv_group(vf[2], 4);
    __builtin_amdgcn_sched_barrier(0);
    lds_reads_done(vf[3]);
    pv_group(vf[3], 6);
    __builtin_amdgcn_sched_barrier(0);
  };

  if (t_lo < t_hi) dma_tile(t_lo, 0);
  for (int t = t_lo; t < t_hi; t += 2) {
    tile_step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < t_hi) tile_step(std::integral_constant<int, 1>{}, t + 1);
  }

  if (a.n_parts > 1) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float* pp = a.part_sums + ((tblk * a.n_parts + piece) * kRows + wave * (16 * QB) + qb * 16 + lq) * (D + 4);
#pragma unroll
      for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(pp + db * 16 + lh * 4) = acc[qb][db];
      const float l = xor_sum(l_run[qb]);
      if (lh == 0) {
        pp[D] = m_run[qb];
        pp[D + 1] = l;
      }
    }
    continue;
  }
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qrow = q0 + qb * 16 + lq;
    const float l = xor_sum(l_run[qb]);
    const float inv = 1.0f / l;
    if (qrow < S) {
      uint16_t* cp = a.C + (tok0 + qrow) * a.ldc + int64_t(head) * D + lh * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        u16x4 o;
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = ntp_gemm::f32_to_bf16(acc[qb][db][r] * inv);
        *reinterpret_cast<u16x4*>(cp + db * 16) = o;
      }
      if (lh == 0 && a.LSE) a.LSE[int64_t(head) * (int64_t(a.n_seq) * S) + tok0 + qrow] = (m_run[qb] + log2f(l)) * 0.6931471805599453f;
    }
  }
  }  // the workgroup's passes
}

// Merges the pieces of a cut forward walk: with m = max_p m_p, the row is sum_p 2^(m_p - m) O_p over
// sum_p 2^(m_p - m) l_p.  One thread per 4 output values; a piece that saw no key has m_p = -inf, l_p = 0.
template <int D>
__global__ __launch_bounds__(256) void attn_core_fwd_merge_kernel(const CoreArgs a, int64_t n_blk) {
  constexpr int Q = D / 4, W = D + 4;
  const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int c = int(idx % Q) * 4, row = int((idx / Q) % 64);
  const int64_t blk = idx / (Q * 64);
  if (blk >= n_blk) return;
  const int qt = a.causal ? a.q_tiles - 1 - int(blk % a.q_tiles) : int(blk % a.q_tiles);
  const int64_t sh = blk / a.q_tiles;
  const int seq = int(sh % a.n_seq), head = int(sh / a.n_seq);
  const int qrow = qt * 64 + row;
  if (qrow >= a.seq_len) return;
  const float* p = a.part_sums + (blk * a.n_parts * 64 + row) * W;
  float m = -INFINITY;
  for (int i = 0; i < a.n_parts; ++i) m = fmaxf(m, p[int64_t(i) * 64 * W + D]);
  f32x4 o = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int i = 0; i < a.n_parts; ++i) {
    const float* pi = p + int64_t(i) * 64 * W;
    const float w = fast_exp2(pi[D] - m);  // every row sees at least one key, so m is finite
    o = o + *reinterpret_cast<const f32x4*>(pi + c) * w;
    l += pi[D + 1] * w;
  }
  const float inv = 1.0f / l;
  u16x4 out;
#pragma unroll
  for (int r = 0; r < 4; ++r) out[r] = ntp_gemm::f32_to_bf16(o[r] * inv);
  const int64_t tok = int64_t(seq) * a.seq_len + qrow;
  *reinterpret_cast<u16x4*>(a.C + tok * a.ldc + int64_t(head) * D + c) = out;
  if (c == 0 && a.LSE) a.LSE[int64_t(head) * (int64_t(a.n_seq) * a.seq_len) + tok] = (m + log2f(l)) * 0.6931471805599453f;
}

// ---- backward ---------------------------------------------------------------------------------
// With P = softmax rows (rebuilt from the saved log-sum-exp), dP = dC V^T and
// delta_i = sum_d dC_id C_id:  dS = P .* (dP - delta),  dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d),
// dV = P^T dC.  Two kernels, no atomics: one owns query rows and walks over the keys (dQ, and delta on
// the way), one owns keys and walks over the query rows of every local query head that reads them
// (dK, dV).  Both keep the owned index on the lane axis like the forward kernel.
struct CoreBwdArgs {
  const uint16_t* QKV;
  const uint16_t* C;
  const uint16_t* dC;
  const float* LSE;
  float* Delta;
  uint16_t* dQKV;
  int64_t ld, ldc, lddc, ldd;
  int32_t n_seq, seq_len, q_cnt, kv_cnt, q_off, kv_off, group, causal;
  int32_t tiles;        // query tiles (dQ kernel) or key tiles (dK/dV kernel) per sequence
  float scale_log2;     // log2(e) / sqrt(d)
  float scale;          // 1 / sqrt(d)
  // n_parts > 1: the walk of every workgroup is cut into n_parts pieces, one workgroup each, which store
  // their fp32 sums to part_sums ([workgroup][part][64 rows][row length]); a second kernel adds them
  float* part_sums;
  int32_t n_parts;
  // pairs > 0 (causal mask): a workgroup takes two tiles one after the other, one from each end of the sequence, so
  // that every workgroup's walk has the same length (tiles + 1 tiles, cut into n_parts); pairs = (tiles + 1) / 2
  // workgroups per (sequence, head)
  int32_t pairs;
  // 1: the dQ kernel does not store the rows' delta values (a kernel before it has)
  int32_t delta_stored;
};

typedef __attribute__((address_space(3))) s16x4 lds_s16x4_t;

// Operand A[i = column c0 + lane%16][k = row slot] of a row-major LDS tile: rows 4 (lane/16) .. + 3 from
// r0 on for slots 0..3 and the same 16 rows further down for slots 4..7 (see the forward kernel).
__device__ __forceinline__ bf16x8 tr_frag(const uint16_t* tile, int ldt, int r0, int c0, int lq, int lh) {
  const uint16_t* vp = tile + (r0 + lh * 4 + (lq >> 2)) * ldt + c0 + (lq & 3) * 4;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(vp));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(vp + 16 * ldt));
  const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  return __builtin_bit_cast(bf16x8, both);
}

// dQ (and delta): a workgroup takes 64 QB query rows of one (sequence, head), a wavefront 16 QB of them.
template <int D, int QB, bool PAIRED>
__global__ __attribute__((amdgpu_flat_work_group_size(kThreads, kThreads), amdgpu_waves_per_eu(QB == 1 ? 3 : 2, QB == 1 ? 3 : 2))) void
attn_core_bwd_dq_kernel(const CoreBwdArgs a) {
  constexpr int kRows = 64 * QB;
  constexpr int LDT = D + 16, KS = D / 32, DB = D / 16, CPR = D / 8, NLD = kBKV * CPR / kThreads;
  __shared__ __attribute__((aligned(16))) uint16_t sK[kBKV * LDT];
  __shared__ __attribute__((aligned(16))) uint16_t sV[kBKV * LDT];
  const uint32_t bid = xcd_major(blockIdx.x, gridDim.x);
  const int piece = a.n_parts > 1 ? int(bid % a.n_parts) : 0;
  const int blk = a.n_parts > 1 ? int(bid / a.n_parts) : int(bid);
  const int per_seq = PAIRED ? a.pairs : a.tiles;
  const int u = blk % per_seq;
  const int sh = blk / per_seq;
  const int seq = sh % a.n_seq, head = sh / a.n_seq;
  const int g = (a.q_off + head) / a.group - a.kv_off;
  const int S = a.seq_len;
  const int64_t tok0 = int64_t(seq) * S, Mtot = int64_t(a.n_seq) * S;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lq = lane & 15, lh = lane >> 4;
  const uint16_t* Qp = a.QKV + int64_t(head) * D;
  const uint16_t* Kp = a.QKV + int64_t(a.q_cnt + g) * D;
  const uint16_t* Vp = a.QKV + int64_t(a.q_cnt + a.kv_cnt + g) * D;
  ntp_gemm::u16x8 rk[NLD], rv[NLD];
  uint32_t voff[NLD];
  TileSrc<D>::tile_offsets(a.ld, voff);
  TileSrc<D> srcK, srcV;
  srcK.init(Kp + tok0 * a.ld, a.ld, S);
  srcV.init(Vp + tok0 * a.ld, a.ld, S);

  for (int seg = 0; seg < (PAIRED ? 2 : 1); ++seg) {
  const int qt = PAIRED ? (seg == 0 ? a.tiles - 1 - u : u) : (a.causal ? a.tiles - 1 - u : u);
  if (seg == 1) {
    if (qt == a.tiles - 1 - u) break;  // odd tile count: the middle tile has no partner
    __syncthreads();                   // the first pass's last tile has been read by everyone
  }
  // the tile's number in the order the reduce kernel counts them (late tiles first under the causal mask)
  const int64_t tblk = int64_t(sh) * a.tiles + (a.causal ? a.tiles - 1 - qt : qt);
  const int q0 = qt * kRows + wave * (16 * QB);

  // query and output-gradient fragments (operand B: j = query row), delta and the log-sum-exp of the rows
  bf16x8 qf[QB][KS], gf[QB][KS];
  float lse2[QB], delta[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qr = min(q0 + qb * 16 + lq, S - 1);
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[qb][ks] = *reinterpret_cast<const bf16x8*>(Qp + (tok0 + qr) * a.ld + ks * 32 + lh * 8);
      gf[qb][ks] = *reinterpret_cast<const bf16x8*>(a.dC + (tok0 + qr) * a.lddc + int64_t(head) * D + ks * 32 + lh * 8);
      const bf16x8 of = *reinterpret_cast<const bf16x8*>(a.C + (tok0 + qr) * a.ldc + int64_t(head) * D + ks * 32 + lh * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) part += float(gf[qb][ks][e]) * float(of[e]);
    }
    delta[qb] = xor_sum(part);
    lse2[qb] = a.LSE[int64_t(head) * Mtot + tok0 + qr] * 1.4426950408889634f;
    if (lh == 0 && piece == 0 && q0 + qb * 16 + lq < S) a.Delta[int64_t(head) * Mtot + tok0 + qr] = delta[qb];
  }

  f32x4 acc[QB][DB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb)
#pragma unroll
    for (int db = 0; db < DB; ++db) acc[qb][db] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int kv_end = a.causal ? min(S, qt * kRows + kRows) : S;
  const int n_tiles = (kv_end + kBKV - 1) / kBKV;
  auto load_tile = [&](int t) {  // rows past the sequence end arrive as zeros (masked below)
    srcK.load(t, voff, rk);
    srcV.load(t, voff, rv);
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int c = threadIdx.x + i * kThreads;
      const int o = (c / CPR) * LDT + (c % CPR) * 8;
      *reinterpret_cast<ntp_gemm::u16x8*>(sK + o) = rk[i];
      *reinterpret_cast<ntp_gemm::u16x8*>(sV + o) = rv[i];
    }
  };

  // this workgroup's share of the key tiles (all of them unless the walk is cut into parts)
  const int t_lo = a.n_parts > 1 ? int(int64_t(piece) * n_tiles / a.n_parts) : 0;
  const int t_hi = a.n_parts > 1 ? int(int64_t(piece + 1) * n_tiles / a.n_parts) : n_tiles;
  if (t_lo < t_hi) load_tile(t_lo);
  for (int t = t_lo; t < t_hi; ++t) {
    __syncthreads();
    store_tile();
    __syncthreads();
    if (t + 1 < t_hi) load_tile(t + 1);
    const int kv0 = t * kBKV;
    if (a.causal && kv0 > q0 + 16 * QB - 1) continue;  // nothing of this tile is visible to the wavefront's rows
    // S^T and dP^T blocks: [key kb*16 + (lane/16)*4 + r][query qb*16 + lane%16]
    f32x4 st[4][QB], dpt[4][QB];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        st[kb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
        dpt[kb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
      }
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + (kb * 16 + lq) * LDT + ks * 32 + lh * 8);
        const bf16x8 vf = *reinterpret_cast<const bf16x8*>(sV + (kb * 16 + lq) * LDT + ks * 32 + lh * 8);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          st[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf, qf[qb][ks], st[kb][qb], 0, 0, 0);
          dpt[kb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf, gf[qb][ks], dpt[kb][qb], 0, 0, 0);
        }
      }
    }
    const bool edge = kv0 + kBKV > S || (a.causal && kv0 + kBKV - 1 > q0);
    bf16x8 dsf[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int qrow = q0 + qb * 16 + lq;
      float ds[4][4];
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) ds[kb][r] = fast_exp2(fmaf(st[kb][qb][r], a.scale_log2, -lse2[qb]));
      if (edge) {
#pragma unroll
        for (int kb = 0; kb < 4; ++kb)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int key = kv0 + kb * 16 + lh * 4 + r;
            if (key >= S || (a.causal && key > qrow)) ds[kb][r] = 0.f;
          }
      }
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) ds[kb][r] *= dpt[kb][qb][r] - delta[qb];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        bf16x8 f;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          f[r] = static_cast<__bf16>(ds[2 * s2][r]);
          f[4 + r] = static_cast<__bf16>(ds[2 * s2 + 1][r]);
        }
        dsf[qb][s2] = f;
      }
    }
    // dQ^T += K^T dS^T
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 kt = tr_frag(sK, LDT, s2 * 32, db * 16, lq, lh);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) acc[qb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kt, dsf[qb][s2], acc[qb][db], 0, 0, 0);
      }
  }
  if (a.n_parts > 1) {
    // unscaled fp32 sums of this part: row (wavefront, block, lane % 16) of the workgroup's 64 QB rows
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      float* pp = a.part_sums + ((tblk * a.n_parts + piece) * kRows + wave * (16 * QB) + qb * 16 + lq) * D + lh * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(pp + db * 16) = acc[qb][db];
    }
    continue;
  }
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int qrow = q0 + qb * 16 + lq;
    if (qrow >= S) continue;
    uint16_t* op = a.dQKV + (tok0 + qrow) * a.ldd + int64_t(head) * D + lh * 4;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      u16x4 o;
#pragma unroll
      for (int r = 0; r < 4; ++r) o[r] = ntp_gemm::f32_to_bf16(acc[qb][db][r] * a.scale);
      *reinterpret_cast<u16x4*>(op + db * 16) = o;
    }
  }
  }  // the workgroup's passes
}

// The dQ kernel with the key / value tiles brought to LDS by DMA (see attn_core_fwd_dma_kernel: the same chunk-permuted
// rows, two buffers per matrix, one barrier per tile, LDS reads as inline assembly with their waits).  Head
// dimension 128, 16 query rows per wavefront.
// (bid: the workgroup's number in its launch, or in its share of a launch; sKV: 4 tiles of LDS, key buffers 0 and
// 1, then value buffers 0 and 1: one base address per lane, the rest are immediates)
template <bool PAIRED>
__device__ __forceinline__ void bwd_dq_dma_body(const CoreBwdArgs& a, const uint32_t b_launch, const uint32_t total, uint16_t* sKV) {
  const uint32_t bid = xcd_major(b_launch, total);
  constexpr int D = 128, KS = D / 32, DB = D / 16, kRows = 64;
  constexpr int TILE = kDmaTile;           // elements of one tile
  constexpr int NI = TILE * 2 / 1024 / 4;  // DMA instructions per wavefront, matrix and tile
  const int piece = a.n_parts > 1 ? int(bid % a.n_parts) : 0;
  const int blk = a.n_parts > 1 ? int(bid / a.n_parts) : int(bid);
  const int per_seq = PAIRED ? a.pairs : a.tiles;
  const int u = blk % per_seq;
  const int sh = blk / per_seq;
  const int seq = sh % a.n_seq, head = sh / a.n_seq;
  const int g = (a.q_off + head) / a.group - a.kv_off;
  const int S = a.seq_len;
  const int64_t tok0 = int64_t(seq) * S, Mtot = int64_t(a.n_seq) * S;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lq = lane & 15, lh = lane >> 4;
  const uint16_t* Qp = a.QKV + int64_t(head) * D;
  const uint16_t* Kp = a.QKV + int64_t(a.q_cnt + g) * D;
  const uint16_t* Vp = a.QKV + int64_t(a.q_cnt + a.kv_cnt + g) * D;
  TileSrc<D> srcK, srcV;
  srcK.init(Kp + tok0 * a.ld, a.ld, S);
  srcV.init(Vp + tok0 * a.ld, a.ld, S);
  uint32_t voff[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int p = (wave * NI + j) * 64 + lane;
    const int row = p >> 4, slot = p & 15;
    voff[j] = uint32_t((int64_t(row) * a.ld + int64_t(uint32_t(slot) ^ row_swz(row)) * 8) * 2);
  }
  auto dma_tile = [&](int t, int buf) {  // rows past the sequence end lie outside the buffer views: zeros
    const uint32_t soff = uint32_t(t) * srcK.step;
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      dma_16(srcK.rs, sKV + buf * TILE + (wave * NI + j) * 512, voff[j], soff);
      dma_16(srcV.rs, sKV + (2 + buf) * TILE + (wave * NI + j) * 512, voff[j], soff);
    }
  };
  uint32_t ak[KS], at[DB];  // addresses of the row-fragment reads and of the transposing reads in key buffer 0
  {
    const uint32_t base = uint32_t(reinterpret_cast<uintptr_t>(sKV));
    const uint32_t xk = row_swz(lq);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ak[ks] = base + uint32_t(lq) * 256u + ((uint32_t(ks * 4 + lh) ^ xk) * 16u);
    const int rv = lh * 4 + (lq >> 2);
    const uint32_t xv = row_swz(rv);
#pragma unroll
    for (int db = 0; db < DB; ++db)
      at[db] = base + uint32_t(rv) * 256u + uint32_t(lq & 1) * 8u + ((uint32_t(db * 2 + ((lq & 3) >> 1)) ^ xv) * 16u);
  }

  for (int seg = 0; seg < (PAIRED ? 2 : 1); ++seg) {
  const int qt = PAIRED ? (seg == 0 ? a.tiles - 1 - u : u) : (a.causal ? a.tiles - 1 - u : u);
  if (seg == 1) {
    if (qt == a.tiles - 1 - u) break;  // odd tile count: the middle tile has no partner
    __syncthreads();                   // the first pass's last tile has been read by everyone
  }
  const int64_t tblk = int64_t(sh) * a.tiles + (a.causal ? a.tiles - 1 - qt : qt);
  const int q0 = qt * kRows + wave * 16;

  bf16x8 qf[KS], gf[KS];
  float lse2, delta;
  {
    const int qr = min(q0 + lq, S - 1);
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      qf[ks] = *reinterpret_cast<const bf16x8*>(Qp + (tok0 + qr) * a.ld + ks * 32 + lh * 8);
      gf[ks] = *reinterpret_cast<const bf16x8*>(a.dC + (tok0 + qr) * a.lddc + int64_t(head) * D + ks * 32 + lh * 8);
      const bf16x8 of = *reinterpret_cast<const bf16x8*>(a.C + (tok0 + qr) * a.ldc + int64_t(head) * D + ks * 32 + lh * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) part += float(gf[ks][e]) * float(of[e]);
    }
    delta = xor_sum(part);
    lse2 = a.LSE[int64_t(head) * Mtot + tok0 + qr] * 1.4426950408889634f;
    if (lh == 0 && piece == 0 && !a.delta_stored && q0 + lq < S) a.Delta[int64_t(head) * Mtot + tok0 + qr] = delta;
  }
  f32x4 acc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) acc[db] = f32x4{0.f, 0.f, 0.f, 0.f};
  const int kv_end = a.causal ? min(S, qt * kRows + kRows) : S;
  const int n_tiles = (kv_end + kBKV - 1) / kBKV;
  const int t_lo = a.n_parts > 1 ? int(int64_t(piece) * n_tiles / a.n_parts) : 0;
  const int t_hi = a.n_parts > 1 ? int(int64_t(piece + 1) * n_tiles / a.n_parts) : n_tiles;

  // one key tile out of buffer BUF (a compile-time constant, so that every LDS offset is an immediate)
  auto tile_step = [&](auto bufc, int t) {
    constexpr int BUF = decltype(bufc)::value;
    constexpr int KO = BUF * TILE * 2, VO = (2 + BUF) * TILE * 2;  // byte offsets of the two buffers
    dma_done();        // this wavefront's share of tile t has landed ...
    __syncthreads();   // ... and everyone's; everyone has finished reading tile t - 1 in the other buffers
    if (t + 1 < t_hi) dma_tile(t + 1, BUF ^ 1);
    const int kv0 = t * kBKV;
    if (a.causal && kv0 > q0 + 15) return;  // nothing of this tile is visible to the wavefront's rows
    // S^T and dP^T blocks: [key kb*16 + (lane/16)*4 + r][query lane%16]; key blocks 0-1 first, 2-3 behind them
    attn_u32x4 k01[8], v01[8], k23[8], v23[8];  // [(kb % 2) * 4 + ks]
    k01[0] = lds_frag_b128<KO + 0 * 4096>(ak[0]);
    k01[1] = lds_frag_b128<KO + 0 * 4096>(ak[1]);
    k01[2] = lds_frag_b128<KO + 0 * 4096>(ak[2]);
    k01[3] = lds_frag_b128<KO + 0 * 4096>(ak[3]);
    k01[4] = lds_frag_b128<KO + 1 * 4096>(ak[0]);
    k01[5] = lds_frag_b128<KO + 1 * 4096>(ak[1]);
    k01[6] = lds_frag_b128<KO + 1 * 4096>(ak[2]);
    k01[7] = lds_frag_b128<KO + 1 * 4096>(ak[3]);
    v01[0] = lds_frag_b128<VO + 0 * 4096>(ak[0]);
    v01[1] = lds_frag_b128<VO + 0 * 4096>(ak[1]);
    v01[2] = lds_frag_b128<VO + 0 * 4096>(ak[2]);
    v01[3] = lds_frag_b128<VO + 0 * 4096>(ak[3]);
    v01[4] = lds_frag_b128<VO + 1 * 4096>(ak[0]);
    v01[5] = lds_frag_b128<VO + 1 * 4096>(ak[1]);
    v01[6] = lds_frag_b128<VO + 1 * 4096>(ak[2]);
    v01[7] = lds_frag_b128<VO + 1 * 4096>(ak[3]);
    lds_reads_done(k01);
    lds_reads_tied(v01);
    k23[0] = lds_frag_b128<KO + 2 * 4096>(ak[0]);
    k23[1] = lds_frag_b128<KO + 2 * 4096>(ak[1]);
    k23[2] = lds_frag_b128<KO + 2 * 4096>(ak[2]);
    k23[3] = lds_frag_b128<KO + 2 * 4096>(ak[3]);
    k23[4] = lds_frag_b128<KO + 3 * 4096>(ak[0]);
    k23[5] = lds_frag_b128<KO + 3 * 4096>(ak[1]);
    k23[6] = lds_frag_b128<KO + 3 * 4096>(ak[2]);
    k23[7] = lds_frag_b128<KO + 3 * 4096>(ak[3]);
    f32x4 st[4], dpt[4];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      st[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
      dpt[kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        st[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k01[kb * 4 + ks]), qf[ks], st[kb], 0, 0, 0);
        dpt[kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v01[kb * 4 + ks]), gf[ks], dpt[kb], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    v23[0] = lds_frag_b128<VO + 2 * 4096>(ak[0]);
    v23[1] = lds_frag_b128<VO + 2 * 4096>(ak[1]);
    v23[2] = lds_frag_b128<VO + 2 * 4096>(ak[2]);
    v23[3] = lds_frag_b128<VO + 2 * 4096>(ak[3]);
    v23[4] = lds_frag_b128<VO + 3 * 4096>(ak[0]);
    v23[5] = lds_frag_b128<VO + 3 * 4096>(ak[1]);
    v23[6] = lds_frag_b128<VO + 3 * 4096>(ak[2]);
    v23[7] = lds_frag_b128<VO + 3 * 4096>(ak[3]);
    lds_reads_left<8>(k23);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      st[2 + kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        st[2 + kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, k23[kb * 4 + ks]), qf[ks], st[2 + kb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    lds_reads_done(v23);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      dpt[2 + kb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        dpt[2 + kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v23[kb * 4 + ks]), gf[ks], dpt[2 + kb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // transposed key fragments of the third product: requested now, needed after the arithmetic on the scores
    attn_u32x2 kt[4][8];  // [db / 2][(db % 2) * 4 + s2 * 2 + half]: keys s2*32 + half*16 .. of the tile
    kt[0][0] = lds_tr_b64<KO + 0>(at[0]); kt[0][1] = lds_tr_b64<KO + 4096>(at[0]); kt[0][2] = lds_tr_b64<KO + 8192>(at[0]); kt[0][3] = lds_tr_b64<KO + 12288>(at[0]);
    kt[0][4] = lds_tr_b64<KO + 0>(at[1]); kt[0][5] = lds_tr_b64<KO + 4096>(at[1]); kt[0][6] = lds_tr_b64<KO + 8192>(at[1]); kt[0][7] = lds_tr_b64<KO + 12288>(at[1]);
    kt[1][0] = lds_tr_b64<KO + 0>(at[2]); kt[1][1] = lds_tr_b64<KO + 4096>(at[2]); kt[1][2] = lds_tr_b64<KO + 8192>(at[2]); kt[1][3] = lds_tr_b64<KO + 12288>(at[2]);
    kt[1][4] = lds_tr_b64<KO + 0>(at[3]); kt[1][5] = lds_tr_b64<KO + 4096>(at[3]); kt[1][6] = lds_tr_b64<KO + 8192>(at[3]); kt[1][7] = lds_tr_b64<KO + 12288>(at[3]);
    kt[2][0] = lds_tr_b64<KO + 0>(at[4]); kt[2][1] = lds_tr_b64<KO + 4096>(at[4]); kt[2][2] = lds_tr_b64<KO + 8192>(at[4]); kt[2][3] = lds_tr_b64<KO + 12288>(at[4]);
    kt[2][4] = lds_tr_b64<KO + 0>(at[5]); kt[2][5] = lds_tr_b64<KO + 4096>(at[5]); kt[2][6] = lds_tr_b64<KO + 8192>(at[5]); kt[2][7] = lds_tr_b64<KO + 12288>(at[5]);
    kt[3][0] = lds_tr_b64<KO + 0>(at[6]); kt[3][1] = lds_tr_b64<KO + 4096>(at[6]); kt[3][2] = lds_tr_b64<KO + 8192>(at[6]); kt[3][3] = lds_tr_b64<KO + 12288>(at[6]);
    kt[3][4] = lds_tr_b64<KO + 0>(at[7]); kt[3][5] = lds_tr_b64<KO + 4096>(at[7]); kt[3][6] = lds_tr_b64<KO + 8192>(at[7]); kt[3][7] = lds_tr_b64<KO + 12288>(at[7]);

    const bool edge = kv0 + kBKV > S || (a.causal && kv0 + kBKV - 1 > q0);
    const int qrow = q0 + lq;
    float ds[4][4];
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int r = 0; r < 4; ++r) ds[kb][r] = fast_exp2(fmaf(st[kb][r], a.scale_log2, -lse2));
    if (edge) {
#pragma unroll
      for (int kb = 0; kb < 4; ++kb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int key = kv0 + kb * 16 + lh * 4 + r;
          if (key >= S || (a.causal && key > qrow)) ds[kb][r] = 0.f;
        }
    }
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int r = 0; r < 4; ++r) ds[kb][r] *= dpt[kb][r] - delta;
    bf16x8 dsf[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      bf16x8 f;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        f[r] = static_cast<__bf16>(ds[2 * s2][r]);
        f[4 + r] = static_cast<__bf16>(ds[2 * s2 + 1][r]);
      }
      dsf[s2] = f;
    }
    lds_reads_done(kt[0]);
    lds_reads_tied(kt[1]);
    lds_reads_tied(kt[2]);
    lds_reads_tied(kt[3]);
    // dQ^T += K^T dS^T
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = kt[db >> 1][(db & 1) * 4 + s2 * 2], hi = kt[db >> 1][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        acc[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), dsf[s2], acc[db], 0, 0, 0);
      }
  };

  if (t_lo < t_hi) dma_tile(t_lo, 0);
  for (int t = t_lo; t < t_hi; t += 2) {
    tile_step(std::integral_constant<int, 0>{}, t);
    if (t + 1 < t_hi) tile_step(std::integral_constant<int, 1>{}, t + 1);
  }

  if (a.n_parts > 1) {
    // unscaled fp32 sums of this part: row (wavefront, lane % 16) of the workgroup's 64 rows
    float* pp = a.part_sums + ((tblk * a.n_parts + piece) * kRows + wave * 16 + lq) * D + lh * 4;
#pragma unroll
    for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(pp + db * 16) = acc[db];
    continue;
  }
  {
    const int qrow = q0 + lq;
    if (qrow < S) {
      uint16_t* op = a.dQKV + (tok0 + qrow) * a.ldd + int64_t(head) * D + lh * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        u16x4 o;
#pragma unroll
        for (int r = 0; r < 4; ++r) o[r] = ntp_gemm::f32_to_bf16(acc[db][r] * a.scale);
        *reinterpret_cast<u16x4*>(op + db * 16) = o;
      }
    }
  }
  }  // the workgroup's passes
}

// dK and dV: a workgroup takes 64 KB keys of one (sequence, KV head), a wavefront 16 KB of them, and walks
// over the query rows (tiles of 64) of every local query head that reads this KV head.  KB = 2 does twice
// the matrix work per LDS read but needs 440 registers (one wavefront per SIMD); KB = 1 fits in 256, two
// workgroups share a compute unit and it measured 7-35 % faster at every size: only KB = 1 is built.
template <int D, int KB, bool PAIRED>
__global__ __launch_bounds__(kThreads, 2) void attn_core_bwd_dkv_kernel(const CoreBwdArgs a) {
  constexpr int LDT = D + 16, KS = D / 32, DB = D / 16, CPR = D / 8, NLD = kBKV * CPR / kThreads;
  __shared__ __attribute__((aligned(16))) uint16_t sQ[kBKV * LDT];
  __shared__ __attribute__((aligned(16))) uint16_t sG[kBKV * LDT];
  __shared__ __attribute__((aligned(16))) float sL[kBKV];
  __shared__ __attribute__((aligned(16))) float sD[kBKV];
  const uint32_t bid = xcd_major(blockIdx.x, gridDim.x);
  const int part = a.n_parts > 1 ? int(bid % a.n_parts) : 0;
  const int blk = a.n_parts > 1 ? int(bid / a.n_parts) : int(bid);
  const int per_seq = PAIRED ? a.pairs : a.tiles;
  const int u = blk % per_seq;
  const int sh = blk / per_seq;
  const int seq = sh % a.n_seq, g = sh / a.n_seq;  // g: local KV head
  const int S = a.seq_len;
  const int64_t tok0 = int64_t(seq) * S, Mtot = int64_t(a.n_seq) * S;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lq = lane & 15, lh = lane >> 4;
  const uint16_t* Kp = a.QKV + int64_t(a.q_cnt + g) * D;
  const uint16_t* Vp = a.QKV + int64_t(a.q_cnt + a.kv_cnt + g) * D;
  ntp_gemm::u16x8 rq[NLD], rg[NLD];
  uint32_t voffq[NLD], voffg[NLD];
  TileSrc<D>::tile_offsets(a.ld, voffq);
  TileSrc<D>::tile_offsets(a.lddc, voffg);

  for (int seg = 0; seg < (PAIRED ? 2 : 1); ++seg) {
  // this pass's key tile: with pairing an early one (whose keys most query tiles see), then its partner from the end
  const int kt = PAIRED && seg == 1 ? a.tiles - 1 - u : u;
  if (seg == 1 && kt == u) break;  // odd tile count: the middle tile has no partner
  const int64_t tblk = int64_t(sh) * a.tiles + kt;
  const int k0 = kt * (64 * KB) + wave * (16 * KB);  // first key of this wavefront

  // key and value fragments (operand B: j = key)
  bf16x8 kf[KB][KS], vf[KB][KS];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    const int kr = min(k0 + kb * 16 + lq, S - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[kb][ks] = *reinterpret_cast<const bf16x8*>(Kp + (tok0 + kr) * a.ld + ks * 32 + lh * 8);
      vf[kb][ks] = *reinterpret_cast<const bf16x8*>(Vp + (tok0 + kr) * a.ld + ks * 32 + lh * 8);
    }
  }
  f32x4 dk[KB][DB], dv[KB][DB];
#pragma unroll
  for (int kb = 0; kb < KB; ++kb)
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      dk[kb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
      dv[kb][db] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

  // query tiles this workgroup needs: all, or from the tile that holds its first key on
  const int q_first = a.causal ? (kt * (64 * KB)) / kBKV : 0;
  const int q_tiles = (S + kBKV - 1) / kBKV;
  // The walk is a list of (query head, query tile) units, head-major; part p of n_parts takes an even,
  // contiguous share of it.
  const int nt = max(q_tiles - q_first, 0);
  int heads_here = 0;
  for (int head = 0; head < a.q_cnt; ++head) heads_here += (a.q_off + head) / a.group - a.kv_off == g ? 1 : 0;
  const int units = heads_here * nt;
  const int u_lo = a.n_parts > 1 ? int(int64_t(part) * units / a.n_parts) : 0;
  const int u_hi = a.n_parts > 1 ? int(int64_t(part + 1) * units / a.n_parts) : units;
  int head_idx = 0;
  float rl = 0.f, rd = 0.f;
  for (int head = 0; head < a.q_cnt; ++head) {
    if ((a.q_off + head) / a.group - a.kv_off != g) continue;  // the same for the whole workgroup
    const int u_base = head_idx * nt;
    ++head_idx;
    const int t_lo = q_first + max(u_lo - u_base, 0), t_hi = q_first + min(u_hi - u_base, nt);
    if (t_lo >= t_hi) continue;
    const uint16_t* Qp = a.QKV + int64_t(head) * D;
    const uint16_t* Gp = a.dC + int64_t(head) * D;
    TileSrc<D> srcQ, srcG;
    srcQ.init(Qp + tok0 * a.ld, a.ld, S);
    srcG.init(Gp + tok0 * a.lddc, a.lddc, S);
    auto load_tile = [&](int t) {  // rows past the sequence end arrive as zeros (masked below)
      srcQ.load(t, voffq, rq);
      srcG.load(t, voffg, rg);
      if (threadIdx.x < kBKV) {
        const int row = min(t * kBKV + int(threadIdx.x), S - 1);
        rl = a.LSE[int64_t(head) * Mtot + tok0 + row] * 1.4426950408889634f;
        rd = a.Delta[int64_t(head) * Mtot + tok0 + row];
      }
    };
    auto store_tile = [&]() {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int c = threadIdx.x + i * kThreads;
        const int o = (c / CPR) * LDT + (c % CPR) * 8;
        *reinterpret_cast<ntp_gemm::u16x8*>(sQ + o) = rq[i];
        *reinterpret_cast<ntp_gemm::u16x8*>(sG + o) = rg[i];
      }
      if (threadIdx.x < kBKV) {
        sL[threadIdx.x] = rl;
        sD[threadIdx.x] = rd;
      }
    };
    load_tile(t_lo);
    for (int t = t_lo; t < t_hi; ++t) {
      __syncthreads();
      store_tile();
      __syncthreads();
      if (t + 1 < t_hi) load_tile(t + 1);
      const int qbase = t * kBKV;
      if (a.causal && qbase + kBKV - 1 < k0) continue;  // every query row of the tile comes before this wavefront's keys
      // S and dP blocks: [query qb*16 + (lane/16)*4 + r][key kb*16 + lane%16]
      f32x4 sc[4][KB], dp[4][KB];
#pragma unroll
      for (int qb = 0; qb < 4; ++qb) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
          sc[qb][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
          dp[qb][kb] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          const bf16x8 qa = *reinterpret_cast<const bf16x8*>(sQ + (qb * 16 + lq) * LDT + ks * 32 + lh * 8);
          const bf16x8 ga = *reinterpret_cast<const bf16x8*>(sG + (qb * 16 + lq) * LDT + ks * 32 + lh * 8);
#pragma unroll
          for (int kb = 0; kb < KB; ++kb) {
            sc[qb][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa, kf[kb][ks], sc[qb][kb], 0, 0, 0);
            dp[qb][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ga, vf[kb][ks], dp[qb][kb], 0, 0, 0);
          }
        }
      }
      // the mask is needed only where the tile reaches past the sequence end, or (causal) where some query
      // row of the tile comes before the wavefront's last key
      const bool edge = qbase + kBKV > S || k0 + 16 * KB > S || (a.causal && qbase < k0 + 16 * KB - 1);
      bf16x8 pf[KB][2], dsf[KB][2];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        const int key = k0 + kb * 16 + lq;
        float p[4][4], ds[4][4];
#pragma unroll
        for (int qb = 0; qb < 4; ++qb) {
          const f32x4 l4 = *reinterpret_cast<const f32x4*>(sL + qb * 16 + lh * 4);
          const f32x4 d4 = *reinterpret_cast<const f32x4*>(sD + qb * 16 + lh * 4);
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            p[qb][r] = fast_exp2(fmaf(sc[qb][kb][r], a.scale_log2, -l4[r]));
            ds[qb][r] = dp[qb][kb][r] - d4[r];
          }
        }
        if (edge) {
#pragma unroll
          for (int qb = 0; qb < 4; ++qb)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const int qrow = qbase + qb * 16 + lh * 4 + r;
              if (qrow >= S || key >= S || (a.causal && key > qrow)) p[qb][r] = 0.f;
            }
        }
#pragma unroll
        for (int qb = 0; qb < 4; ++qb)
#pragma unroll
          for (int r = 0; r < 4; ++r) ds[qb][r] *= p[qb][r];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          bf16x8 f, h;
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            f[r] = static_cast<__bf16>(p[2 * s2][r]);
            f[4 + r] = static_cast<__bf16>(p[2 * s2 + 1][r]);
            h[r] = static_cast<__bf16>(ds[2 * s2][r]);
            h[4 + r] = static_cast<__bf16>(ds[2 * s2 + 1][r]);
          }
          pf[kb][s2] = f;
          dsf[kb][s2] = h;
        }
      }
      // dV^T += dC^T P, dK^T += Q^T dS (query slots in the order the scores sit in the registers)
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const bf16x8 gt = tr_frag(sG, LDT, s2 * 32, db * 16, lq, lh);
          const bf16x8 qt2 = tr_frag(sQ, LDT, s2 * 32, db * 16, lq, lh);
#pragma unroll
          for (int kb = 0; kb < KB; ++kb) {
            dv[kb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gt, pf[kb][s2], dv[kb][db], 0, 0, 0);
            dk[kb][db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qt2, dsf[kb][s2], dk[kb][db], 0, 0, 0);
          }
        }
    }
    __syncthreads();  // the next head's first tile overwrites LDS
  }
  if (a.n_parts > 1) {
    // unscaled fp32 sums of this part: per key a row of [dK | dV]
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
      float* pp = a.part_sums + ((tblk * a.n_parts + part) * (64 * KB) + wave * (16 * KB) + kb * 16 + lq) * (2 * D) + lh * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        *reinterpret_cast<f32x4*>(pp + db * 16) = dk[kb][db];
        *reinterpret_cast<f32x4*>(pp + D + db * 16) = dv[kb][db];
      }
    }
    continue;
  }
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    const int key = k0 + kb * 16 + lq;
    if (key >= S) continue;
    uint16_t* kp = a.dQKV + (tok0 + key) * a.ldd + int64_t(a.q_cnt + g) * D + lh * 4;
    uint16_t* vp = a.dQKV + (tok0 + key) * a.ldd + int64_t(a.q_cnt + a.kv_cnt + g) * D + lh * 4;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      u16x4 ok, ov;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        ok[r] = ntp_gemm::f32_to_bf16(dk[kb][db][r] * a.scale);
        ov[r] = ntp_gemm::f32_to_bf16(dv[kb][db][r]);
      }
      *reinterpret_cast<u16x4*>(kp + db * 16) = ok;
      *reinterpret_cast<u16x4*>(vp + db * 16) = ov;
    }
  }
  }  // the workgroup's passes
}

// The dK / dV kernel with the query and output-gradient tiles brought to LDS by DMA (the layout and the read
// discipline of attn_core_fwd_dma_kernel; head dimension 128, 16 keys per wavefront).  The walk over (query head, query
// tile) units is one stream through the two buffers; the rows' log-sum-exp and delta values go through registers
// into a small LDS array of their own, stored before the tile's barrier.
// (sQG: 4 tiles of LDS, query buffers 0 and 1, then output-gradient buffers 0 and 1; sLD: 4 x 64 floats,
// [buffer][log-sum-exp, delta][row])
template <bool PAIRED>
__device__ __forceinline__ void bwd_dkv_dma_body(const CoreBwdArgs& a, const uint32_t b_launch, const uint32_t total, uint16_t* sQG, float* sLD) {
  const uint32_t bid = xcd_major(b_launch, total);
  constexpr int D = 128, KS = D / 32, DB = D / 16;
  constexpr int TILE = kDmaTile;           // elements of one tile
  constexpr int NI = TILE * 2 / 1024 / 4;  // DMA instructions per wavefront, matrix and tile
  const int part = a.n_parts > 1 ? int(bid % a.n_parts) : 0;
  const int blk = a.n_parts > 1 ? int(bid / a.n_parts) : int(bid);
  const int per_seq = PAIRED ? a.pairs : a.tiles;
  const int u = blk % per_seq;
  const int sh = blk / per_seq;
  const int seq = sh % a.n_seq, g = sh / a.n_seq;  // g: local KV head
  const int S = a.seq_len;
  const int64_t tok0 = int64_t(seq) * S, Mtot = int64_t(a.n_seq) * S;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lq = lane & 15, lh = lane >> 4;
  const uint16_t* Kp = a.QKV + int64_t(a.q_cnt + g) * D;
  const uint16_t* Vp = a.QKV + int64_t(a.q_cnt + a.kv_cnt + g) * D;
  uint32_t voffq[NI], voffg[NI];
#pragma unroll
  for (int j = 0; j < NI; ++j) {
    const int p = (wave * NI + j) * 64 + lane;
    const int row = p >> 4, slot = p & 15;
    const int64_t c8 = int64_t(uint32_t(slot) ^ row_swz(row)) * 8;
    voffq[j] = uint32_t((int64_t(row) * a.ld + c8) * 2);
    voffg[j] = uint32_t((int64_t(row) * a.lddc + c8) * 2);
  }
  uint32_t ak[KS], at[DB], al;  // read addresses in query buffer 0 and in the first log-sum-exp row
  {
    const uint32_t base = uint32_t(reinterpret_cast<uintptr_t>(sQG));
    const uint32_t xk = row_swz(lq);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) ak[ks] = base + uint32_t(lq) * 256u + ((uint32_t(ks * 4 + lh) ^ xk) * 16u);
    const int rv = lh * 4 + (lq >> 2);
    const uint32_t xv = row_swz(rv);
#pragma unroll
    for (int db = 0; db < DB; ++db)
      at[db] = base + uint32_t(rv) * 256u + uint32_t(lq & 1) * 8u + ((uint32_t(db * 2 + ((lq & 3) >> 1)) ^ xv) * 16u);
    al = uint32_t(reinterpret_cast<uintptr_t>(sLD)) + uint32_t(lh) * 16u;
  }
  // the local query heads that read this KV head are consecutive
  int head_first = 0, heads_here = 0;
  for (int head = a.q_cnt - 1; head >= 0; --head)
    if ((a.q_off + head) / a.group - a.kv_off == g) {
      head_first = head;
      ++heads_here;
    }

  for (int seg = 0; seg < (PAIRED ? 2 : 1); ++seg) {
  const int kt = PAIRED && seg == 1 ? a.tiles - 1 - u : u;
  if (seg == 1) {
    if (kt == u) break;  // odd tile count: the middle tile has no partner
    __syncthreads();     // the first pass's last tile has been read by everyone
  }
  const int64_t tblk = int64_t(sh) * a.tiles + kt;
  const int k0 = kt * 64 + wave * 16;  // first key of this wavefront

  bf16x8 kf[KS], vf[KS];  // key and value fragments (operand B: j = key)
  {
    const int kr = min(k0 + lq, S - 1);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8*>(Kp + (tok0 + kr) * a.ld + ks * 32 + lh * 8);
      vf[ks] = *reinterpret_cast<const bf16x8*>(Vp + (tok0 + kr) * a.ld + ks * 32 + lh * 8);
    }
  }
  f32x4 dk[DB], dv[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    dk[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    dv[db] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  // query tiles this workgroup needs: all, or from the tile that holds its first key on; the walk is the list of
  // (query head, query tile) units, head-major, and part p of n_parts takes an even, contiguous share of it
  const int q_first = a.causal ? (kt * 64) / kBKV : 0;
  const int q_tiles = (S + kBKV - 1) / kBKV;
  const int nt = max(q_tiles - q_first, 0);
  const int units = heads_here * nt;
  const int u_lo = a.n_parts > 1 ? int(int64_t(part) * units / a.n_parts) : 0;
  const int u_hi = a.n_parts > 1 ? int(int64_t(part + 1) * units / a.n_parts) : units;

  float rl = 0.f, rd = 0.f;
  // unit w: DMA of its two tiles into buffer `buf`, and this thread's log-sum-exp / delta value of it into registers
  auto fetch_unit = [&](int head, int t, int buf) {
    TileSrc<D> srcQ, srcG;  // rows past the sequence end lie outside the views: zeros
    srcQ.init(a.QKV + int64_t(head) * D + tok0 * a.ld, a.ld, S);
    srcG.init(a.dC + int64_t(head) * D + tok0 * a.lddc, a.lddc, S);
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      dma_16(srcQ.rs, sQG + buf * TILE + (wave * NI + j) * 512, voffq[j], uint32_t(t) * srcQ.step);
      dma_16(srcG.rs, sQG + (2 + buf) * TILE + (wave * NI + j) * 512, voffg[j], uint32_t(t) * srcG.step);
    }
    if (threadIdx.x < kBKV) {  // (buffer loads as well: scalar base, rows past the sequence end read as zeros)
      const __amdgpu_buffer_rsrc_t rsL = __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.LSE + int64_t(head) * Mtot + tok0), 0, S * 4, 0x00020000);
      const __amdgpu_buffer_rsrc_t rsD = __builtin_amdgcn_make_buffer_rsrc(a.Delta + int64_t(head) * Mtot + tok0, 0, S * 4, 0x00020000);
      // (used, and scaled, only when the next step stores it: arithmetic here would wait for the DMA issued above)
      rl = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsL, threadIdx.x * 4u, uint32_t(t) * (kBKV * 4), 0));
      rd = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsD, threadIdx.x * 4u, uint32_t(t) * (kBKV * 4), 0));
    }
  };

  // one unit out of buffer BUF (a compile-time constant, so that every LDS offset is an immediate)
  auto tile_step = [&](auto bufc, int t, bool more, int head_next, int t_next) {
    constexpr int BUF = decltype(bufc)::value;
    constexpr int QO = BUF * TILE * 2, GO = (2 + BUF) * TILE * 2, LO = BUF * 2 * kBKV * 4;  // byte offsets
    dma_done();  // this wavefront's share of the unit has landed (and rl, rd have arrived) ...
    if (threadIdx.x < kBKV) {
      sLD[BUF * 2 * kBKV + threadIdx.x] = rl * 1.4426950408889634f;
      sLD[BUF * 2 * kBKV + kBKV + threadIdx.x] = rd;
    }
    __syncthreads();  // ... and everyone's; everyone has finished reading the unit before in the other buffers
    if (more) fetch_unit(head_next, t_next, BUF ^ 1);
    const int qbase = t * kBKV;
    if (a.causal && qbase + kBKV - 1 < k0) return;  // every query row of the tile comes before this wavefront's keys
    // S and dP blocks: [query qb*16 + (lane/16)*4 + r][key lane%16]; query blocks 0-1 first, 2-3 behind them
    attn_u32x4 q01[8], g01[8], q23[8], g23[8];  // [(qb % 2) * 4 + ks]
    q01[0] = lds_frag_b128<QO + 0 * 4096>(ak[0]);
    q01[1] = lds_frag_b128<QO + 0 * 4096>(ak[1]);
    q01[2] = lds_frag_b128<QO + 0 * 4096>(ak[2]);
    q01[3] = lds_frag_b128<QO + 0 * 4096>(ak[3]);
    q01[4] = lds_frag_b128<QO + 1 * 4096>(ak[0]);
    q01[5] = lds_frag_b128<QO + 1 * 4096>(ak[1]);
    q01[6] = lds_frag_b128<QO + 1 * 4096>(ak[2]);
    q01[7] = lds_frag_b128<QO + 1 * 4096>(ak[3]);
    g01[0] = lds_frag_b128<GO + 0 * 4096>(ak[0]);
    g01[1] = lds_frag_b128<GO + 0 * 4096>(ak[1]);
    g01[2] = lds_frag_b128<GO + 0 * 4096>(ak[2]);
    g01[3] = lds_frag_b128<GO + 0 * 4096>(ak[3]);
    g01[4] = lds_frag_b128<GO + 1 * 4096>(ak[0]);
    g01[5] = lds_frag_b128<GO + 1 * 4096>(ak[1]);
    g01[6] = lds_frag_b128<GO + 1 * 4096>(ak[2]);
    g01[7] = lds_frag_b128<GO + 1 * 4096>(ak[3]);
    lds_reads_done(q01);
    lds_reads_tied(g01);
    q23[0] = lds_frag_b128<QO + 2 * 4096>(ak[0]);
    q23[1] = lds_frag_b128<QO + 2 * 4096>(ak[1]);
    q23[2] = lds_frag_b128<QO + 2 * 4096>(ak[2]);
    q23[3] = lds_frag_b128<QO + 2 * 4096>(ak[3]);
    q23[4] = lds_frag_b128<QO + 3 * 4096>(ak[0]);
    q23[5] = lds_frag_b128<QO + 3 * 4096>(ak[1]);
    q23[6] = lds_frag_b128<QO + 3 * 4096>(ak[2]);
    q23[7] = lds_frag_b128<QO + 3 * 4096>(ak[3]);
    f32x4 sc[4], dp[4];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      sc[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
      dp[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        sc[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, q01[qb * 4 + ks]), kf[ks], sc[qb], 0, 0, 0);
        dp[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, g01[qb * 4 + ks]), vf[ks], dp[qb], 0, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    g23[0] = lds_frag_b128<GO + 2 * 4096>(ak[0]);
    g23[1] = lds_frag_b128<GO + 2 * 4096>(ak[1]);
    g23[2] = lds_frag_b128<GO + 2 * 4096>(ak[2]);
    g23[3] = lds_frag_b128<GO + 2 * 4096>(ak[3]);
    g23[4] = lds_frag_b128<GO + 3 * 4096>(ak[0]);
    g23[5] = lds_frag_b128<GO + 3 * 4096>(ak[1]);
    g23[6] = lds_frag_b128<GO + 3 * 4096>(ak[2]);
    g23[7] = lds_frag_b128<GO + 3 * 4096>(ak[3]);
    lds_reads_left<8>(q23);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      sc[2 + qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        sc[2 + qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, q23[qb * 4 + ks]), kf[ks], sc[2 + qb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    // the rows' log-sum-exp and delta values ([0..3]: log-sum-exp of query block qb, [4..7]: delta), then the
    // transposed output-gradient fragments of the dV product: needed after the arithmetic on the scores
    attn_u32x4 ld8[8];
    ld8[0] = lds_frag_b128<LO + 0>(al);
    ld8[1] = lds_frag_b128<LO + 64>(al);
    ld8[2] = lds_frag_b128<LO + 128>(al);
    ld8[3] = lds_frag_b128<LO + 192>(al);
    ld8[4] = lds_frag_b128<LO + 256>(al);
    ld8[5] = lds_frag_b128<LO + 320>(al);
    ld8[6] = lds_frag_b128<LO + 384>(al);
    ld8[7] = lds_frag_b128<LO + 448>(al);
    lds_reads_left<8>(g23);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      dp[2 + qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < KS; ++ks)
        dp[2 + qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, g23[qb * 4 + ks]), vf[ks], dp[2 + qb], 0, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    lds_reads_done(ld8);
    // transposed fragments of the last two products, 8 reads (one pair of 16-column blocks) per group: two groups of
    // the output gradient are requested now and land under the arithmetic on the scores
    attn_u32x2 gt[4][8], qt[4][8];  // [db / 2][(db % 2) * 4 + s2 * 2 + half]: query rows s2*32 + half*16 .. of the tile
    gt[0][0] = lds_tr_b64<GO + 0>(at[0]); gt[0][1] = lds_tr_b64<GO + 4096>(at[0]); gt[0][2] = lds_tr_b64<GO + 8192>(at[0]); gt[0][3] = lds_tr_b64<GO + 12288>(at[0]);
    gt[0][4] = lds_tr_b64<GO + 0>(at[1]); gt[0][5] = lds_tr_b64<GO + 4096>(at[1]); gt[0][6] = lds_tr_b64<GO + 8192>(at[1]); gt[0][7] = lds_tr_b64<GO + 12288>(at[1]);
    gt[1][0] = lds_tr_b64<GO + 0>(at[2]); gt[1][1] = lds_tr_b64<GO + 4096>(at[2]); gt[1][2] = lds_tr_b64<GO + 8192>(at[2]); gt[1][3] = lds_tr_b64<GO + 12288>(at[2]);
    gt[1][4] = lds_tr_b64<GO + 0>(at[3]); gt[1][5] = lds_tr_b64<GO + 4096>(at[3]); gt[1][6] = lds_tr_b64<GO + 8192>(at[3]); gt[1][7] = lds_tr_b64<GO + 12288>(at[3]);

    // the mask is needed only where the tile reaches past the sequence end, or (causal) where some query
    // row of the tile comes before the wavefront's last key
    const bool edge = qbase + kBKV > S || k0 + 16 > S || (a.causal && qbase < k0 + 15);
    const int key = k0 + lq;
    float p[4][4], ds[4][4];
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
      const f32x4 l4 = __builtin_bit_cast(f32x4, ld8[qb]);
      const f32x4 d4 = __builtin_bit_cast(f32x4, ld8[4 + qb]);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        p[qb][r] = fast_exp2(fmaf(sc[qb][r], a.scale_log2, -l4[r]));
        ds[qb][r] = dp[qb][r] - d4[r];
      }
    }
    if (edge) {
#pragma unroll
      for (int qb = 0; qb < 4; ++qb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int qrow = qbase + qb * 16 + lh * 4 + r;
          if (qrow >= S || key >= S || (a.causal && key > qrow)) p[qb][r] = 0.f;
        }
    }
#pragma unroll
    for (int qb = 0; qb < 4; ++qb)
#pragma unroll
      for (int r = 0; r < 4; ++r) ds[qb][r] *= p[qb][r];
    bf16x8 pf[2], dsf[2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      bf16x8 f, h;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        f[r] = static_cast<__bf16>(p[2 * s2][r]);
        f[4 + r] = static_cast<__bf16>(p[2 * s2 + 1][r]);
        h[r] = static_cast<__bf16>(ds[2 * s2][r]);
        h[4 + r] = static_cast<__bf16>(ds[2 * s2 + 1][r]);
      }
      pf[s2] = f;
      dsf[s2] = h;
    }
    // dV^T += dC^T P, dK^T += Q^T dS (query slots in the order the scores sit in the registers); every group of
    // reads lands under the matrix instructions of the groups before it
    lds_reads_done(gt[0]);
    lds_reads_tied(gt[1]);
    __builtin_amdgcn_sched_barrier(0);
    gt[2][0] = lds_tr_b64<GO + 0>(at[4]); gt[2][1] = lds_tr_b64<GO + 4096>(at[4]); gt[2][2] = lds_tr_b64<GO + 8192>(at[4]); gt[2][3] = lds_tr_b64<GO + 12288>(at[4]);
    gt[2][4] = lds_tr_b64<GO + 0>(at[5]); gt[2][5] = lds_tr_b64<GO + 4096>(at[5]); gt[2][6] = lds_tr_b64<GO + 8192>(at[5]); gt[2][7] = lds_tr_b64<GO + 12288>(at[5]);
    gt[3][0] = lds_tr_b64<GO + 0>(at[6]); gt[3][1] = lds_tr_b64<GO + 4096>(at[6]); gt[3][2] = lds_tr_b64<GO + 8192>(at[6]); gt[3][3] = lds_tr_b64<GO + 12288>(at[6]);
    gt[3][4] = lds_tr_b64<GO + 0>(at[7]); gt[3][5] = lds_tr_b64<GO + 4096>(at[7]); gt[3][6] = lds_tr_b64<GO + 8192>(at[7]); gt[3][7] = lds_tr_b64<GO + 12288>(at[7]);
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = gt[0][(db & 1) * 4 + s2 * 2], hi = gt[0][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        dv[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pf[s2], dv[db], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int db = 2; db < 4; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = gt[1][(db & 1) * 4 + s2 * 2], hi = gt[1][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        dv[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pf[s2], dv[db], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
    qt[0][0] = lds_tr_b64<QO + 0>(at[0]); qt[0][1] = lds_tr_b64<QO + 4096>(at[0]); qt[0][2] = lds_tr_b64<QO + 8192>(at[0]); qt[0][3] = lds_tr_b64<QO + 12288>(at[0]);
    qt[0][4] = lds_tr_b64<QO + 0>(at[1]); qt[0][5] = lds_tr_b64<QO + 4096>(at[1]); qt[0][6] = lds_tr_b64<QO + 8192>(at[1]); qt[0][7] = lds_tr_b64<QO + 12288>(at[1]);
    lds_reads_left<8>(gt[2]);
    lds_reads_tied(gt[3]);
#pragma unroll
    for (int db = 4; db < 6; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = gt[2][(db & 1) * 4 + s2 * 2], hi = gt[2][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        dv[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pf[s2], dv[db], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int db = 6; db < 8; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = gt[3][(db & 1) * 4 + s2 * 2], hi = gt[3][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        dv[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), pf[s2], dv[db], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
    qt[1][0] = lds_tr_b64<QO + 0>(at[2]); qt[1][1] = lds_tr_b64<QO + 4096>(at[2]); qt[1][2] = lds_tr_b64<QO + 8192>(at[2]); qt[1][3] = lds_tr_b64<QO + 12288>(at[2]);
    qt[1][4] = lds_tr_b64<QO + 0>(at[3]); qt[1][5] = lds_tr_b64<QO + 4096>(at[3]); qt[1][6] = lds_tr_b64<QO + 8192>(at[3]); qt[1][7] = lds_tr_b64<QO + 12288>(at[3]);
    lds_reads_left<8>(qt[0]);
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = qt[0][(db & 1) * 4 + s2 * 2], hi = qt[0][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        dk[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), dsf[s2], dk[db], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
    qt[2][0] = lds_tr_b64<QO + 0>(at[4]); qt[2][1] = lds_tr_b64<QO + 4096>(at[4]); qt[2][2] = lds_tr_b64<QO + 8192>(at[4]); qt[2][3] = lds_tr_b64<QO + 12288>(at[4]);
    qt[2][4] = lds_tr_b64<QO + 0>(at[5]); qt[2][5] = lds_tr_b64<QO + 4096>(at[5]); qt[2][6] = lds_tr_b64<QO + 8192>(at[5]); qt[2][7] = lds_tr_b64<QO + 12288>(at[5]);
    lds_reads_left<8>(qt[1]);
#pragma unroll
    for (int db = 2; db < 4; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = qt[1][(db & 1) * 4 + s2 * 2], hi = qt[1][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        dk[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), dsf[s2], dk[db], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
    qt[3][0] = lds_tr_b64<QO + 0>(at[6]); qt[3][1] = lds_tr_b64<QO + 4096>(at[6]); qt[3][2] = lds_tr_b64<QO + 8192>(at[6]); qt[3][3] = lds_tr_b64<QO + 12288>(at[6]);
    qt[3][4] = lds_tr_b64<QO + 0>(at[7]); qt[3][5] = lds_tr_b64<QO + 4096>(at[7]); qt[3][6] = lds_tr_b64<QO + 8192>(at[7]); qt[3][7] = lds_tr_b64<QO + 12288>(at[7]);
    lds_reads_left<8>(qt[2]);
#pragma unroll
    for (int db = 4; db < 6; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = qt[2][(db & 1) * 4 + s2 * 2], hi = qt[2][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        dk[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), dsf[s2], dk[db], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
    lds_reads_done(qt[3]);
#pragma unroll
    for (int db = 6; db < 8; ++db)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const attn_u32x2 lo = qt[3][(db & 1) * 4 + s2 * 2], hi = qt[3][(db & 1) * 4 + s2 * 2 + 1];
        const attn_u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
        dk[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, both), dsf[s2], dk[db], 0, 0, 0);
      }
    __builtin_amdgcn_sched_barrier(0);
  };

  if (u_lo < u_hi) {
    // (head, tile) of the unit in hand and of the next one
    int head = head_first + u_lo / nt, t = q_first + u_lo % nt;
    fetch_unit(head, t, 0);
    for (int w = u_lo; w < u_hi; w += 2) {
      int hn = t + 1 < q_tiles ? head : head + 1, tn = t + 1 < q_tiles ? t + 1 : q_first;
      tile_step(std::integral_constant<int, 0>{}, t, w + 1 < u_hi, hn, tn);
      head = hn;
      t = tn;
      if (w + 1 < u_hi) {
        hn = t + 1 < q_tiles ? head : head + 1;
        tn = t + 1 < q_tiles ? t + 1 : q_first;
        tile_step(std::integral_constant<int, 1>{}, t, w + 2 < u_hi, hn, tn);
        head = hn;
        t = tn;
      }
    }
  }

  if (a.n_parts > 1) {
    // unscaled fp32 sums of this part: per key a row of [dK | dV]
    float* pp = a.part_sums + ((tblk * a.n_parts + part) * 64 + wave * 16 + lq) * (2 * D) + lh * 4;
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      *reinterpret_cast<f32x4*>(pp + db * 16) = dk[db];
      *reinterpret_cast<f32x4*>(pp + D + db * 16) = dv[db];
    }
    continue;
  }
  {
    const int key = k0 + lq;
    if (key < S) {
      uint16_t* kp = a.dQKV + (tok0 + key) * a.ldd + int64_t(a.q_cnt + g) * D + lh * 4;
      uint16_t* vp = a.dQKV + (tok0 + key) * a.ldd + int64_t(a.q_cnt + a.kv_cnt + g) * D + lh * 4;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        u16x4 ok, ov;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          ok[r] = ntp_gemm::f32_to_bf16(dk[db][r] * a.scale);
          ov[r] = ntp_gemm::f32_to_bf16(dv[db][r]);
        }
        *reinterpret_cast<u16x4*>(kp + db * 16) = ok;
        *reinterpret_cast<u16x4*>(vp + db * 16) = ov;
      }
    }
  }
  }  // the workgroup's passes
}

template <bool PAIRED>
__global__ __attribute__((amdgpu_flat_work_group_size(kThreads, kThreads), amdgpu_waves_per_eu(2, 2))) void
attn_core_bwd_dq_dma_kernel(const CoreBwdArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t tiles[4 * kDmaTile];
  bwd_dq_dma_body<PAIRED>(a, blockIdx.x, gridDim.x, tiles);
}

template <bool PAIRED>
__global__ __launch_bounds__(kThreads, 2) void attn_core_bwd_dkv_dma_kernel(const CoreBwdArgs a) {
  __shared__ __attribute__((aligned(1024))) uint16_t tiles[4 * kDmaTile];
  __shared__ __attribute__((aligned(16))) float row_values[2 * 2 * kBKV];
  bwd_dkv_dma_body<PAIRED>(a, blockIdx.x, gridDim.x, tiles, row_values);
}

// Both backward kernels in one launch: the first n_dkv workgroups are dK/dV workgroups, the rest dQ workgroups.
// Each kernel alone keeps the matrix pipe and the vector ALU busy in turn; at the launch sizes of a few heads
// and a few thousand tokens either leaves most SIMDs with one wavefront, and nothing overlaps.  Launched together a
// compute unit holds one workgroup of each kind (65 KB + 64 KB of LDS), whose phases differ (14 heads x 2048
// tokens, causal: 50 + 60 us one after the other, 76 us together).  The dK/dV workgroups need every row's delta
// before they start, so a small kernel stores those first (attn_core_delta_kernel).
// Order of the workgroups: a compute unit holds two of them, and the kinds should meet there.  Measured, a launch of
// 224 dK/dV workgroups followed by 224 dQ workgroups behaves like the two kernels on two streams (workgroups are
// spread one per compute unit before any gets its second), while kinds that alternate every 8 workgroups ran 8 %
// slower.  So the kinds alternate in chunks of `chunk` = compute units workgroups, dK/dV first, over the first
// 2 `paired` workgroups (paired: a multiple of chunk, at most either kind's count); the rest of the dK/dV
// workgroups and then the rest of the dQ workgroups follow.
struct BothOrder {
  uint32_t n_dkv, paired, chunk;
};

template <bool PAIRED>
__global__ __launch_bounds__(kThreads, 2) void attn_core_bwd_both_kernel(const CoreBwdArgs adq, const CoreBwdArgs adkv, const BothOrder o) {
  __shared__ __attribute__((aligned(1024))) uint16_t tiles[4 * kDmaTile];
  __shared__ __attribute__((aligned(16))) float row_values[2 * 2 * kBKV];
  uint32_t b = blockIdx.x;
  bool dkv;
  if (b < 2 * o.paired) {
    const uint32_t c = b / o.chunk;
    dkv = (c & 1) == 0;
    b = (c >> 1) * o.chunk + b % o.chunk;
  } else {
    b -= 2 * o.paired;
    dkv = b < o.n_dkv - o.paired;
    b = dkv ? o.paired + b : o.paired + b - (o.n_dkv - o.paired);
  }
  // (each kind renumbered by itself: its workgroups with equal b % 8 share an XCD whatever the other kind's count)
  if (dkv) bwd_dkv_dma_body<PAIRED>(adkv, b, o.n_dkv, tiles, row_values);
  else bwd_dq_dma_body<PAIRED>(adq, b, gridDim.x - o.n_dkv, tiles);
}

// delta[head][row] = sum_d dC[row][head D + d] C[row][head D + d]: 16 lanes per (row, head), 8 values each
template <int D>
__global__ __launch_bounds__(256) void attn_core_delta_kernel(const CoreBwdArgs a, int64_t rows) {
  constexpr int LPR = D / 8;  // lanes per (row, head): 16 or 8
  const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int c = int(idx % LPR);
  const int64_t rh = idx / LPR;
  const int head = int(rh % a.q_cnt);
  const int64_t row = rh / a.q_cnt;
  float part = 0.f;
  if (row < rows) {
    const bf16x8 g = *reinterpret_cast<const bf16x8*>(a.dC + row * a.lddc + int64_t(head) * D + c * 8);
    const bf16x8 o = *reinterpret_cast<const bf16x8*>(a.C + row * a.ldc + int64_t(head) * D + c * 8);
#pragma unroll
    for (int e = 0; e < 8; ++e) part += float(g[e]) * float(o[e]);
  }
#pragma unroll
  for (int m = LPR / 2; m >= 1; m >>= 1) part += __shfl_xor(part, m);
  if (c == 0 && row < rows) a.Delta[int64_t(head) * rows + row] = part;
}

// Adds the parts of a cut walk and stores the gradient as bf16.  `rows` rows per workgroup of the cut
// kernel, `width` fp32 values per row: D (dQ) or 2 D ([dK | dV]).  One thread per 4 values.
template <int D, bool DKV>
__global__ __launch_bounds__(256) void attn_core_part_reduce_kernel(const CoreBwdArgs a, int64_t n_blk) {
  constexpr int W = DKV ? 2 * D : D, Q = W / 4;
  const int64_t idx = int64_t(blockIdx.x) * 256 + threadIdx.x;
  const int c = int(idx % Q) * 4, row = int((idx / Q) % 64);
  const int64_t blk = idx / (Q * 64);
  if (blk >= n_blk) return;
  const int tile = DKV || !a.causal ? int(blk % a.tiles) : a.tiles - 1 - int(blk % a.tiles);
  const int64_t sh = blk / a.tiles;
  const int seq = int(sh % a.n_seq), hd = int(sh / a.n_seq);  // local KV head (dK, dV) or query head (dQ)
  const int tok = tile * 64 + row;
  if (tok >= a.seq_len) return;
  const float* p = a.part_sums + (blk * a.n_parts * 64 + row) * W + c;
  f32x4 sum = *reinterpret_cast<const f32x4*>(p);
  for (int part = 1; part < a.n_parts; ++part) sum = sum + *reinterpret_cast<const f32x4*>(p + int64_t(part) * 64 * W);
  const bool is_v = DKV && c >= D;
  const int col = is_v ? c - D : c;
  const int64_t slot = DKV ? int64_t(a.q_cnt) + (is_v ? a.kv_cnt : 0) + hd : hd;
  const float f = is_v ? 1.0f : a.scale;
  u16x4 o;
#pragma unroll
  for (int r = 0; r < 4; ++r) o[r] = ntp_gemm::f32_to_bf16(sum[r] * f);
  *reinterpret_cast<u16x4*>(a.dQKV + (int64_t(seq) * a.seq_len + tok) * a.ldd + slot * D + col) = o;
}

// Parts to cut each workgroup's walk into.  wgs: workgroups the launch has uncut; walk: key (or query) tiles each
// walks over; slots x parts x bytes_per_part must fit ws_bytes (no workspace: no cut).  Measured on 2 to 14 heads x
// 2048 to 8192 tokens: the best count brings the launch to fill x compute units workgroups (fill = 2 under the causal
// mask, where paired tiles make all walks equal, and for the dK/dV kernel; 3 for the unmasked forward and dQ
// kernels), as long as a part keeps at least 6 tiles; launches that already have more workgroups than compute units
// gain only from parts of more than 16 tiles (the merge pass and the per-workgroup prologue cost more than shorter
// parts gain); a causal walk of 40 tiles or more per part takes one part more.
int choose_parts(const ntp_handle* h, int64_t ws_bytes, int64_t wgs, int64_t slots, int64_t walk, int64_t bytes_per_part, double fill,
                 int64_t cap, bool causal) {
  if (ws_bytes <= 0 || wgs <= 0) return 1;
  const int64_t cus = h->compute_units;
  int64_t parts = std::min<int64_t>(cap, std::max<int64_t>(1, int64_t(fill * double(cus) / double(wgs) + 0.5)));
  parts = std::min<int64_t>(parts, std::max<int64_t>(1, walk / 6));
  if (wgs > cus)
    while (parts > 1 && walk / parts <= 16) --parts;
  if (causal && parts < cap && walk / parts >= 40 && wgs * parts < 3 * cus) ++parts;
  // tests reach every cut through this override (1..16 parts at any size)
  if (const int64_t f = h->opt[NTP_OPT_ATTN_PARTS]) parts = std::min<int64_t>(16, std::max<int64_t>(1, f));
  while (parts > 1 && slots * parts * bytes_per_part > ws_bytes) --parts;
  return int(std::max<int64_t>(parts, 1));
}

// The same for the kernels that copy by DMA (two workgroups of 64-65 KB LDS per compute unit), from a sweep over 2 to
// 32 heads x 1024 to 8192 tokens, both masks, 1-8 parts, one and two backward launches: the walk is cut until the
// launch has `slots` workgroups (forward: two per compute unit; dQ and dK/dV: one per compute unit each, they share a
// launch), never into parts of fewer than 8 tiles, and into parts of fewer than `long_part` tiles only while the
// launch still leaves compute units idle (fewer than `idle` workgroups): short parts cost their second pass and
// their prologues, and once every compute unit has work they no longer buy anything.
int choose_parts_dma(const ntp_handle* h, int64_t ws_bytes, int64_t wgs, int64_t slots_ws, int64_t walk, int64_t bytes_per_part,
                     int64_t slots, int64_t long_part, int64_t idle) {
  if (ws_bytes <= 0 || wgs <= 0) return 1;
  const int64_t pmax = std::min<int64_t>(16, std::max<int64_t>(1, slots / wgs));
  int64_t parts = 1;
  while (parts + 1 <= pmax && walk / (parts + 1) >= 8 && (walk / (parts + 1) >= long_part || wgs * parts < idle)) ++parts;
  // tests reach every cut through this override (1..16 parts at any size)
  if (const int64_t f = h->opt[NTP_OPT_ATTN_PARTS]) parts = std::min<int64_t>(16, std::max<int64_t>(1, f));
  while (parts > 1 && slots_ws * parts * bytes_per_part > ws_bytes) --parts;
  return int(std::max<int64_t>(parts, 1));
}

// Launch decisions of the three kernels for a (checked) shape.
struct CoreChoice {
  int fwd_rows;  // query rows per wavefront of the forward kernel: 16 or 32
  int fwd_parts, dq_parts, dkv_parts;
  int64_t ws_bytes;  // workspace bytes the cut launches use (the largest of the three)
  bool dq_dma, dkv_dma;  // the dQ / the dK, dV kernel brings its tiles to LDS by DMA
  bool bwd_both;         // both backward kernels go out as one launch
  int64_t dkv_ws_offset; // then: byte offset of the dK/dV parts in the workspace (behind the dQ parts)
};
CoreChoice choose_core(const ntp_handle* h, int64_t ws_bytes, const ntp_attn_core_shape_t* s) {
  CoreChoice c{16, 1, 1, 1, 0, false, false, false, 0};
  const bool causal = s->causal != 0;
  const int64_t tiles = (s->seq_len + kBKV - 1) / kBKV;
  // under the causal mask a workgroup takes a pair of tiles, one from each end of the sequence
  const int64_t per_seq = causal ? (tiles + 1) / 2 : tiles, walk = causal ? tiles + 1 : tiles;
  // 16-row query blocks per wavefront: two (twice the matrix work per LDS read, two workgroups per CU), or
  // one (three workgroups per CU, twice as many of them) when two would leave compute units short of work
  // (the same count with and without the mask: the causal pairs make the 128-row tiles' walks equal, 14 heads x
  // 8192 tokens causal 375 -> 309 us with two)
  const int64_t blocks2 = int64_t((s->seq_len + 127) / 128) * s->n_seq * s->q_cnt;
  c.fwd_rows = blocks2 < 1.5 * h->compute_units ? 16 : 32;
  // with few heads even the 64-row workgroups leave compute units idle while each walks over up to
  // seq_len / 64 key tiles: cut the walks then (needs a workspace)
  const int64_t bq = tiles * s->n_seq * s->q_cnt, bk = tiles * s->n_seq * s->kv_cnt;  // tiles: one partial-sum slot each
  const int64_t wq = per_seq * s->n_seq * s->q_cnt, wk = per_seq * s->n_seq * s->kv_cnt;
  const int64_t bf = int64_t(64) * (s->head_dim + 4) * 4, bdq = int64_t(64) * s->head_dim * 4, bdkv = int64_t(64) * 2 * s->head_dim * 4;
  const double fill = causal ? 2.0 : 3.0;
  const bool dma = s->head_dim == 128 && h->opt[NTP_OPT_ATTN_COPY] != 1;
  const int64_t cus = h->compute_units;
  // a dK/dV workgroup walks over the query tiles of every query head that reads its KV head
  const int64_t heads_per_kv = std::min<int64_t>(s->group, s->q_cnt);
  if (dma) {
    // (a launch that occupies 3/4 of the compute units uncut needs parts of 24 tiles to gain from a cut: 14 heads x
    // 2048 tokens causal forward 42 us cut in two, 39 us whole; 8 heads x 2048 unmasked 36 and 33 us)
    c.fwd_parts = choose_parts_dma(h, ws_bytes, wq, bq, walk, bf, 2 * cus, wq * 4 >= cus * 3 ? 24 : 16, cus * 3 / 4);
    c.dq_parts = choose_parts_dma(h, ws_bytes, wq, bq, walk, bdq, cus, 10, cus * 3 / 8);
    c.dkv_parts = choose_parts_dma(h, ws_bytes, wk, bk, heads_per_kv * walk, bdkv, cus, 10, cus * 3 / 8);
  } else {
    c.fwd_parts = choose_parts(h, ws_bytes, wq, bq, walk, bf, fill, 12, causal);
    c.dq_parts = choose_parts(h, ws_bytes, wq, bq, walk, bdq, fill, 12, causal);
    c.dkv_parts = choose_parts(h, ws_bytes, wk, bk, heads_per_kv * walk, bdkv, 2.0, 16, false);
  }
  if (c.fwd_parts > 1) c.fwd_rows = 16;
  c.dq_dma = c.dkv_dma = dma;
  if (c.fwd_parts > 1) c.ws_bytes = std::max(c.ws_bytes, bq * c.fwd_parts * bf);
  const int64_t dq_bytes = c.dq_parts > 1 ? bq * c.dq_parts * bdq : 0, dkv_bytes = c.dkv_parts > 1 ? bk * c.dkv_parts * bdkv : 0;
  // the two DMA kernels share a launch (attn_core_bwd_both_kernel) where the workspace holds both kernels' parts
  // at once; NTP_OPT_ATTN_BWD_LAUNCHES: 1 always two launches, 2 one launch wherever the kernels allow
  c.dkv_ws_offset = (dq_bytes + 255) / 256 * 256;
  // Where it pays (the sweep above): wherever the two launches, uncut, have at most 3 workgroups per compute unit
  // between them (14 heads x 2048 causal: 98 -> 77 us; 8 heads x 4096 causal 175 -> 143; 4 heads x 4096 unmasked
  // 146 -> 122); larger launches fill the device on their own and lose 1-4 % to the extra kernel.
  const bool pays = wq + wk <= 3 * cus;
  c.bwd_both = c.dq_dma && c.dkv_dma && h->opt[NTP_OPT_ATTN_BWD_LAUNCHES] != 1 && (pays || h->opt[NTP_OPT_ATTN_BWD_LAUNCHES] == 2) &&
               (dkv_bytes == 0 || c.dkv_ws_offset + dkv_bytes <= ws_bytes);
  c.ws_bytes = std::max(c.ws_bytes, c.bwd_both ? (dkv_bytes ? c.dkv_ws_offset + dkv_bytes : dq_bytes) : std::max(dq_bytes, dkv_bytes));
  return c;
}

int check_core_shape(const ntp_attn_core_shape_t* s) {
  if (!s || s->n_seq < 0 || s->seq_len < 0 || s->q_cnt < 0 || s->kv_cnt < 0 || s->group < 1 || s->q_off < 0 || s->kv_off < 0)
    return NTP_ERR_INVALID_ARG;
  if (s->head_dim != 64 && s->head_dim != 128) return NTP_ERR_UNSUPPORTED;
  if (int64_t(s->n_seq) * s->seq_len > 0x7fffffffll) return NTP_ERR_UNSUPPORTED;
  // every local query head must read a local KV head
  for (int32_t j = 0; j < s->q_cnt; ++j) {
    const int64_t g = int64_t(s->q_off + j) / s->group - s->kv_off;
    if (g < 0 || g >= s->kv_cnt) return NTP_ERR_INVALID_ARG;
  }
  return NTP_OK;
}

}  // namespace

int ntp::attn_core_workspace_wish(const ntp_handle* h, const ntp_attn_core_shape_t* s, int64_t* bytes) {
  const int st = check_core_shape(s);
  if (st != NTP_OK) return st == NTP_ERR_UNSUPPORTED ? NTP_ERR_INVALID_ARG : st;
  *bytes = choose_core(h, INT64_MAX / 2, s).ws_bytes;
  return NTP_OK;
}

extern "C" int ntp_attn_core_choice(const ntp_handle_t* h, const ntp_attn_core_shape_t* s, ntp_attn_core_choice_t* out) {
  const int st = check_core_shape(s);
  if (st != NTP_OK) return st;
  if (!h || !out) return NTP_ERR_INVALID_ARG;
  const CoreChoice c = choose_core(h, h->workspace ? h->workspace_bytes : 0, s);
  *out = ntp_attn_core_choice_t{c.fwd_rows, c.fwd_parts, c.dq_parts, c.dkv_parts};
  return NTP_OK;
}

extern "C" int ntp_attn_core_shard_fwd(ntp_handle_t* h, const ntp_attn_core_shape_t* s, const void* QKV, int64_t ldqkv,
                                       void* C, int64_t ldc, float* LSE, void* stream) {
  int st = check_core_shape(s);
  if (st != NTP_OK) return st;
  if (!h) return NTP_ERR_INVALID_ARG;
  const int64_t M = int64_t(s->n_seq) * s->seq_len;
  if (M == 0 || s->q_cnt == 0) return NTP_OK;
  if (h->device < 0) return NTP_ERR_NO_DEVICE;
  if (!QKV || !C) return NTP_ERR_INVALID_ARG;
  const int64_t wq = int64_t(s->q_cnt + 2 * s->kv_cnt) * s->head_dim, wo = int64_t(s->q_cnt) * s->head_dim;
  if (ldqkv < wq || ldc < wo) return NTP_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(QKV) & 15) || (reinterpret_cast<uintptr_t>(C) & 15) || ldqkv % 8 || ldc % 8 ||
      (reinterpret_cast<uintptr_t>(LSE) & 3))
    return NTP_ERR_ALIGNMENT;
  // the tile loads address one sequence's rows with 32-bit byte offsets
  if (int64_t(s->seq_len) * ldqkv * 2 > 0x7fffffffll) return NTP_ERR_UNSUPPORTED;
  CoreArgs a{};
  a.QKV = static_cast<const uint16_t*>(QKV);
  a.C = static_cast<uint16_t*>(C);
  a.LSE = LSE;
  a.ld = ldqkv;
  a.ldc = ldc;
  a.n_seq = s->n_seq;
  a.seq_len = s->seq_len;
  a.q_cnt = s->q_cnt;
  a.kv_cnt = s->kv_cnt;
  a.q_off = s->q_off;
  a.kv_off = s->kv_off;
  a.group = s->group;
  a.causal = s->causal ? 1 : 0;
  // 16-row query blocks per wavefront: two (twice the matrix work per LDS read, two workgroups per CU), or
  // one (three workgroups per CU, twice as many of them) when two would leave compute units short of work
  const CoreChoice cc = choose_core(h, h->workspace ? h->workspace_bytes : 0, s);
  const int qbw = cc.fwd_rows / 16;
  a.part_sums = static_cast<float*>(h->workspace);
  a.n_parts = cc.fwd_parts;
  a.q_tiles = (s->seq_len + 64 * qbw - 1) / (64 * qbw);
  a.pairs = s->causal ? (a.q_tiles + 1) / 2 : 0;
  a.scale_log2 = float(1.4426950408889634 / std::sqrt(double(s->head_dim)));
  const int64_t blocks = int64_t(a.q_tiles) * s->n_seq * s->q_cnt;  // query tiles
  const int64_t wgs = int64_t(a.pairs > 0 ? a.pairs : a.q_tiles) * s->n_seq * s->q_cnt;
  if (blocks * std::max(a.n_parts, 1) > 0x7fffffffll) return NTP_ERR_UNSUPPORTED;
  hipStream_t hs = static_cast<hipStream_t>(stream);
  if (ntp::timing_on(h)) {
    char name[48];
    snprintf(name, sizeof(name), "attn_core_fwd%s%s", s->causal ? "_causal" : "", a.n_parts > 1 ? "_cut" : "");
    ntp::timing_begin(h, stream, name,
                      (s->causal ? 2.0 : 4.0) * double(s->n_seq) * double(s->seq_len) * double(s->seq_len) * s->head_dim * s->q_cnt, 0.0);
  }
  const dim3 grid(uint32_t(wgs * std::max(a.n_parts, 1)));
  auto launch = [&](auto d, auto q, auto paired) {
    hipLaunchKernelGGL((attn_core_fwd_kernel<decltype(d)::value, decltype(q)::value, decltype(paired)::value>), grid, dim3(kThreads), 0, hs, a);
  };
  using std::integral_constant;
  auto by_pairing = [&](auto d, auto q) {
    if (a.pairs > 0) launch(d, q, std::true_type{});
    else launch(d, q, std::false_type{});
  };
  const bool by_dma = s->head_dim == 128 && qbw == 1 && h->opt[NTP_OPT_ATTN_COPY] != 1;
  if (by_dma) {
    if (a.pairs > 0) hipLaunchKernelGGL((attn_core_fwd_dma_kernel<true>), grid, dim3(kThreads), 0, hs, a);
    else hipLaunchKernelGGL((attn_core_fwd_dma_kernel<false>), grid, dim3(kThreads), 0, hs, a);
  } else if (s->head_dim == 128 && qbw == 2 && h->opt[NTP_OPT_ATTN_COPY] != 1) {
    if (a.pairs > 0) hipLaunchKernelGGL((attn_core_fwd_dma2_kernel<true>), grid, dim3(kThreads), 0, hs, a);
    else hipLaunchKernelGGL((attn_core_fwd_dma2_kernel<false>), grid, dim3(kThreads), 0, hs, a);
  } else if (s->head_dim == 128 && qbw == 2) by_pairing(integral_constant<int, 128>{}, integral_constant<int, 2>{});
  else if (s->head_dim == 128) by_pairing(integral_constant<int, 128>{}, integral_constant<int, 1>{});
  else if (qbw == 2) by_pairing(integral_constant<int, 64>{}, integral_constant<int, 2>{});
  else by_pairing(integral_constant<int, 64>{}, integral_constant<int, 1>{});
  bool ok = hipGetLastError() == hipSuccess;
  if (ok && a.n_parts > 1) {
    const dim3 rgrid(uint32_t((blocks * 64 * (s->head_dim / 4) + 255) / 256));
    if (s->head_dim == 128)
      hipLaunchKernelGGL((attn_core_fwd_merge_kernel<128>), rgrid, dim3(256), 0, hs, a, blocks);
    else
      hipLaunchKernelGGL((attn_core_fwd_merge_kernel<64>), rgrid, dim3(256), 0, hs, a, blocks);
    ok = hipGetLastError() == hipSuccess;
  }
  ntp::timing_end(h, stream);
  return ok ? NTP_OK : NTP_ERR_LAUNCH;
}

extern "C" int ntp_attn_core_shard_bwd(ntp_handle_t* h, const ntp_attn_core_shape_t* s, const void* QKV, int64_t ldqkv,
                                       const void* C, int64_t ldc, const void* dC, int64_t lddc, const float* LSE,
                                       float* Delta, void* dQKV, int64_t lddqkv, void* stream) {
  int st = check_core_shape(s);
  if (st != NTP_OK) return st;
  if (!h) return NTP_ERR_INVALID_ARG;
  const int64_t M = int64_t(s->n_seq) * s->seq_len;
  if (M == 0 || (s->q_cnt == 0 && s->kv_cnt == 0)) return NTP_OK;
  if (h->device < 0) return NTP_ERR_NO_DEVICE;
  if (!QKV || !dQKV || (s->q_cnt > 0 && (!C || !dC || !LSE || !Delta))) return NTP_ERR_INVALID_ARG;
  const int64_t wq = int64_t(s->q_cnt + 2 * s->kv_cnt) * s->head_dim, wo = int64_t(s->q_cnt) * s->head_dim;
  if (ldqkv < wq || lddqkv < wq || ldc < wo || lddc < wo) return NTP_ERR_INVALID_ARG;
  auto mis = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; };
  if (mis(QKV) || mis(dQKV) || mis(C) || mis(dC) || ldqkv % 8 || lddqkv % 8 || ldc % 8 || lddc % 8 ||
      (reinterpret_cast<uintptr_t>(LSE) & 3) || (reinterpret_cast<uintptr_t>(Delta) & 3))
    return NTP_ERR_ALIGNMENT;
  if (int64_t(s->seq_len) * std::max(ldqkv, lddc) * 2 > 0x7fffffffll) return NTP_ERR_UNSUPPORTED;
  CoreBwdArgs a{};
  a.QKV = static_cast<const uint16_t*>(QKV);
  a.C = static_cast<const uint16_t*>(C);
  a.dC = static_cast<const uint16_t*>(dC);
  a.LSE = LSE;
  a.Delta = Delta;
  a.dQKV = static_cast<uint16_t*>(dQKV);
  a.ld = ldqkv;
  a.ldc = ldc;
  a.lddc = lddc;
  a.ldd = lddqkv;
  a.n_seq = s->n_seq;
  a.seq_len = s->seq_len;
  a.q_cnt = s->q_cnt;
  a.kv_cnt = s->kv_cnt;
  a.q_off = s->q_off;
  a.kv_off = s->kv_off;
  a.group = s->group;
  a.causal = s->causal ? 1 : 0;
  // the dQ kernel with 16 query rows per wavefront (three workgroups per CU, no register spills) measured
  // faster than with 32 at almost every size: only that variant is built
  constexpr int qbw = 1;
  a.tiles = (s->seq_len + 64 * qbw - 1) / (64 * qbw);
  constexpr int kb = 1;  // 64 keys per workgroup of the dK/dV kernel
  const int32_t key_tiles = (s->seq_len + 64 * kb - 1) / (64 * kb);
  a.scale = float(1.0 / std::sqrt(double(s->head_dim)));
  a.scale_log2 = float(1.4426950408889634 / std::sqrt(double(s->head_dim)));
  hipStream_t hs = static_cast<hipStream_t>(stream);
  const double pair_flops = (s->causal ? 1.0 : 2.0) * double(s->n_seq) * double(s->seq_len) * double(s->seq_len) * s->head_dim * s->q_cnt;
  bool ok = true;
  const int64_t bq = int64_t(a.tiles) * s->n_seq * s->q_cnt, bk = int64_t(key_tiles) * s->n_seq * s->kv_cnt;
  if (bq > 0x7fffffffll || bk > 0x7fffffffll) return NTP_ERR_UNSUPPORTED;
  a.part_sums = static_cast<float*>(h->workspace);
  const CoreChoice cc = choose_core(h, h->workspace ? h->workspace_bytes : 0, s);
  const int32_t q_pairs = s->causal ? (a.tiles + 1) / 2 : 0, k_pairs = s->causal ? (key_tiles + 1) / 2 : 0;
  const int64_t dq_wgs = int64_t(q_pairs > 0 ? q_pairs : a.tiles) * s->n_seq * s->q_cnt * cc.dq_parts;
  const int64_t dkv_wgs = int64_t(k_pairs > 0 ? k_pairs : key_tiles) * s->n_seq * s->kv_cnt * cc.dkv_parts;
  auto reduce_parts = [&](auto dkv, int64_t blocks) {
    constexpr bool DKV = decltype(dkv)::value;
    const dim3 rgrid(uint32_t((blocks * 64 * ((DKV ? 2 : 1) * s->head_dim / 4) + 255) / 256));
    if (s->head_dim == 128)
      hipLaunchKernelGGL((attn_core_part_reduce_kernel<128, DKV>), rgrid, dim3(256), 0, hs, a, blocks);
    else
      hipLaunchKernelGGL((attn_core_part_reduce_kernel<64, DKV>), rgrid, dim3(256), 0, hs, a, blocks);
    return hipGetLastError() == hipSuccess;
  };
  const int64_t delta_wgs = (M * s->q_cnt * 16 + 255) / 256;
  if (dq_wgs > 0x7fffffffll || dkv_wgs > 0x7fffffffll) return NTP_ERR_UNSUPPORTED;
  if (cc.bwd_both && bq > 0 && bk > 0 && dq_wgs + dkv_wgs <= 0x7fffffffll && delta_wgs <= 0x7fffffffll) {
    // one launch for both kernels, after the rows' delta values (5 algorithmic + 2 recomputed products per pair)
    CoreBwdArgs adq = a, adkv = a;
    adq.n_parts = cc.dq_parts;
    adq.pairs = q_pairs;
    adq.delta_stored = 1;
    adkv.tiles = key_tiles;
    adkv.n_parts = cc.dkv_parts;
    adkv.pairs = k_pairs;
    adkv.part_sums = a.part_sums + cc.dkv_ws_offset / 4;
    if (ntp::timing_on(h)) ntp::timing_begin(h, stream, cc.dq_parts > 1 || cc.dkv_parts > 1 ? "attn_core_bwd_both_cut" : "attn_core_bwd_both", 7.0 * pair_flops, 0.0);
    hipLaunchKernelGGL((attn_core_delta_kernel<128>), dim3(uint32_t(delta_wgs)), dim3(256), 0, hs, a, M);
    ok = hipGetLastError() == hipSuccess;
    const dim3 grid(uint32_t(dq_wgs + dkv_wgs));
    if (ok) {
      BothOrder order;
      order.n_dkv = uint32_t(dkv_wgs);
      order.chunk = uint32_t(std::max(h->compute_units, 1));
      order.paired = uint32_t(std::min(dq_wgs, dkv_wgs) / order.chunk * order.chunk);
      if (s->causal) hipLaunchKernelGGL((attn_core_bwd_both_kernel<true>), grid, dim3(kThreads), 0, hs, adq, adkv, order);
      else hipLaunchKernelGGL((attn_core_bwd_both_kernel<false>), grid, dim3(kThreads), 0, hs, adq, adkv, order);
      ok = hipGetLastError() == hipSuccess;
    }
    if (ok && cc.dq_parts > 1) {
      a = adq;
      ok = reduce_parts(std::false_type{}, bq);
    }
    if (ok && cc.dkv_parts > 1) {
      a = adkv;
      ok = reduce_parts(std::true_type{}, bk);
    }
    ntp::timing_end(h, stream);
    return ok ? NTP_OK : NTP_ERR_LAUNCH;
  }
  if (bq > 0) {
    // dQ and delta: three products per (query, key) pair.  With few heads the launch is short of
    // workgroups and each walks over up to seq_len / 64 key tiles: cut the walks then.
    a.n_parts = cc.dq_parts;
    a.pairs = q_pairs;
    if (ntp::timing_on(h)) ntp::timing_begin(h, stream, a.n_parts > 1 ? "attn_core_bwd_dq_cut" : "attn_core_bwd_dq", 3.0 * pair_flops, 0.0);
    const dim3 grid{uint32_t(dq_wgs)};
    if (cc.dq_dma) {
      if (a.pairs > 0) hipLaunchKernelGGL((attn_core_bwd_dq_dma_kernel<true>), grid, dim3(kThreads), 0, hs, a);
      else hipLaunchKernelGGL((attn_core_bwd_dq_dma_kernel<false>), grid, dim3(kThreads), 0, hs, a);
    } else if (s->head_dim == 128 && a.pairs > 0)
      hipLaunchKernelGGL((attn_core_bwd_dq_kernel<128, qbw, true>), grid, dim3(kThreads), 0, hs, a);
    else if (s->head_dim == 128)
      hipLaunchKernelGGL((attn_core_bwd_dq_kernel<128, qbw, false>), grid, dim3(kThreads), 0, hs, a);
    else if (a.pairs > 0)
      hipLaunchKernelGGL((attn_core_bwd_dq_kernel<64, qbw, true>), grid, dim3(kThreads), 0, hs, a);
    else
      hipLaunchKernelGGL((attn_core_bwd_dq_kernel<64, qbw, false>), grid, dim3(kThreads), 0, hs, a);
    ok = hipGetLastError() == hipSuccess;
    if (ok && a.n_parts > 1) ok = reduce_parts(std::false_type{}, bq);
    ntp::timing_end(h, stream);
    if (!ok) return NTP_ERR_LAUNCH;
  }
  if (bk > 0) {
    // dK and dV: four products per pair
    // a workgroup walks over the query tiles of every query head that reads its KV head
    a.tiles = key_tiles;
    a.n_parts = cc.dkv_parts;
    a.pairs = k_pairs;
    if (ntp::timing_on(h)) ntp::timing_begin(h, stream, a.n_parts > 1 ? "attn_core_bwd_dkv_cut" : "attn_core_bwd_dkv", 4.0 * pair_flops, 0.0);
    const dim3 grid{uint32_t(dkv_wgs)};
    if (cc.dkv_dma) {
      if (a.pairs > 0) hipLaunchKernelGGL((attn_core_bwd_dkv_dma_kernel<true>), grid, dim3(kThreads), 0, hs, a);
      else hipLaunchKernelGGL((attn_core_bwd_dkv_dma_kernel<false>), grid, dim3(kThreads), 0, hs, a);
    } else if (s->head_dim == 128 && a.pairs > 0)
      hipLaunchKernelGGL((attn_core_bwd_dkv_kernel<128, kb, true>), grid, dim3(kThreads), 0, hs, a);
    else if (s->head_dim == 128)
      hipLaunchKernelGGL((attn_core_bwd_dkv_kernel<128, kb, false>), grid, dim3(kThreads), 0, hs, a);
    else if (a.pairs > 0)
      hipLaunchKernelGGL((attn_core_bwd_dkv_kernel<64, kb, true>), grid, dim3(kThreads), 0, hs, a);
    else
      hipLaunchKernelGGL((attn_core_bwd_dkv_kernel<64, kb, false>), grid, dim3(kThreads), 0, hs, a);
    ok = hipGetLastError() == hipSuccess;
    if (ok && a.n_parts > 1) ok = reduce_parts(std::true_type{}, bk);
    ntp::timing_end(h, stream);
  }
  return ok ? NTP_OK : NTP_ERR_LAUNCH;
}
