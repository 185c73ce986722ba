// Ping-pong form of the ring GEMM kernel (8 wavefronts).  Same tiles, LDS ring, slot layouts, DMA addressing
// and epilogues as gemm_ring_kernel (ntp_gemm_ring.h); what differs is who does what when in the K loop.
//
// The two wavefronts of a SIMD (w and w + 4: wavefronts are dealt to the four SIMDs in turn) alternate between
// two kinds of slot, with a workgroup barrier after every slot:
//   memory slot   read all fragments of one K-step (32 k) of the current K tile from LDS into registers, start
//                 this wavefront's DMA instructions, wait for the fragments;
//   compute slot  MI x NI matrix instructions on those fragments, nothing else.
// Wavefronts 0-3 ("early") run M0 C0 M1 C1 per K tile, wavefronts 4-7 ("late") the same one slot behind, so
// in every slot one wavefront of each SIMD computes while the other one's LDS latency, address arithmetic and DMA
// issue hide behind it, instead of sharing an instruction stream with the matrix instructions.
//
// LDS ring (five operand slots): K tile t (P = t mod 5) has A in slot 2P and B in slot 2P+1.  The last reader
// of tile t is the late group's M1, the fourth slot of the tile; after that slot's barrier both are free.
// Every wavefront moves an eighth of both operands, so that each of a tile's four slots carries a quarter of the
// tile's DMA instructions (the vector memory path takes about 18 cycles per 1 KiB instruction and compute unit:
// 64 of them per K tile are two thirds of the tile's matrix time, and have to be spread evenly to hide):
//   in M0 of tile t a wavefront starts its share of B of tile t+1 -> slot 2P+3 (where A of tile t-1 was),
//   in M1 its share of A of tile t+2 -> slot 2P+4 (where B of tile t-1 was), and the L2 prefetch;
//   before the barrier that ends the tile's fourth slot (early group: after C1, late group: after M1) it waits
//   for its DMA instructions up to that share of B (the NA + 1 newer ones may stay in flight).
// After that barrier tile t+1 is complete in LDS.  Past the last tile the schedule keeps loading the last tile
// (clamped index) into slots nobody reads, so that instruction counts stay static.
//
// LDS reads in the loop are inline assembly: the compiler then neither sees nor guards them (it would put a
// wait for every DMA in flight in front of each), and the waits above are the only ones.
#ifndef NTP_GEMM_PP_H_
#define NTP_GEMM_PP_H_

#include "ntp_gemm_ring.h"

namespace ntp_gemm {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

// 32-bit LDS address of an object in shared memory
__device__ __forceinline__ uint32_t lds_addr(const void* p) { return uint32_t(reinterpret_cast<uintptr_t>(p)); }

// Fragment I (16 rows) of K-step KS of an operand slot, by inline-assembly LDS reads (see FragAddr for the layout).
// The caller waits for lgkmcnt before using the result.
template <bool KC, int R, int NF, int I, int KS>
__device__ __forceinline__ bf16x8 frag_read_asm(const FragAddr<KC, R, NF>& f, uint32_t slot_addr) {
#if !defined(__HIP_DEVICE_COMPILE__)
  // (the host pass only needs the signature: its compiler does not know the GPU's register constraints)
  return bf16x8{};
#else
  if constexpr (KC) {
    u32x4_t v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(slot_addr + f.o[KS] * 2u), "n"(I * 16 * DK * 2) : "memory");
    return __builtin_bit_cast(bf16x8, v);
  } else {
    u32x2_t lo, hi;
    const uint32_t a = slot_addr + f.o[I] * 2u;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(a), "n"(KS * 32 * R * 2) : "memory");
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(a), "n"(KS * 32 * R * 2 + 4 * R * 2) : "memory");
    const u32x4_t v = {lo[0], lo[1], hi[0], hi[1]};
    return __builtin_bit_cast(bf16x8, v);
  }
#endif
}

// one DMA instruction: 64 lanes x 16 bytes from the buffer view (lane offset voff + scalar offset soff) to 1 KiB of LDS at dst
__device__ __forceinline__ void dma_issue(__amdgpu_buffer_rsrc_t rsrc, uint16_t* dst, uint32_t voff, uint32_t soff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)dst, 16, voff, soff, 0, 0);
}

template <int... Is, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, Is...>, F&& f) {
  (f(Int<Is>{}), ...);
}

template <bool AKC, bool BKC, int EPI, int BM_, int BN_, int WGM, int WGN>
__global__ __launch_bounds__(512) void gemm_pp_kernel(const GemmArgs g) {
  static_assert(WGM * WGN == 8, "wavefront w is paired with wavefront w + 4");
  constexpr int TM = BM_ / WGM, TN = BN_ / WGN;  // wavefront tile
  constexpr int MI = TM / 16, NI = TN / 16;      // 16 x 16 accumulator blocks
  static_assert(TM % 16 == 0 && TN % 16 == 0, "wavefront tile: 16 x 16 blocks");
  constexpr int RA = slot_rows(AKC, BM_), RB = slot_rows(BKC, BN_);
  static_assert(BM_ <= 256 && BN_ <= 256, "tile sides up to 256");
  constexpr int SLOT = (RA > RB ? RA : RB) * DK;
  // DMA instructions per K tile and wavefront for A and for B
  constexpr int NAI = RA * DK * 2 / 1024 / 8, NBI = RB * DK * 2 / 1024 / 8;
  static_assert((RA * DK * 2 / 1024) % 8 == 0 && (RB * DK * 2 / 1024) % 8 == 0, "operands split evenly over the wavefronts");
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
  const bool late = wave >= 4;  // uniform within a wavefront

  // persistent workgroups, XCD-aware tile walk: as in gemm_ring_kernel
  const int nblk = g.tiles_m * g.tiles_n;
  struct Pos {
    int tile_m, tile_n, row0, col0;
  };
  auto place = [&](int v) {
    const TilePos t = place_tile(v, g.tiles_m, g.tiles_n);
    return Pos{t.tile_m, t.tile_n, t.tile_m * BM_, t.tile_n * BN_};
  };
  int vblk = blockIdx.x;
  const int K = g.K;
  Pos pos = place(vblk);
  int row0 = pos.row0, col0 = pos.col0;

  f32x4 acc[MI][NI];
  const int64_t astep = AKC ? DK : DK * g.lda, bstep = BKC ? DK : DK * g.ldb;  // elements per K tile
  constexpr bool RT = AKC && !BKC;
  // range-checked buffer views of the operands (see gemm_ring_kernel); a wavefront uses the one of the operand it moves
  const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(g.A), 0, int(g.a_extent), 0x00020000);
  const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(g.B), 0, int(g.b_extent), 0x00020000);
  const uint32_t astep_b = uint32_t(astep) * 2, bstep_b = uint32_t(bstep) * 2;
  FragAddr<AKC, RA, MI> fra;
  FragAddr<BKC, RB, NI> frb;
  fra.init(wm * TM, lane);
  frb.init(wn * TN, lane);

  const int nfull = K / DK;
  const bool ring_tail = RT && g.ring_tail != 0 && nfull * DK < K;
  const int nk = nfull + (ring_tail ? 1 : 0);

  // L2 prefetch four K tiles ahead, by turns among the workgroups that share an operand tile: as in gemm_ring_kernel
  constexpr int PFD = 4;
  uint32_t pf_sink = 0;
  const bool pf_is_a = wave < 4;
  const int pf_mask = pf_is_a ? 3 : 7;
  const bool pf_ok = pf_is_a ? (AKC || g.M >= 2) : (BKC || g.N >= 2);
  const char* const pf_base = reinterpret_cast<const char*>(pf_is_a ? g.A : g.B);
  const int64_t pf_step = (pf_is_a ? astep : bstep) * 2;  // bytes per K tile
  int pf_turn = 0, pf_turn_next = -1;  // -1: there is no next output tile
  uint32_t pf_voff = 0, pf_voff_next = 0;
  auto pf_params = [&](const Pos& p, int& turn, uint32_t& voff) {
    turn = pf_is_a ? (p.tile_n & 3) : (p.tile_m & 7);
    voff = pf_is_a ? DmaOperand<AKC, RA, 8>::prefetch_offset(g.lda, p.row0, g.M, wave & 3, lane)
                   : DmaOperand<BKC, RB, 8>::prefetch_offset(g.ldb, p.col0, g.N, wave & 3, lane);
  };
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

  // this wavefront's DMA offsets
  uint32_t offa[NAI], offb[NBI];
  auto setup_tile = [&] {
#pragma unroll
    for (int i = 0; i < NAI; ++i) {
      int line, chunk;
      slot_src<AKC, RA>((wave * NAI + i) * 64 + lane, line, chunk);
      offa[i] = dma_offset<AKC>(g.lda, row0, g.M, line, chunk);
    }
#pragma unroll
    for (int i = 0; i < NBI; ++i) {
      int line, chunk;
      slot_src<BKC, RB>((wave * NBI + i) * 64 + lane, line, chunk);
      offb[i] = dma_offset<BKC>(g.ldb, col0, g.N, line, chunk);
    }
    pf_params(pos, pf_turn, pf_voff);
  };
  // Byte offset of this wavefront's first DMA destination inside a slot.  It passes through an empty assembly
  // statement at every use, so that the compiler adds it to the slot's address then and there (one scalar add per
  // instruction) instead of keeping forty precomputed LDS addresses alive across the loop.
  uint32_t dsta = uint32_t(wave) * NAI * 1024u, dstb = uint32_t(wave) * NBI * 1024u;
  auto dma_a = [&](int kt, uint16_t* sl) {
    asm volatile("" : "+s"(dsta));
#pragma unroll
    for (int i = 0; i < NAI; ++i) dma_issue(ra, reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(sl) + dsta) + i * 512, offa[i], uint32_t(kt) * astep_b);
  };
  auto dma_b = [&](int kt, uint16_t* sl) {
    asm volatile("" : "+s"(dstb));
#pragma unroll
    for (int i = 0; i < NBI; ++i) dma_issue(rb, reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(sl) + dstb) + i * 512, offb[i], uint32_t(kt) * bstep_b);
  };
  // first DMA instructions of an output tile: K tile 0 whole and A of K tile 1
  auto first_dma = [&] {
    if (nk > 0) {
      dma_a(0, r0);
      dma_b(0, r1);
      dma_a(min(1, nk - 1), r2);
    }
  };

  bf16x8 fa[MI], fb[NI];
  auto read_frags = [&](auto kss, uint32_t sa_addr, uint32_t sb_addr) {
    constexpr int ks = decltype(kss)::value;
    static_for(std::make_integer_sequence<int, MI>{}, [&](auto i) { fa[decltype(i)::value] = frag_read_asm<AKC, RA, MI, decltype(i)::value, ks>(fra, sa_addr); });
    static_for(std::make_integer_sequence<int, NI>{}, [&](auto j) { fb[decltype(j)::value] = frag_read_asm<BKC, RB, NI, decltype(j)::value, ks>(frb, sb_addr); });
  };
  auto compute_slot = [&] {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
    // operands swapped so that each lane ends up with 4 consecutive columns of one row
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto pp_tile = [&](auto p, int t) {
    constexpr int P = decltype(p)::value;
    uint16_t* const sa = slot(Int<(2 * P) % 5>{});
    uint16_t* const sb = slot(Int<(2 * P + 1) % 5>{});
    uint16_t* const nss = slot(Int<(2 * P + 3) % 5>{});
    uint16_t* const fsl = slot(Int<(2 * P + 4) % 5>{});
    const uint32_t sa_addr = lds_addr(sa), sb_addr = lds_addr(sb);
    const int t1 = min(t + 1, nk - 1), t2 = min(t + 2, nk - 1);
    // M0
    __builtin_amdgcn_sched_barrier(0);
    read_frags(Int<0>{}, sa_addr, sb_addr);
    __builtin_amdgcn_sched_barrier(0);
    dma_b(t1, nss);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(lgkm0_imm());
    __builtin_amdgcn_s_barrier();
    compute_slot();  // C0
    __builtin_amdgcn_s_barrier();
    // M1
    __builtin_amdgcn_sched_barrier(0);
    read_frags(Int<1>{}, sa_addr, sb_addr);
    __builtin_amdgcn_sched_barrier(0);
    dma_a(t2, fsl);
    prefetch(t);
    __builtin_amdgcn_sched_barrier(0);
    // late group: this is the tile's fourth slot; its share of B of tile t+1 (started in M0) has landed, the
    // NAI + 1 newer instructions may fly on
    if (late) __builtin_amdgcn_s_waitcnt(vmcnt_lgkm0_imm(NAI + 1));
    else __builtin_amdgcn_s_waitcnt(lgkm0_imm());
    __builtin_amdgcn_s_barrier();
    compute_slot();  // C1
    // early group: its C1 is the tile's fourth slot
    if (!late) __builtin_amdgcn_s_waitcnt(vmcnt_imm(NAI + 1));
    __builtin_amdgcn_s_barrier();
  };

  // vector memory instructions a wavefront issues in the epilogue of an interior tile (see gemm_ring_kernel)
  constexpr bool PAIRED = EPI == ntp::EPI_BF16 || EPI == ntp::EPI_GELU || EPI == ntp::EPI_DGELU;
  constexpr int NPAIR = NI / 2, NODD = NI & 1;
  constexpr int NEPI = EPI == ntp::EPI_BF16    ? MI * (NPAIR + NODD)
                       : EPI == ntp::EPI_GELU  ? MI * 2 * (NPAIR + NODD)
                       : EPI == ntp::EPI_DGELU ? MI * (3 * NPAIR + 2 * NODD)
                       : EPI == ntp::EPI_F32   ? MI * NI
                                               : MI * NI * 2;
  bool stores_in_flight = false;
  setup_tile();
  first_dma();
  while (true) {
    const int vnext = vblk + int(gridDim.x);
    const bool more = vnext < nblk;
    const Pos npos = more ? place(vnext) : pos;
    if (more) pf_params(npos, pf_turn_next, pf_voff_next);
    else pf_turn_next = -1;
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    if (nk > 0) {
      // the first DMA instructions of this output tile have landed (the previous tile's NEPI epilogue
      // instructions, issued after them, may stay in flight: the counter is in order)
      if (stores_in_flight) __builtin_amdgcn_s_waitcnt(vmcnt_imm(NEPI <= 63 ? NEPI : 63));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __builtin_amdgcn_s_barrier();
      // Every wavefront passes 4 nk + 1 barriers in the loop: the late group one before its first slot, the
      // early group one after its last (nk is the same for the whole workgroup).
      if (late) __builtin_amdgcn_s_barrier();
      for (int t = 0; t < nk; t += 5) {
        pp_tile(Int<0>{}, t);
        if (t + 1 < nk) pp_tile(Int<1>{}, t + 1);
        if (t + 2 < nk) pp_tile(Int<2>{}, t + 2);
        if (t + 3 < nk) pp_tile(Int<3>{}, t + 3);
        if (t + 4 < nk) pp_tile(Int<4>{}, t + 4);
      }
      if (!late) __builtin_amdgcn_s_barrier();
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));  // the clamped DMA instructions of the last tiles
    // K tail (K % 64 != 0) through registers with element masks, not overlapped
    if (!ring_tail && nfull * DK < K) {
      __syncthreads();
      {
        DmaOperand<AKC, RA, 8> ta;
        ta.init(g.lda, row0, g.M, wave, lane);
        ta.tail(g.A, astep, nfull, K, r0, wave, lane);
        DmaOperand<BKC, RB, 8> tb;
        tb.init(g.ldb, col0, g.N, wave, lane);
        tb.tail(g.B, bstep, nfull, K, r1, wave, lane);
      }
      __syncthreads();
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[i] = fra.read(r0, i, ks);
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[j] = frb.read(r1, j, ks);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
      }
    }
    const int erow0 = row0, ecol0 = col0;
    vblk = vnext;
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
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int m = erow0 + wm * TM + i * 16 + (lane & 15);
      if constexpr (PAIRED) {
#pragma unroll
        for (int j = 0; j + 1 < NI; j += 2) store8_pair<EPI>(g, m, ecol0 + wn * TN + j * 16, lane >> 4, acc[i][j], acc[i][j + 1]);
      }
#pragma unroll
      for (int j = PAIRED ? NI - NODD : 0; j < NI; ++j) store4<EPI>(g, m, ecol0 + wn * TN + j * 16 + (lane >> 4) * 4, acc[i][j]);
    }
    if (!more) break;
  }
  asm volatile("" : "+v"(pf_sink));  // the prefetch register stays reserved up to here
}

}  // namespace ntp_gemm

#endif  // NTP_GEMM_PP_H_
