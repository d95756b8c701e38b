// Ring contraction kernel for one K-contiguous (ROWK) and one K-major (KROW) operand, bf16.
//
// Same contract, tile shape, MFMA schedule and epilogues as gemm_dma4_kernel (gemm_dma4.h); what differs is how
// the K-contiguous operand A travels.  In a 32-deep K block a row of A is 64 bytes, half a cache line, so the
// ring of gemm_dma4.h asks the L2 for every line of A twice (once per half, in consecutive blocks).  Here A
// moves in 64-deep blocks of whole lines, one every second iteration, while B keeps its 32-deep blocks (rows of
// B are whole lines at any depth): LDS holds three 64-deep tiles of A (3 x 32 KB) and four 32-deep tiles of B
// (4 x 16 KB), 160 KB in all.  Block kb multiplies A tile (kb / 2) % 3, steps 2 (kb % 2) and 2 (kb % 2) + 1,
// with B tile kb % 4.  Loads per wave: B(kb + 3) every iteration (2), A((kb + 3) / 2) on odd iterations (4);
// any two consecutive iterations issue 8, so "at most 8 loads outstanding" again means that everything the next
// block needs has landed.
#pragma once
#include "gemm_dma4.h"

namespace rnnlm_dev {

#if defined(__HIP_DEVICE_COMPILE__)
// 64-deep K-contiguous tile [ROWS][64 k], loads written as inline assembly (see DmaLoader32 for why).
template <int ROWS, int NT>
struct DmaLoader64Asm {
  static constexpr int BLOCKS = ROWS * 128 / 1024;
  static constexpr int NW = NT / 64;
  static constexpr int PER = BLOCKS / NW;
  static_assert(BLOCKS % NW == 0 && PER >= 1, "tile does not divide over the waves");
  typedef int i32x4_t __attribute__((ext_vector_type(4)));
  int off[PER];
  i32x4_t rsrc;

  __device__ inline void init(const char *op, long op_bytes, long ld_bytes, long row0, long k0, int tid) {
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int q = (wave + i * NW) * 64 + lane;  // physical chunk index inside the tile
      const int r = q >> 3, p = q & 7;
      off[i] = (int)(r * ld_bytes + ((p ^ rowk_swz(r)) << 4));
    }
    const long start = row0 * ld_bytes + k0 * 2;
    const long left = op_bytes - start;
    const unsigned records = left > 0xffffffffL ? 0xffffffffu : (unsigned)left;
    const unsigned long long base = reinterpret_cast<unsigned long long>(op + start);
    rsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
    rsrc[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((base >> 32) & 0xffffu));
    rsrc[2] = __builtin_amdgcn_readfirstlane((int)records);
    rsrc[3] = 0x00020000;
  }
  __device__ inline void issue(char *tile, int kb64, int tid) const {  // 64-deep block kb64 (relative to the first)
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int soff = kb64 * 128;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const unsigned lds_addr = (unsigned)(unsigned long long)(lds_void_ptr)(tile + (wave + i * NW) * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :
                   : "s"(lds_addr), "v"(off[i]), "s"(rsrc), "s"(soff)
                   : "memory", "m0");
    }
  }
};
#endif  // __HIP_DEVICE_COMPILE__

template <int BM, int BN, int WGM, int WGN, class Epi, bool PERSIST>
__global__ void __launch_bounds__(WGM *WGN * 64) gemm_ring64_kernel(const GemmShape g, const Epi epi) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int NT = WGM * WGN * 64;
  constexpr int BK = 32;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int ASLOT = BM * 128, BSLOT = BN * 64;
  static_assert(Epi::template lds_bytes<BM, BN>() == 0, "the ring takes the whole LDS");
  static_assert(3 * ASLOT + 4 * BSLOT <= 160 * 1024, "tile does not fit the 160 KB of LDS");
  __shared__ __attribute__((aligned(1024))) char lds[3 * ASLOT + 4 * BSLOT];
  char *const a_tiles = lds;
  char *const b_tiles = lds + 3 * ASLOT;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int nwork = g.perXcd * NUM_XCD;
  const int stride = PERSIST ? (int)gridDim.x : nwork;
  DmaLoader64Asm<BM, NT> la;
  DmaLoader32<BN, KROW, NT> lb;
  constexpr int LOADS_TWO_ITERATIONS = DmaLoader64Asm<BM, NT>::PER + 2 * DmaLoader32<BN, KROW, NT>::PER;
  static_assert(LOADS_TWO_ITERATIONS <= 15, "outstanding-load count must fit the low bits of vmcnt");
  constexpr int WAIT_NEXT = LOADS_TWO_ITERATIONS | (7 << 4);  // vmcnt, expcnt at its maximum, lgkmcnt 0
  const int lr = lane & 31;
  static_assert(TM <= 4 && TN <= 4, "fragment addressing covers up to four 32-row blocks per wave");
  DmaFragAddr<BM, ROWK> addr_a;
  DmaFragAddr32<BN, KROW> addr_b;
  addr_a.init(wm * WTM + lr, lane);
  addr_b.init(wn * WTN + lr, lane);

  bool prefetched = false;  // the loaders are set up for this tile and its first blocks are in flight
  for (int wid = blockIdx.x; wid < nwork; wid += stride) {
    int tile_m, tile_n, split;
    if (!map_workgroup(g, wid, split, tile_m, tile_n)) continue;  // uniform for the workgroup (never after a prefetch)
    // g.kBlocks counts 64-deep blocks; the loop walks 32-deep ones (an even number of them)
    const int kb0 = 2 * split * g.kBlocksPerSplit;
    const int kb1 = 2 * min((split + 1) * g.kBlocksPerSplit, g.kBlocks);
    const int nk = kb1 - kb0;

    f32x16_t acc[TM][TN];
    epi.template init<TM, TN>(acc, tile_m * BM + wm * WTM, tile_n * BN + wn * WTN, lane, split);

    // block / pair index clamped to the last one: the final iterations re-fetch it (into a tile nobody reads
    // any more) instead of branching, so the number of loads per iteration and wave keeps its pattern
    auto fetch_b = [&](int kb, int nblocks) { lb.issue(b_tiles + (kb & 3) * BSLOT, min(kb, nblocks - 1), tid); };
    auto fetch_a = [&](int pair, int nblocks) { la.issue(a_tiles + (pair % 3) * ASLOT, min(pair, nblocks / 2 - 1), tid); };
    auto first_fetches = [&](int nblocks) {  // everything blocks 0 .. 2 need, in the order the waits assume
      fetch_a(0, nblocks);
      fetch_b(0, nblocks);
      fetch_b(1, nblocks);
      fetch_a(1, nblocks);
      fetch_b(2, nblocks);
    };
    if (!prefetched) {
      la.init(static_cast<const char *>(g.A), g.bytesA, g.lda * 2, (long)tile_m * BM, (long)kb0 * BK, tid);
      lb.init(static_cast<const char *>(g.B), g.bytesB, g.ldb * 2, (long)tile_n * BN, (long)kb0 * BK, tid);
    }

    bf16x8_t fa[2][TM], fb[2][TN];
    auto read_frags = [&](int kb, int step, int buf) {  // 16-wide step `step` (0, 1) of block kb
      const char *sa = a_tiles + ((kb >> 1) % 3) * ASLOT;
      const char *sb = b_tiles + (kb & 3) * BSLOT;
      const int st = 2 * (kb & 1) + step;
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[buf][i] = addr_a.get(sa, i, st);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[buf][j] = addr_b.get(sb, j, step);
    };
    auto mfmas = [&](int buf) {
      __builtin_amdgcn_s_setprio(3);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) mma16(acc[i][j], fa[buf][i], fb[buf][j]);
      __builtin_amdgcn_s_setprio(0);
    };
    // One K block (its step-0 fragments are already in buffer 0).  ODD: also the A tile three blocks ahead.
    auto block = [&](int kb, bool odd) {
      fetch_b(kb + 3, nk);
      if (odd) fetch_a((kb + 3) >> 1, nk);
      read_frags(kb, 1, 1);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(0);
      // this wave's share of block kb + 1 has landed and its reads of block kb have returned
      __builtin_amdgcn_s_waitcnt(WAIT_NEXT);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      read_frags(kb + 1, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(1);
    };

    if (nk > 0) {
      if (!prefetched) first_fetches(nk);
      __builtin_amdgcn_s_waitcnt(WAIT_NEXT);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      read_frags(0, 0, 0);
#pragma unroll 1
      for (int kb = 0; kb < nk; kb += 2) {
        block(kb, false);
        block(kb + 1, true);
      }
    }
    __builtin_amdgcn_s_waitcnt(7 << 4);  // vmcnt(0) lgkmcnt(0): every load of this wave has landed
    __syncthreads();  // ... and everyone's, and all fragment reads are done
    const int this_m = tile_m, this_n = tile_n, this_split = split;
    prefetched = false;
    if (PERSIST) {
      // the next work item of this workgroup: loaders re-aimed, first blocks requested (older than every access
      // of the epilogue below, so the waits of the next main loop still count the right loads)
      int nm, nn, ns;
      if (wid + stride < nwork && map_workgroup(g, wid + stride, ns, nm, nn)) {
        const int nkb0 = 2 * ns * g.kBlocksPerSplit;
        const int nnk = 2 * min((ns + 1) * g.kBlocksPerSplit, g.kBlocks) - nkb0;
        if (nnk > 0) {
          la.init(static_cast<const char *>(g.A), g.bytesA, g.lda * 2, (long)nm * BM, (long)nkb0 * BK, tid);
          lb.init(static_cast<const char *>(g.B), g.bytesB, g.ldb * 2, (long)nn * BN, (long)nkb0 * BK, tid);
          first_fetches(nnk);
          prefetched = true;
        }
      }
    }
    EpiCtx ctx;
    ctx.smem_lo = ctx.smem_hi = nullptr;
    ctx.q[0] = ctx.q[1] = ctx.q[2] = ctx.q[3] = nullptr;
    ctx.tile_row0 = this_m * BM;
    ctx.tile_col0 = this_n * BN;
    ctx.wrow = wm * WTM;
    ctx.wcol = wn * WTN;
    ctx.lane = lane;
    ctx.tid = tid;
    ctx.split = this_split;
    epi.template run<BM, BN, TM, TN, NT>(acc, ctx);
  }
#endif  // __HIP_DEVICE_COMPILE__
}

template <int BM, int BN, int WGM, int WGN, class Epi>
inline hipError_t launch_gemm_ring64(hipStream_t stream, const void *A, long lda, const void *B, long ldb, long Mg,
                                     long Ng, long K, int splits, const Epi &epi, int band = 4) {
  constexpr int BK = 64;
  if (Mg <= 0 || Ng <= 0 || K < 0 || Mg % BM || Ng % BN || K % BK || splits < 1) return hipErrorInvalidValue;
  GemmShape g;
  g.A = A;
  g.B = B;
  g.lda = lda;
  g.ldb = ldb;
  g.bytesA = 2 * lda * Mg;
  g.bytesB = 2 * ldb * K;
  if (K * ldb * 2 >= (1L << 31) || lda * 2 * BM >= (1L << 31)) return hipErrorInvalidValue;
  g.tilesM = (int)(Mg / BM);
  g.tilesN = (int)(Ng / BN);
  g.kBlocks = (int)(K / BK);
  g.kBlocksPerSplit = (g.kBlocks + splits - 1) / splits;
  g.splits = splits;
  const long total = (long)g.tilesM * g.tilesN * splits;
  if (band == 0 || total > (1L << 30)) return hipErrorInvalidValue;
  g.perXcd = (int)((total + NUM_XCD - 1) / NUM_XCD);
  g.bandOverN = band < 0;
  g.band = band < 0 ? -band : band;
  unsigned grid = (unsigned)(g.perXcd * NUM_XCD);
  if (grid > 256u) grid = 256u;  // one persistent workgroup per compute unit
  hipLaunchKernelGGL((gemm_ring64_kernel<BM, BN, WGM, WGN, Epi, true>), dim3(grid), dim3(WGM * WGN * 64), 0, stream,
                     g, epi);
  return hipGetLastError();
}

}  // namespace rnnlm_dev
