// bf16 MFMA contraction with direct global->LDS loads and a FOUR-stage ring of 32-deep K blocks.
//
// Same contract and data path as gemm_dma_kernel (gemm_dma.h), different pipeline depth.  What the main
// loop of the two-stage kernel waits for is operand data: with one 64 KB stage in flight per compute unit
// and a loaded L2/fabric latency of about 1.5 us, a compute unit can pull about 43 GB/s, less than the
// 71 GB/s a 256x256 tile consumes at full MFMA rate.  Here the same 128 KB of LDS holds four stages of
// 32 KB (K blocks of 32), three of which can be in flight while the fourth is multiplied, so 96 KB per
// compute unit are outstanding.  One barrier per K block; it is a bare s_barrier preceded by an explicit
// s_waitcnt for "at most two blocks of this wave's loads still outstanding" (a __syncthreads would wait for
// all of them).  The stages are four separate arrays and the loop is unrolled by four so that the compiler
// can tell the loads in flight into one stage from the fragment reads of another.
//
// LDS layouts (64 banks x 4 bytes):
//   ROWK tile [rows][32 k]: rows of 64 bytes = 4 chunks of 16 bytes, 16 rows per kilobyte.  A 16-byte
//   fragment read is served 16 lanes (16 consecutive rows, one logical chunk) per clock, which must cover
//   all 16 chunk positions of a 256-byte bank line: physical chunk = logical ^ ((row >> 2) & 3).
//   KROW tile [32 k][rows]: as in gemm_dma.h (physical chunk = logical ^ (4 * (k & 3))).
#pragma once
#include "gemm_dma.h"

namespace rnnlm_dev {

__device__ inline int rowk32_swz(int row) { return (row >> 2) & 3; }

#if defined(__HIP_DEVICE_COMPILE__)
template <int ROWS, int LAYOUT, int NT>
struct DmaLoader32 {
  static constexpr int BLOCKS = ROWS * 64 / 1024;  // kilobyte blocks per tile
  static constexpr int NW = NT / 64;
  static constexpr int PER = BLOCKS / NW;
  static_assert(BLOCKS % NW == 0 && PER >= 1, "tile does not divide over the waves");
  typedef int i32x4_t __attribute__((ext_vector_type(4)));
  int off[PER];  // this lane's byte offset inside a k block for each of its kilobyte blocks
  i32x4_t rsrc;  // buffer resource: base, stride 0, extent in bytes, raw 32-bit addressing
  int kstep;     // bytes to advance per k block

  __device__ inline void init(const char *op, long op_bytes, long ld_bytes, long row0, long k0, int tid) {
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int q = (wave + i * NW) * 64 + lane;  // physical chunk index inside the tile
      if (LAYOUT == ROWK) {
        const int r = q >> 2, p = q & 3;
        off[i] = (int)(r * ld_bytes + ((p ^ rowk32_swz(r)) << 4));
      } else {
        constexpr int CPR = ROWS / 8;
        const int k = q / CPR, p = q % CPR;
        off[i] = (int)(k * ld_bytes + ((p ^ krow_swz(k)) << 4));
      }
    }
    const long start = (LAYOUT == ROWK) ? row0 * ld_bytes + k0 * 2 : k0 * ld_bytes + row0 * 2;
    kstep = (LAYOUT == ROWK) ? 64 : (int)(32 * ld_bytes);
    const long left = op_bytes - start;
    const unsigned records = left > 0xffffffffL ? 0xffffffffu : (unsigned)left;
    const unsigned long long base = reinterpret_cast<unsigned long long>(op + start);
    // every word is uniform over the workgroup: keep the descriptor in scalar registers
    rsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
    rsrc[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((base >> 32) & 0xffffu));
    rsrc[2] = __builtin_amdgcn_readfirstlane((int)records);
    rsrc[3] = 0x00020000;
  }
  // The loads are written as inline assembly on purpose: the compiler then neither counts them in vmcnt nor
  // treats them as LDS writes, so it places no waits of its own between them and the fragment reads of the
  // other stages (with the intrinsic it waited for all but the newest block at every loop head, which
  // defeats the ring); the kernel's explicit s_waitcnt + s_barrier pairs order them instead.  M0 carries
  // the LDS address of the kilobyte a wave instruction fills (64 lanes x 16 bytes, contiguous).
  __device__ inline void issue(char *tile, int kb, int tid) const {
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int soff = kb * kstep;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const unsigned lds_addr =
          (unsigned)(unsigned long long)(lds_void_ptr)(tile + (wave + i * NW) * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :
                   : "s"(lds_addr), "v"(off[i]), "s"(rsrc), "s"(soff)
                   : "memory", "m0");
    }
  }
};
#endif  // __HIP_DEVICE_COMPILE__

// Fragment addressing for 32-deep tiles (two 16-wide steps st = 0, 1).
//   ROWK: row r = r0 + 32 i: r*64 + (((2 st + h) ^ swz(r)) << 4), h = lane / 32; swz uses row bits 2..3, which
//         do not depend on i: pre[st] = r0*64 + (((2 st + h) ^ swz) << 4), immediate = i * 2048.
//   KROW: as DmaFragAddr<ROWS, KROW>, with two steps per tile.
template <int ROWS, int LAYOUT>
struct DmaFragAddr32;
template <int ROWS>
struct DmaFragAddr32<ROWS, ROWK> {
  int pre[2];
  __device__ inline void init(int r0, int lane) {
    const int h = lane >> 5, sw = rowk32_swz(r0);
#pragma unroll
    for (int st = 0; st < 2; ++st) pre[st] = r0 * 64 + (((2 * st + h) ^ sw) << 4);
  }
  __device__ inline bf16x8_t get(const char *tile, int i, int st) const {
    return *reinterpret_cast<const bf16x8_t *>(tile + pre[st] + i * 2048);
  }
};
template <int ROWS>
struct DmaFragAddr32<ROWS, KROW> : DmaFragAddr<ROWS, KROW> {};

template <int BM, int BN, class Epi>
constexpr int dma4_stage_bytes() {
  constexpr int loop = (BM + BN) * 64;
  constexpr int epi = (Epi::template lds_bytes<BM, BN>() + 3) / 4;
  constexpr int need = loop > epi ? loop : epi;
  return (need + 1023) / 1024 * 1024;
}

// PERSIST (epilogues that leave the LDS alone): the grid is one workgroup per compute unit and each walks the
// work items id, id + grid, ... (the grid is a multiple of 8, so a workgroup stays on the XCD whose chunk of
// tiles it walks); the first three K blocks of the next tile are requested before the current tile's epilogue
// starts, so the next main loop finds them in LDS instead of waiting a memory round trip per tile.
template <int BM, int BN, int WGM, int WGN, int LA, int LB, class Epi, bool PERSIST = false>
__global__ void __launch_bounds__(WGM *WGN * 64) gemm_dma4_kernel(const GemmShape g, const Epi epi) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int NT = WGM * WGN * 64;
  constexpr int BK = 32;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int SBYTES = dma4_stage_bytes<BM, BN, Epi>();
  __shared__ __attribute__((aligned(1024))) char stage0[SBYTES];
  __shared__ __attribute__((aligned(1024))) char stage1[SBYTES];
  __shared__ __attribute__((aligned(1024))) char stage2[SBYTES];
  __shared__ __attribute__((aligned(1024))) char stage3[SBYTES];

  static_assert(!PERSIST || Epi::template lds_bytes<BM, BN>() == 0, "the next tile's blocks land while the epilogue runs");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int nwork = g.perXcd * NUM_XCD;
  const int stride = PERSIST ? (int)gridDim.x : nwork;
  DmaLoader32<BM, LA, NT> la;
  DmaLoader32<BN, LB, NT> lb;
  bool prefetched = false;  // the loaders are set up for this tile and its first three blocks are in flight
  for (int wid = blockIdx.x; wid < nwork; wid += stride) {
  int tile_m, tile_n, split;
  if (!map_workgroup(g, wid, split, tile_m, tile_n)) continue;  // uniform for the workgroup (never after a prefetch)
  // g.kBlocks counts 64-deep blocks; this kernel walks 32-deep ones
  const int kb0 = 2 * split * g.kBlocksPerSplit;
  const int kb1 = 2 * min((split + 1) * g.kBlocksPerSplit, g.kBlocks);
  const int nk = kb1 - kb0;

  f32x16_t acc[TM][TN];
  epi.template init<TM, TN>(acc, tile_m * BM + wm * WTM, tile_n * BN + wn * WTN, lane, split);

  if (!prefetched) {
    la.init(static_cast<const char *>(g.A), g.bytesA, g.lda * 2, (long)tile_m * BM, (long)kb0 * BK, tid);
    lb.init(static_cast<const char *>(g.B), g.bytesB, g.ldb * 2, (long)tile_n * BN, (long)kb0 * BK, tid);
  }
  const int lr = lane & 31;

  // block index clamped to the last one: the final iterations re-fetch it (into a stage nobody reads any
  // more) instead of branching, so the number of loads per block and wave is always the same
  auto fetch_of = [&](char *stage, int kb, int nblocks) {
    kb = min(kb, nblocks - 1);
    la.issue(stage, kb, tid);
    lb.issue(stage + BM * 64, kb, tid);
  };
  auto fetch = [&](char *stage, int kb) { fetch_of(stage, kb, nk); };
  constexpr int LOADS_PER_BLOCK = DmaLoader32<BM, LA, NT>::PER + DmaLoader32<BN, LB, NT>::PER;
  static_assert(2 * LOADS_PER_BLOCK <= 15, "outstanding-load count must fit the low bits of vmcnt");
  // "this wave's loads of all but the two youngest blocks have landed, and its LDS reads have returned":
  // vmcnt = 2 * LOADS_PER_BLOCK, lgkmcnt = 0, expcnt left at its maximum (gfx9 encoding:
  // vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8])
  constexpr int WAIT_TWO_BLOCKS = (2 * LOADS_PER_BLOCK) | (7 << 4);

  static_assert(TM <= 4 && TN <= 4, "fragment addressing covers up to four 32-row blocks per wave");
  bf16x8_t fa[2][TM], fb[2][TN];
  DmaFragAddr32<BM, LA> addr_a;
  DmaFragAddr32<BN, LB> addr_b;
  addr_a.init(wm * WTM + lr, lane);
  addr_b.init(wn * WTN + lr, lane);
  auto read_frags = [&](const char *stage, int step, int buf) {
    const char *sa = stage;
    const char *sb = stage + BM * 64;
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[buf][i] = addr_a.get(sa, i, step);
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
  // One K block: `cur` holds the block being multiplied (its step-0 fragments are already in buffer 0),
  // `next` the one after it, `refill` the stage of the block before it (free once every wave has passed the
  // previous barrier), which receives the block three ahead.
  auto block = [&](const char *cur, const char *next, char *refill, int kb_refill) {
    fetch(refill, kb_refill);
    read_frags(cur, 1, 1);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(0);
    // this wave's share of `next` has landed and its reads of `cur` have returned (so `cur` may be
    // refilled by whoever passes the barrier first)
    __builtin_amdgcn_s_waitcnt(WAIT_TWO_BLOCKS);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    read_frags(next, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(1);
  };

  if (nk > 0) {
    if (!prefetched) {
      fetch(stage0, 0);
      fetch(stage1, 1);
      fetch(stage2, 2);
    }
    __builtin_amdgcn_s_waitcnt(WAIT_TWO_BLOCKS);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    read_frags(stage0, 0, 0);
#pragma unroll 1
    for (int it = 0; it < nk; it += 4) {
      block(stage0, stage1, stage3, it + 3);
      if (it + 1 < nk) block(stage1, stage2, stage0, it + 4);
      if (it + 2 < nk) block(stage2, stage3, stage1, it + 5);
      if (it + 3 < nk) block(stage3, stage0, stage2, it + 6);
    }
  }
  __builtin_amdgcn_s_waitcnt(7 << 4);  // vmcnt(0) lgkmcnt(0): every load of this wave has landed
  __syncthreads();  // ... and everyone's, and all fragment reads are done: the epilogue reuses the stages
  const int this_m = tile_m, this_n = tile_n, this_split = split;
  prefetched = false;
  if (PERSIST) {
    // the next work item of this workgroup: loaders re-aimed, first three blocks requested (older than every
    // access of the epilogue below, so the waits of the next main loop still count the right loads)
    int nm, nn, ns;
    if (wid + stride < nwork && map_workgroup(g, wid + stride, ns, nm, nn)) {
      const int nkb0 = 2 * ns * g.kBlocksPerSplit;
      const int nnk = 2 * min((ns + 1) * g.kBlocksPerSplit, g.kBlocks) - nkb0;
      if (nnk > 0) {
        la.init(static_cast<const char *>(g.A), g.bytesA, g.lda * 2, (long)nm * BM, (long)nkb0 * BK, tid);
        lb.init(static_cast<const char *>(g.B), g.bytesB, g.ldb * 2, (long)nn * BN, (long)nkb0 * BK, tid);
        fetch_of(stage0, 0, nnk);
        fetch_of(stage1, 1, nnk);
        fetch_of(stage2, 2, nnk);
        prefetched = true;
      }
    }
  }
  EpiCtx ctx;
  ctx.smem_lo = stage0;
  ctx.smem_hi = stage2;
  ctx.q[0] = stage0;
  ctx.q[1] = stage1;
  ctx.q[2] = stage2;
  ctx.q[3] = stage3;
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

template <int BM, int BN, int WGM, int WGN, int LA, int LB, bool PERSIST = false, class Epi>
inline hipError_t launch_gemm_dma4(hipStream_t stream, const void *A, long lda, const void *B, long ldb, long Mg,
                                   long Ng, long K, int splits, const Epi &epi, int band = 4) {
  constexpr int BK = 64;  // splits are made of 64-deep blocks, as in launch_gemm_dma
  if (Mg <= 0 || Ng <= 0 || K < 0 || Mg % BM || Ng % BN || K % BK || splits < 1) return hipErrorInvalidValue;
  static_assert(4 * dma4_stage_bytes<BM, BN, Epi>() <= 160 * 1024, "tile does not fit the 160 KB of LDS");
  GemmShape g;
  g.A = A;
  g.B = B;
  g.lda = lda;
  g.ldb = ldb;
  g.bytesA = 2 * lda * (LA == ROWK ? Mg : K);
  g.bytesB = 2 * ldb * (LB == ROWK ? Ng : K);
  // one k block of a K-major operand must stay within a 32-bit scalar offset
  if ((LA == KROW && K * lda * 2 >= (1L << 31)) || (LB == KROW && K * ldb * 2 >= (1L << 31)) ||
      lda * 2 * BM >= (1L << 31) || ldb * 2 * BN >= (1L << 31))
    return hipErrorInvalidValue;
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
  if (PERSIST && grid > 256u) grid = 256u;  // one workgroup per compute unit
  hipLaunchKernelGGL((gemm_dma4_kernel<BM, BN, WGM, WGN, LA, LB, Epi, PERSIST>), dim3(grid), dim3(WGM * WGN * 64), 0,
                     stream, g, epi);
  return hipGetLastError();
}

}  // namespace rnnlm_dev
