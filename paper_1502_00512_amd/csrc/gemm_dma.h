// bf16 MFMA contraction with direct global->LDS loads (gfx950 global_load_lds_dwordx4).
//
// Same contract as gemm_kernel (C[m][n] = sum_k A(m,k) B(n,k), tile-padded operands, ROWK or KROW
// layouts, fused epilogues), different data path: operand tiles never pass through registers.  Each
// wave-level load deposits 64 lanes x 16 bytes as one contiguous kilobyte of LDS, so tiles are
// stored unpadded and bank conflicts are avoided by an XOR swizzle of the 16-byte chunk index, applied
// when choosing which global chunk a lane fetches and undone when fragments are read.  The two LDS
// stages are two separate arrays and the loop is unrolled by two, so the compiler can tell that the
// loads in flight into one stage do not alias the fragment reads from the other and does not wait
// for them until the barrier that ends the iteration.
#pragma once
#include "gemm.h"

namespace rnnlm_dev {

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *global_void_ptr;

// Swizzles, chosen for the 64 banks x 4 bytes of the gfx950 LDS (256 bytes per clock; measured: zero
// SQ_LDS_BANK_CONFLICT with these, half of all LDS cycles conflicting with a 32-bank choice).
// ROWK tile: rows of 128 bytes = 8 chunks of 16 bytes; a 16-byte fragment read is served 16 lanes
// (16 consecutive rows) per clock, which must cover all 16 chunk positions of a 256-byte bank line:
// physical chunk = logical ^ ((row >> 1) & 7).
// KROW tile: one row per k, ROWS*2 bytes; a transposing 8-byte read is served 32 lanes per clock =
// 4 k rows x 64 contiguous bytes, which must land in 4 distinct 64-byte bank groups:
// physical chunk = logical ^ (4 * (k & 3)) (a multiple of 4, so each 64-byte run stays contiguous).
__device__ inline int rowk_swz(int row) { return (row >> 1) & 7; }
__device__ inline int krow_swz(int k) { return (k & 3) << 2; }

// (Device pass only: the buffer-resource type does not exist for the host target, and a kernel template
// whose body fails to instantiate there loses its launch stub.)
#if defined(__HIP_DEVICE_COMPILE__)
// Loads go through a buffer resource (base + 32-bit per-lane offset + scalar offset): no 64-bit
// address arithmetic in the loop, one VGPR per load, and reads past the operand return zero instead
// of faulting.
template <int ROWS, int LAYOUT, int NT>
struct DmaLoader {
  static constexpr int BLOCKS = ROWS * 128 / 1024;  // kilobyte blocks per tile
  static constexpr int NW = NT / 64;
  static constexpr int PER = BLOCKS / NW;
  static_assert(BLOCKS % NW == 0, "tile does not divide over the waves");
  int off[PER];  // this lane's byte offset inside a k block for each of its kilobyte blocks
  __amdgpu_buffer_rsrc_t rsrc;
  int kstep;     // bytes to advance per k block

  // op: operand base; op_bytes: its extent; (row0, k0): first tile row and first k of this workgroup
  __device__ inline void init(const char *op, long op_bytes, long ld_bytes, long row0, long k0, int tid) {
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int q = (wave + i * NW) * 64 + lane;  // physical chunk index inside the tile
      if (LAYOUT == ROWK) {
        const int r = q >> 3, p = q & 7;
        off[i] = (int)(r * ld_bytes + ((p ^ rowk_swz(r)) << 4));
      } else {
        constexpr int CPR = ROWS / 8;
        const int k = q / CPR, p = q % CPR;
        off[i] = (int)(k * ld_bytes + ((p ^ krow_swz(k)) << 4));
      }
    }
    const long start = (LAYOUT == ROWK) ? row0 * ld_bytes + k0 * 2 : k0 * ld_bytes + row0 * 2;
    kstep = (LAYOUT == ROWK) ? 128 : (int)(64 * ld_bytes);
    const long left = op_bytes - start;
    const unsigned records = left > 0xffffffffL ? 0xffffffffu : (unsigned)left;
    rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(op + start), 0, (int)records, 0x00020000);
  }
  // issues the loads of k block kb (relative to the first) into `tile` (LDS)
  __device__ inline void issue(char *tile, int kb, int tid) const {
    const int wave = tid >> 6;
    const int soff = kb * kstep;
#pragma unroll
    for (int i = 0; i < PER; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)(tile + (wave + i * NW) * 1024), 16, off[i], soff, 0, 0);
  }
};

#endif  // __HIP_DEVICE_COMPILE__

// Fragment addressing.  A lane's byte offsets inside an operand tile are split into a per-lane part
// computed once (4 registers per operand) and compile-time parts that fold into the instruction's
// immediate offset, so the loop spends no VALU work on addresses.
//   ROWK: row r = r0 + 32 i, 16-wide step st: r*128 + ((2 st + h) ^ swz(r)) * 16 with h = lane / 32.
//         swz(r) does not depend on i (it uses row bits 1..3), so: pre[st] = r0*128 + (((2 st + h) ^ swz) << 4),
//         immediate = i * 4096.
//   KROW: transposing reads (see FragReader<bf16_t, ROWS, KROW> in gemm.h): source lane s of a 16-lane
//         block points at tile[k][n .. n+3], k = 16 st + 8 h + s/4 (+4 for the second read),
//         n = r0' + 32 i + 4 (s % 4); byte offset k*ROWS*2 + (((n >> 3) ^ swz(k)) << 4) + (n & 7)*2, and
//         swz(k) = 4 (s/4 & 3) is a per-lane constant: pre[i] = (8 h + s/4)*ROWS*2 + that chunk term,
//         immediate = st * 16 * ROWS * 2 (+ 4 * ROWS * 2).
template <int ROWS, int LAYOUT>
struct DmaFragAddr;
template <int ROWS>
struct DmaFragAddr<ROWS, ROWK> {
  int pre[4];
  __device__ inline void init(int r0, int lane) {  // r0: the lane's row in the wave's first 32-row block
    const int h = lane >> 5, sw = rowk_swz(r0);
#pragma unroll
    for (int st = 0; st < 4; ++st) pre[st] = r0 * 128 + (((2 * st + h) ^ sw) << 4);
  }
  __device__ inline bf16x8_t get(const char *tile, int i, int st) const {
    return *reinterpret_cast<const bf16x8_t *>(tile + pre[st] + i * 4096);
  }
};
template <int ROWS>
struct DmaFragAddr<ROWS, KROW> {
  int pre[4];
  __device__ inline void init(int r0, int lane) {
    const int h = lane >> 5, s = lane & 15;
    const int k = 8 * h + (s >> 2);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = (r0 - s) + 32 * i + 4 * (s & 3);
      pre[i] = k * (ROWS * 2) + ((((n >> 3) ^ krow_swz(k)) << 4) | ((n & 7) << 1));
    }
  }
  __device__ inline bf16x8_t get(const char *tile, int i, int st) const {
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4_t *lds_ptr_t;
    const char *p = tile + pre[i] + st * (16 * ROWS * 2);
    union {
      s16x4_t hh[2];
      bf16x8_t f;
    } u;
    u.hh[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    u.hh[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * ROWS * 2));
    return u.f;
  }
};

template <int BM, int BN, class Epi>
constexpr int dma_stage_bytes() {
  constexpr int loop = (BM + BN) * 128;
  constexpr int epi = Epi::template lds_bytes<BM, BN>() / 2;
  return loop > epi ? loop : epi;
}

// PERSIST: the grid is one workgroup per compute unit and each walks the work items id, id + grid, ... (the
// grid is a multiple of 8, so a workgroup stays on the XCD whose chunk of tiles it walks): the next tile's
// first loads are issued while the previous tile's stores drain, and no workgroup is relaunched per tile.
template <int BM, int BN, int WGM, int WGN, int LA, int LB, class Epi, bool PERSIST = false>
__global__ void __launch_bounds__(WGM *WGN * 64) gemm_dma_kernel(const GemmShape g, const Epi epi) {
#if defined(__HIP_DEVICE_COMPILE__)
  constexpr int NT = WGM * WGN * 64;
  constexpr int BK = 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int SBYTES = dma_stage_bytes<BM, BN, Epi>();
  __shared__ __attribute__((aligned(1024))) char stage0[SBYTES];
  __shared__ __attribute__((aligned(1024))) char stage1[SBYTES];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int nwork = g.perXcd * NUM_XCD;
  for (int wid = blockIdx.x; wid < nwork; wid += PERSIST ? (int)gridDim.x : nwork) {
  int tile_m, tile_n, split;
  if (!map_workgroup(g, wid, split, tile_m, tile_n)) continue;  // uniform for the workgroup
  const int kb0 = split * g.kBlocksPerSplit;
  const int kb1 = min(kb0 + g.kBlocksPerSplit, g.kBlocks);
  const int nk = kb1 - kb0;

  f32x16_t acc[TM][TN];
  epi.template init<TM, TN>(acc, tile_m * BM + wm * WTM, tile_n * BN + wn * WTN, lane, split);

  DmaLoader<BM, LA, NT> la;
  DmaLoader<BN, LB, NT> lb;
  la.init(static_cast<const char *>(g.A), g.bytesA, g.lda * 2, (long)tile_m * BM, (long)kb0 * BK, tid);
  lb.init(static_cast<const char *>(g.B), g.bytesB, g.ldb * 2, (long)tile_n * BN, (long)kb0 * BK, tid);
  const int lr = lane & 31;

  // tile index is clamped to the last one: the final iterations re-fetch it instead of branching
  auto fetch = [&](char *stage, int kb) {
    kb = min(kb, nk - 1);
    la.issue(stage, kb, tid);
    lb.issue(stage + BM * 128, kb, tid);
  };
  // Software pipeline over the four 16-wide steps of a tile, with fragments double buffered in
  // registers: the reads of step k+1 are issued before the MFMAs of step k.  The barrier that
  // publishes the next tile sits BEFORE the last step's MFMAs, and the next tile's first fragments
  // are read right after it, so their LDS latency is covered by those MFMAs instead of stalling the
  // start of the next iteration.
  static_assert(TM <= 4 && TN <= 4, "fragment addressing covers up to four 32-row blocks per wave");
  bf16x8_t fa[2][TM], fb[2][TN];
  DmaFragAddr<BM, LA> addr_a;
  DmaFragAddr<BN, LB> addr_b;
  addr_a.init(wm * WTM + lr, lane);
  addr_b.init(wn * WTN + lr, lane);
  auto read_frags = [&](const char *stage, int step, int buf) {
    const char *sa = stage;
    const char *sb = stage + BM * 128;
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[buf][i] = addr_a.get(sa, i, step);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[buf][j] = addr_b.get(sb, j, step);
  };
  // MFMA clusters run at raised wave priority so that, of the two waves sharing a SIMD, the one with
  // operands ready wins the issue slot over the one still issuing loads.
  auto mfmas = [&](int buf) {
    __builtin_amdgcn_s_setprio(3);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) mma16(acc[i][j], fa[buf][i], fb[buf][j]);
    __builtin_amdgcn_s_setprio(0);
  };
  constexpr int KSTEPS = BK / 16;
  // steps 0 .. KSTEPS-2 of the tile in `stage` (its step-0 fragments are already in buffer 0)
  auto head_steps = [&](const char *stage) {
#pragma unroll
    for (int step = 0; step + 1 < KSTEPS; ++step) {
      read_frags(stage, step + 1, (step + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);
      mfmas(step & 1);
    }
  };
  // last step of the current tile, overlapped with the first fragment reads of the tile in `next`
  // (read unconditionally: after the last tile they fetch stale but in-bounds LDS and are unused)
  auto tail_step = [&](const char *next) {
    read_frags(next, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfmas((KSTEPS - 1) & 1);
  };

  if (nk > 0) {
    fetch(stage0, 0);
    __syncthreads();  // waits for this wave's loads, then for everyone's
    read_frags(stage0, 0, 0);
#pragma unroll 1
    for (int it = 0; it < nk; it += 2) {
      fetch(stage1, it + 1);
      head_steps(stage0);
      __syncthreads();  // tile it+1 has landed; every wave has finished reading stage0
      tail_step(stage1);
      if (it + 1 < nk) {
        fetch(stage0, it + 2);
        head_steps(stage1);
        __syncthreads();
        tail_step(stage0);
      }
    }
  }
  __syncthreads();  // all loads have landed and all fragment reads are done: the epilogue reuses both stages
  EpiCtx ctx;
  ctx.smem_lo = stage0;
  ctx.smem_hi = stage1;
  ctx.q[0] = stage0;
  ctx.q[1] = stage0 + (BM / 4) * StageGeom<BN>::PITCH;
  ctx.q[2] = stage1;
  ctx.q[3] = stage1 + (BM / 4) * StageGeom<BN>::PITCH;
  ctx.tile_row0 = tile_m * BM;
  ctx.tile_col0 = tile_n * BN;
  ctx.wrow = wm * WTM;
  ctx.wcol = wn * WTN;
  ctx.lane = lane;
  ctx.tid = tid;
  ctx.split = split;
  epi.template run<BM, BN, TM, TN, NT>(acc, ctx);
  if (PERSIST) {
    // the epilogue's LDS reads have returned (lgkmcnt 0; its global stores may still be in flight: vmcnt and
    // expcnt are left alone) before anyone's next loads overwrite the stages
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();
  }
  }
#endif  // __HIP_DEVICE_COMPILE__
}

template <int BM, int BN, int WGM, int WGN, int LA, int LB, bool PERSIST = false, class Epi>
inline hipError_t launch_gemm_dma(hipStream_t stream, const void *A, long lda, const void *B, long ldb, long Mg,
                                  long Ng, long K, int splits, const Epi &epi, int band = 4) {
  constexpr int BK = 64;
  if (Mg <= 0 || Ng <= 0 || K < 0 || Mg % BM || Ng % BN || K % BK || splits < 1) return hipErrorInvalidValue;
  static_assert(2 * dma_stage_bytes<BM, BN, Epi>() <= 160 * 1024, "tile does not fit the 160 KB of LDS");
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
  hipLaunchKernelGGL((gemm_dma_kernel<BM, BN, WGM, WGN, LA, LB, Epi, PERSIST>), dim3(grid), dim3(WGM * WGN * 64), 0,
                     stream, g, epi);
  return hipGetLastError();
}

}  // namespace rnnlm_dev
