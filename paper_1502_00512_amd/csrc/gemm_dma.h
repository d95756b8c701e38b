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

template <int ROWS, int LAYOUT, int NT>
struct DmaLoader {
  static constexpr int BLOCKS = ROWS * 128 / 1024;  // kilobyte blocks per tile
  static constexpr int NW = NT / 64;
  static constexpr int PER = BLOCKS / NW;
  static_assert(BLOCKS % NW == 0, "tile does not divide over the waves");
  const char *gp[PER];  // this lane's global source of each of its blocks, at k block 0
  long kstep;           // bytes to advance per k block

  __device__ inline void init(const char *base, long ld_bytes, long row0, long k0, int tid) {
    const int wave = tid >> 6, lane = tid & 63;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int q = (wave + i * NW) * 64 + lane;  // physical chunk index inside the tile
      if (LAYOUT == ROWK) {
        const int r = q >> 3, p = q & 7;
        gp[i] = base + (row0 + r) * ld_bytes + k0 * 2 + ((p ^ rowk_swz(r)) << 4);
      } else {
        constexpr int CPR = ROWS / 8;
        const int k = q / CPR, p = q % CPR;
        gp[i] = base + (k0 + k) * ld_bytes + row0 * 2 + ((p ^ krow_swz(k)) << 4);
      }
    }
    kstep = (LAYOUT == ROWK) ? 128 : 64 * ld_bytes;
  }
  // issues the loads of the next k block into `tile` (LDS) and advances
  __device__ inline void issue(char *tile, int tid) {
    const int wave = tid >> 6;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      __builtin_amdgcn_global_load_lds((global_void_ptr)gp[i], (lds_void_ptr)(tile + (wave + i * NW) * 1024), 16, 0, 0);
      gp[i] += kstep;
    }
  }
};

template <int ROWS, int LAYOUT>
struct DmaFragReader;
template <int ROWS>
struct DmaFragReader<ROWS, ROWK> {
  // 8 consecutive-k elements of tile row r starting at k offset ks (a multiple of 8)
  __device__ static inline bf16x8_t get(const char *tile, int r, int ks) {
    return *reinterpret_cast<const bf16x8_t *>(tile + r * 128 + (((ks >> 3) ^ rowk_swz(r)) << 4));
  }
};
template <int ROWS>
struct DmaFragReader<ROWS, KROW> {
  // transposing reads, see FragReader<bf16_t, ROWS, KROW>: source lane s of a 16-lane block points at
  // tile[ks + s/4][r0 + 4*(s%4) .. +3]
  __device__ static inline bf16x8_t get(const char *tile, int r, int ks) {
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4_t *lds_ptr_t;
    const int lane = threadIdx.x & 63;
    const int s = lane & 15;
    const int k = ks + (s >> 2);
    const int n = (r - s) + 4 * (s & 3);
    const char *p = tile + k * (ROWS * 2) + ((((n >> 3) ^ krow_swz(k)) << 4) | ((n & 7) << 1));
    union {
      s16x4_t h[2];
      bf16x8_t f;
    } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * ROWS * 2));
    return u.f;
  }
};

template <int BM, int BN, class Epi>
constexpr int dma_stage_bytes() {
  constexpr int loop = (BM + BN) * 128;
  constexpr int epi = Epi::template lds_bytes<BM, BN>() / 2;
  return loop > epi ? loop : epi;
}

template <int BM, int BN, int WGM, int WGN, int LA, int LB, class Epi>
__global__ void __launch_bounds__(WGM *WGN * 64) gemm_dma_kernel(const GemmShape g, const Epi epi) {
  constexpr int NT = WGM * WGN * 64;
  constexpr int BK = 64;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int SBYTES = dma_stage_bytes<BM, BN, Epi>();
  __shared__ __attribute__((aligned(1024))) char stage0[SBYTES];
  __shared__ __attribute__((aligned(1024))) char stage1[SBYTES];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  int tile_m, tile_n, split;
  if (!map_workgroup(g, blockIdx.x, split, tile_m, tile_n)) return;  // uniform for the workgroup
  const int kb0 = split * g.kBlocksPerSplit;
  const int kb1 = min(kb0 + g.kBlocksPerSplit, g.kBlocks);
  const int nk = kb1 - kb0;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  DmaLoader<BM, LA, NT> la;
  DmaLoader<BN, LB, NT> lb;
  la.init(static_cast<const char *>(g.A), g.lda * 2, (long)tile_m * BM, (long)kb0 * BK, tid);
  lb.init(static_cast<const char *>(g.B), g.ldb * 2, (long)tile_n * BN, (long)kb0 * BK, tid);
  const int lr = lane & 31, lk = (lane >> 5) * 8;

  auto fetch = [&](char *stage) {
    la.issue(stage, tid);
    lb.issue(stage + BM * 128, tid);
  };
  auto multiply = [&](const char *stage) {
    const char *sa = stage;
    const char *sb = stage + BM * 128;
    bf16x8_t fa[2][TM], fb[2][TN];
    auto read_frags = [&](int step, int buf) {
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[buf][i] = DmaFragReader<BM, LA>::get(sa, wm * WTM + i * 32 + lr, step * 16 + lk);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[buf][j] = DmaFragReader<BN, LB>::get(sb, wn * WTN + j * 32 + lr, step * 16 + lk);
    };
    read_frags(0, 0);
#pragma unroll
    for (int step = 0; step < BK / 16; ++step) {
      if (step + 1 < BK / 16) read_frags(step + 1, (step + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);  // keep the next step's LDS reads ahead of this step's MFMAs
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) mma16(acc[i][j], fa[step & 1][i], fb[step & 1][j]);
    }
  };

  if (nk > 0) {
    fetch(stage0);
    __syncthreads();  // waits for this wave's loads, then for everyone's
  }
  for (int it = 0; it < nk; it += 2) {
    if (it + 1 < nk) fetch(stage1);
    multiply(stage0);
    __syncthreads();
    if (it + 1 < nk) {
      if (it + 2 < nk) fetch(stage0);
      multiply(stage1);
      __syncthreads();
    }
  }
  EpiCtx ctx;
  ctx.smem_lo = stage0;
  ctx.smem_hi = stage1;
  ctx.tile_row0 = tile_m * BM;
  ctx.tile_col0 = tile_n * BN;
  ctx.wrow = wm * WTM;
  ctx.wcol = wn * WTN;
  ctx.lane = lane;
  ctx.tid = tid;
  ctx.split = split;
  epi.template run<BM, BN, TM, TN, NT>(acc, ctx);
}

template <int BM, int BN, int WGM, int WGN, int LA, int LB, class Epi>
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
  hipLaunchKernelGGL((gemm_dma_kernel<BM, BN, WGM, WGN, LA, LB, Epi>), dim3((unsigned)(g.perXcd * NUM_XCD)),
                     dim3(WGM * WGN * 64), 0, stream, g, epi);
  return hipGetLastError();
}

}  // namespace rnnlm_dev
