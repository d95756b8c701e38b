// MFMA contraction kernel for gfx950 and the fused epilogues of the RNNLM step.
//
// C[m][n] = sum_k A(m,k) * B(n,k), both operands in tile-padded buffers (no bounds checks in the
// main loop).  Each operand is stored either K-contiguous ("ROWK": [rows][K]) or row-contiguous
// ("KROW": [K][rows]); the kernel stages 128-byte-deep K tiles of both through LDS (double
// buffered, global loads for tile i+1 in flight while tile i is multiplied) and feeds
// v_mfma_f32_32x32x16_bf16 (bf16 operands) or v_mfma_f32_32x32x2_f32 (fp32 operands), always with
// fp32 accumulation.  One workgroup owns a BM x BN tile; its WGM x WGN waves own sub-tiles made of
// 32x32 MFMA blocks.
#pragma once
#include "common.h"

namespace rnnlm_dev {

enum : int { ROWK = 0, KROW = 1 };

struct GemmShape {
  const void *A, *B;
  long lda, ldb;        // leading dimensions in elements
  long bytesA, bytesB;  // extents of the operands (used by the buffer-resource loads)
  int tilesM, tilesN;   // output tiles
  int kBlocks;          // K / BK
  int kBlocksPerSplit;  // K blocks handled by one split
  int splits;
  // Workgroup -> (split, tile) mapping.  Workgroups are dealt to the 8 XCDs (each with its own L2)
  // round-robin by id, so id % 8 picks a contiguous chunk of `perXcd` work items and id / 8 walks it:
  // neighbours in that walk run on one XCD at about the same time and share operand panels in its
  // L2.  Inside a split, tiles are walked in bands of `band` tile rows (bandOverN = 0) or tile
  // columns (bandOverN = 1), the other index running fastest.
  int perXcd, band, bandOverN;
};

constexpr int NUM_XCD = 8;

__device__ inline bool map_workgroup(const GemmShape &g, int id, int &split, int &tile_m, int &tile_n) {
  const int tiles = g.tilesM * g.tilesN;
  const int lin = (id % NUM_XCD) * g.perXcd + id / NUM_XCD;
  if (id / NUM_XCD >= g.perXcd || lin >= tiles * g.splits) return false;
  split = lin / tiles;
  const int t = lin % tiles;
  const int major = g.bandOverN ? g.tilesN : g.tilesM;  // banded index
  const int minor = g.bandOverN ? g.tilesM : g.tilesN;
  const int perBand = g.band * minor;
  const int b = t / perBand, r = t % perBand;
  const int width = min(g.band, major - b * g.band);
  const int imajor = b * g.band + r % width, iminor = r / width;
  tile_m = g.bandOverN ? iminor : imajor;
  tile_n = g.bandOverN ? imajor : iminor;
  return true;
}

// KBYTES = bytes of K held by one LDS tile row (128 or 64): BK = KBYTES / sizeof(T) elements.
template <typename T, int ROWS, int LAYOUT, int KBYTES>
struct TileGeom {
  static constexpr int ES = sizeof(T);
  static constexpr int BK = KBYTES / ES;
  static constexpr int ROWK_STRIDE = KBYTES + 16;     // +16 B: 16-byte reads of 8 consecutive rows hit distinct banks
  static constexpr int KROW_STRIDE = ROWS * ES + 64;  // +64 B: the 4 k rows x 64 B that a transposing read touches per clock hit distinct banks
  static constexpr int BYTES = (LAYOUT == ROWK) ? ROWS * ROWK_STRIDE : BK * KROW_STRIDE;
};

// Moves one ROWS x BK operand tile global -> registers -> LDS in 16-byte pieces.
template <typename T, int ROWS, int LAYOUT, int NT, int KBYTES>
struct TileLoader {
  using G = TileGeom<T, ROWS, LAYOUT, KBYTES>;
  static constexpr int CPK = KBYTES / 16;  // 16-byte chunks along K per tile row
  static constexpr int CHUNKS = ROWS * CPK;
  static constexpr int PER = CHUNKS / NT;
  static_assert(CHUNKS % NT == 0, "tile does not divide over the workgroup");
  u32x4_t regs[PER];

  __device__ inline void load(const char *base, long ld_bytes, long row0, long k0, int tid) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid + i * NT;
      const char *p;
      if (LAYOUT == ROWK) {
        const int r = c / CPK, kc = c % CPK;
        p = base + (row0 + r) * ld_bytes + k0 * G::ES + kc * 16;
      } else {
        constexpr int CPR = ROWS * G::ES / 16;
        const int kk = c / CPR, mc = c % CPR;
        p = base + (k0 + kk) * ld_bytes + row0 * G::ES + mc * 16;
      }
      regs[i] = *reinterpret_cast<const u32x4_t *>(p);
    }
  }
  __device__ inline void store(char *tile, int tid) const {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid + i * NT;
      int off;
      if (LAYOUT == ROWK) {
        off = (c / CPK) * G::ROWK_STRIDE + (c % CPK) * 16;
      } else {
        constexpr int CPR = ROWS * G::ES / 16;
        off = (c / CPR) * G::KROW_STRIDE + (c % CPR) * 16;
      }
      *reinterpret_cast<u32x4_t *>(tile + off) = regs[i];
    }
  }
};

struct F32x8 {
  float v[8];
};
template <typename T>
struct FragT;
template <>
struct FragT<bf16_t> {
  typedef bf16x8_t type;
};
template <>
struct FragT<float> {
  typedef F32x8 type;
};

// FragReader::get returns the 8 consecutive-k elements of tile row r starting at k offset ks (a
// multiple of 8).
template <typename T, int ROWS, int LAYOUT, int KBYTES>
struct FragReader;

template <int ROWS, int KBYTES>
struct FragReader<bf16_t, ROWS, ROWK, KBYTES> {
  __device__ static inline bf16x8_t get(const char *tile, int r, int ks) {
    return *reinterpret_cast<const bf16x8_t *>(tile + r * (KBYTES + 16) + ks * 2);
  }
};
// K-major bf16 tile: ds_read_b64_tr_b16 transposes on the way out of LDS.  Within each block of 16
// lanes, source lane s points at 4 row-contiguous elements and destination lane i receives element
// i%4 of source lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4 (layout measured on gfx950).  Pointing source lane s
// at tile[kb + s/4][r0 + 4*(s%4)] therefore hands lane i the four k-consecutive values
// tile[kb .. kb+3][r0 + i]: two such reads give the 8 values an MFMA operand lane needs.
template <int ROWS, int KBYTES>
struct FragReader<bf16_t, ROWS, KROW, KBYTES> {
  __device__ static inline bf16x8_t get(const char *tile, int r, int ks) {
    constexpr int S = TileGeom<bf16_t, ROWS, KROW, KBYTES>::KROW_STRIDE;
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4_t *lds_ptr_t;
    const int lane = threadIdx.x & 63;
    const int s = lane & 15;
    // r = tile row of this lane; its 16-lane block starts at row r - s
    const char *p = tile + (ks + (s >> 2)) * S + ((r - s) + 4 * (s & 3)) * 2;
    union {
      s16x4_t h[2];
      bf16x8_t f;
    } u;
    u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p));
    u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * S));
    return u.f;
  }
};
template <int ROWS, int KBYTES>
struct FragReader<float, ROWS, ROWK, KBYTES> {
  __device__ static inline F32x8 get(const char *tile, int r, int ks) {
    F32x8 f;
    const f32x4_t a = *reinterpret_cast<const f32x4_t *>(tile + r * (KBYTES + 16) + ks * 4);
    const f32x4_t b = *reinterpret_cast<const f32x4_t *>(tile + r * (KBYTES + 16) + ks * 4 + 16);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f.v[e] = a[e];
      f.v[4 + e] = b[e];
    }
    return f;
  }
};
template <int ROWS, int KBYTES>
struct FragReader<float, ROWS, KROW, KBYTES> {
  __device__ static inline F32x8 get(const char *tile, int r, int ks) {
    constexpr int S = TileGeom<float, ROWS, KROW, KBYTES>::KROW_STRIDE;
    F32x8 f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f.v[e] = *reinterpret_cast<const float *>(tile + (ks + e) * S + r * 4);
    return f;
  }
};

// One 32x32 block update over 16 values of k.  Lane l holds row/col (l & 31) and the 8 k values
// 8*(l >> 5) .. +7 of both operands.  fp32: the e-th 32x32x2 instruction contracts k = e (lanes
// 0-31) and k = 8 + e (lanes 32-63), so eight of them cover the same 16 values.
__device__ inline void mma16(f32x16_t &acc, const bf16x8_t &a, const bf16x8_t &b) {
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}
__device__ inline void mma16(f32x16_t &acc, const F32x8 &a, const F32x8 &b) {
#pragma unroll
  for (int e = 0; e < 8; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[e], b.v[e], acc, 0, 0, 0);
}

// Pitch (bytes) of the bf16 staging tile: 144 dwords = 16 (mod 64), so the two rows and two
// half-waves of one staged write land in distinct banks.
template <int BN>
struct StageGeom {
  static constexpr int PITCH = BN * 2 + 64;
};

// Start value of the accumulators.  Every epilogue provides init<TM, TN>(acc, row0, col0, lane, split),
// called before the main loop with the origin of the wave's sub-tile in C; the default is zero.
struct EpiZeroInit {
  template <int TM, int TN>
  __device__ inline void init(f32x16_t (&acc)[TM][TN], int, int, int, int) const {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;
  }
};

// What an epilogue sees: the workgroup's LDS (reusable: the main loop ends with a barrier), the
// origin of the workgroup tile in C, the origin of this wave's sub-tile inside it, and ids.
struct EpiCtx {
  char *smem_lo, *smem_hi;  // LDS for staging the upper / lower half of the tile's rows
  char *q[4];               // the same LDS seen as four regions, one per quarter of the tile's rows
  int tile_row0, tile_col0;
  int wrow, wcol;
  int lane, tid, split;
};

// PF = tiles of global loads in flight ahead of the tile being multiplied (1 or 2).  With PF = 2 the
// loads of tile i+2 are issued before tile i is multiplied and land in LDS one iteration later, which
// covers about two multiply phases of memory latency.
template <typename T, int BM, int BN, int WGM, int WGN, int LA, int LB, class Epi, int KBYTES, int MINWG, int PF>
__global__ void __launch_bounds__(WGM *WGN * 64, MINWG) gemm_kernel(const GemmShape g, const Epi epi) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int NT = WGM * WGN * 64;
  constexpr int ES = sizeof(T);
  constexpr int BK = KBYTES / ES;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 blocks");
  using GA = TileGeom<T, BM, LA, KBYTES>;
  using GB = TileGeom<T, BN, LB, KBYTES>;
  constexpr int STAGE = GA::BYTES + GB::BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  int tile_m, tile_n, split;
  if (!map_workgroup(g, blockIdx.x, split, tile_m, tile_n)) return;  // uniform for the workgroup
  const int kb0 = split * g.kBlocksPerSplit;
  const int kb1 = min(kb0 + g.kBlocksPerSplit, g.kBlocks);
  const int nk = kb1 - kb0;

  f32x16_t acc[TM][TN];
  epi.template init<TM, TN>(acc, tile_m * BM + wm * WTM, tile_n * BN + wn * WTN, lane, split);

  TileLoader<T, BM, LA, NT, KBYTES> la[PF];
  TileLoader<T, BN, LB, NT, KBYTES> lb[PF];
  const char *Ab = static_cast<const char *>(g.A);
  const char *Bb = static_cast<const char *>(g.B);
  const long lda_b = g.lda * ES, ldb_b = g.ldb * ES;
  const long arow0 = (long)tile_m * BM, brow0 = (long)tile_n * BN;
  const int lr = lane & 31, lk = (lane >> 5) * 8;

  // one multiply phase on the LDS stage `it & 1`: operand fragments are double buffered so that the
  // LDS reads of 16-wide step k+1 are in flight while the MFMAs of step k issue
  auto multiply = [&](int it) {
    const char *sa = smem + (it & 1) * STAGE;
    const char *sb = sa + GA::BYTES;
    constexpr int KSTEPS = BK / 16;
    typename FragT<T>::type fa[2][TM], fb[2][TN];
    auto read_frags = [&](int step, int buf) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
        fa[buf][i] = FragReader<T, BM, LA, KBYTES>::get(sa, wm * WTM + i * 32 + lr, step * 16 + lk);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        fb[buf][j] = FragReader<T, BN, LB, KBYTES>::get(sb, wn * WTN + j * 32 + lr, step * 16 + lk);
    };
    read_frags(0, 0);
#pragma unroll
    for (int step = 0; step < KSTEPS; ++step) {
      if (step + 1 < KSTEPS) read_frags(step + 1, (step + 1) & 1);
      __builtin_amdgcn_sched_barrier(0);  // keep the next step's LDS reads ahead of this step's MFMAs
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) mma16(acc[i][j], fa[step & 1][i], fb[step & 1][j]);
    }
  };
  // tile j travels through register set j % PF and LDS stage j & 1
  auto fetch = [&](int j, int set) {
    la[set].load(Ab, lda_b, arow0, (long)(kb0 + j) * BK, tid);
    lb[set].load(Bb, ldb_b, brow0, (long)(kb0 + j) * BK, tid);
  };
  auto land = [&](int j, int set) {
    char *d = smem + (j & 1) * STAGE;
    la[set].store(d, tid);
    lb[set].store(d + GA::BYTES, tid);
  };

  if (nk > 0) {
    fetch(0, 0);
    land(0, 0);
    if (PF == 2) {
      if (nk > 1) fetch(1, 1 % PF);
    }
    __syncthreads();
  }
  if (PF == 1) {
    for (int it = 0; it < nk; ++it) {
      const bool more = it + 1 < nk;
      if (more) fetch(it + 1, 0);
      multiply(it);
      if (more) land(it + 1, 0);
      __syncthreads();
    }
  } else {
    // unrolled by two so that register sets are addressed statically
    for (int it = 0; it < nk; it += 2) {
      if (it + 2 < nk) fetch(it + 2, 0);
      multiply(it);
      if (it + 1 < nk) land(it + 1, 1 % PF);
      __syncthreads();
      if (it + 1 < nk) {
        if (it + 3 < nk) fetch(it + 3, 1 % PF);
        multiply(it + 1);
        if (it + 2 < nk) land(it + 2, 0);
        __syncthreads();
      }
    }
  }
  EpiCtx ctx;
  ctx.smem_lo = smem;
  ctx.smem_hi = smem + (BM / 2) * StageGeom<BN>::PITCH;
#pragma unroll
  for (int qi = 0; qi < 4; ++qi) ctx.q[qi] = smem + qi * (BM / 4) * StageGeom<BN>::PITCH;
  ctx.tile_row0 = tile_m * BM;
  ctx.tile_col0 = tile_n * BN;
  ctx.wrow = wm * WTM;
  ctx.wcol = wn * WTN;
  ctx.lane = lane;
  ctx.tid = tid;
  ctx.split = split;
  epi.template run<BM, BN, TM, TN, NT>(acc, ctx);
}

// LDS region of quarter qi of the tile's rows (a select chain: indexing the pointer array with a run-time
// value would move it to scratch memory).
__device__ inline char *quarter_ptr(const EpiCtx &c, int qi) {
  return qi == 0 ? c.q[0] : (qi == 1 ? c.q[1] : (qi == 2 ? c.q[2] : c.q[3]));
}

// Accumulator element r (0..15) of a 32x32 block lives at row 8*(r/4) + 4*(lane/32) + r%4,
// column lane%32.
#define RNNLM_ACC_ROW(r, lane) ((((r) >> 2) << 3) + (((lane) >> 5) << 2) + ((r)&3))

// ---- Tile store helpers --------------------------------------------------------------------------


// Writes the workgroup's BM x BN tile of values (already final, in MFMA accumulator layout) to
// out[row][col] (leading dimension ld, no bounds: the caller's buffer is tile-padded).
// fp32: direct stores, 32 lanes cover 128 contiguous bytes of a row.
template <int BM, int BN, int TM, int TN, int NT>
__device__ inline void store_tile(const f32x16_t (&val)[TM][TN], const EpiCtx &c, float *out, long ld) {
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const long col = c.tile_col0 + c.wcol + j * 32 + (c.lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const long row = c.tile_row0 + c.wrow + i * 32 + RNNLM_ACC_ROW(r, c.lane);
        out[row * ld + col] = val[i][j][r];
      }
    }
}
// bf16: a lane holds one column and runs of 4 consecutive rows.  Neighbouring lanes swap one packed
// pair so that each lane owns two adjacent columns of one row (one dword), the tile is assembled in
// LDS (which the main loop no longer needs; four regions, one per quarter of the rows) and leaves as
// 16-byte row-contiguous stores, marked nontemporal: the tile is hundreds of megabytes per launch, is read
// once by the next kernel, and ordinary stores cost the contraction 6 % (they displace the operand panels
// the other workgroups of the XCD are re-reading from its L2).
template <int BM, int BN, int TM, int TN, int NT>
__device__ inline void store_tile(const f32x16_t (&val)[TM][TN], const EpiCtx &c, bf16_t *out, long ld) {
  constexpr int PITCH = StageGeom<BN>::PITCH;
  constexpr int QR = BM / 4;  // rows per LDS region
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const bool odd = c.lane & 1;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    // with at least 32 rows per region a 32-row block lies in one region: its base is uniform for the wave
    const int blk = c.wrow + i * 32;
    char *blk_base = quarter_ptr(c, blk / QR) + (blk % QR) * PITCH;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = c.wcol + j * 32 + (c.lane & 31);
#pragma unroll
      for (int q = 0; q < 8; ++q) {  // rows 2q, 2q+1 of this lane's 16
        const int r0 = 2 * q;
        union {
          bf16x2_t h;
          unsigned u;
        } pk;
        pk.h[0] = (bf16_t)val[i][j][r0];
        pk.h[1] = (bf16_t)val[i][j][r0 + 1];
        const unsigned mine = pk.u;
        const unsigned theirs = (unsigned)__builtin_amdgcn_mov_dpp((int)mine, 0xB1, 0xF, 0xF, true);  // lane ^ 1
        const unsigned word = odd ? ((theirs >> 16) | (mine & 0xffff0000u)) : ((mine & 0xffffu) | (theirs << 16));
        const int rin = RNNLM_ACC_ROW(r0, c.lane) + (odd ? 1 : 0);  // row inside the 32-row block
        if constexpr (QR >= 32) {
          *reinterpret_cast<unsigned *>(blk_base + rin * PITCH + (col & ~1) * 2) = word;
        } else {
          const int row = blk + rin;
          *reinterpret_cast<unsigned *>(quarter_ptr(c, row / QR) + (row % QR) * PITCH + (col & ~1) * 2) = word;
        }
      }
    }
  }
  __syncthreads();
  constexpr int CPR = BN * 2 / 16;  // 16-byte chunks per row
  constexpr int RPI = NT / CPR;     // rows the workgroup moves per iteration
  if constexpr (NT % CPR == 0 && QR % RPI == 0 && BM % RPI == 0) {
    // an iteration's rows lie in one region, known at compile time once the loop is unrolled
    const int r_lo = c.tid / CPR, ch = c.tid % CPR;
#pragma unroll
    for (int k = 0; k < BM / RPI; ++k) {
      const int row = k * RPI + r_lo;
      const char *quarter = c.q[(k * RPI) / QR];
      const u32x4_t v = *reinterpret_cast<const u32x4_t *>(quarter + ((k * RPI) % QR + r_lo) * PITCH + ch * 16);
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(out + (long)(c.tile_row0 + row) * ld + c.tile_col0 + ch * 8));
    }
  } else {
#pragma unroll 4
    for (int idx = c.tid; idx < BM * CPR; idx += NT) {
      const int row = idx / CPR, ch = idx % CPR;
      const char *quarter = quarter_ptr(c, row / QR);
      const u32x4_t v = *reinterpret_cast<const u32x4_t *>(quarter + (row % QR) * PITCH + ch * 16);
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t *>(out + (long)(c.tile_row0 + row) * ld + c.tile_col0 + ch * 8));
    }
  }
}
template <typename T, int BM, int BN>
constexpr int stage_lds_bytes() {
  return sizeof(T) == 2 ? BM * StageGeom<BN>::PITCH : 0;
}

// ---- Epilogues ---------------------------------------------------------------------------------
// Each provides run<BM, BN, TM, TN, NT>(acc, ctx), executed by every thread of the workgroup after
// the main loop's final barrier (so LDS may be reused and barriers are allowed), and
// lds_bytes<BM, BN>() = LDS it needs.

// Recurrent forward step (Sec. 4.1): h = sigmoid(X + Hprev U^T).  Rows = streams, cols = units.
template <typename T>
struct EpiRnnFwd : EpiZeroInit {
  const float *X;   // [Bp][ld]  gathered embedding rows of this timestep
  T *Hnext;         // [Bp][ld]  hidden state slot of this timestep (padding written as zero)
  float *h_state;   // [B][H] or nullptr: carried state, written at the window's last step
  int B, H, ld;
  template <int BM, int BN>
  static constexpr int lds_bytes() { return 0; }
  template <int BM, int BN, int TM, int TN, int NT>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], const EpiCtx &c) const {
    const int row0 = c.tile_row0 + c.wrow, col0 = c.tile_col0 + c.wcol, lane = c.lane;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = col0 + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
          const bool ok = row < B && col < H;
          float hval = 0.0f;
          if (ok) hval = sigmoidf_(acc[i][j][r] + X[(long)row * ld + col]);
          Hnext[(long)row * ld + col] = from_f32<T>(hval);
          if (ok && h_state) h_state[(long)row * H + col] = hval;
        }
      }
  }
};

// Output layer forward: z[v][m] = Wo[v] . h[m] + b[v] (rows = vocabulary, cols = window positions),
// stored vocabulary-major for the softmax pass and both gradient contractions, plus per-(wave row
// block, position) partial (max, sum exp) statistics of the fp32 logits and the fp32 logit of each
// position's target word.  A lane owns one position (column), so its statistics need no cross-lane
// traffic except one exchange between the two half-waves.
template <typename T>
struct EpiOutFwd : EpiZeroInit {
  const float *b;   // [V]
  T *ZT;            // [Vp][ldz]
  float2 *part;     // [Vp / BM][ldz]: one (max, sum exp) per tile row block and position
  const int *yp;    // [Mp] target id per position, -1 on padding
  float *zy;        // [Mp] target logit
  int V;
  long ldz;
  template <int BM, int BN>
  static constexpr int lds_bytes() {
    return stage_lds_bytes<T, BM, BN>() > 8 * BN * 8 ? stage_lds_bytes<T, BM, BN>() : 8 * BN * 8;
  }
  // The accumulators start at the bias of their vocabulary row (0 for rows >= V): the bias costs neither
  // an addition per logit nor a load whose latency the epilogue would have to wait for.  The contraction
  // is never split for this epilogue.
  template <int TM, int TN>
  __device__ inline void init(f32x16_t (&acc)[TM][TN], int row0, int, int lane, int) const {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int v = row0 + i * 32 + 8 * g + ((lane >> 5) << 2);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float bv = (v + e < V) ? b[v + e] : 0.0f;
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j][4 * g + e] = bv;
        }
      }
  }
  template <int BM, int BN, int TM, int TN, int NT>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], const EpiCtx &c) const {
    const int row0 = c.tile_row0 + c.wrow, col0 = c.tile_col0 + c.wcol, lane = c.lane;
    float2 *red = reinterpret_cast<float2 *>(c.smem_lo);  // [waves along rows][BN] statistics exchange
    const bool interior = c.tile_row0 + BM <= V;  // every vocabulary row of the tile exists (all but the last row block)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int m = col0 + j * 32 + (lane & 31);
      const int target = yp[m];
      float mx = -INFINITY;
      float sum = 0.0f;
      if (interior) {
        // no per-row checks; the exponentials work in base 2 with the scale folded into one multiply-add
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            mx = fmaxf(mx, acc[i][j][r]);
          }
        constexpr float LOG2E = 1.4426950408889634f;
        const float off = -mx * LOG2E;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += __builtin_amdgcn_exp2f(fmaf(acc[i][j][r], LOG2E, off));
        // the target's logit: only if it lies in this wave's rows (rare), then a compare chain over the registers
        const int trel = target - row0 - ((lane >> 5) << 2);  // row offset inside the wave tile, this half-wave's share removed
        if (trel >= 0 && trel < 32 * TM && ((trel >> 2) & 1) == 0) {
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              if (trel == i * 32 + 8 * (r >> 2) + (r & 3)) zy[m] = acc[i][j][r];
        }
      } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int v = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
            float z = 0.0f;
            if (v < V) {
              z = acc[i][j][r];
              mx = fmaxf(mx, z);
              if (v == target) zy[m] = z;
            }
            acc[i][j][r] = z;
          }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int v = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
            if (v < V) sum += __expf(acc[i][j][r] - mx);
          }
      }
      // the other half-wave holds the other rows of the same position
      const float omx = __shfl_xor(mx, 32, 64);
      const float osum = __shfl_xor(sum, 32, 64);
      const float nmx = fmaxf(mx, omx);
      float tot = 0.0f;
      if (sum > 0.0f) tot += sum * __expf(mx - nmx);
      if (osum > 0.0f) tot += osum * __expf(omx - nmx);
      if (lane < 32) red[(c.wrow / (32 * TM)) * BN + c.wcol + j * 32 + lane] = make_float2(nmx, tot);
    }
    // merge the statistics of the waves stacked along the vocabulary rows of this tile, in fixed order
    __syncthreads();
    constexpr int WGM = BM / (32 * TM);
    if (c.tid < BN) {
      float2 a = red[c.tid];
#pragma unroll
      for (int w = 1; w < WGM; ++w) {
        const float2 q = red[w * BN + c.tid];
        const float nm = fmaxf(a.x, q.x);
        float t = 0.0f;
        if (a.y > 0.0f) t += a.y * __expf(a.x - nm);
        if (q.y > 0.0f) t += q.y * __expf(q.x - nm);
        a = make_float2(nm, t);
      }
      part[(long)(c.tile_row0 / BM) * ldz + c.tile_col0 + c.tid] = a;
    }
    __syncthreads();
    store_tile<BM, BN, TM, TN, NT>(acc, c, ZT, ldz);
  }
};

// Split-K partial sums: part[split][row][col] = acc.
struct EpiPartial : EpiZeroInit {
  float *part;
  long ld;           // columns
  long split_stride; // elements between splits
  template <int BM, int BN>
  static constexpr int lds_bytes() { return 0; }
  template <int BM, int BN, int TM, int TN, int NT>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], const EpiCtx &c) const {
    store_tile<BM, BN, TM, TN, NT>(acc, c, part + (long)c.split * split_stride, ld);
  }
};

// Plain store of the tile into a tile-padded buffer, in fp32 (out32) and/or in the compute type (outc).
template <typename T>
struct EpiStore : EpiZeroInit {
  float *out32;
  T *outc;
  long ld;
  template <int BM, int BN>
  static constexpr int lds_bytes() { return 0; }
  template <int BM, int BN, int TM, int TN, int NT>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], const EpiCtx &c) const {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const long col = c.tile_col0 + c.wcol + j * 32 + (c.lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const long row = c.tile_row0 + c.wrow + i * 32 + RNNLM_ACC_ROW(r, c.lane);
          if (out32) out32[row * ld + col] = acc[i][j][r];
          if (outc) outc[row * ld + col] = from_f32<T>(acc[i][j][r]);
        }
      }
  }
};

// Fused SGD (Sec. 4.2) on a weight-gradient contraction computed TRANSPOSED: the accumulator tile is
// C[j][r] = dLoss/dW[r][j] (rows = columns j of the weight matrix, columns = its rows r), so a lane
// holds runs of 4 consecutive j for one weight row and updates W[r][j..j+3] with one 16-byte
// read-modify-write.  out = alpha*W - lr*acc for the R x C valid entries; training passes out = W (in
// place, alpha = 1) and also refreshes the compute copy Wc; the gradient-export call passes out =
// caller buffer, alpha = 0, lr = -1, Wc = nullptr.  Padding entries of Wc are never written (they
// stay zero).  WcT, when given, receives the same values transposed (the recurrent matrix keeps both).
template <typename T>
struct EpiSgdT : EpiZeroInit {
  const float *W;
  float *out;
  T *Wc;
  T *WcT = nullptr;  // optional: the transposed compute copy (leading dimension ldc), refreshed as well
  long ldw, ldc;  // ldw: W/out leading dimension; ldc: compute copy leading dimension
  int R, C;       // valid weight rows (tile columns) and weight columns (tile rows)
  float alpha, lr;
  template <int BM, int BN>
  static constexpr int lds_bytes() { return 0; }
  __device__ static inline void store4(float *p, const f32x4_t &v) { *reinterpret_cast<f32x4_t *>(p) = v; }
  __device__ static inline void store4(bf16_t *p, const f32x4_t &v) {
    bf16x4_t h;
#pragma unroll
    for (int e = 0; e < 4; ++e) h[e] = (bf16_t)v[e];
    *reinterpret_cast<bf16x4_t *>(p) = h;
  }
  template <int BM, int BN, int TM, int TN, int NT>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], const EpiCtx &c) const {
    const int row0 = c.tile_row0 + c.wrow, col0 = c.tile_col0 + c.wcol, lane = c.lane;
    const bool vec_ok = ((ldw | ldc) & 3) == 0;
    if (vec_ok && row0 + 32 * TM <= C) {
      // Interior of the matrix along the weight columns: no per-element checks, and the master values of
      // a batch of 8 (or 4) 16-byte groups are all requested before any of them is used.  W and out are
      // the same array when training in place, so the compiler keeps loads behind earlier stores; issuing
      // a batch's loads first is what keeps several memory round trips in flight per wave.
      constexpr int IB = (TM % 4 == 0) ? 4 : ((TM % 2 == 0) ? 2 : 1);  // 32-row blocks per batch
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int r = col0 + j * 32 + (lane & 31);  // weight row
        if (r >= R) continue;
#pragma unroll
        for (int i0 = 0; i0 < TM; i0 += IB) {
          f32x4_t w[IB][4];
          if (alpha != 0.0f) {
#pragma unroll
            for (int ii = 0; ii < IB; ++ii)
#pragma unroll
              for (int g = 0; g < 4; ++g) {
                const int j0 = row0 + (i0 + ii) * 32 + 8 * g + ((lane >> 5) << 2);
                w[ii][g] = *reinterpret_cast<const f32x4_t *>(W + (long)r * ldw + j0);
              }
          }
#pragma unroll
          for (int ii = 0; ii < IB; ++ii)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const int j0 = row0 + (i0 + ii) * 32 + 8 * g + ((lane >> 5) << 2);
              f32x4_t nv;
#pragma unroll
              for (int e = 0; e < 4; ++e)
                nv[e] = ((alpha != 0.0f) ? alpha * w[ii][g][e] : 0.0f) - lr * acc[i0 + ii][j][4 * g + e];
              *reinterpret_cast<f32x4_t *>(out + (long)r * ldw + j0) = nv;
              if (Wc) store4(Wc + (long)r * ldc + j0, nv);
              if (WcT) {
#pragma unroll
                for (int e = 0; e < 4; ++e) WcT[(long)(j0 + e) * ldc + r] = from_f32<T>(nv[e]);
              }
            }
        }
      }
      return;
    }
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int r = col0 + j * 32 + (lane & 31);  // weight row
      if (r >= R) continue;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int j0 = row0 + i * 32 + 8 * g + ((lane >> 5) << 2);  // first of 4 weight columns
          if (j0 >= C) continue;
          const long idx = (long)r * ldw + j0;
          if (vec_ok && j0 + 3 < C) {
            f32x4_t nv;
            if (alpha != 0.0f) {
              const f32x4_t w = *reinterpret_cast<const f32x4_t *>(W + idx);
#pragma unroll
              for (int e = 0; e < 4; ++e) nv[e] = alpha * w[e] - lr * acc[i][j][4 * g + e];
            } else {
#pragma unroll
              for (int e = 0; e < 4; ++e) nv[e] = -lr * acc[i][j][4 * g + e];
            }
            *reinterpret_cast<f32x4_t *>(out + idx) = nv;
            if (Wc) store4(Wc + (long)r * ldc + j0, nv);
            if (WcT) {
#pragma unroll
              for (int e = 0; e < 4; ++e) WcT[(long)(j0 + e) * ldc + r] = from_f32<T>(nv[e]);
            }
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (j0 + e < C) {
                const float w = (alpha != 0.0f) ? alpha * W[idx + e] : 0.0f;
                const float nv = w - lr * acc[i][j][4 * g + e];
                out[idx + e] = nv;
                if (Wc) Wc[(long)r * ldc + j0 + e] = from_f32<T>(nv);
                if (WcT) WcT[(long)(j0 + e) * ldc + r] = from_f32<T>(nv);
              }
          }
        }
    }
  }
};

// Fused SGD on a weight-gradient contraction computed in the matrix's own orientation: tile rows = weight
// rows, tile columns = weight columns, so the 32 lanes that share an accumulator register hold 32 consecutive
// columns of one weight row: every 4-byte access of a half-wave falls into one 128-byte line (two lines per
// wave instruction).  The transposed form above moves 16 bytes per lane but spreads a wave instruction over
// 32 weight rows, i.e. 32 lines, and the vector memory path then spends its time on line look-ups; for the
// large output matrix that made the epilogue several times longer than its traffic needs.  Same contract as
// EpiSgdT otherwise (out = alpha*W - lr*acc on the R x C valid entries, optional compute copy Wc).
template <typename T>
struct EpiSgd : EpiZeroInit {
  const float *W;
  float *out;
  T *Wc;
  long ldw, ldc;
  int R, C;
  float alpha, lr;
  template <int BM, int BN>
  static constexpr int lds_bytes() { return 0; }
  template <int BM, int BN, int TM, int TN, int NT>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], const EpiCtx &c) const {
    const int row0 = c.tile_row0 + c.wrow, col0 = c.tile_col0 + c.wcol, lane = c.lane;
    const int lc = lane & 31;
#if defined(__HIP_DEVICE_COMPILE__)
    if (row0 + 32 * TM <= R && col0 + 32 * TN <= C && (ldc & 1) == 0) {
      // Interior wave tile: no checks.  What bounds this epilogue is memory latency (a compute unit moves 640 KB
      // per tile; its matrix cores idle meanwhile), so the master values of TWO 32-row blocks are in flight at
      // any time: block i + 2 is requested as soon as block i has been stored.  All accesses go through buffer
      // resources based at the wave tile's origin: one lane-dependent offset register serves every access and
      // the row part is a scalar, which leaves the registers for the 2 x TN x 16 values in flight (with pointer
      // arithmetic the addresses alone would not fit).  W and out are the same array when training in place:
      // buffer accesses are kept in program order.  The copy in the compute type leaves as packed pairs:
      // neighbouring lanes swap one value so that each lane owns two adjacent columns of one row.
      // (the wave tile's origin is the same for all lanes: say so, or every access becomes a loop over lanes)
      const long origin = (long)__builtin_amdgcn_readfirstlane(row0) * ldw + __builtin_amdgcn_readfirstlane(col0);
      const long origin_c = (long)__builtin_amdgcn_readfirstlane(row0) * ldc + __builtin_amdgcn_readfirstlane(col0);
      auto uniform = [](auto *p) {
        const unsigned long long v = reinterpret_cast<unsigned long long>(p);
        const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
        const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
        return reinterpret_cast<decltype(p)>(((unsigned long long)hi << 32) | lo);
      };
      const __amdgpu_buffer_rsrc_t rw =
          __builtin_amdgcn_make_buffer_rsrc(uniform(const_cast<float *>(W) + origin), 0, 0x7fffffff, 0x00020000);
      const __amdgpu_buffer_rsrc_t ro =
          __builtin_amdgcn_make_buffer_rsrc(uniform(out + origin), 0, 0x7fffffff, 0x00020000);
      const __amdgpu_buffer_rsrc_t rc = __builtin_amdgcn_make_buffer_rsrc(
          uniform(Wc ? Wc + origin_c : reinterpret_cast<T *>(out + origin)), 0, 0x7fffffff, 0x00020000);
      const int half = lane >> 5;
      const int voff = (int)((half * 4 * ldw + lc) * 4);  // this lane's byte offset inside a 32-row block
      const bool odd = lane & 1;
      const int voffc = (int)(((half * 4 + (odd ? 1 : 0)) * ldc + (lc & ~1)) * (long)sizeof(T));
      const int ldw4 = (int)(ldw * 4), ldcb = (int)(ldc * (long)sizeof(T));
      auto request = [&](int i, float (&w)[TN][16]) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            w[j][r] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                          rw, voff, (i * 32 + 8 * (r >> 2) + (r & 3)) * ldw4 + j * 128, 0));
      };
      auto apply = [&](int i, const float (&w)[TN][16]) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          float nv[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            nv[r] = ((alpha != 0.0f) ? alpha * w[j][r] : 0.0f) - lr * acc[i][j][r];
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, nv[r]), ro, voff,
                                                  (i * 32 + 8 * (r >> 2) + (r & 3)) * ldw4 + j * 128, 0);
          }
          if (Wc) {
            if constexpr (sizeof(T) == 2) {
              typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
#pragma unroll
              for (int q = 0; q < 8; ++q) {  // rows 2q, 2q+1 of this lane's 16: even lanes keep 2q, odd lanes 2q+1
                union {
                  bf16x2_t h;
                  unsigned u;
                } pk;
                pk.h[0] = (bf16_t)nv[2 * q];
                pk.h[1] = (bf16_t)nv[2 * q + 1];
                const unsigned mine = pk.u;
                const unsigned theirs = (unsigned)__builtin_amdgcn_mov_dpp((int)mine, 0xB1, 0xF, 0xF, true);  // lane ^ 1
                const unsigned word = odd ? ((theirs >> 16) | (mine & 0xffff0000u)) : ((mine & 0xffffu) | (theirs << 16));
                const int r0 = 2 * q;
                __builtin_amdgcn_raw_buffer_store_b32(word, rc, voffc,
                                                      (i * 32 + 8 * (r0 >> 2) + (r0 & 3)) * ldcb + j * 32 * (int)sizeof(T), 0);
              }
            } else {
#pragma unroll
              for (int r = 0; r < 16; ++r)
                __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, nv[r]), rc, (int)((half * 4 * ldc + lc) * 4),
                                                      (i * 32 + 8 * (r >> 2) + (r & 3)) * ldcb + j * 128, 0);
            }
          }
        }
      };
      if (alpha != 0.0f) {
        static_assert(TM % 2 == 0, "two row blocks in flight");
        // (scheduling barriers: left alone, the compiler starts applying the first values after a third of the
        // requests and issues the rest only when those have arrived, one memory round trip later)
        float wa[TN][16], wb[TN][16];
        request(0, wa);
        request(1, wb);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < TM; i += 2) {
          apply(i, wa);
          __builtin_amdgcn_sched_barrier(0);
          if (i + 2 < TM) request(i + 2, wa);
          __builtin_amdgcn_sched_barrier(0);
          apply(i + 1, wb);
          __builtin_amdgcn_sched_barrier(0);
          if (i + 3 < TM) request(i + 3, wb);
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
        float wz[TN][16];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) wz[j][r] = 0.0f;
#pragma unroll
        for (int i = 0; i < TM; ++i) apply(i, wz);
      }
      return;
    }
#endif
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = col0 + j * 32 + lc;
        if (col >= C) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const long row = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
          if (row >= R) continue;
          const float w = (alpha != 0.0f) ? alpha * W[row * ldw + col] : 0.0f;
          const float nv = w - lr * acc[i][j][r];
          out[row * ldw + col] = nv;
          if (Wc) Wc[row * ldc + col] = from_f32<T>(nv);
        }
      }
  }
};

// Recurrent backward step: dA = (dH_out + dA_next U) * h * (1 - h).  Rows = streams, cols = units.
template <typename T>
struct EpiRnnBwd : EpiZeroInit {
  const float *dHs;  // [Bp][ld] gradient arriving from the output layer at this timestep
  const T *Hs;       // [Bp][ld] hidden state of this timestep
  float *dA32;       // [Bp][ld]
  T *dAc;            // [Bp][ld]
  int B, H, ld;
  template <int BM, int BN>
  static constexpr int lds_bytes() { return 0; }
  template <int BM, int BN, int TM, int TN, int NT>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], const EpiCtx &c) const {
    const int row0 = c.tile_row0 + c.wrow, col0 = c.tile_col0 + c.wcol, lane = c.lane;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = col0 + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
          const long idx = (long)row * ld + col;
          float d = 0.0f;
          if (row < B && col < H) {
            const float hv = to_f32(Hs[idx]);
            d = (dHs[idx] + acc[i][j][r]) * hv * (1.0f - hv);
          }
          dA32[idx] = d;
          dAc[idx] = from_f32<T>(d);
        }
      }
  }
};

// ---- Host launcher -----------------------------------------------------------------------------

// band > 0: tiles walked in bands of `band` tile rows; band < 0: bands of -band tile columns.
template <typename T, int BM, int BN, int WGM, int WGN, int LA, int LB, int KBYTES = 128, int MINWG = 1, int PF = 2,
          class Epi>
inline hipError_t launch_gemm(hipStream_t stream, const void *A, long lda, const void *B, long ldb, long Mg, long Ng,
                              long K, int splits, const Epi &epi, int band = 4) {
  constexpr int BK = KBYTES / (int)sizeof(T);
  if (Mg <= 0 || Ng <= 0 || K < 0 || Mg % BM || Ng % BN || K % BK || splits < 1) return hipErrorInvalidValue;
  constexpr int loop_bytes = 2 * (TileGeom<T, BM, LA, KBYTES>::BYTES + TileGeom<T, BN, LB, KBYTES>::BYTES);
  constexpr int epi_bytes = Epi::template lds_bytes<BM, BN>();
  constexpr int smem_bytes = loop_bytes > epi_bytes ? loop_bytes : epi_bytes;
  static_assert(smem_bytes <= 160 * 1024, "tile does not fit the 160 KB of LDS");
  auto kern = gemm_kernel<T, BM, BN, WGM, WGN, LA, LB, Epi, KBYTES, MINWG, PF>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes);
    if (e != hipSuccess) return e;
    configured = true;
  }
  GemmShape g;
  g.A = A;
  g.B = B;
  g.lda = lda;
  g.ldb = ldb;
  g.bytesA = g.bytesB = 0;
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
  dim3 grid((unsigned)(g.perXcd * NUM_XCD));
  hipLaunchKernelGGL(kern, grid, dim3(WGM * WGN * 64), smem_bytes, stream, g, epi);
  return hipGetLastError();
}

}  // namespace rnnlm_dev
