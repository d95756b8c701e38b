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
  int tilesM, tilesN;   // output tiles
  int kBlocks;          // K / BK
  int kBlocksPerSplit;  // K blocks handled by one blockIdx.y
};

constexpr int LDS_ROWK_STRIDE = 128 + 16;  // bytes per tile row, padded against bank conflicts

template <typename T, int ROWS, int LAYOUT>
struct TileGeom {
  static constexpr int ES = sizeof(T);
  static constexpr int BK = Elem<T>::BK;
  static constexpr int KROW_STRIDE = ROWS * ES + 16;
  static constexpr int BYTES = (LAYOUT == ROWK) ? ROWS * LDS_ROWK_STRIDE : BK * KROW_STRIDE;
};

// Moves one ROWS x BK operand tile global -> registers -> LDS in 16-byte pieces.
template <typename T, int ROWS, int LAYOUT, int NT>
struct TileLoader {
  using G = TileGeom<T, ROWS, LAYOUT>;
  static constexpr int CHUNKS = ROWS * 8;
  static constexpr int PER = CHUNKS / NT;
  static_assert(CHUNKS % NT == 0, "tile does not divide over the workgroup");
  uint4 regs[PER];

  __device__ inline void load(const char *base, long ld_bytes, long row0, long k0, int tid) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid + i * NT;
      const char *p;
      if (LAYOUT == ROWK) {
        const int r = c >> 3, kc = c & 7;
        p = base + (row0 + r) * ld_bytes + k0 * G::ES + kc * 16;
      } else {
        constexpr int CPR = ROWS * G::ES / 16;
        const int kk = c / CPR, mc = c % CPR;
        p = base + (k0 + kk) * ld_bytes + row0 * G::ES + mc * 16;
      }
      regs[i] = *reinterpret_cast<const uint4 *>(p);
    }
  }
  __device__ inline void store(char *tile, int tid) const {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int c = tid + i * NT;
      int off;
      if (LAYOUT == ROWK) {
        off = (c >> 3) * LDS_ROWK_STRIDE + (c & 7) * 16;
      } else {
        constexpr int CPR = ROWS * G::ES / 16;
        off = (c / CPR) * G::KROW_STRIDE + (c % CPR) * 16;
      }
      *reinterpret_cast<uint4 *>(tile + off) = regs[i];
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
template <typename T, int ROWS, int LAYOUT>
struct FragReader;

template <int ROWS>
struct FragReader<bf16_t, ROWS, ROWK> {
  __device__ static inline bf16x8_t get(const char *tile, int r, int ks) {
    return *reinterpret_cast<const bf16x8_t *>(tile + r * LDS_ROWK_STRIDE + ks * 2);
  }
};
template <int ROWS>
struct FragReader<bf16_t, ROWS, KROW> {
  __device__ static inline bf16x8_t get(const char *tile, int r, int ks) {
    constexpr int S = TileGeom<bf16_t, ROWS, KROW>::KROW_STRIDE;
    bf16x8_t f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = *reinterpret_cast<const bf16_t *>(tile + (ks + e) * S + r * 2);
    return f;
  }
};
template <int ROWS>
struct FragReader<float, ROWS, ROWK> {
  __device__ static inline F32x8 get(const char *tile, int r, int ks) {
    F32x8 f;
    const f32x4_t a = *reinterpret_cast<const f32x4_t *>(tile + r * LDS_ROWK_STRIDE + ks * 4);
    const f32x4_t b = *reinterpret_cast<const f32x4_t *>(tile + r * LDS_ROWK_STRIDE + ks * 4 + 16);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f.v[e] = a[e];
      f.v[4 + e] = b[e];
    }
    return f;
  }
};
template <int ROWS>
struct FragReader<float, ROWS, KROW> {
  __device__ static inline F32x8 get(const char *tile, int r, int ks) {
    constexpr int S = TileGeom<float, ROWS, KROW>::KROW_STRIDE;
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

template <typename T, int BM, int BN, int WGM, int WGN, int LA, int LB, class Epi>
__global__ void __launch_bounds__(WGM *WGN * 64) gemm_kernel(const GemmShape g, const Epi epi) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int NT = WGM * WGN * 64;
  constexpr int BK = Elem<T>::BK;
  constexpr int ES = sizeof(T);
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  static_assert(WTM % 32 == 0 && WTN % 32 == 0, "wave tile must be made of 32x32 blocks");
  using GA = TileGeom<T, BM, LA>;
  using GB = TileGeom<T, BN, LB>;
  constexpr int STAGE = GA::BYTES + GB::BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave % WGM, wn = wave / WGM;
  const int tile_m = blockIdx.x % g.tilesM, tile_n = blockIdx.x / g.tilesM;
  const int split = blockIdx.y;
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

  TileLoader<T, BM, LA, NT> la;
  TileLoader<T, BN, LB, NT> lb;
  const char *Ab = static_cast<const char *>(g.A);
  const char *Bb = static_cast<const char *>(g.B);
  const long lda_b = g.lda * ES, ldb_b = g.ldb * ES;
  const long arow0 = (long)tile_m * BM, brow0 = (long)tile_n * BN;

  if (nk > 0) {
    la.load(Ab, lda_b, arow0, (long)kb0 * BK, tid);
    lb.load(Bb, ldb_b, brow0, (long)kb0 * BK, tid);
    la.store(smem, tid);
    lb.store(smem + GA::BYTES, tid);
    __syncthreads();
  }
  const int lr = lane & 31, lk = (lane >> 5) * 8;
  for (int it = 0; it < nk; ++it) {
    const char *sa = smem + (it & 1) * STAGE;
    const char *sb = sa + GA::BYTES;
    const bool more = it + 1 < nk;
    if (more) {
      la.load(Ab, lda_b, arow0, (long)(kb0 + it + 1) * BK, tid);
      lb.load(Bb, ldb_b, brow0, (long)(kb0 + it + 1) * BK, tid);
    }
#pragma unroll
    for (int ks = 0; ks < BK; ks += 16) {
      typename FragT<T>::type fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = FragReader<T, BM, LA>::get(sa, wm * WTM + i * 32 + lr, ks + lk);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = FragReader<T, BN, LB>::get(sb, wn * WTN + j * 32 + lr, ks + lk);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) mma16(acc[i][j], fa[i], fb[j]);
    }
    if (more) {
      char *da = smem + ((it + 1) & 1) * STAGE;
      la.store(da, tid);
      lb.store(da + GA::BYTES, tid);
    }
    __syncthreads();
  }
  epi.template run<TM, TN>(acc, tile_m * BM + wm * WTM, tile_n * BN + wn * WTN, lane, split);
}

// Accumulator element r (0..15) of a 32x32 block lives at row 8*(r/4) + 4*(lane/32) + r%4,
// column lane%32.
#define RNNLM_ACC_ROW(r, lane) ((((r) >> 2) << 3) + (((lane) >> 5) << 2) + ((r)&3))

// ---- Epilogues ---------------------------------------------------------------------------------

// Recurrent forward step (Sec. 4.1): h = sigmoid(X + Hprev U^T).  Rows = streams, cols = units.
template <typename T>
struct EpiRnnFwd {
  const float *X;   // [Bp][ld]  gathered embedding rows of this timestep
  T *Hnext;         // [Bp][ld]  hidden state slot of this timestep (padding written as zero)
  float *h_state;   // [B][H] or nullptr: carried state, written at the window's last step
  int B, H, ld;
  template <int TM, int TN>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], int row0, int col0, int lane, int) const {
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
// stored transposed (vocabulary-major) for the softmax pass and both gradient contractions, plus
// per-(wave row block, position) partial (max, sum exp) statistics of the fp32 logits and the fp32
// logit of each position's target word.
template <typename T>
struct EpiOutFwd {
  const float *b;   // [V]
  T *ZT;            // [Vp][ldz]
  float2 *part;     // [Vp / (32*TM)][ldz]
  const int *yp;    // [Mp] target id per position, -1 on padding
  float *zy;        // [Mp] target logit
  int V;
  long ldz;
  template <int TM, int TN>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], int row0, int col0, int lane, int) const {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int m = col0 + j * 32 + (lane & 31);
      const int target = yp[m];
      float mx = -INFINITY;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int v = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
          float z = 0.0f;
          if (v < V) {
            z = acc[i][j][r] + b[v];
            mx = fmaxf(mx, z);
            if (v == target) zy[m] = z;
          }
          acc[i][j][r] = z;
          ZT[(long)v * ldz + m] = from_f32<T>(z);
        }
      float sum = 0.0f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int v = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
          if (v < V) sum += __expf(acc[i][j][r] - mx);
        }
      // the other half-wave holds the other rows of the same position
      const float omx = __shfl_xor(mx, 32, 64);
      const float osum = __shfl_xor(sum, 32, 64);
      const float nmx = fmaxf(mx, omx);
      float tot = 0.0f;
      if (sum > 0.0f) tot += sum * __expf(mx - nmx);
      if (osum > 0.0f) tot += osum * __expf(omx - nmx);
      if (lane < 32) part[(long)(row0 / (32 * TM)) * ldz + m] = make_float2(nmx, tot);
    }
  }
};

// Split-K partial sums: part[split][row][col] = acc.
struct EpiPartial {
  float *part;
  long ld;           // columns
  long split_stride; // elements between splits
  template <int TM, int TN>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], int row0, int col0, int lane, int split) const {
    float *p = part + (long)split * split_stride;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = col0 + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
          p[(long)row * ld + col] = acc[i][j][r];
        }
      }
  }
};

// Fused SGD (Sec. 4.2) on a weight-gradient contraction: out = alpha*W - lr*acc for the R x C
// valid entries; training passes out = W (in place, alpha = 1) and also refreshes the compute copy
// Wc; the gradient-export call passes out = caller buffer, alpha = 0, lr = -1, Wc = nullptr.
template <typename T>
struct EpiSgd {
  const float *W;
  float *out;
  T *Wc;
  long ldw, ldc;  // ldw: W/out leading dimension; ldc: compute copy leading dimension
  int R, C;
  float alpha, lr;
  template <int TM, int TN>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], int row0, int col0, int lane, int) const {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = col0 + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = row0 + i * 32 + RNNLM_ACC_ROW(r, lane);
          if (row < R && col < C) {
            const float w = (alpha != 0.0f) ? alpha * W[(long)row * ldw + col] : 0.0f;
            const float nv = w - lr * acc[i][j][r];
            out[(long)row * ldw + col] = nv;
            if (Wc) Wc[(long)row * ldc + col] = from_f32<T>(nv);
          }
        }
      }
  }
};

// Recurrent backward step: dA = (dH_out + dA_next U) * h * (1 - h).  Rows = streams, cols = units.
template <typename T>
struct EpiRnnBwd {
  const float *dHs;  // [Bp][ld] gradient arriving from the output layer at this timestep
  const T *Hs;       // [Bp][ld] hidden state of this timestep
  float *dA32;       // [Bp][ld]
  T *dAc;            // [Bp][ld]
  int B, H, ld;
  template <int TM, int TN>
  __device__ inline void run(f32x16_t (&acc)[TM][TN], int row0, int col0, int lane, int) const {
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

template <typename T, int BM, int BN, int WGM, int WGN, int LA, int LB, class Epi>
inline hipError_t launch_gemm(hipStream_t stream, const void *A, long lda, const void *B, long ldb, long Mg, long Ng,
                              long K, int splits, const Epi &epi) {
  constexpr int BK = Elem<T>::BK;
  if (Mg <= 0 || Ng <= 0 || K < 0 || Mg % BM || Ng % BN || K % BK || splits < 1) return hipErrorInvalidValue;
  constexpr int smem_bytes = 2 * (TileGeom<T, BM, LA>::BYTES + TileGeom<T, BN, LB>::BYTES);
  auto kern = gemm_kernel<T, BM, BN, WGM, WGN, LA, LB, Epi>;
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
  g.tilesM = (int)(Mg / BM);
  g.tilesN = (int)(Ng / BN);
  g.kBlocks = (int)(K / BK);
  g.kBlocksPerSplit = (g.kBlocks + splits - 1) / splits;
  dim3 grid((unsigned)(g.tilesM * g.tilesN), (unsigned)splits);
  hipLaunchKernelGGL(kern, grid, dim3(WGM * WGN * 64), smem_bytes, stream, g, epi);
  return hipGetLastError();
}

}  // namespace rnnlm_dev
