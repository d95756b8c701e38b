// Host side of the C ABI declared in include/rnnlm.h: argument validation, workspace carving and
// the kernel sequence of one window (Sec. 4.1 / 4.2 of the paper; see the header for the model).
#include "../../include/rnnlm.h"

#include <math.h>
#include <stdlib.h>

#include <algorithm>
#include <mutex>
#include <new>
#include <vector>

#include "common.h"
#include "gemm.h"
#include "gemm_dma.h"
#include "gemm_dma4.h"
#include "kernels.h"
#include "nce.h"
#include "rmsprop.h"
#include "gemm_ring64.h"
#include "rnn_persistent.h"
#include "rnn_resident.h"

using namespace rnnlm_dev;

#define HIP_TRY(expr)                        \
  do {                                       \
    hipError_t e_ = (expr);                  \
    if (e_ != hipSuccess) return RNNLM_ERR_HIP; \
  } while (0)

struct WsLayout {
  size_t Wo_c, U_c, UT_c, Hs_c, ZT, dA_c, X32, dHs32, dA32, part32, stat, lse, zy, logp_int, xp, yp, perm, seg, xtmp, ytmp,
      scalars, total;
  // noise-contrastive calls (present when K_max > 0)
  size_t Wn_c, S32, dS_c, G32, noff, ndt, nct, gcol, ids, perm2, seg2;
  // rmsprop calls (present when cfg.rmsprop != 0): gradient buffers the redirected update epilogues fill
  size_t gWo, gU, gb, gN, gbN;
  // compressed architecture (present when cfg.P > 0; then Wo_c holds the compute copy of the tied matrix E)
  size_t A_c, C_c, Xp_c, P_c, dP32, dP_c, dX32;
  // partial sums of the chip-resident recurrent kernel (present for Hp = 4096, 256 streams, bf16)
  size_t part_res, sync;
  bool has_part_res;
  long partElems;
};

struct EventPair {
  hipEvent_t start, stop;
  int stage;
};

struct rnnlm {
  rnnlm_config cfg;
  rnnlm_buffers buf;
  int Hp, Vp, Bp, MpMax;
  int Pp;     // cfg.P rounded up to the tile size (0: plain architecture)
  int D, Dp;  // width of the output layer's input: H / Hp, or P / Pp for the compressed architecture
  int KpMax;  // K_max rounded up to the tile size (0: no noise-contrastive workspace)
  int nPart;
  WsLayout L;
  char *ws;
  // stage timing (host-side only)
  // the integer helpers of the row updates (sort by id, run starts) depend on the token ids only: they run
  // on a second stream (default priority) next to the recurrent forward pass and are joined before the updates
  hipStream_t side = nullptr;
  hipEvent_t ev_fork[2] = {nullptr, nullptr}, ev_join[2] = {nullptr, nullptr};
  bool xcd_local = false;        // the probe at init saw round-robin placement over 8 XCDs
  int exchange_mode = RNNLM_EXCHANGE_AUTO;  // how the persistent recurrent kernels exchange state between workgroups
  unsigned spin_limit = 1u << 18;  // polls of a grid barrier before giving up (about a second)
  uint32_t prof_mask = 0;
  std::vector<EventPair> prof_pool;
  size_t prof_used = 0;
  long prof_open[RNNLM_STAGE_COUNT] = {0};
  double prof_ms[RNNLM_STAGE_COUNT] = {0};
  int64_t prof_n[RNNLM_STAGE_COUNT] = {0};
};

namespace {
constexpr size_t PROF_MAX_PAIRS = 16384;

// Records a start event now and a stop event when it goes out of scope, if the stage is enabled.
struct StageTimer {
  rnnlm *h;
  hipStream_t st;
  EventPair *p = nullptr;
  bool close_;
  // open/close: a stage made of several launches opens its pair at the first launch and closes it at
  // the last (stage < 0: nothing to do for the launches in between).
  StageTimer(rnnlm *h_, int stage, hipStream_t st_, bool open = true, bool close = true)
      : h(h_), st(st_), close_(close) {
    if (stage < 0 || !(h->prof_mask & (1u << stage))) return;
    if (!open) {
      if (h->prof_open[stage] >= 0) p = &h->prof_pool[h->prof_open[stage]];
      return;
    }
    h->prof_open[stage] = -1;
    if (h->prof_used == h->prof_pool.size()) {
      if (h->prof_pool.size() >= PROF_MAX_PAIRS) return;
      EventPair e;
      if (hipEventCreate(&e.start) != hipSuccess) return;
      if (hipEventCreate(&e.stop) != hipSuccess) {
        (void)hipEventDestroy(e.start);
        return;
      }
      h->prof_pool.push_back(e);
    }
    h->prof_open[stage] = (long)h->prof_used;
    p = &h->prof_pool[h->prof_used++];
    p->stage = stage;
    (void)hipEventRecord(p->start, st);
  }
  ~StageTimer() {
    if (p && close_) (void)hipEventRecord(p->stop, st);
  }
};
}  // namespace

namespace {

// Tile shape of the three output-layer contractions and of the recurrent weight gradient: 256x256
// output tile, 8 waves as 2 x 4 (wave tile 128 x 64).
constexpr int BIG = 256;
// The large contractions: bf16 operands take the direct global->LDS kernel (four-stage ring), fp32 the
// register-staged one.
// RING4: the four-stage ring of 32-deep K blocks (deeper prefetch; pays when at least one operand is
// K-major, whose 32-deep blocks are still made of full cache lines) instead of two stages of 64.
template <typename T, int WGM, int WGN, int LA, int LB, bool RING4, class Epi>
hipError_t big_gemm(hipStream_t st, const void *A, long lda, const void *B, long ldb, long Mg, long Ng, long K,
                    int splits, const Epi &epi, int band = 4) {
  if constexpr (sizeof(T) == 2 && RING4) {
    // epilogues that leave the LDS alone run as one persistent workgroup per compute unit, which requests the
    // next tile's first K blocks before its epilogue
    constexpr bool PERSIST = Epi::template lds_bytes<BIG, BIG>() == 0;
    return launch_gemm_dma4<BIG, BIG, WGM, WGN, LA, LB, PERSIST>(st, A, lda, B, ldb, Mg, Ng, K, splits, epi, band);
  } else if constexpr (sizeof(T) == 2) {
    return launch_gemm_dma<BIG, BIG, WGM, WGN, LA, LB>(st, A, lda, B, ldb, Mg, Ng, K, splits, epi, band);
  } else {
    return launch_gemm<T, BIG, BIG, 2, 4, LA, LB>(st, A, lda, B, ldb, Mg, Ng, K, splits, epi, band);
  }
}

// The mid-sized contractions (128x128 output tiles: noise-panel products, the layers of the compressed
// architecture): bf16 operands take the direct global->LDS kernels (the ring when an operand is K-major), fp32
// the register-staged one.
template <typename T, int LA, int LB, class Epi>
hipError_t mid_gemm(hipStream_t st, const void *A, long lda, const void *B, long ldb, long Mg, long Ng, long K,
                    int splits, const Epi &epi, int band = 4) {
  // the direct-load kernels address a K-major operand's k blocks with a 32-bit scalar offset
  const bool fits = !((LA == KROW && K * lda * 2 >= (1L << 31)) || (LB == KROW && K * ldb * 2 >= (1L << 31)) ||
                      lda * 2 * 128 >= (1L << 31) || ldb * 2 * 128 >= (1L << 31));
  if constexpr (sizeof(T) == 2 && (LA == KROW || LB == KROW)) {
    if (fits) return launch_gemm_dma4<128, 128, 2, 2, LA, LB>(st, A, lda, B, ldb, Mg, Ng, K, splits, epi, band);
    return launch_gemm<T, 128, 128, 2, 2, LA, LB>(st, A, lda, B, ldb, Mg, Ng, K, splits, epi, band);
  } else if constexpr (sizeof(T) == 2) {
    if (fits) return launch_gemm_dma<128, 128, 2, 2, LA, LB>(st, A, lda, B, ldb, Mg, Ng, K, splits, epi, band);
    return launch_gemm<T, 128, 128, 2, 2, LA, LB>(st, A, lda, B, ldb, Mg, Ng, K, splits, epi, band);
  } else {
    return launch_gemm<T, 128, 128, 2, 2, LA, LB>(st, A, lda, B, ldb, Mg, Ng, K, splits, epi, band);
  }
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

bool cfg_ok(const rnnlm_config *c) {
  if (!c) return false;
  if (c->V <= 0 || c->H <= 0 || c->B <= 0 || c->T_max <= 0) return false;
  if (c->precision != RNNLM_FP32 && c->precision != RNNLM_BF16_FP32MASTER) return false;
  if (c->device < 0) return false;
  if (c->K_max < 0 || c->K_max > 65536) return false;
  if (c->rmsprop != 0 && c->rmsprop != 1) return false;
  if ((long)c->B * c->T_max > (1L << 24)) return false;
  if (c->P < 0 || (c->P > 0 && (c->K_max != 0 || c->rmsprop != 0))) return false;
  return true;
}

int desired_splits(long Mp, long Hp, long kBlocks) {
  const long tiles = (Mp / BIG) * (Hp / BIG);
  long s = 256 / tiles;  // one workgroup per compute unit: stay within one round
  if (s > 16) s = 16;
  if (s > kBlocks) s = kBlocks;
  if (s < 1) s = 1;
  return (int)s;
}

void make_layout(const rnnlm_config &c, int &Hp, int &Vp, int &Bp, int &MpMax, int &nPart, int &KpMax, WsLayout &L) {
  const size_t es = (c.precision == RNNLM_FP32) ? 4 : 2;
  const int Pp = (int)round_up(c.P, PAD_H);
  Hp = (int)round_up(c.H, PAD_H);
  const int Dp = Pp > 0 ? Pp : Hp;
  Vp = (int)round_up(c.V, PAD_V);
  Bp = (int)round_up(c.B, PAD_B);
  MpMax = (int)round_up((long)c.T_max * Bp, PAD_M);
  nPart = Vp / BIG;  // one softmax-statistics partial per tile row block
  const int BK = (es == 4) ? 32 : 64;
  const int S = desired_splits(MpMax, Dp, Vp / BK);
  L.partElems = (long)S * MpMax * Dp;
  size_t o = 0;
  auto take = [&](size_t bytes) {
    size_t at = o;
    o = align256(o + bytes);
    return at;
  };
  L.Wo_c = take((size_t)Vp * Dp * es);
  L.U_c = take((size_t)Hp * Hp * es);
  L.UT_c = take((size_t)Hp * Hp * es);
  L.Hs_c = take((size_t)(MpMax + Bp) * Hp * es);
  L.ZT = take((size_t)Vp * MpMax * es);
  L.dA_c = take((size_t)(MpMax + Bp) * Hp * es);
  L.X32 = take((size_t)MpMax * Hp * 4);
  L.dHs32 = take((size_t)MpMax * Hp * 4);
  L.dA32 = take((size_t)MpMax * Hp * 4);
  L.part32 = take((size_t)L.partElems * 4);
  L.stat = take((size_t)nPart * MpMax * 8);
  L.lse = take((size_t)MpMax * 4);
  L.zy = take((size_t)MpMax * 4);
  L.logp_int = take((size_t)MpMax * 4);
  L.xp = take((size_t)MpMax * 4);
  L.yp = take((size_t)MpMax * 4);
  L.perm = take((size_t)MpMax * 4);
  L.seg = take((size_t)(MpMax + 1) * 4);
  L.xtmp = take((size_t)c.T_max * c.B * 4);
  L.ytmp = take((size_t)c.T_max * c.B * 4);
  KpMax = (int)round_up(c.K_max, 256);
  L.Wn_c = L.S32 = L.dS_c = L.G32 = L.noff = L.ndt = L.nct = L.gcol = L.ids = L.perm2 = L.seg2 = 0;
  if (KpMax > 0) {
    const size_t nent = (size_t)KpMax + (size_t)c.T_max * c.B;
    L.Wn_c = take((size_t)KpMax * Hp * es);
    L.S32 = take((size_t)MpMax * KpMax * 4);
    L.dS_c = take((size_t)MpMax * KpMax * es);
    L.G32 = take((size_t)KpMax * Hp * 4);
    L.noff = take((size_t)KpMax * 4);
    L.ndt = take((size_t)MpMax * 4);
    L.nct = take((size_t)MpMax * 4);
    L.gcol = take((size_t)NCE_COLSUM_PARTS * KpMax * 4);  // 16 row-block partials of the noise words' bias gradient
    L.ids = take(nent * 4);
    L.perm2 = take(nent * 4);
    L.seg2 = take((nent + 1) * 4);
  }
  L.gWo = L.gU = L.gb = 0;
  if (c.rmsprop) {
    L.gWo = take((size_t)c.V * c.H * 4);
    L.gU = take((size_t)c.H * c.H * 4);
    L.gb = take((size_t)c.V * 4);
  }
  L.gN = L.gbN = 0;
  if (c.rmsprop && KpMax > 0) {  // compact per-touched-word gradient rows of the noise-contrastive calls
    const size_t nent = (size_t)KpMax + (size_t)c.T_max * c.B;
    L.gN = take(nent * Hp * 4);
    L.gbN = take(nent * 4);
  }
  L.A_c = L.C_c = L.Xp_c = L.P_c = L.dP32 = L.dP_c = L.dX32 = 0;
  if (Pp > 0) {
    L.A_c = take((size_t)Hp * Pp * es);
    L.C_c = take((size_t)Pp * Hp * es);
    L.Xp_c = take((size_t)MpMax * Pp * es);
    L.P_c = take((size_t)MpMax * Pp * es);
    L.dP32 = take((size_t)MpMax * Pp * 4);
    L.dP_c = take((size_t)MpMax * Pp * es);
    L.dX32 = take((size_t)MpMax * Pp * 4);
  }
  L.part_res = 0;
  L.has_part_res = es == 2 && Pp == 0 && Hp == RES_HP && Bp == RES_BP;
  if (L.has_part_res) L.part_res = take((size_t)RES_PART_STEP * 4);
  L.sync = take((size_t)SYNC_WORDS * 4);  // barrier / ticket counters of the persistent recurrent kernels
  L.scalars = take(256);  // [0]: int nseg, [4]: int nseg of the noise-contrastive update list, [8..19]: int flags[3], [32]: double sum, [40]: double running
  L.total = o;
}

template <typename P>
P *at(rnnlm_t *h, size_t off) {
  return reinterpret_cast<P *>(h->ws + off);
}
int32_t *p_nseg(rnnlm_t *h) { return at<int32_t>(h, h->L.scalars); }
int32_t *p_nseg2(rnnlm_t *h) { return at<int32_t>(h, h->L.scalars + 4); }
int32_t *p_flags(rnnlm_t *h) { return at<int32_t>(h, h->L.scalars + 8); }
double *p_sum(rnnlm_t *h) { return at<double>(h, h->L.scalars + 32); }
double *p_running(rnnlm_t *h) { return at<double>(h, h->L.scalars + 40); }
unsigned *p_counter(rnnlm_t *h) { return at<unsigned>(h, h->L.sync); }

inline unsigned blocks_for(long n, int per) { return (unsigned)((n + per - 1) / per); }

template <typename T>
int sync_copies(rnnlm_t *h, hipStream_t st) {
  const rnnlm_config &c = h->cfg;
  const long nWo = (long)h->Vp * h->Dp, nU = (long)h->Hp * h->Hp;
  // the output layer's matrix: Wo, or the tied matrix E of the compressed architecture
  hipLaunchKernelGGL(to_compute_copy_kernel<T>, dim3(std::min<long>(blocks_for(nWo, 256), 65535)), dim3(256), 0, st,
                     c.P > 0 ? h->buf.E : h->buf.Wo, c.V, h->D, h->Dp, nWo, at<T>(h, h->L.Wo_c));
  if (c.P > 0) {
    const long nA = (long)h->Hp * h->Pp;
    hipLaunchKernelGGL(to_compute_copy_kernel<T>, dim3(std::min<long>(blocks_for(nA, 256), 65535)), dim3(256), 0, st,
                       h->buf.A, c.H, c.P, h->Pp, nA, at<T>(h, h->L.A_c));
    hipLaunchKernelGGL(to_compute_copy_kernel<T>, dim3(std::min<long>(blocks_for(nA, 256), 65535)), dim3(256), 0, st,
                       h->buf.C, c.P, c.H, h->Hp, nA, at<T>(h, h->L.C_c));
  }
  hipLaunchKernelGGL(to_compute_copy_kernel<T>, dim3(std::min<long>(blocks_for(nU, 256), 65535)), dim3(256), 0, st,
                     h->buf.U, c.H, c.H, h->Hp, nU, at<T>(h, h->L.U_c));
  hipLaunchKernelGGL(transpose_kernel<T>, dim3(h->Hp / 32, h->Hp / 32), dim3(256), 0, st, at<T>(h, h->L.U_c), h->Hp,
                     at<T>(h, h->L.UT_c));
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

// The persistent recurrent kernel applies when each wave's share of the contraction fits its register
// file (4 waves up to Hp = 1024, 8 waves up to Hp = 2048) and the grid is small enough to be co-resident
// with a wide margin (at most half of what the chip can hold at once).
bool persistent_ok(const rnnlm_t *h) {
  const long grid = (long)(h->Bp / 32) * (h->Hp / 32);
  if (h->Hp <= 1024) return h->Hp % 256 == 0 && grid <= 256;
  // the 8-wave variant has half the registers per wave: bf16 fragments only
  if (h->Hp <= 2048) return h->cfg.precision == RNNLM_BF16_FP32MASTER && h->Hp % 256 == 0 && grid <= 256;
  return false;
}

// Per-step recurrent path for shapes the persistent kernel does not cover: with whole blocks of 256 streams
// and a wide hidden layer the step's contraction is split over its contraction dimension (0: not split).
// bf16: 256 x 128 tiles through the direct global->LDS kernels; fp32: 256 x 64 tiles through the register-staged one.
int rnn_step_tile_n(const rnnlm_t *h) { return h->cfg.precision == RNNLM_FP32 ? 64 : 128; }
int rnn_step_splits(const rnnlm_t *h) {
  if (h->Bp % 256 != 0 || h->Hp < 2048) return 0;
  const long tiles = (long)(h->Bp / 256) * (h->Hp / rnn_step_tile_n(h));
  long S = std::max<long>(1, 256 / tiles);
  const int BK = (h->cfg.precision == RNNLM_FP32) ? 32 : 64;
  S = std::min<long>(std::min<long>(S, 8), std::min<long>(h->Hp / BK, h->L.partElems / ((long)h->Bp * h->Hp)));
  return S >= 2 ? (int)S : 0;
}

// Workgroups of a kernel that one compute unit holds at once, as the runtime computes it (asked once).
template <auto Kern>
int blocks_per_cu(int threads) {
  static int n = -1;
  if (n < 0) {
    int v = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, Kern, threads, 0) != hipSuccess) v = 0;
    n = v;
  }
  return n;
}

template <typename T, bool BACKWARD>
int launch_rnn_persistent(rnnlm_t *h, int Tn, bool advance_state, hipStream_t st) {
  RnnPersistArgs a;
  a.W = BACKWARD ? at<T>(h, h->L.UT_c) : at<T>(h, h->L.U_c);
  a.Hs = at<T>(h, h->L.Hs_c);
  a.X = BACKWARD ? at<float>(h, h->L.dHs32) : at<float>(h, h->L.X32);
  a.dA32 = at<float>(h, h->L.dA32);
  a.dAc = at<T>(h, h->L.dA_c);
  a.h_state = (!BACKWARD && advance_state) ? h->buf.h_state : nullptr;
  a.counter = p_counter(h);
  a.flags = p_flags(h);
  a.T = Tn;
  a.B = h->cfg.B;
  a.H = h->cfg.H;
  a.Bp = h->Bp;
  a.Hp = h->Hp;
  a.spin_limit = h->spin_limit;
  // the counters are zero here: cleared by the token-preparation kernel (forward) and by the
  // log-probability sum (backward), which always run before this launch on the same stream
  // XCD-local mode: one group of Hp/32 workgroups per block of 32 streams, group x on XCD x
  const bool xcd = h->xcd_local && h->exchange_mode != RNNLM_EXCHANGE_CHIP_WIDE && h->Bp / 32 <= NUM_XCD;
  const dim3 grid(xcd ? (unsigned)(NUM_XCD * (h->Hp / 32)) : (unsigned)((h->Bp / 32) * (h->Hp / 32)));
  // bf16, XCD-local, whole [32][64] blocks per wave: the state goes through LDS (coalesced loads): 4 waves keep
  // their blocks resident; 8 waves (1024 < Hp <= 2048) take the wide kernel, 64 units per workgroup and one
  // workgroup per compute unit, provided the runtime confirms that it fits one
#define RNNLM_LAUNCH_PERSIST(KS, NW)                                                                        \
  do {                                                                                                      \
    if constexpr (sizeof(T) == 2 && KS % 4 == 0 && NW == 8) {                                               \
      if (xcd && blocks_per_cu<rnn_persistent_wide_kernel<KS, BACKWARD>>(512) >= 1) {                       \
        hipLaunchKernelGGL((rnn_persistent_wide_kernel<KS, BACKWARD>), dim3(NUM_XCD * (h->Hp / 64)), dim3(512), 0, st, a); \
        break;                                                                                              \
      }                                                                                                     \
    }                                                                                                       \
    if constexpr (sizeof(T) == 2 && KS % 4 == 0 && NW == 4) {                                               \
      if (xcd && 32 * blocks_per_cu<rnn_persistent_kernel<T, KS, NW, BACKWARD, true, true>>(64 * NW) >= h->Hp / 32) { \
        hipLaunchKernelGGL((rnn_persistent_kernel<T, KS, NW, BACKWARD, true, true>), grid, dim3(64 * NW), 0, st, a); \
        break;                                                                                              \
      }                                                                                                     \
    }                                                                                                       \
    if (xcd) hipLaunchKernelGGL((rnn_persistent_kernel<T, KS, NW, BACKWARD, true>), grid, dim3(64 * NW), 0, st, a); \
    else hipLaunchKernelGGL((rnn_persistent_kernel<T, KS, NW, BACKWARD, false>), grid, dim3(64 * NW), 0, st, a);    \
  } while (0)
  switch (h->Hp / 256) {
    case 1: RNNLM_LAUNCH_PERSIST(4, 4); break;
    case 2: RNNLM_LAUNCH_PERSIST(8, 4); break;
    case 3: RNNLM_LAUNCH_PERSIST(12, 4); break;
    case 4: RNNLM_LAUNCH_PERSIST(16, 4); break;
    case 5: RNNLM_LAUNCH_PERSIST(10, 8); break;
    case 6: RNNLM_LAUNCH_PERSIST(12, 8); break;
    case 7: RNNLM_LAUNCH_PERSIST(14, 8); break;
    case 8: RNNLM_LAUNCH_PERSIST(16, 8); break;
    default: return RNNLM_ERR_ARG;
  }
#undef RNNLM_LAUNCH_PERSIST
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

// Widest layer (Hp = 4096, 256 streams, bf16): one launch of 256 workgroups, one per compute unit, with the whole
// state-to-state matrix resident in registers.  Needs the round-robin placement the init probe checks (32
// workgroups on every XCD); RNNLM_EXCHANGE_CHIP_WIDE selects the per-step launches instead.
bool resident_ok(const rnnlm_t *h) {
  return h->L.has_part_res && h->xcd_local && h->exchange_mode != RNNLM_EXCHANGE_CHIP_WIDE &&
         blocks_per_cu<rnn_resident_kernel<false>>(512) >= 1 && blocks_per_cu<rnn_resident_kernel<true>>(512) >= 1;
}

template <bool BACKWARD>
int launch_rnn_resident(rnnlm_t *h, int Tn, bool advance_state, hipStream_t st) {
  typedef bf16_t T;
  RnnResidentArgs ra;
  RnnPersistArgs &a = ra.p;
  a.W = BACKWARD ? at<T>(h, h->L.UT_c) : at<T>(h, h->L.U_c);
  a.Hs = at<T>(h, h->L.Hs_c);
  a.X = BACKWARD ? at<float>(h, h->L.dHs32) : at<float>(h, h->L.X32);
  a.dA32 = at<float>(h, h->L.dA32);
  a.dAc = at<T>(h, h->L.dA_c);
  a.h_state = (!BACKWARD && advance_state) ? h->buf.h_state : nullptr;
  a.counter = p_counter(h);  // zero here, as for the other persistent kernels
  a.flags = p_flags(h);
  a.T = Tn;
  a.B = h->cfg.B;
  a.H = h->cfg.H;
  a.Bp = h->Bp;
  a.Hp = h->Hp;
  a.spin_limit = h->spin_limit;
  ra.part = at<float>(h, h->L.part_res);
  hipLaunchKernelGGL((rnn_resident_kernel<BACKWARD>), dim3(256), dim3(512), 0, st, ra);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

struct UpdateTargets {
  // where each fused update writes: training -> the masters (alpha 1, lr), gradient export -> caller
  // buffers (alpha 0, lr -1, no compute-copy refresh, no state advance)
  float *E, *U, *Wo, *b;
  float alpha, lr;
  bool refresh_copies;
  bool advance_state;
  int e_compact_ld = 0;  // > 0: the embedding rows go to a compact [runs][e_compact_ld] buffer (one row per run)
  int wo_compact_ld = 0; // > 0: likewise the touched rows of Wo and entries of b of the noise-contrastive calls
  // compressed architecture: Wo is unused, E is the tied matrix (output-side update first, then the input rows)
  float *A = nullptr, *C = nullptr;
};

// Forward half of a window: tokens -> padded ids, state -> slot 0, gather, T recurrent steps,
// output layer with fused statistics, log-probabilities.
// Fork: work enqueued on the side stream after this call starts once everything enqueued on `st` so far has
// finished.  Join: `st` waits for everything enqueued on the side stream so far.  slot = which event pair.
int side_fork(rnnlm_t *h, int slot, hipStream_t st) {
  HIP_TRY(hipEventRecord(h->ev_fork[slot], st));
  HIP_TRY(hipStreamWaitEvent(h->side, h->ev_fork[slot], 0));
  return RNNLM_OK;
}
int side_join(rnnlm_t *h, int slot, hipStream_t st) {
  HIP_TRY(hipEventRecord(h->ev_join[slot], h->side));
  HIP_TRY(hipStreamWaitEvent(st, h->ev_join[slot], 0));
  return RNNLM_OK;
}

template <typename T>
int sort_segments(rnnlm_t *h, int Tn, int32_t *perm, int32_t *seg, int32_t *nseg, hipStream_t st);

// sort_inputs: the window will be trained on, so the sort of its input ids for the embedding update is
// started on the side stream as soon as the padded ids exist (joined in backward_window).
template <typename T>
int forward_window(rnnlm_t *h, const int32_t *x, const int32_t *y, int Tn, float *logp_out, bool advance_state,
                   bool with_output, hipStream_t st, bool sort_inputs = false, bool need_feat = false) {
  const rnnlm_config &c = h->cfg;
  const int Hp = h->Hp, Bp = h->Bp, Vp = h->Vp;
  const int Mrows = Tn * Bp;
  const int Mp = (int)round_up(Mrows, PAD_M);
  const long ldz = h->MpMax;
  T *Hs_c = at<T>(h, h->L.Hs_c);
  float *X32 = at<float>(h, h->L.X32);
  int32_t *xp = at<int32_t>(h, h->L.xp), *yp = at<int32_t>(h, h->L.yp);
  float *lse = at<float>(h, h->L.lse), *zy = at<float>(h, h->L.zy);

  {
    StageTimer tm(h, RNNLM_STAGE_PREP, st);
    const int prep_blocks = (int)blocks_for(std::max<long>(Mp, (long)Bp * Hp), 256);
    if (c.P > 0) {  // compressed architecture: the gathered rows are operands of the contraction below
      hipLaunchKernelGGL(prep_tokens_kernel<T>, dim3(prep_blocks + Mrows), dim3(256), 0, st, x, y, Tn, c.B, Bp, Mp, c.V,
                         xp, yp, lse, p_flags(h), h->buf.h_state, c.H, Hp, Hs_c, p_counter(h), prep_blocks,
                         (const float *)nullptr, (float *)nullptr, (const T *)at<T>(h, h->L.Wo_c), h->Pp,
                         at<T>(h, h->L.Xp_c));
    } else {
      hipLaunchKernelGGL(prep_tokens_kernel<T>, dim3(prep_blocks + Mrows), dim3(256), 0, st, x, y, Tn, c.B, Bp, Mp, c.V,
                         xp, yp, lse, p_flags(h), h->buf.h_state, c.H, Hp, Hs_c, p_counter(h), prep_blocks, h->buf.E,
                         X32, (const T *)nullptr, 0, (T *)nullptr);
    }
    HIP_TRY(hipGetLastError());
    if (sort_inputs) {
      int rc = side_fork(h, 0, st);
      if (rc) return rc;
      rc = sort_segments<T>(h, Tn, at<int32_t>(h, h->L.perm), at<int32_t>(h, h->L.seg), p_nseg(h), h->side);
      if (rc) return rc;
    }
  }

  if (c.P > 0) {
    // layer below the state: X[m][i] = sum_p x_m[p] A[i][p], the additive input of every recurrent step
    StageTimer tm(h, RNNLM_STAGE_PROJ, st);
    EpiPartial epi;
    epi.part = X32;
    epi.ld = Hp;
    epi.split_stride = 0;
    HIP_TRY((mid_gemm<T, ROWK, ROWK>(st, at<T>(h, h->L.Xp_c), h->Pp, at<T>(h, h->L.A_c), h->Pp, Mp,
                                                        Hp, h->Pp, 1, epi)));
  }

  if (persistent_ok(h)) {
    StageTimer tm(h, RNNLM_STAGE_RNN_FWD, st);
    int rc = launch_rnn_persistent<T, false>(h, Tn, advance_state, st);
    if (rc) return rc;
  } else if (sizeof(T) == 2 && resident_ok(h)) {
    StageTimer tm(h, RNNLM_STAGE_RNN_FWD, st);
    int rc = launch_rnn_resident<false>(h, Tn, advance_state, st);
    if (rc) return rc;
  } else
  for (int t = 0; t < Tn; ++t) {
    StageTimer tm(h, (t == 0 || t == Tn - 1) ? RNNLM_STAGE_RNN_FWD : -1, st, t == 0, t == Tn - 1);
    EpiRnnFwd<T> epi;
    epi.X = X32 + (long)t * Bp * Hp;
    epi.Hnext = Hs_c + (long)(t + 1) * Bp * Hp;
    epi.h_state = (advance_state && t == Tn - 1) ? h->buf.h_state : nullptr;
    epi.B = c.B;
    epi.H = c.H;
    epi.ld = Hp;
    const T *A_ = Hs_c + (long)t * Bp * Hp;
    const T *B_ = at<T>(h, h->L.U_c);
    const int S = rnn_step_splits(h);
    if (S > 0) {
      // wide step: all streams x 128 (fp32: 64) units per workgroup, contraction split S ways, then sum + sigmoid
      const long per = (long)Bp * Hp;
      EpiPartial ep;
      ep.part = at<float>(h, h->L.part32);
      ep.ld = Hp;
      ep.split_stride = per;
      if constexpr (sizeof(T) == 2) {
        HIP_TRY((launch_gemm_dma<256, 128, 4, 2, ROWK, ROWK>(st, A_, Hp, B_, Hp, Bp, Hp, Hp, S, ep)));
      } else {
        HIP_TRY((launch_gemm<T, 256, 64, 4, 2, ROWK, ROWK>(st, A_, Hp, B_, Hp, Bp, Hp, Hp, S, ep)));
      }
      hipLaunchKernelGGL(rnn_step_fwd_kernel<T>, dim3(blocks_for(per / 4, 256)), dim3(256), 0, st,
                         at<float>(h, h->L.part32), per, S, epi.X, c.B, c.H, Hp, per / 4, epi.Hnext, epi.h_state);
      HIP_TRY(hipGetLastError());
    } else {
      HIP_TRY((launch_gemm<T, 32, 64, 1, 2, ROWK, ROWK>(st, A_, Hp, B_, Hp, Bp, Hp, Hp, 1, epi)));
    }
  }
  if (!with_output && !(need_feat && c.P > 0)) return RNNLM_OK;  // the noise-contrastive calls score the hidden states themselves
  const T *feat = Hs_c + (long)Bp * Hp;  // what the output layer reads: the states, or the layer above them
  if (c.P > 0) {
    StageTimer tm(h, RNNLM_STAGE_PROJ, st);
    EpiStore<T> epi;
    epi.out32 = nullptr;
    epi.outc = at<T>(h, h->L.P_c);
    epi.ld = h->Pp;
    HIP_TRY((mid_gemm<T, ROWK, ROWK>(st, Hs_c + (long)Bp * Hp, Hp, at<T>(h, h->L.C_c), Hp, Mp,
                                                        h->Pp, Hp, 1, epi)));
    feat = at<T>(h, h->L.P_c);
  }
  if (!with_output) return RNNLM_OK;  // the scoring calls only wanted the layer above the states
  {
    StageTimer tm(h, RNNLM_STAGE_OUT_FWD, st);
    EpiOutFwd<T> epi;
    epi.b = h->buf.b;
    epi.ZT = at<T>(h, h->L.ZT);
    epi.part = at<float2>(h, h->L.stat);
    epi.yp = yp;
    epi.zy = zy;
    epi.V = c.V;
    epi.ldz = ldz;
    if constexpr (sizeof(T) == 2) {
      // thousands of short tiles: one persistent workgroup per compute unit walks them, in bands of 8 vocabulary
      // row panels (the 32 tiles an XCD works on at a time then share 8 row panels and 4 position panels in its L2:
      // measured best of 1..16 on all three large configurations)
      HIP_TRY((launch_gemm_dma<BIG, BIG, 4, 2, ROWK, ROWK, true>(st, at<T>(h, h->L.Wo_c), h->Dp, feat, h->Dp, Vp, Mp,
                                                                 h->Dp, 1, epi, 8)));
    } else {
      HIP_TRY((big_gemm<T, 4, 2, ROWK, ROWK, false>(st, at<T>(h, h->L.Wo_c), h->Dp, feat, h->Dp, Vp, Mp, h->Dp, 1, epi)));
    }
  }
  StageTimer tm(h, RNNLM_STAGE_STATS, st);
  hipLaunchKernelGGL(merge_stats_kernel, dim3(blocks_for(Mrows, 64)), dim3(1024), 0, st, at<float2>(h, h->L.stat),
                     Vp / BIG, ldz, Tn, c.B, Bp, zy, lse, at<float>(h, h->L.logp_int), logp_out);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

template <typename T>
int sort_segments(rnnlm_t *h, int Tn, int32_t *perm, int32_t *seg, int32_t *nseg, hipStream_t st) {
  const int M = Tn * h->cfg.B;
  hipLaunchKernelGGL(rank_sort_kernel, dim3(blocks_for(M, 64)), dim3(1024), 0, st, at<int32_t>(h, h->L.xp), M,
                     h->cfg.B, h->Bp, perm);
  hipLaunchKernelGGL(segment_kernel, dim3(1), dim3(1024), 0, st, at<int32_t>(h, h->L.xp), perm, M, h->cfg.B, h->Bp,
                     seg, nseg);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

// One call of the noise-contrastive criterion (Sec. 4.2): K noise words shared by the window.
struct NceCall {
  const int32_t *noise;
  int K;
  const float *lnq;
  float lnZ;
  float *J_out;
  bool sort_ids;  // the call updates (or exports) rows: sort the touched-word list
};

// Scores of all positions against the gathered noise rows, the targets' own scores, then the
// elementwise pass: coefficients dS (contraction operand), target coefficients, losses, bias column sums.
template <typename T>
int nce_forward(rnnlm_t *h, int Tn, const NceCall &n, hipStream_t st) {
  const rnnlm_config &c = h->cfg;
  const int Hp = h->Hp, Bp = h->Bp;
  const int Mrows = Tn * Bp, Mp = (int)round_up(Mrows, PAD_M), M = Tn * c.B;
  const int K = n.K, Kp = (int)round_up(K, 256);
  T *Hs1 = at<T>(h, h->L.Hs_c) + (long)Bp * Hp;
  T *Wn = at<T>(h, h->L.Wn_c);
  float *S = at<float>(h, h->L.S32);
  int32_t *yp = at<int32_t>(h, h->L.yp);
  const float lnZ_lnK = n.lnZ + logf((float)K);
  const float scale = 1.0f / (float)M;
  {
    StageTimer tm(h, RNNLM_STAGE_NCE_SCORE, st);
    hipLaunchKernelGGL(nce_prep_kernel<T>, dim3(Kp + blocks_for(M, 256)), dim3(256), 0, st, n.noise, K, Kp, c.V, n.lnq,
                       h->buf.b, lnZ_lnK, yp, M, c.B, Bp, at<T>(h, h->L.Wo_c), Hp, Wn, at<float>(h, h->L.noff),
                       at<int32_t>(h, h->L.ids), p_flags(h));
    if (n.sort_ids) {  // the touched-word list is complete: sort it next to the contractions
      int rc = side_fork(h, 1, st);
      if (rc) return rc;
      const int nent = K + M;
      int32_t *ids = at<int32_t>(h, h->L.ids);
      // the sort helpers index keys as key[(i / B) * Bp + i % B]: B = Bp = 1 reads the compact list
      hipLaunchKernelGGL(rank_sort_kernel, dim3(blocks_for(nent, 64)), dim3(1024), 0, h->side, ids, nent, 1, 1,
                         at<int32_t>(h, h->L.perm2));
      hipLaunchKernelGGL(segment_kernel, dim3(1), dim3(1024), 0, h->side, ids, at<int32_t>(h, h->L.perm2), nent, 1, 1,
                         at<int32_t>(h, h->L.seg2), p_nseg2(h));
    }
    hipLaunchKernelGGL(nce_target_score_kernel<T>, dim3(blocks_for(Mrows, 4)), dim3(256), 0, st, Hs1,
                       at<T>(h, h->L.Wo_c), Hp, yp, h->buf.b, n.lnq, lnZ_lnK, Mrows, c.B, Bp, at<float>(h, h->L.ndt),
                       (float *)nullptr);
    HIP_TRY(hipGetLastError());
    EpiPartial epi;
    epi.part = S;
    epi.ld = Kp;
    epi.split_stride = 0;
    HIP_TRY((mid_gemm<T, ROWK, ROWK>(st, Hs1, Hp, Wn, Hp, Mp, Kp, Hp, 1, epi)));
  }
  StageTimer tm(h, RNNLM_STAGE_NCE_GRAD, st);
  hipLaunchKernelGGL(nce_grad_kernel<T>, dim3(Mp), dim3(256), 0, st, S, Kp, K, at<float>(h, h->L.noff),
                     at<float>(h, h->L.ndt), Tn, c.B, Bp, scale, at<T>(h, h->L.dS_c), at<float>(h, h->L.nct),
                     at<float>(h, h->L.logp_int), n.J_out);
  // bias-gradient column sums of the noise words: 16 row-block partials, added in order by the row update
  hipLaunchKernelGGL(nce_colsum_kernel, dim3(Kp / 64, NCE_COLSUM_PARTS), dim3(1024), 0, st, S, Kp, K,
                     at<float>(h, h->L.noff), Tn, c.B, Bp, scale, at<float>(h, h->L.gcol));
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

// dHs = dS . Wn + ct * Wo[target]  (what the output layer sends back to the hidden states)
template <typename T>
int nce_backward_h(rnnlm_t *h, int Tn, const NceCall &n, hipStream_t st) {
  const int Hp = h->Hp, Bp = h->Bp;
  const int Mrows = Tn * Bp, Mp = (int)round_up(Mrows, PAD_M);
  const int Kp = (int)round_up(n.K, 256);
  float *dHs32 = at<float>(h, h->L.dHs32);
  StageTimer tm(h, RNNLM_STAGE_NCE_BWD_H, st);
  EpiPartial epi;
  epi.part = dHs32;
  epi.ld = Hp;
  epi.split_stride = 0;
  HIP_TRY((mid_gemm<T, ROWK, KROW>(st, at<T>(h, h->L.dS_c), Kp, at<T>(h, h->L.Wn_c), Hp, Mp, Hp, Kp,
                                                      1, epi)));
  hipLaunchKernelGGL(nce_target_dhs_kernel<T>, dim3(Mrows), dim3(256), 0, st, at<T>(h, h->L.Wo_c), Hp,
                     at<int32_t>(h, h->L.yp), at<float>(h, h->L.nct), dHs32);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

// Gradient rows of the noise words (G = dS^T . Hs), then the order-fixed update of every touched row of
// Wo and entry of b (noise words and targets together).
template <typename T>
int nce_update(rnnlm_t *h, int Tn, const NceCall &n, const UpdateTargets &u, hipStream_t st) {
  const rnnlm_config &c = h->cfg;
  const int Hp = h->Hp, Bp = h->Bp;
  const int Mrows = Tn * Bp, Mp = (int)round_up(Mrows, PAD_M), M = Tn * c.B;
  const int K = n.K, Kp = (int)round_up(K, 256);
  T *Hs1 = at<T>(h, h->L.Hs_c) + (long)Bp * Hp;
  float *G = at<float>(h, h->L.G32);
  {
    StageTimer tm(h, RNNLM_STAGE_NCE_BWD_W, st);
    const long per = (long)Kp * Hp;
    constexpr int BK = Elem<T>::BK;
    long S = 256 / ((long)(Kp / 128) * (Hp / 128));  // aim at one round of workgroups
    S = std::min<long>(std::min<long>(S, 8), std::min<long>(Mp / BK, h->L.partElems / per));
    if (S < 1) S = 1;
    EpiPartial epi;
    epi.part = (S == 1) ? G : at<float>(h, h->L.part32);
    epi.ld = Hp;
    epi.split_stride = per;
    HIP_TRY((mid_gemm<T, KROW, KROW>(st, at<T>(h, h->L.dS_c), Kp, Hs1, Hp, Kp, Hp, Mp, (int)S, epi)));
    if (S > 1) {
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks_for(per / 4, 256)), dim3(256), 0, st,
                         at<float>(h, h->L.part32), per, per, (int)S, G);
      HIP_TRY(hipGetLastError());
    }
  }
  StageTimer tm(h, RNNLM_STAGE_NCE_UPDATE, st);
  const int nent = K + M;
  int32_t *ids = at<int32_t>(h, h->L.ids), *perm = at<int32_t>(h, h->L.perm2), *seg = at<int32_t>(h, h->L.seg2);
  {  // the sort of the list was started on the side stream by nce_forward
    int rc = side_join(h, 1, st);
    if (rc) return rc;
  }
  T *Wc = u.refresh_copies ? at<T>(h, h->L.Wo_c) : nullptr;
  if (c.H % 4 == 0) {
    hipLaunchKernelGGL((nce_row_update_kernel<T, 4>), dim3(nent, (c.H + 255) / 256), dim3(1024), 0, st, G, Hs1, Hp,
                       c.H, K, c.B, Bp, at<float>(h, h->L.nct), ids, perm, seg, p_nseg2(h), h->buf.Wo, u.Wo, Wc,
                       at<float>(h, h->L.gcol), Kp, h->buf.b, u.b, u.alpha, u.lr, u.wo_compact_ld);
  } else {
    hipLaunchKernelGGL((nce_row_update_kernel<T, 1>), dim3(nent, (c.H + 63) / 64), dim3(1024), 0, st, G, Hs1, Hp,
                       c.H, K, c.B, Bp, at<float>(h, h->L.nct), ids, perm, seg, p_nseg2(h), h->buf.Wo, u.Wo, Wc,
                       at<float>(h, h->L.gcol), Kp, h->buf.b, u.b, u.alpha, u.lr, u.wo_compact_ld);
  }
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

// Backward half of a window + fused updates.
template <typename T>
int backward_window(rnnlm_t *h, int Tn, const UpdateTargets &u, const NceCall *nce, hipStream_t st) {
  const rnnlm_config &c = h->cfg;
  const int Hp = h->Hp, Bp = h->Bp, Vp = h->Vp;
  const int Mrows = Tn * Bp;
  const int Mp = (int)round_up(Mrows, PAD_M);
  const long ldz = h->MpMax;
  constexpr int BK = Elem<T>::BK;
  T *Hs_c = at<T>(h, h->L.Hs_c);
  T *ZT = at<T>(h, h->L.ZT);
  T *Wo_c = at<T>(h, h->L.Wo_c);
  T *U_c = at<T>(h, h->L.U_c);
  T *dA_c = at<T>(h, h->L.dA_c);
  float *dA32 = at<float>(h, h->L.dA32);
  float *dHs32 = at<float>(h, h->L.dHs32);
  int32_t *xp = at<int32_t>(h, h->L.xp), *yp = at<int32_t>(h, h->L.yp);
  int32_t *perm = at<int32_t>(h, h->L.perm), *seg = at<int32_t>(h, h->L.seg);

  // the integer helpers of the embedding update were started on the side stream by forward_window

  if (nce) {
    int rc = nce_backward_h<T>(h, Tn, *nce, st);
    if (rc) return rc;
  } else {
  // fused softmax gradient + bias update, in place on the vocabulary-major logits
  {
    StageTimer tm(h, RNNLM_STAGE_SOFTMAX_GRAD, st);
    hipLaunchKernelGGL(softmax_grad_kernel<T>, dim3(Vp / 16), dim3(256), 0, st, ZT, ldz, Mp, c.V, Vp,
                       at<float>(h, h->L.lse), yp, 1.0f / (float)(Tn * c.B), h->buf.b, u.b, u.alpha, u.lr);
    HIP_TRY(hipGetLastError());
  }

  // dHs[m][j] = sum_v dz[v][m] Wo[v][j]   (contraction over the vocabulary, split-K); compressed
  // architecture: the same contraction with the tied matrix gives the gradient of the layer above the state
  {
    const int Dp = h->Dp;
    float *dF32 = c.P > 0 ? at<float>(h, h->L.dP32) : dHs32;
    int S = desired_splits(Mp, Dp, Vp / BK);
    const long per = (long)Mp * Dp;
    if ((long)S * per > h->L.partElems) S = (int)(h->L.partElems / per);
    if (S < 1) S = 1;
    EpiPartial epi;
    epi.part = (S == 1) ? dF32 : at<float>(h, h->L.part32);
    epi.ld = Dp;
    epi.split_stride = per;
    {
      StageTimer tm(h, RNNLM_STAGE_OUT_BWD_H, st);
      HIP_TRY((big_gemm<T, 2, 4, KROW, KROW, true>(st, ZT, ldz, Wo_c, Dp, Mp, Dp, Vp, S, epi)));
    }
    if (S > 1) {
      StageTimer tm(h, RNNLM_STAGE_REDUCE, st);
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks_for(per / 4, 256)), dim3(256), 0, st,
                         at<float>(h, h->L.part32), per, per, S, dF32);
      HIP_TRY(hipGetLastError());
    }
  }
  if (c.P > 0) {
    // through the layer above the state: dHs[m][j] = sum_p dp[m][p] C[p][j]
    StageTimer tm(h, RNNLM_STAGE_PROJ, st);
    const long n = (long)Mp * h->Pp;
    T *dP_c = at<T>(h, h->L.dP_c);
    hipLaunchKernelGGL(to_compute_kernel<T>, dim3(blocks_for(n, 256)), dim3(256), 0, st, at<float>(h, h->L.dP32), n, dP_c);
    HIP_TRY(hipGetLastError());
    EpiPartial epi;
    epi.part = dHs32;
    epi.ld = Hp;
    epi.split_stride = 0;
    HIP_TRY((mid_gemm<T, ROWK, KROW>(st, dP_c, h->Pp, at<T>(h, h->L.C_c), Hp, Mp, Hp, h->Pp, 1, epi)));
  }
  }

  // rows [Mrows, Mp) of dA take part in the dU contraction: keep them zero
  if (Mp > Mrows) {
    const long n = (long)(Mp - Mrows) * Hp * (long)sizeof(T) / 4;
    hipLaunchKernelGGL(fill_kernel<uint32_t>, dim3(blocks_for(n, 256)), dim3(256), 0, st,
                       reinterpret_cast<uint32_t *>(dA_c + (long)Mrows * Hp), n, 0u);
  }

  // back-propagation through time over the window (stops at the window start)
  if (persistent_ok(h)) {
    StageTimer tm(h, RNNLM_STAGE_RNN_BWD, st);
    int rc = launch_rnn_persistent<T, true>(h, Tn, false, st);
    if (rc) return rc;
  } else if (sizeof(T) == 2 && resident_ok(h)) {
    StageTimer tm(h, RNNLM_STAGE_RNN_BWD, st);
    int rc = launch_rnn_resident<true>(h, Tn, false, st);
    if (rc) return rc;
  } else
  for (int t = Tn - 1; t >= 0; --t) {
    StageTimer tm(h, (t == 0 || t == Tn - 1) ? RNNLM_STAGE_RNN_BWD : -1, st, t == Tn - 1, t == 0);
    EpiRnnBwd<T> epi;
    epi.dHs = dHs32 + (long)t * Bp * Hp;
    epi.Hs = Hs_c + (long)(t + 1) * Bp * Hp;
    epi.dA32 = dA32 + (long)t * Bp * Hp;
    epi.dAc = dA_c + (long)t * Bp * Hp;
    epi.B = c.B;
    epi.H = c.H;
    epi.ld = Hp;
    const long K = (t == Tn - 1) ? 0 : Hp;
    const T *A_ = dA_c + (long)(t + 1) * Bp * Hp;
    const int S = rnn_step_splits(h);
    if (S > 0) {
      const long per = (long)Bp * Hp;
      EpiPartial ep;
      ep.part = at<float>(h, h->L.part32);
      ep.ld = Hp;
      ep.split_stride = per;
      if (K > 0) {
        if constexpr (sizeof(T) == 2) {
          HIP_TRY((launch_gemm_dma4<256, 128, 4, 2, ROWK, KROW>(st, A_, Hp, U_c, Hp, Bp, Hp, K, S, ep)));
        } else {
          HIP_TRY((launch_gemm<T, 256, 64, 4, 2, ROWK, KROW>(st, A_, Hp, U_c, Hp, Bp, Hp, K, S, ep)));
        }
      }
      hipLaunchKernelGGL(rnn_step_bwd_kernel<T>, dim3(blocks_for(per / 4, 256)), dim3(256), 0, st,
                         at<float>(h, h->L.part32), per, K > 0 ? S : 0, epi.dHs, epi.Hs, c.B, c.H, Hp, per / 4,
                         epi.dA32, epi.dAc);
      HIP_TRY(hipGetLastError());
    } else {
      HIP_TRY((launch_gemm<T, 32, 64, 1, 2, ROWK, KROW>(st, A_, Hp, U_c, Hp, Bp, Hp, K, 1, epi)));
    }
  }

  // E[w] -= lr * sum_{m: x[m] = w} dA[m]: on the side stream, behind the sort helpers already queued there (joined at
  // the end of this function).
  auto embedding_update = [&]() -> int {
  {
    StageTimer tm(h, RNNLM_STAGE_EMB, h->side);
    // plain: rows of dA, width H.  Compressed: rows of dx, width P, added on top of the output-side update the
    // same matrix has just received (training: in the master; gradient export: in the caller's buffer), and
    // the compute copy of the tied matrix follows.
    const float *rows = c.P > 0 ? at<float>(h, h->L.dX32) : dA32;
    const float *src = (c.P > 0 && !u.refresh_copies) ? u.E : h->buf.E;
    const float e_alpha = (c.P > 0 && !u.refresh_copies) ? 1.0f : u.alpha;
    T *Ec = (c.P > 0 && u.refresh_copies) ? Wo_c : nullptr;
    const int W = h->D, Wp = h->Dp;
    if (W % 4 == 0) {
      hipLaunchKernelGGL((scatter_update_kernel<4, T>), dim3(Tn * c.B, (W + 1023) / 1024), dim3(256), 0, h->side, rows,
                         Wp, W, c.B, Bp, xp, perm, seg, p_nseg(h), src, u.E, e_alpha, u.lr, u.e_compact_ld, Ec, Wp);
    } else {
      hipLaunchKernelGGL((scatter_update_kernel<1, T>), dim3(Tn * c.B, (W + 255) / 256), dim3(256), 0, h->side, rows,
                         Wp, W, c.B, Bp, xp, perm, seg, p_nseg(h), src, u.E, e_alpha, u.lr, u.e_compact_ld, Ec, Wp);
    }
    HIP_TRY(hipGetLastError());
  }
    return RNNLM_OK;
  };
  // U[i][j] -= lr * sum_m dA[m][i] Hprev[m][j], contracted transposed (tile rows = j, tile columns = i)
  auto recurrent_update = [&](hipStream_t rs) -> int {
  {
    StageTimer tm(h, RNNLM_STAGE_REC_W, rs);
    EpiSgdT<T> epi;
    epi.W = h->buf.U;
    epi.out = u.U;
    epi.Wc = u.refresh_copies ? U_c : nullptr;
    epi.WcT = u.refresh_copies ? at<T>(h, h->L.UT_c) : nullptr;  // the backward pass reads the transposed copy
    epi.ldw = c.H;
    epi.ldc = Hp;
    epi.R = c.H;
    epi.C = c.H;
    epi.alpha = u.alpha;
    epi.lr = u.lr;
    if (sizeof(T) == 2 && (long)(Hp / BIG) * (Hp / BIG) >= 64) {
      HIP_TRY((big_gemm<T, 2, 4, KROW, KROW, true>(rs, Hs_c, Hp, dA_c, Hp, Hp, Hp, Mp, 1, epi)));
    } else if (Hp <= 1024) {  // small matrix: 64x64 tiles give up to 256 workgroups
      HIP_TRY((launch_gemm<T, 64, 64, 2, 2, KROW, KROW>(rs, Hs_c, Hp, dA_c, Hp, Hp, Hp, Mp, 1, epi)));
    } else {
      HIP_TRY((launch_gemm<T, 128, 128, 2, 2, KROW, KROW>(rs, Hs_c, Hp, dA_c, Hp, Hp, Hp, Mp, 1, epi)));
    }
  }
    return RNNLM_OK;
  };
  // Plain architecture with the normalised criterion: the embedding update and the recurrent weight update need
  // nothing from the output weight update: started on the side stream BEFORE it, they run on the compute units
  // that its last, partly empty round of tiles leaves idle (window time -2 % at H = 2048, -1.3 % at H = 1024).  At
  // H = 4096 the recurrent update is a full round of 256 tiles by itself and keeps its place after the output
  // weight update; the embedding update goes first there as well.
  const bool early_side = !nce && c.P == 0;
  const bool early_rec = early_side && (long)(Hp / BIG) * (Hp / BIG) < 256;
  if (early_side) {
    int rc = side_fork(h, 0, st);
    if (rc) return rc;
    rc = embedding_update();
    if (rc) return rc;
    if (early_rec) {
      rc = recurrent_update(h->side);
      if (rc) return rc;
    }
  }
  if (nce) {
    int rc = nce_update<T>(h, Tn, *nce, u, st);
    if (rc) return rc;
  } else {
    if (c.P > 0) {
      // C[p][j] -= lr * sum_m dp[m][p] h[m][j], contracted transposed (tile rows = j, tile columns = p)
      StageTimer tm(h, RNNLM_STAGE_PROJ, st);
      EpiSgdT<T> epi;
      epi.W = h->buf.C;
      epi.out = u.C;
      epi.Wc = u.refresh_copies ? at<T>(h, h->L.C_c) : nullptr;
      epi.ldw = c.H;
      epi.ldc = Hp;
      epi.R = c.P;
      epi.C = c.H;
      epi.alpha = u.alpha;
      epi.lr = u.lr;
      HIP_TRY((launch_gemm<T, 64, 64, 2, 2, KROW, KROW>(st, Hs_c + (long)Bp * Hp, Hp, at<T>(h, h->L.dP_c), h->Pp, Hp,
                                                        h->Pp, Mp, 1, epi)));
    }
    {
    // Wo[v][j] -= lr * sum_m dz[v][m] Hs[m][j]: bf16 in the matrix's own orientation, fp32 and the compressed
    // architecture contracted transposed (tile rows = j, tile columns = v); compressed architecture: the
    // output-side update of the tied matrix, E[v][p] -= lr * sum_m dz[v][m] p[m][p]
    StageTimer tm(h, RNNLM_STAGE_OUT_BWD_W, st);
    if (sizeof(T) == 2 && c.P == 0) {
      // bf16 path: contracted in the matrix's own orientation (tile rows = v, tile columns = j), whose update
      // epilogue touches two 128-byte lines per wave instruction instead of 32.  Tiles are walked in bands of 4
      // (wide matrices: 8) tile columns, so that the 32 tiles an XCD works on at a time share few operand panels
      // in its L2 (8 x 4 or 4 x 8 instead of 2 x 16: 4 % faster on the widest configuration)
      EpiSgd<T> e2;
      e2.W = h->buf.Wo;
      e2.out = u.Wo;
      e2.Wc = u.refresh_copies ? Wo_c : nullptr;
      e2.ldw = c.H;
      e2.ldc = Hp;
      e2.R = c.V;
      e2.C = c.H;
      e2.alpha = u.alpha;
      e2.lr = u.lr;
      if constexpr (sizeof(T) == 2) {
        // dz is the K-contiguous operand: up to 8 tile columns its tiles travel as whole cache lines (64-deep
        // blocks, gemm_ring64.h: 8-9 % faster at H = 1024 and 2048); the widest layer runs at the chip's power
        // limit, where the symmetric ring measured 0.5 % better
        if (Hp / BIG >= 16) {
          HIP_TRY((big_gemm<T, 2, 4, ROWK, KROW, true>(st, ZT, ldz, Hs_c + (long)Bp * Hp, Hp, Vp, Hp, Mp, 1, e2, -8)));
        } else {
          HIP_TRY((launch_gemm_ring64<BIG, BIG, 2, 4>(st, ZT, ldz, Hs_c + (long)Bp * Hp, Hp, Vp, Hp, Mp, 1, e2, -4)));
        }
      }
    } else {
    EpiSgdT<T> epi;
    epi.W = c.P > 0 ? h->buf.E : h->buf.Wo;
    epi.out = c.P > 0 ? u.E : u.Wo;
    epi.Wc = u.refresh_copies ? Wo_c : nullptr;
    epi.ldw = h->D;
    epi.ldc = h->Dp;
    epi.R = c.V;
    epi.C = h->D;
    epi.alpha = u.alpha;
    epi.lr = u.lr;
    const T *feat = c.P > 0 ? at<T>(h, h->L.P_c) : Hs_c + (long)Bp * Hp;
    if ((long)(h->Dp / BIG) * (Vp / BIG) < 128) {  // a narrow layer above the state: smaller tiles fill the chip
      if constexpr (sizeof(T) == 2) {
        HIP_TRY((launch_gemm_dma4<128, BIG, 2, 4, KROW, ROWK>(st, feat, h->Dp, ZT, ldz, h->Dp, Vp, Mp, 1, epi, -4)));
      } else {
        HIP_TRY((launch_gemm<T, 128, 128, 2, 2, KROW, ROWK>(st, feat, h->Dp, ZT, ldz, h->Dp, Vp, Mp, 1, epi, -2)));
      }
    } else {
      HIP_TRY((big_gemm<T, 2, 4, KROW, ROWK, true>(st, feat, h->Dp, ZT, ldz, h->Dp, Vp, Mp, 1, epi, -2)));
    }
    }
    }
    if (c.P > 0) {
      // through the layer below the state: dx[m][p] = sum_i da[m][i] A[i][p] (before A is updated)
      StageTimer tm(h, RNNLM_STAGE_PROJ, st);
      EpiPartial epi;
      epi.part = at<float>(h, h->L.dX32);
      epi.ld = h->Pp;
      epi.split_stride = 0;
      HIP_TRY((mid_gemm<T, ROWK, KROW>(st, dA_c, Hp, at<T>(h, h->L.A_c), h->Pp, Mp, h->Pp, Hp, 1, epi)));
    }
  }
  if (!early_side) {
    int rc = side_fork(h, 0, st);  // the side stream waits for everything queued so far
    if (rc) return rc;
    rc = embedding_update();
    if (rc) return rc;
  }
  if (c.P > 0) {
    // A[i][p] -= lr * sum_m da[m][i] x[m][p], contracted transposed (tile rows = p, tile columns = i)
    StageTimer tm(h, RNNLM_STAGE_PROJ, st);
    EpiSgdT<T> epi;
    epi.W = h->buf.A;
    epi.out = u.A;
    epi.Wc = u.refresh_copies ? at<T>(h, h->L.A_c) : nullptr;
    epi.ldw = c.P;
    epi.ldc = h->Pp;
    epi.R = c.H;
    epi.C = c.P;
    epi.alpha = u.alpha;
    epi.lr = u.lr;
    HIP_TRY((launch_gemm<T, 64, 64, 2, 2, KROW, KROW>(st, at<T>(h, h->L.Xp_c), h->Pp, dA_c, Hp, h->Pp, Hp, Mp, 1, epi)));
  }

  if (!early_rec) {
    int rc = recurrent_update(st);
    if (rc) return rc;
  }
  // wait for the embedding update running on the side stream
  return side_join(h, 0, st);
}

template <typename T>
int window_call(rnnlm_t *h, const int32_t *x, const int32_t *y, int Tn, float *logp, double *sum_logp,
                const UpdateTargets *u, bool advance_state, hipStream_t st, const NceCall *nce = nullptr) {
  int rc = forward_window<T>(h, x, y, Tn, logp, advance_state, nce == nullptr, st, u != nullptr);
  if (rc) return rc;
  if (nce) {  // per-position losses take the place of the log-probabilities
    rc = nce_forward<T>(h, Tn, *nce, st);
    if (rc) return rc;
  }
  if (sum_logp || u) {
    hipLaunchKernelGGL(sum_logp_kernel, dim3(1), dim3(1024), 0, st, at<float>(h, h->L.logp_int), Tn * h->cfg.B,
                       sum_logp ? sum_logp : p_sum(h), (double *)nullptr, p_flags(h), u ? p_counter(h) : nullptr);
    HIP_TRY(hipGetLastError());
  }
  if (u) rc = backward_window<T>(h, Tn, *u, nce, st);
  return rc;
}

template <typename T>
int score_call(rnnlm_t *h, const int32_t *x, const int32_t *y, int Tn, float lnZ, float *score, hipStream_t st) {
  int rc = forward_window<T>(h, x, y, Tn, nullptr, true, false, st, false, true);
  if (rc) return rc;
  const int Mrows = Tn * h->Bp;
  StageTimer tm(h, RNNLM_STAGE_NCE_SCORE, st);
  // what the output layer reads: the states, or (compressed architecture) the layer above them
  const T *feat = h->cfg.P > 0 ? at<T>(h, h->L.P_c) : at<T>(h, h->L.Hs_c) + (long)h->Bp * h->Hp;
  // the per-position scratch of the log-probability path holds the padded result
  hipLaunchKernelGGL(nce_target_score_kernel<T>, dim3(blocks_for(Mrows, 4)), dim3(256), 0, st, feat,
                     at<T>(h, h->L.Wo_c), h->Dp, at<int32_t>(h, h->L.yp), h->buf.b, (const float *)nullptr, lnZ, Mrows,
                     h->cfg.B, h->Bp, at<float>(h, h->L.zy), score);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

// Forward pass, then the scores of C candidate words per position (no targets: y = nullptr).
template <typename T>
int shortlist_call(rnnlm_t *h, const int32_t *x, const int32_t *cand, int C, int Tn, float lnZ, float *score,
                   hipStream_t st) {
  int rc = forward_window<T>(h, x, nullptr, Tn, nullptr, true, false, st, false, true);
  if (rc) return rc;
  StageTimer tm(h, RNNLM_STAGE_NCE_SCORE, st);
  const T *feat = h->cfg.P > 0 ? at<T>(h, h->L.P_c) : at<T>(h, h->L.Hs_c) + (long)h->Bp * h->Hp;
  const long total = (long)Tn * h->cfg.B * C;
  hipLaunchKernelGGL(score_candidates_kernel<T>, dim3(blocks_for(total, 4)), dim3(256), 0, st, feat,
                     at<T>(h, h->L.Wo_c), h->Dp, cand, C, h->cfg.V, h->buf.b, lnZ, total, h->cfg.B, h->Bp, p_flags(h),
                     score);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

template <typename T>
int quantize_call(rnnlm_t *h, const rnnlm_quantized &q, hipStream_t st) {
  const rnnlm_config &c = h->cfg;
  hipLaunchKernelGGL(quantize_rows_kernel<T>, dim3(c.V), dim3(256), 0, st, h->buf.E, c.P, q.qE, q.sE,
                     reinterpret_cast<T *>(h->ws + h->L.Wo_c), h->Pp);
  hipLaunchKernelGGL(quantize_rows_kernel<T>, dim3(c.H), dim3(256), 0, st, h->buf.A, c.P, q.qA, q.sA,
                     reinterpret_cast<T *>(h->ws + h->L.A_c), h->Pp);
  hipLaunchKernelGGL(quantize_rows_kernel<T>, dim3(c.H), dim3(256), 0, st, h->buf.U, c.H, q.qU, q.sU,
                     reinterpret_cast<T *>(h->ws + h->L.U_c), h->Hp);
  hipLaunchKernelGGL(quantize_rows_kernel<T>, dim3(c.P), dim3(256), 0, st, h->buf.C, c.H, q.qC, q.sC,
                     reinterpret_cast<T *>(h->ws + h->L.C_c), h->Hp);
  hipLaunchKernelGGL(transpose_kernel<T>, dim3(h->Hp / 32, h->Hp / 32), dim3(256), 0, st,
                     reinterpret_cast<T *>(h->ws + h->L.U_c), h->Hp, reinterpret_cast<T *>(h->ws + h->L.UT_c));
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

bool window_args_ok(rnnlm_t *h, const int32_t *x, const int32_t *y, int T) {
  return h && x && y && T >= 1 && T <= h->cfg.T_max;
}

}  // namespace

extern "C" {

size_t rnnlm_workspace_bytes(const rnnlm_config *cfg) {
  if (!cfg_ok(cfg)) return 0;
  int Hp, Vp, Bp, MpMax, nPart, KpMax;
  WsLayout L;
  make_layout(*cfg, Hp, Vp, Bp, MpMax, nPart, KpMax, L);
  return L.total;
}

int rnnlm_init(const rnnlm_config *cfg, const rnnlm_buffers *buf, rnnlm_t **out) {
  if (!out) return RNNLM_ERR_ARG;
  *out = nullptr;
  if (!cfg_ok(cfg) || !buf) return RNNLM_ERR_ARG;
  if (!buf->E || !buf->U || !buf->b || !buf->h_state || !buf->workspace) return RNNLM_ERR_ARG;
  if (cfg->P > 0 ? (buf->Wo || !buf->A || !buf->C) : (!buf->Wo || buf->A || buf->C)) return RNNLM_ERR_ARG;
  if (reinterpret_cast<uintptr_t>(buf->workspace) & 255) return RNNLM_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(buf->E) | reinterpret_cast<uintptr_t>(buf->U) |
       reinterpret_cast<uintptr_t>(buf->Wo) | reinterpret_cast<uintptr_t>(buf->b) |
       reinterpret_cast<uintptr_t>(buf->h_state) | reinterpret_cast<uintptr_t>(buf->A) |
       reinterpret_cast<uintptr_t>(buf->C)) & 15)
    return RNNLM_ERR_ARG;
  rnnlm_t *h = new (std::nothrow) rnnlm_t;
  if (!h) return RNNLM_ERR_NOMEM;
  h->cfg = *cfg;
  h->buf = *buf;
  make_layout(*cfg, h->Hp, h->Vp, h->Bp, h->MpMax, h->nPart, h->KpMax, h->L);
  h->Pp = (int)round_up(cfg->P, PAD_H);
  h->D = cfg->P > 0 ? cfg->P : cfg->H;
  h->Dp = cfg->P > 0 ? h->Pp : h->Hp;
  if (buf->workspace_bytes < h->L.total) {
    delete h;
    return RNNLM_ERR_ARG;
  }
  h->ws = static_cast<char *>(buf->workspace);
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || cfg->device >= ndev || hipSetDevice(cfg->device) != hipSuccess) {
    delete h;
    return RNNLM_ERR_HIP;
  }
  int rc = RNNLM_OK;
  if (hipMemsetAsync(h->ws, 0, h->L.total, nullptr) != hipSuccess ||
      hipMemsetAsync(buf->h_state, 0, sizeof(float) * (size_t)cfg->B * cfg->H, nullptr) != hipSuccess)
    rc = RNNLM_ERR_HIP;
  if (rc == RNNLM_OK)
    rc = (cfg->precision == RNNLM_FP32) ? sync_copies<float>(h, nullptr) : sync_copies<bf16_t>(h, nullptr);
  if (rc == RNNLM_OK && hipDeviceSynchronize() != hipSuccess) rc = RNNLM_ERR_HIP;
  if (rc == RNNLM_OK) {
    // where do the workgroups of a grid land?  (uses the start of the not-yet-used logits buffer)
    constexpr int N = 64 * NUM_XCD;
    int32_t *dev = at<int32_t>(h, h->L.X32);
    int32_t host[N];
    hipLaunchKernelGGL(xcd_probe_kernel, dim3(N), dim3(64), 0, nullptr, dev);
    if (hipMemcpy(host, dev, sizeof(host), hipMemcpyDeviceToHost) != hipSuccess ||
        hipMemsetAsync(dev, 0, sizeof(host), nullptr) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
      rc = RNNLM_ERR_HIP;
    } else {
      // round-robin from whatever XCD the dispatcher had reached: block i on XCD (first + i) mod 8.  The start
      // rotates from launch to launch (it continues where the previous grid ended); what the XCD-local kernels
      // need is only that a grid of 8 n workgroups puts exactly n on every XCD, which any rotation gives.
      bool rr = host[0] >= 0 && host[0] < NUM_XCD;
      for (int i = 0; i < N; ++i) rr = rr && host[i] == (host[0] + i) % NUM_XCD;
      h->xcd_local = rr;
    }
  }
  if (rc == RNNLM_OK) {
    bool ok = hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking) == hipSuccess;
    for (int i = 0; i < 2 && ok; ++i)
      ok = hipEventCreateWithFlags(&h->ev_fork[i], hipEventDisableTiming) == hipSuccess &&
           hipEventCreateWithFlags(&h->ev_join[i], hipEventDisableTiming) == hipSuccess;
    if (!ok) rc = RNNLM_ERR_HIP;
  }
  if (rc != RNNLM_OK) {
    rnnlm_free(h);
    return rc;
  }
  *out = h;
  return RNNLM_OK;
}

void rnnlm_free(rnnlm_t *h) {
  if (!h) return;
  for (EventPair &e : h->prof_pool) {
    (void)hipEventDestroy(e.start);
    (void)hipEventDestroy(e.stop);
  }
  for (int i = 0; i < 2; ++i) {
    if (h->ev_fork[i]) (void)hipEventDestroy(h->ev_fork[i]);
    if (h->ev_join[i]) (void)hipEventDestroy(h->ev_join[i]);
  }
  if (h->side) {
    (void)hipStreamSynchronize(h->side);
    (void)hipStreamDestroy(h->side);
  }
  delete h;
}

int rnnlm_stream_chunk(rnnlm_t *h, const int32_t *tok, int64_t N, int64_t k, int32_t T, int32_t *x, int32_t *y,
                       void *stream) {
  if (!h || !tok || !x || !y || N < 2 || T < 1 || T > h->cfg.T_max) return RNNLM_ERR_ARG;
  const long L = (long)((N - 1) / h->cfg.B);
  if (k < 0 || k >= L / T) return RNNLM_ERR_ARG;
  hipLaunchKernelGGL(stream_chunk_kernel, dim3(blocks_for((long)T * h->cfg.B, 256)), dim3(256), 0, (hipStream_t)stream,
                     tok, L, (long)k, T, h->cfg.B, x, y);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

int rnnlm_forward_logprob(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float *logp, void *stream) {
  if (!window_args_ok(h, x, y, T) || !logp) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  return (h->cfg.precision == RNNLM_FP32) ? window_call<float>(h, x, y, T, logp, nullptr, nullptr, true, st)
                                          : window_call<bf16_t>(h, x, y, T, logp, nullptr, nullptr, true, st);
}

int rnnlm_train_chunk(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float lr, float *logp,
                      double *sum_logp, void *stream) {
  if (!window_args_ok(h, x, y, T) || !(lr == lr)) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  UpdateTargets u{h->buf.E, h->buf.U, h->buf.Wo, h->buf.b, 1.0f, lr, true, true};
  u.A = h->buf.A;
  u.C = h->buf.C;
  return (h->cfg.precision == RNNLM_FP32) ? window_call<float>(h, x, y, T, logp, sum_logp, &u, true, st)
                                          : window_call<bf16_t>(h, x, y, T, logp, sum_logp, &u, true, st);
}

int rnnlm_grad_chunk(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float *dE, float *dU, float *dWo,
                     float *db, float *logp, void *stream) {
  if (!window_args_ok(h, x, y, T) || !dE || !dU || !dWo || !db || h->cfg.P > 0) return RNNLM_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(dE) | reinterpret_cast<uintptr_t>(dU) | reinterpret_cast<uintptr_t>(dWo) |
       reinterpret_cast<uintptr_t>(db)) & 15)
    return RNNLM_ERR_ARG;  // the update epilogues use 16-byte accesses
  hipStream_t st = (hipStream_t)stream;
  const long nE = (long)h->cfg.V * h->cfg.H;
  hipLaunchKernelGGL(fill_kernel<float>, dim3(std::min<long>(blocks_for(nE, 256), 65535)), dim3(256), 0, st, dE, nE,
                     0.0f);
  HIP_TRY(hipGetLastError());
  UpdateTargets u{dE, dU, dWo, db, 0.0f, -1.0f, false, false};
  return (h->cfg.precision == RNNLM_FP32) ? window_call<float>(h, x, y, T, logp, nullptr, &u, false, st)
                                          : window_call<bf16_t>(h, x, y, T, logp, nullptr, &u, false, st);
}

int rnnlm_grad_chunk_compressed(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float *dE, float *dA,
                                float *dU, float *dC, float *db, float *logp, void *stream) {
  if (!window_args_ok(h, x, y, T) || !dE || !dA || !dU || !dC || !db || h->cfg.P <= 0) return RNNLM_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(dE) | reinterpret_cast<uintptr_t>(dA) | reinterpret_cast<uintptr_t>(dU) |
       reinterpret_cast<uintptr_t>(dC) | reinterpret_cast<uintptr_t>(db)) & 15)
    return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  // every entry of dE is written by the output-side contraction; the input rows are then added on top
  UpdateTargets u{dE, dU, nullptr, db, 0.0f, -1.0f, false, false};
  u.A = dA;
  u.C = dC;
  return (h->cfg.precision == RNNLM_FP32) ? window_call<float>(h, x, y, T, logp, nullptr, &u, false, st)
                                          : window_call<bf16_t>(h, x, y, T, logp, nullptr, &u, false, st);
}

int rnnlm_quantize_weights(rnnlm_t *h, const rnnlm_quantized *q, void *stream) {
  if (!h || !q || h->cfg.P <= 0) return RNNLM_ERR_ARG;
  if (!q->qE || !q->sE || !q->qA || !q->sA || !q->qU || !q->sU || !q->qC || !q->sC) return RNNLM_ERR_ARG;
  return (h->cfg.precision == RNNLM_FP32) ? quantize_call<float>(h, *q, (hipStream_t)stream)
                                          : quantize_call<bf16_t>(h, *q, (hipStream_t)stream);
}

namespace {
bool nce_args_ok(rnnlm_t *h, const int32_t *noise, int32_t K, const float *lnq, float lnZ) {
  return h && noise && lnq && K >= 1 && K <= h->cfg.K_max && (lnZ == lnZ);
}
}  // namespace

int rnnlm_nce_train_chunk(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, const int32_t *noise, int32_t K,
                          const float *lnq, float lnZ, float lr, float *J, double *sum_J, void *stream) {
  if (!window_args_ok(h, x, y, T) || !nce_args_ok(h, noise, K, lnq, lnZ) || !(lr == lr)) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  UpdateTargets u{h->buf.E, h->buf.U, h->buf.Wo, h->buf.b, 1.0f, lr, true, true};
  NceCall n{noise, K, lnq, lnZ, J, true};
  return (h->cfg.precision == RNNLM_FP32) ? window_call<float>(h, x, y, T, nullptr, sum_J, &u, true, st, &n)
                                          : window_call<bf16_t>(h, x, y, T, nullptr, sum_J, &u, true, st, &n);
}

int rnnlm_nce_grad_chunk(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, const int32_t *noise, int32_t K,
                         const float *lnq, float lnZ, float *dE, float *dU, float *dWo, float *db, float *J,
                         void *stream) {
  if (!window_args_ok(h, x, y, T) || !nce_args_ok(h, noise, K, lnq, lnZ) || !dE || !dU || !dWo || !db)
    return RNNLM_ERR_ARG;
  if ((reinterpret_cast<uintptr_t>(dE) | reinterpret_cast<uintptr_t>(dU) | reinterpret_cast<uintptr_t>(dWo) |
       reinterpret_cast<uintptr_t>(db)) & 15)
    return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  const long nE = (long)h->cfg.V * h->cfg.H;
  const unsigned fb = (unsigned)std::min<long>(blocks_for(nE, 256), 65535);
  hipLaunchKernelGGL(fill_kernel<float>, dim3(fb), dim3(256), 0, st, dE, nE, 0.0f);
  hipLaunchKernelGGL(fill_kernel<float>, dim3(fb), dim3(256), 0, st, dWo, nE, 0.0f);
  hipLaunchKernelGGL(fill_kernel<float>, dim3(blocks_for(h->cfg.V, 256)), dim3(256), 0, st, db, (long)h->cfg.V, 0.0f);
  HIP_TRY(hipGetLastError());
  UpdateTargets u{dE, dU, dWo, db, 0.0f, -1.0f, false, false};
  NceCall n{noise, K, lnq, lnZ, J, true};
  return (h->cfg.precision == RNNLM_FP32) ? window_call<float>(h, x, y, T, nullptr, nullptr, &u, false, st, &n)
                                          : window_call<bf16_t>(h, x, y, T, nullptr, nullptr, &u, false, st, &n);
}

int rnnlm_forward_score(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float lnZ, float *score,
                        void *stream) {
  if (!window_args_ok(h, x, y, T) || !score || !(lnZ == lnZ)) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  return (h->cfg.precision == RNNLM_FP32) ? score_call<float>(h, x, y, T, lnZ, score, st)
                                          : score_call<bf16_t>(h, x, y, T, lnZ, score, st);
}

int rnnlm_forward_score_shortlist(rnnlm_t *h, const int32_t *x, const int32_t *cand, int32_t C, int32_t T, float lnZ,
                                  float *score, void *stream) {
  if (!h || !x || !cand || !score || T < 1 || T > h->cfg.T_max || C < 1 || C > 65536 || !(lnZ == lnZ))
    return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  return (h->cfg.precision == RNNLM_FP32) ? shortlist_call<float>(h, x, cand, C, T, lnZ, score, st)
                                          : shortlist_call<bf16_t>(h, x, cand, C, T, lnZ, score, st);
}

namespace {
bool rms_args_ok(rnnlm_t *h, float lr, float rho, float eps, const rnnlm_rmsprop_state *s) {
  if (!h || !h->cfg.rmsprop || !s || !s->rE || !s->rU || !s->rWo || !s->rb) return false;
  return (lr == lr) && rho >= 0.0f && rho <= 1.0f && eps >= 0.0f;
}
}  // namespace

int rnnlm_train_chunk_rmsprop(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float lr, float rho,
                              float eps, const rnnlm_rmsprop_state *state, float *logp, double *sum_logp,
                              void *stream) {
  if (!window_args_ok(h, x, y, T) || !rms_args_ok(h, lr, rho, eps, state)) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  const rnnlm_config &c = h->cfg;
  // gradients through the plain step's kernels, update epilogues redirected (out = 0*W + 1*g); the
  // embedding rows go to a compact buffer (one row per distinct input word): the hidden-state gradient
  // buffer, which is free once back-propagation through time is done
  float *gWo = reinterpret_cast<float *>(h->ws + h->L.gWo), *gU = reinterpret_cast<float *>(h->ws + h->L.gU),
        *gb = reinterpret_cast<float *>(h->ws + h->L.gb), *gE = reinterpret_cast<float *>(h->ws + h->L.dHs32);
  UpdateTargets u{gE, gU, gWo, gb, 0.0f, -1.0f, false, true, h->Hp};
  const bool f32 = c.precision == RNNLM_FP32;
  int rc = f32 ? window_call<float>(h, x, y, T, logp, sum_logp, &u, true, st)
               : window_call<bf16_t>(h, x, y, T, logp, sum_logp, &u, true, st);
  if (rc) return rc;
  StageTimer tm(h, RNNLM_STAGE_RMSPROP, st);
  const long nU = (long)c.H * c.H;
  const int32_t *xp = reinterpret_cast<int32_t *>(h->ws + h->L.xp), *perm = reinterpret_cast<int32_t *>(h->ws + h->L.perm),
                *seg = reinterpret_cast<int32_t *>(h->ws + h->L.seg);
  hipLaunchKernelGGL(rms_decay_kernel, dim3(blocks_for(c.V, 256)), dim3(256), 0, st, state->rE, (long)c.V, rho);
  if (f32) {
    float *Wo_c = reinterpret_cast<float *>(h->ws + h->L.Wo_c), *U_c = reinterpret_cast<float *>(h->ws + h->L.U_c);
    hipLaunchKernelGGL(rms_row_apply_kernel<float>, dim3(c.V), dim3(256), 0, st, gWo, (long)c.H, nullptr, nullptr,
                       nullptr, nullptr, c.B, h->Bp, c.H, h->Hp, h->buf.Wo, Wo_c, state->rWo, rho, lr, eps);
    hipLaunchKernelGGL(rms_elem_apply_kernel<float>, dim3(blocks_for(nU, 256)), dim3(256), 0, st, gU, c.H, c.H, h->buf.U,
                       U_c, h->Hp, state->rU, rho, lr, eps);
    hipLaunchKernelGGL(transpose_kernel<float>, dim3(h->Hp / 32, h->Hp / 32), dim3(256), 0, st, U_c, h->Hp,
                       reinterpret_cast<float *>(h->ws + h->L.UT_c));
    hipLaunchKernelGGL(rms_row_apply_kernel<float>, dim3(T * c.B), dim3(256), 0, st, gE, (long)h->Hp, xp, perm, seg,
                       p_nseg(h), c.B, h->Bp, c.H, h->Hp, h->buf.E, (float *)nullptr, state->rE, rho, lr, eps);
  } else {
    bf16_t *Wo_c = reinterpret_cast<bf16_t *>(h->ws + h->L.Wo_c), *U_c = reinterpret_cast<bf16_t *>(h->ws + h->L.U_c);
    hipLaunchKernelGGL(rms_row_apply_kernel<bf16_t>, dim3(c.V), dim3(256), 0, st, gWo, (long)c.H, nullptr, nullptr,
                       nullptr, nullptr, c.B, h->Bp, c.H, h->Hp, h->buf.Wo, Wo_c, state->rWo, rho, lr, eps);
    hipLaunchKernelGGL(rms_elem_apply_kernel<bf16_t>, dim3(blocks_for(nU, 256)), dim3(256), 0, st, gU, c.H, c.H,
                       h->buf.U, U_c, h->Hp, state->rU, rho, lr, eps);
    hipLaunchKernelGGL(transpose_kernel<bf16_t>, dim3(h->Hp / 32, h->Hp / 32), dim3(256), 0, st, U_c, h->Hp,
                       reinterpret_cast<bf16_t *>(h->ws + h->L.UT_c));
    hipLaunchKernelGGL(rms_row_apply_kernel<bf16_t>, dim3(T * c.B), dim3(256), 0, st, gE, (long)h->Hp, xp, perm, seg,
                       p_nseg(h), c.B, h->Bp, c.H, h->Hp, h->buf.E, (bf16_t *)nullptr, state->rE, rho, lr, eps);
  }
  hipLaunchKernelGGL(rms_elem_apply_kernel<float>, dim3(blocks_for(c.V, 256)), dim3(256), 0, st, gb, 1, c.V, h->buf.b,
                     (float *)nullptr, 0, state->rb, rho, lr, eps);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

int rnnlm_nce_train_chunk_rmsprop(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, const int32_t *noise,
                                  int32_t K, const float *lnq, float lnZ, float lr, float rho, float eps,
                                  const rnnlm_rmsprop_state *state, float *J, double *sum_J, void *stream) {
  if (!window_args_ok(h, x, y, T) || !nce_args_ok(h, noise, K, lnq, lnZ) || !rms_args_ok(h, lr, rho, eps, state))
    return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  const rnnlm_config &c = h->cfg;
  float *gU = reinterpret_cast<float *>(h->ws + h->L.gU), *gE = reinterpret_cast<float *>(h->ws + h->L.dHs32),
        *gN = reinterpret_cast<float *>(h->ws + h->L.gN), *gbN = reinterpret_cast<float *>(h->ws + h->L.gbN);
  // gradients through the plain step's kernels; the touched rows of Wo / entries of b and the embedding rows
  // go to compact one-row-per-word buffers
  UpdateTargets u{gE, gU, gN, gbN, 0.0f, -1.0f, false, true, h->Hp, h->Hp};
  NceCall n{noise, K, lnq, lnZ, J, true};
  const bool f32 = c.precision == RNNLM_FP32;
  int rc = f32 ? window_call<float>(h, x, y, T, nullptr, sum_J, &u, true, st, &n)
               : window_call<bf16_t>(h, x, y, T, nullptr, sum_J, &u, true, st, &n);
  if (rc) return rc;
  StageTimer tm(h, RNNLM_STAGE_RMSPROP, st);
  const long nU = (long)c.H * c.H;
  const int nent = K + T * c.B;
  const int32_t *xp = reinterpret_cast<int32_t *>(h->ws + h->L.xp), *perm = reinterpret_cast<int32_t *>(h->ws + h->L.perm),
                *seg = reinterpret_cast<int32_t *>(h->ws + h->L.seg);
  const int32_t *ids = reinterpret_cast<int32_t *>(h->ws + h->L.ids),
                *perm2 = reinterpret_cast<int32_t *>(h->ws + h->L.perm2),
                *seg2 = reinterpret_cast<int32_t *>(h->ws + h->L.seg2);
  const unsigned vb = blocks_for(c.V, 256);
  hipLaunchKernelGGL(rms_decay_kernel, dim3(vb), dim3(256), 0, st, state->rE, (long)c.V, rho);
  hipLaunchKernelGGL(rms_decay_kernel, dim3(vb), dim3(256), 0, st, state->rWo, (long)c.V, rho);
  hipLaunchKernelGGL(rms_decay_kernel, dim3(vb), dim3(256), 0, st, state->rb, (long)c.V, rho);
  if (f32) {
    float *Wo_c = reinterpret_cast<float *>(h->ws + h->L.Wo_c), *U_c = reinterpret_cast<float *>(h->ws + h->L.U_c);
    // the sort helpers' key indexing key[(i / B) * Bp + i % B] with B = Bp = 1 reads the compact id list
    hipLaunchKernelGGL(rms_row_apply_kernel<float>, dim3(nent), dim3(256), 0, st, gN, (long)h->Hp, ids, perm2, seg2,
                       p_nseg2(h), 1, 1, c.H, h->Hp, h->buf.Wo, Wo_c, state->rWo, rho, lr, eps);
    hipLaunchKernelGGL(rms_elem_apply_kernel<float>, dim3(blocks_for(nU, 256)), dim3(256), 0, st, gU, c.H, c.H, h->buf.U,
                       U_c, h->Hp, state->rU, rho, lr, eps);
    hipLaunchKernelGGL(transpose_kernel<float>, dim3(h->Hp / 32, h->Hp / 32), dim3(256), 0, st, U_c, h->Hp,
                       reinterpret_cast<float *>(h->ws + h->L.UT_c));
    hipLaunchKernelGGL(rms_row_apply_kernel<float>, dim3(T * c.B), dim3(256), 0, st, gE, (long)h->Hp, xp, perm, seg,
                       p_nseg(h), c.B, h->Bp, c.H, h->Hp, h->buf.E, (float *)nullptr, state->rE, rho, lr, eps);
  } else {
    bf16_t *Wo_c = reinterpret_cast<bf16_t *>(h->ws + h->L.Wo_c), *U_c = reinterpret_cast<bf16_t *>(h->ws + h->L.U_c);
    hipLaunchKernelGGL(rms_row_apply_kernel<bf16_t>, dim3(nent), dim3(256), 0, st, gN, (long)h->Hp, ids, perm2, seg2,
                       p_nseg2(h), 1, 1, c.H, h->Hp, h->buf.Wo, Wo_c, state->rWo, rho, lr, eps);
    hipLaunchKernelGGL(rms_elem_apply_kernel<bf16_t>, dim3(blocks_for(nU, 256)), dim3(256), 0, st, gU, c.H, c.H,
                       h->buf.U, U_c, h->Hp, state->rU, rho, lr, eps);
    hipLaunchKernelGGL(transpose_kernel<bf16_t>, dim3(h->Hp / 32, h->Hp / 32), dim3(256), 0, st, U_c, h->Hp,
                       reinterpret_cast<bf16_t *>(h->ws + h->L.UT_c));
    hipLaunchKernelGGL(rms_row_apply_kernel<bf16_t>, dim3(T * c.B), dim3(256), 0, st, gE, (long)h->Hp, xp, perm, seg,
                       p_nseg(h), c.B, h->Bp, c.H, h->Hp, h->buf.E, (bf16_t *)nullptr, state->rE, rho, lr, eps);
  }
  hipLaunchKernelGGL(rms_bias_compact_kernel, dim3(blocks_for(nent, 256)), dim3(256), 0, st, gbN, ids, perm2, seg2,
                     p_nseg2(h), h->buf.b, state->rb, rho, lr, eps);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

int rnnlm_reset_state(rnnlm_t *h, void *stream) {
  if (!h) return RNNLM_ERR_ARG;
  const long n = (long)h->cfg.B * h->cfg.H;
  hipLaunchKernelGGL(fill_kernel<float>, dim3(blocks_for(n, 256)), dim3(256), 0, (hipStream_t)stream, h->buf.h_state, n,
                     0.0f);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

int rnnlm_sync_compute_copies(rnnlm_t *h, void *stream) {
  if (!h) return RNNLM_ERR_ARG;
  return (h->cfg.precision == RNNLM_FP32) ? sync_copies<float>(h, (hipStream_t)stream)
                                          : sync_copies<bf16_t>(h, (hipStream_t)stream);
}

int rnnlm_check(rnnlm_t *h, void *stream) {
  if (!h) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  int32_t flags[3] = {0, 0, 0};
  HIP_TRY(hipMemcpyAsync(flags, p_flags(h), sizeof(flags), hipMemcpyDeviceToHost, st));
  hipLaunchKernelGGL(fill_kernel<int32_t>, dim3(1), dim3(64), 0, st, p_flags(h), 3L, 0);
  HIP_TRY(hipStreamSynchronize(st));
  if (flags[2]) return RNNLM_ERR_TIMEOUT;
  if (flags[0]) return RNNLM_ERR_TOKEN_RANGE;
  if (flags[1]) return RNNLM_ERR_NONFINITE;
  return RNNLM_OK;
}

int rnnlm_perplexity(rnnlm_t *h, const int32_t *tok, int64_t N, int32_t T, double *ppl, int64_t *scored,
                     void *stream) {
  if (!h || !tok || !ppl || N < 2 || T < 1 || T > h->cfg.T_max) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  const int B = h->cfg.B;
  const long L = (long)((N - 1) / B);
  const long nchunks = L / T;
  if (nchunks < 1) return RNNLM_ERR_ARG;
  int rc = rnnlm_reset_state(h, stream);
  if (rc) return rc;
  hipLaunchKernelGGL(fill_kernel<double>, dim3(1), dim3(64), 0, st, p_running(h), 1L, 0.0);
  int32_t *xt = at<int32_t>(h, h->L.xtmp), *yt = at<int32_t>(h, h->L.ytmp);
  for (long k = 0; k < nchunks; ++k) {
    hipLaunchKernelGGL(stream_chunk_kernel, dim3(blocks_for((long)T * B, 256)), dim3(256), 0, st, tok, L, k, T, B, xt,
                       yt);
    rc = (h->cfg.precision == RNNLM_FP32) ? forward_window<float>(h, xt, yt, T, nullptr, true, true, st)
                                          : forward_window<bf16_t>(h, xt, yt, T, nullptr, true, true, st);
    if (rc) return rc;
    hipLaunchKernelGGL(sum_logp_kernel, dim3(1), dim3(1024), 0, st, at<float>(h, h->L.logp_int), T * B,
                       (double *)nullptr, p_running(h), p_flags(h), (unsigned *)nullptr);
  }
  HIP_TRY(hipGetLastError());
  double total = 0.0;
  HIP_TRY(hipMemcpyAsync(&total, p_running(h), sizeof(double), hipMemcpyDeviceToHost, st));
  rc = rnnlm_check(h, stream);
  if (rc) return rc;
  const long n = nchunks * (long)B * T;
  *ppl = exp(-total / (double)n);
  if (scored) *scored = n;
  if (!(total == total) || total - total != 0.0) return RNNLM_ERR_NONFINITE;
  return RNNLM_OK;
}

int rnnlm_sort_segments(rnnlm_t *h, const int32_t *x, int32_t T, int32_t *perm, int32_t *seg_start, int32_t *nseg,
                        void *stream) {
  if (!h || !x || !perm || !seg_start || !nseg || T < 1 || T > h->cfg.T_max) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  const int Mp = (int)round_up((long)T * h->Bp, PAD_M);
  const int prep_blocks = (int)blocks_for(Mp, 256);
  hipLaunchKernelGGL(prep_tokens_kernel<float>, dim3(prep_blocks), dim3(256), 0, st, x, (const int32_t *)nullptr, T,
                     h->cfg.B, h->Bp, Mp, h->cfg.V, at<int32_t>(h, h->L.xp), (int32_t *)nullptr,
                     at<float>(h, h->L.lse), p_flags(h), (const float *)nullptr, 0, 0, (float *)nullptr,
                     (unsigned *)nullptr, prep_blocks, (const float *)nullptr, (float *)nullptr,
                     (const float *)nullptr, 0, (float *)nullptr);
  HIP_TRY(hipGetLastError());
  return sort_segments<float>(h, T, perm, seg_start, nseg, st);
}

// ---- the entry point that allocates nothing ----------------------------------------------------------------
namespace {
constexpr int STATIC_MAX_POSITIONS = 65536;  // padded window positions the static scratch holds
struct StaticScratch {
  int32_t xp[STATIC_MAX_POSITIONS];  // padded, range-checked ids
  float lse[STATIC_MAX_POSITIONS];   // the token-preparation kernel marks padded positions here
  int32_t flags[64];                 // [0]: an id was out of range
};
constexpr int STATIC_MAX_DEVICES = 64;
}  // namespace
// One copy per GPU, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress: kernels get the address that call returns for the current device.
static __device__ __align__(256) unsigned char scratch[sizeof(StaticScratch)];
namespace {
std::mutex static_mutex;
StaticScratch *static_ptr[STATIC_MAX_DEVICES] = {nullptr};

// Address of the current device's copy of the scratch array (asked once per device, with that device current).
int static_scratch(StaticScratch **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return RNNLM_ERR_HIP;
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return RNNLM_ERR_ARG;
  std::lock_guard<std::mutex> lock(static_mutex);
  if (!static_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return RNNLM_ERR_HIP;
    static_ptr[dev] = static_cast<StaticScratch *>(p);
  }
  *out = static_ptr[dev];
  return RNNLM_OK;
}

// Hands the range flag to the caller (when asked for) and clears it for the next call.
__global__ void static_flag_kernel(int32_t *flags, int32_t *range_flag) {
  if (threadIdx.x == 0) {
    if (range_flag) *range_flag = flags[0] ? 1 : 0;
    flags[0] = 0;
  }
}
}  // namespace

int rnnlm_sort_segments_static(const int32_t *x, int32_t T, int32_t B, int32_t V, int32_t *perm, int32_t *seg_start,
                               int32_t *nseg, int32_t *range_flag, void *stream) {
  if (!x || !perm || !seg_start || !nseg || T < 1 || B < 1 || V < 1) return RNNLM_ERR_ARG;
  const long Bp = round_up(B, PAD_B);
  const long Mp = round_up((long)T * Bp, PAD_M);
  if (Mp > STATIC_MAX_POSITIONS) return RNNLM_ERR_ARG;  // beyond what the static scratch holds
  StaticScratch *sc = nullptr;
  int rc = static_scratch(&sc);
  if (rc) return rc;
  hipStream_t st = (hipStream_t)stream;
  const int M = T * B;
  const int prep_blocks = (int)blocks_for(Mp, 256);
  // the array keeps the previous call's contents: the flag starts at zero, the ids of all Mp positions are rewritten
  hipLaunchKernelGGL(fill_kernel<int32_t>, dim3(1), dim3(64), 0, st, sc->flags, 64L, 0);
  hipLaunchKernelGGL(prep_tokens_kernel<float>, dim3(prep_blocks), dim3(256), 0, st, x, (const int32_t *)nullptr, T, B,
                     (int)Bp, (int)Mp, V, sc->xp, (int32_t *)nullptr, sc->lse, sc->flags, (const float *)nullptr, 0, 0,
                     (float *)nullptr, (unsigned *)nullptr, prep_blocks, (const float *)nullptr, (float *)nullptr,
                     (const float *)nullptr, 0, (float *)nullptr);
  hipLaunchKernelGGL(rank_sort_kernel, dim3(blocks_for(M, 64)), dim3(1024), 0, st, sc->xp, M, B, (int)Bp, perm);
  hipLaunchKernelGGL(segment_kernel, dim3(1), dim3(1024), 0, st, sc->xp, perm, M, B, (int)Bp, seg_start, nseg);
  hipLaunchKernelGGL(static_flag_kernel, dim3(1), dim3(64), 0, st, sc->flags, range_flag);
  HIP_TRY(hipGetLastError());
  return RNNLM_OK;
}

int rnnlm_set_barrier_spin_limit(rnnlm_t *h, uint32_t polls) {
  if (!h || polls == 0) return RNNLM_ERR_ARG;
  h->spin_limit = polls;
  return RNNLM_OK;
}

int rnnlm_set_recurrent_exchange(rnnlm_t *h, int32_t mode) {
  if (!h) return RNNLM_ERR_ARG;
  if (mode != RNNLM_EXCHANGE_AUTO && mode != RNNLM_EXCHANGE_CHIP_WIDE && mode != RNNLM_EXCHANGE_XCD_LOCAL)
    return RNNLM_ERR_ARG;
  // the XCD-local exchange needs the placement the probe at init looks for and at most one block of 32 streams per XCD
  if (mode == RNNLM_EXCHANGE_XCD_LOCAL && !(h->xcd_local && h->Bp / 32 <= NUM_XCD)) return RNNLM_ERR_ARG;
  h->exchange_mode = mode;
  return RNNLM_OK;
}

int rnnlm_measure_peaks(rnnlm_t *h, double *mfma_bf16_random_tflops, double *mfma_bf16_constant_tflops,
                        double *copy_gbs, void *stream) {
  if (!h || !mfma_bf16_random_tflops || !mfma_bf16_constant_tflops || !copy_gbs) return RNNLM_ERR_ARG;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t e0, e1;
  HIP_TRY(hipEventCreate(&e0));
  HIP_TRY(hipEventCreate(&e1));
  // scratch: the logits buffer (rewritten by the next window's forward pass before anything reads it)
  const size_t es = (h->cfg.precision == RNNLM_FP32) ? 4 : 2;
  char *scratch = h->ws + h->L.ZT;
  const size_t avail = (size_t)h->Vp * h->MpMax * es;
  int rc = RNNLM_OK;
  auto timed = [&](auto launch, double &ms_out) {
    launch();  // warm-up
    if (hipEventRecord(e0, st) != hipSuccess) rc = RNNLM_ERR_HIP;
    launch();
    if (hipEventRecord(e1, st) != hipSuccess || hipEventSynchronize(e1) != hipSuccess) rc = RNNLM_ERR_HIP;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = RNNLM_ERR_HIP;
    ms_out = ms;
  };
  const int iters = 50000;
  const double mfma_flops = 256.0 * 8 * iters * 8 * 32.0 * 32 * 16 * 2;
  double ms = 0.0;
  *mfma_bf16_random_tflops = *mfma_bf16_constant_tflops = *copy_gbs = 0.0;
  if (avail >= 256 * 512 * sizeof(float)) {
    float *out = reinterpret_cast<float *>(scratch);
    timed([&] { hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(256), dim3(512), 0, st, out, iters); }, ms);
    if (rc == RNNLM_OK && ms > 0) *mfma_bf16_random_tflops = mfma_flops / ms / 1e9;
    timed([&] { hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(256), dim3(512), 0, st, out, iters); }, ms);
    if (rc == RNNLM_OK && ms > 0) *mfma_bf16_constant_tflops = mfma_flops / ms / 1e9;
  }
  const size_t half = (avail / 2) & ~(size_t)255;
  if (half >= (8u << 20)) {
    const long n16 = (long)(half / 16);
    timed([&] {
      hipLaunchKernelGGL(copy_kernel, dim3(256 * 32), dim3(256), 0, st, reinterpret_cast<const u32x4_t *>(scratch),
                         reinterpret_cast<u32x4_t *>(scratch + half), n16);
    }, ms);
    if (rc == RNNLM_OK && ms > 0) *copy_gbs = 2.0 * half / ms / 1e6;  // read + write
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (rc == RNNLM_OK && hipGetLastError() != hipSuccess) rc = RNNLM_ERR_HIP;
  return rc;
}

int rnnlm_profile_enable(rnnlm_t *h, uint32_t stage_mask) {
  if (!h || stage_mask >= (1u << RNNLM_STAGE_COUNT)) return RNNLM_ERR_ARG;
  h->prof_mask = stage_mask;
  return RNNLM_OK;
}

int rnnlm_profile_read(rnnlm_t *h, int32_t stage, double *total_ms, int64_t *executions) {
  if (!h || stage < 0 || stage >= RNNLM_STAGE_COUNT || !total_ms || !executions) return RNNLM_ERR_ARG;
  for (size_t i = 0; i < h->prof_used; ++i) {
    EventPair &e = h->prof_pool[i];
    HIP_TRY(hipEventSynchronize(e.stop));
    float ms = 0.0f;
    HIP_TRY(hipEventElapsedTime(&ms, e.start, e.stop));
    h->prof_ms[e.stage] += ms;
    h->prof_n[e.stage] += 1;
  }
  h->prof_used = 0;
  *total_ms = h->prof_ms[stage];
  *executions = h->prof_n[stage];
  h->prof_ms[stage] = 0.0;
  h->prof_n[stage] = 0;
  return RNNLM_OK;
}

const char *rnnlm_status_string(int status) {
  switch (status) {
    case RNNLM_OK: return "ok";
    case RNNLM_ERR_ARG: return "invalid argument";
    case RNNLM_ERR_TOKEN_RANGE: return "token id out of range";
    case RNNLM_ERR_NONFINITE: return "non-finite log-probability sum";
    case RNNLM_ERR_HIP: return "HIP runtime error";
    case RNNLM_ERR_NOMEM: return "host allocation failed";
    case RNNLM_ERR_TIMEOUT: return "grid barrier wait expired";
    default: return "unknown status";
  }
}

}  // extern "C"
