// Persistent recurrent kernels: all T dependent timesteps of a window in ONE launch, with the
// state-to-state matrix held in registers for the whole window (Sec. 4.2 marshals the state-to-state
// work into one large matrix product; on this hardware the serial chain is latency-bound instead, so
// the matrix stays on chip and only the B x H state travels between steps).
//
// Decomposition: workgroup (sb, ub) owns streams [32 sb, +32) x hidden units [32 ub, +32).  Its NWAVE
// (4 or 8) waves split the contraction dimension evenly; each keeps its 32 x (Hp/NWAVE) slice of U (forward:
// rows of U; backward: rows of U^T) as MFMA operand fragments in registers, loads the matching part
// of the previous step's state straight from L2 into operand fragments, and the NWAVE partial 32x32
// tiles are summed through LDS.  Steps are separated by a grid-wide barrier (one atomic counter,
// agent-scope release/acquire); the host guarantees the grid is small enough to be co-resident, and
// the spin is bounded: on expiry a flag is raised and every workgroup still runs to completion.
#pragma once
#include "common.h"
#include "gemm.h"
#include "gemm_dma.h"

namespace rnnlm_dev {

struct RnnPersistArgs {
  const void *W;      // forward: U_c [Hp][Hp]; backward: UT_c [Hp][Hp] (row n holds the k-contiguous operand)
  void *Hs;           // hidden-state slots [(T+1)][Bp][Hp] (slot 0 = carried state)
  const float *X;     // forward: gathered embeddings [T][Bp][Hp]; backward: dHs [T][Bp][Hp]
  float *dA32;        // backward: [T][Bp][Hp]
  void *dAc;          // backward: [T][Bp][Hp] compute type
  float *h_state;     // forward: [B][H] or nullptr
  unsigned *counter;  // SYNC_WORDS barrier / ticket counters, zero at launch (see sync_word)
  int32_t *flags;     // flags[2] raised when a barrier wait expires
  int T, B, H, Bp, Hp;
  unsigned spin_limit;
};

// Coherence between workgroups on different XCDs (each XCD has its own L2): everything one step writes
// and the next step reads (the state h, the gradient dA) moves with agent-scope relaxed atomic
// accesses of 64 bits, which carry the agent-scope cache policy on the access itself.  That avoids
// bulk L2 write-back / invalidate operations at every barrier; ordering comes from every wave waiting
// for the acknowledgement of its own stores (s_waitcnt vmcnt(0)) before the workgroup barrier that
// precedes the arrival atomic, and from the poll loop's control dependency before the loads.
// XCD-local mode.  The workgroups that exchange state with one another are exactly those of one block
// of 32 streams.  When such a group runs on ONE accelerator die (XCD) they share its L2, and the step
// barrier and the state exchange need nothing beyond that L2: plain stores (the vector L1 is
// write-through), a counter updated by atomic adds and polled by loads that bypass the L1, and plain loads
// (a step reads only addresses that no wave of its CU has touched since the kernel started, so the L1
// cannot hold a stale copy).  Placement
// does not rely on the dispatch order: every workgroup reads the id of the XCD it runs on, groups are
// bound to XCDs (stream block x <-> XCD x), and a per-XCD ticket counter hands out the unit blocks;
// surplus workgroups and those on XCDs without a group exit at once.  The host enables this mode only
// after a probe launch has shown that an 8*n grid lands n workgroups on each XCD.
__device__ inline int xcc_id() { return __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15; }  // HW_REG_XCC_ID[3:0]

// Release half of a step barrier, executed by every wave: a workgroup-scope release fence only drains the
// LDS/scalar counter on this target, so the wave also waits until each of its vector-memory stores has been
// acknowledged (vmcnt counts stores as well as loads here); only then may the workgroup signal its arrival.
__device__ inline void wait_own_stores() {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
}

// s_waitcnt vmcnt(n) for a compile-time-unrolled n in {0, 4, 8, ..., MAXN} (the instruction takes an immediate).
template <int MAXN>
__device__ inline void wait_vm_loads(int n) {
  static_assert(MAXN <= 60, "the counter has 6 bits");
  switch (n) {
    case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
    case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
    case 12: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
    case 16: asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
    case 20: asm volatile("s_waitcnt vmcnt(20)" ::: "memory"); break;
    case 24: asm volatile("s_waitcnt vmcnt(24)" ::: "memory"); break;
    case 28: asm volatile("s_waitcnt vmcnt(28)" ::: "memory"); break;
    default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
  }
}

__device__ inline void xcd_barrier(unsigned *counter, unsigned target, unsigned spin_limit, int32_t *flags) {
  wait_own_stores();  // this wave's state stores are in the XCD's L2
  __syncthreads();    // ... and so are those of every other wave of the workgroup
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0;
    // an agent-scope OR with 0: a read of the counter that cannot be served by this compute unit's L1 (the
    // compiler emits it as an agent-scope load)
    while (__hip_atomic_fetch_or(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(1);
      if (++spins >= spin_limit) {
        flags[2] = 1;
        break;
      }
    }
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ inline void grid_barrier(unsigned *counter, unsigned target, unsigned spin_limit, int32_t *flags) {
  wait_own_stores();  // this wave's agent-scope state stores have been acknowledged
  __syncthreads();
  if (threadIdx.x == 0) {
    __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned spins = 0;
    while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
      __builtin_amdgcn_s_sleep(1);
      if (++spins >= spin_limit) {
        flags[2] = 1;
        break;
      }
    }
  }
  __syncthreads();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ inline unsigned long long coherent_load64(const void *p) {
  return __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void coherent_store64(void *p, unsigned long long v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// MFMA operand fragment (8 consecutive-k elements) straight from global memory.
template <typename T, bool COHERENT>
__device__ inline typename FragT<T>::type load_frag_global(const T *p);
template <>
__device__ inline bf16x8_t load_frag_global<bf16_t, false>(const bf16_t *p) {
  return *reinterpret_cast<const bf16x8_t *>(p);
}
template <>
__device__ inline bf16x8_t load_frag_global<bf16_t, true>(const bf16_t *p) {
  union {
    unsigned long long q[2];
    bf16x8_t f;
  } u;
  u.q[0] = coherent_load64(p);
  u.q[1] = coherent_load64(p + 4);
  return u.f;
}
template <>
__device__ inline F32x8 load_frag_global<float, false>(const float *p) {
  F32x8 f;
  const f32x4_t a = *reinterpret_cast<const f32x4_t *>(p);
  const f32x4_t b = *reinterpret_cast<const f32x4_t *>(p + 4);
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f.v[e] = a[e];
    f.v[4 + e] = b[e];
  }
  return f;
}
template <>
__device__ inline F32x8 load_frag_global<float, true>(const float *p) {
  union {
    unsigned long long q[4];
    F32x8 f;
  } u;
#pragma unroll
  for (int e = 0; e < 4; ++e) u.q[e] = coherent_load64(p + 2 * e);
  return u.f;
}

// 4 consecutive values (fp32 in registers) to / from the compute type; store4 uses agent-scope accesses,
// store4_plain ordinary ones.
__device__ inline void store4_plain(float *p, const f32x4_t &v) { *reinterpret_cast<f32x4_t *>(p) = v; }
__device__ inline void store4_plain(bf16_t *p, const f32x4_t &v) {
  bf16x4_t h;
#pragma unroll
  for (int e = 0; e < 4; ++e) h[e] = (bf16_t)v[e];
  *reinterpret_cast<bf16x4_t *>(p) = h;
}
template <typename T>
__device__ inline void store4(T *p, const f32x4_t &v);
template <>
__device__ inline void store4<float>(float *p, const f32x4_t &v) {
  union {
    unsigned long long q[2];
    f32x4_t f;
  } u;
  u.f = v;
  coherent_store64(p, u.q[0]);
  coherent_store64(p + 2, u.q[1]);
}
template <>
__device__ inline void store4<bf16_t>(bf16_t *p, const f32x4_t &v) {
  union {
    unsigned long long q;
    bf16x4_t h;
  } u;
#pragma unroll
  for (int e = 0; e < 4; ++e) u.h[e] = (bf16_t)v[e];
  coherent_store64(p, u.q);
}
template <typename T>
__device__ inline f32x4_t load4(const T *p);
template <>
__device__ inline f32x4_t load4<float>(const float *p) {
  return *reinterpret_cast<const f32x4_t *>(p);
}
template <>
__device__ inline f32x4_t load4<bf16_t>(const bf16_t *p) {
  const bf16x4_t h = *reinterpret_cast<const bf16x4_t *>(p);
  f32x4_t v;
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = (float)h[e];
  return v;
}

// STAGED (bf16, XCD-local mode, KS a multiple of 4): the previous step's state reaches the MFMA operand
// registers through LDS instead of straight from the L2.  Loaded straight into fragments, every lane asks for
// 16 bytes of a different row, and the vector L1 handles such a wave instruction as 64 separate line
// look-ups: at 16 instructions per wave and step that address path, not the L2 or the barrier, set the step
// time (counters: the texture addresser busy 58 % of the kernel, 47 M tag look-ups for 0.6 GB).  Staged, each
// wave copies its own [32 streams][64 k] blocks with direct global->LDS loads whose 64 lanes cover one
// contiguous kilobyte of LDS and eight full 128-byte lines of memory (8 look-ups instead of 64), then reads
// the fragments from LDS.  The block layout and its XOR swizzle are those of the 64-deep K-contiguous tile of
// the contraction kernels (physical 16-byte chunk = logical ^ ((row >> 1) & 7)).  A wave reads only what it
// copied itself, so the copy is ordered by that wave's own s_waitcnt; the buffer is reused every step.
// All of a wave's blocks are resident at once (4 waves, up to 16 KB each); 1024 < Hp <= 2048 takes the wide
// kernel further down.
//
// KS = 16-wide contraction steps per wave = Hp / (16 NWAVE).  BACKWARD = false: h_t = sigmoid(X_t + h_{t-1} U^T)
// for t = 0..T-1.  BACKWARD = true: dA_t = (dHs_t + dA_{t+1} U) * h_t * (1 - h_t) for t = T-1..0.
// XCD = true: XCD-local mode (see above); false: the grid spans the chip and uses agent-scope accesses.
// (8 waves: two workgroups share a compute unit when Hp = 2048, so a wave may use at most 128 registers.)
template <typename T, int KS, int NWAVE, bool BACKWARD, bool XCD, bool STAGED = false>
__global__ void __launch_bounds__(64 * NWAVE, NWAVE == 8 ? 4 : 1) rnn_persistent_kernel(const RnnPersistArgs a) {
  static_assert(!STAGED || (XCD && sizeof(T) == 2 && KS % 4 == 0 && NWAVE == 4),
                "staged state loads: bf16, XCD-local, 4 waves, whole blocks");
  constexpr int NBLK = KS / 4;  // [32][64] blocks of this wave's share of the state (STAGED)
  constexpr int WAVE_STAGE = NBLK * 4096;  // bytes of staging per wave
  __shared__ __attribute__((aligned(16))) float red_own[NWAVE][16][64];
  __shared__ __attribute__((aligned(1024))) char stage[STAGED ? NWAVE * WAVE_STAGE : 16];
  __shared__ int s_ticket;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  auto red_at = [&](int q) -> float * { return &red_own[q][0][0]; };  // partial 32x32 tile of wave q
  const int nsb = a.Bp / 32;
  int sb, ub;
  unsigned nwg;
  unsigned *counter;
  if (XCD) {
    const int x = xcc_id();
    if (x >= nsb) return;  // no group lives on this XCD
    if (threadIdx.x == 0)
      s_ticket = (int)__hip_atomic_fetch_add(a.counter + sync_word(2, x), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    sb = x;
    ub = s_ticket;
    nwg = (unsigned)(a.Hp / 32);
    if (ub >= (int)nwg) return;  // surplus workgroup
    counter = a.counter + sync_word(1, x);
  } else {
    sb = blockIdx.x % nsb;
    ub = blockIdx.x / nsb;
    nwg = gridDim.x;
    counter = a.counter;
  }
  const int Hp = a.Hp, Bp = a.Bp;
  const long slot = (long)Bp * Hp;
  const int kq = wave * (KS * 16);  // first contraction index of this wave
  const int lr = lane & 31, lk = (lane >> 5) * 8;

  // this wave's slice of the matrix, resident in registers for all T steps
  typename FragT<T>::type w[KS];
  {
    const T *Wp = static_cast<const T *>(a.W) + (long)(ub * 32 + lr) * Hp + kq + lk;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) w[kk] = load_frag_global<T, false>(Wp + kk * 16);
  }
#if defined(__HIP_DEVICE_COMPILE__)
  // STAGED: buffer resource over the whole state (gradient) buffer and this lane's offsets inside a block
  typedef int i32x4_t __attribute__((ext_vector_type(4)));
  i32x4_t rsrc = {0, 0, 0, 0};
  int goff[4] = {0, 0, 0, 0};
  int frag_off[4] = {0, 0, 0, 0};
  if constexpr (STAGED) {
    const unsigned long long base = reinterpret_cast<unsigned long long>(BACKWARD ? a.dAc : a.Hs);
    rsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
    rsrc[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((base >> 32) & 0xffffu));
    rsrc[2] = __builtin_amdgcn_readfirstlane((int)((long)(a.T + 1) * slot * 2));
    rsrc[3] = 0x00020000;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = i * 8 + (lane >> 3), pch = lane & 7;  // LDS chunk (r, pch) of the block <- memory chunk pch ^ swz(r)
      goff[i] = (int)(((long)(sb * 32 + r) * Hp + kq) * 2 + ((pch ^ rowk_swz(r)) << 4));
    }
#pragma unroll
    for (int st = 0; st < 4; ++st) frag_off[st] = lr * 128 + (((2 * st + (lane >> 5)) ^ rowk_swz(lr)) << 4);
  }
#endif
  // epilogue ownership (first 256 threads): thread -> accumulator element r = tid/16 of lanes
  // 4*(tid%16) .. +3, i.e. one stream and 4 consecutive hidden units
  const bool epi_thread = tid < 256;
  const int er = (tid >> 4) & 15, el = (tid & 15) * 4;
  const int erow = sb * 32 + ((er >> 2) << 3) + ((el >> 5) << 2) + (er & 3);
  const int ecol = ub * 32 + (el & 31);
  const bool row_ok = epi_thread && erow < a.B;
  T *Hs = static_cast<T *>(a.Hs);
  T *dAc = static_cast<T *>(a.dAc);

  for (int step = 0; step < a.T; ++step) {
    const int t = BACKWARD ? a.T - 1 - step : step;
    const long eidx = (long)t * slot + (long)erow * Hp + ecol;
    // operands of the epilogue do not depend on the previous step: fetch them early
    f32x4_t xin = {0.f, 0.f, 0.f, 0.f};
    f32x4_t hcur = {0.f, 0.f, 0.f, 0.f};
    if (row_ok) {
      xin = *reinterpret_cast<const f32x4_t *>(a.X + eidx);
      if (BACKWARD) hcur = load4<T>(Hs + slot + eidx);
    }
    f32x16_t acc, acc2;  // two accumulation chains: consecutive MFMAs do not wait for one another
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = acc2[r] = 0.0f;
    const bool contract = !(BACKWARD && step == 0);  // nothing flows into the window's last position
    if (contract) {
      const T *src = BACKWARD ? dAc + (long)(t + 1) * slot : Hs + (long)t * slot;
      const T *Ap = src + (long)(sb * 32 + lr) * Hp + kq + lk;
      typename FragT<T>::type f[KS];
#if defined(__HIP_DEVICE_COMPILE__)
      if constexpr (STAGED) {
        char *sw = stage + wave * WAVE_STAGE;
        const int soff = (int)((long)(BACKWARD ? t + 1 : t) * slot * 2);
        auto copy_block = [&](int b, char *dst) {  // block b of this wave's share -> 4 KB at dst
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const unsigned lds_addr = (unsigned)(unsigned long long)(lds_void_ptr)(dst + i * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                         :
                         : "s"(lds_addr), "v"(goff[i]), "s"(rsrc), "s"(soff + b * 128)
                         : "memory", "m0");
          }
        };
#pragma unroll
        for (int b = 0; b < NBLK; ++b) copy_block(b, sw + b * 4096);
        // block by block as this wave's copies land in LDS (4 loads per block, returned in order)
#pragma unroll
        for (int b = 0; b < NBLK; ++b) {
          wait_vm_loads<4 * (NBLK - 1)>(4 * (NBLK - 1 - b));
#pragma unroll
          for (int kk = 4 * b; kk < 4 * b + 4; ++kk)
            f[kk] = *reinterpret_cast<const bf16x8_t *>(sw + (kk >> 2) * 4096 + frag_off[kk & 3]);
        }
      } else
#endif
      {
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) f[kk] = load_frag_global<T, !XCD>(Ap + kk * 16);
      }
#pragma unroll
      for (int kk = 0; kk < KS; kk += 2) {
        mma16(acc, f[kk], w[kk]);
        if (kk + 1 < KS) mma16(acc2, f[kk + 1], w[kk + 1]);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] += acc2[r];
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) red_at(wave)[r * 64 + lane] = acc[r];
    __syncthreads();
    f32x4_t s = *reinterpret_cast<const f32x4_t *>(red_at(0) + er * 64 + el);
#pragma unroll
    for (int q = 1; q < NWAVE; ++q) {
      const f32x4_t p = *reinterpret_cast<const f32x4_t *>(red_at(q) + er * 64 + el);
#pragma unroll
      for (int e = 0; e < 4; ++e) s[e] += p[e];
    }
    f32x4_t o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool ok = row_ok && (ecol + e) < a.H;
      if (!BACKWARD) {
        o[e] = ok ? sigmoidf_(s[e] + xin[e]) : 0.0f;
      } else {
        o[e] = ok ? (xin[e] + s[e]) * hcur[e] * (1.0f - hcur[e]) : 0.0f;
      }
    }
    if (!epi_thread) {
      // waves 4..7 only contribute partial sums
    } else if (!BACKWARD) {
      if (XCD) store4_plain(Hs + slot + eidx, o); else store4<T>(Hs + slot + eidx, o);
      if (a.h_state && step == a.T - 1 && row_ok) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (ecol + e < a.H) a.h_state[(long)erow * a.H + ecol + e] = o[e];
      }
    } else {
      *reinterpret_cast<f32x4_t *>(a.dA32 + eidx) = o;
      if (XCD) store4_plain(dAc + eidx, o); else store4<T>(dAc + eidx, o);
    }
    if (step + 1 < a.T) {
      if (XCD) xcd_barrier(counter, (unsigned)(step + 1) * nwg, a.spin_limit, a.flags);
      else grid_barrier(counter, (unsigned)(step + 1) * nwg, a.spin_limit, a.flags);
    }
  }
}

// Wide variant for 1024 < Hp <= 2048 (bf16, XCD-local mode, KS a multiple of 4): a workgroup of 8 waves owns
// 32 streams x 64 hidden units (two 32-unit tiles), so a group is Hp/64 workgroups, ONE per compute unit of
// its XCD: the previous state is copied into LDS once per compute unit and step (128 KB at Hp = 2048, all of
// a wave's blocks resident), each fragment read from LDS feeds two MFMAs, and the weights of both tiles stay
// in registers (128 per wave).  The partial-sum exchange buffer lives in the staging memory: a wave writes
// its two partial tiles over the start of its own region once its fragments are consumed, and the next
// step's copies start only after the step barrier, which every wave reaches after its reads of the exchange
// buffer.  Same arithmetic order per output as the 32-unit kernels (waves' partials added 0..7).
template <int KS, bool BACKWARD>
__global__ void __launch_bounds__(512, 2) rnn_persistent_wide_kernel(const RnnPersistArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef bf16_t T;
  constexpr int NWAVE = 8, UT = 2;
  static_assert(KS % 4 == 0 && KS >= 8, "whole [32][64] blocks, at least 8 KB of staging per wave");
  constexpr int NBLK = KS / 4;
  constexpr int WAVE_STAGE = NBLK * 4096;
  __shared__ __attribute__((aligned(1024))) char stage[NWAVE * WAVE_STAGE];
  __shared__ int s_ticket;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nsb = a.Bp / 32;
  const int x = xcc_id();
  if (x >= nsb) return;  // no group lives on this XCD
  if (threadIdx.x == 0)
    s_ticket = (int)__hip_atomic_fetch_add(a.counter + sync_word(2, x), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  const int sb = x, ub = s_ticket;
  const unsigned nwg = (unsigned)(a.Hp / 64);
  if (ub >= (int)nwg) return;  // surplus workgroup
  unsigned *counter = a.counter + sync_word(1, x);
  const int Hp = a.Hp, Bp = a.Bp;
  const long slot = (long)Bp * Hp;
  const int kq = wave * (KS * 16);
  const int lr = lane & 31, lk = (lane >> 5) * 8;

  bf16x8_t w[UT][KS];
#pragma unroll
  for (int u = 0; u < UT; ++u) {
    const T *Wp = static_cast<const T *>(a.W) + (long)(ub * 64 + u * 32 + lr) * Hp + kq + lk;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) w[u][kk] = load_frag_global<T, false>(Wp + kk * 16);
  }
  typedef int i32x4_t __attribute__((ext_vector_type(4)));
  i32x4_t rsrc;
  int goff[4], frag_off[4];
  {
    const unsigned long long base = reinterpret_cast<unsigned long long>(BACKWARD ? a.dAc : a.Hs);
    rsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
    rsrc[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((base >> 32) & 0xffffu));
    rsrc[2] = __builtin_amdgcn_readfirstlane((int)((long)(a.T + 1) * slot * 2));
    rsrc[3] = 0x00020000;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = i * 8 + (lane >> 3), pch = lane & 7;
      goff[i] = (int)(((long)(sb * 32 + r) * Hp + kq) * 2 + ((pch ^ rowk_swz(r)) << 4));
    }
#pragma unroll
    for (int st = 0; st < 4; ++st) frag_off[st] = lr * 128 + (((2 * st + (lane >> 5)) ^ rowk_swz(lr)) << 4);
  }
  // epilogue ownership: threads 0..255 the first unit tile, 256..511 the second; inside a tile as in the
  // 32-unit kernels (accumulator element r = t/16 of lanes 4*(t%16) .. +3: one stream, 4 consecutive units)
  const int eu = tid >> 8, t8 = tid & 255;
  const int er = (t8 >> 4) & 15, el = (t8 & 15) * 4;
  const int erow = sb * 32 + ((er >> 2) << 3) + ((el >> 5) << 2) + (er & 3);
  const int ecol = ub * 64 + eu * 32 + (el & 31);
  const bool row_ok = erow < a.B;
  T *Hs = static_cast<T *>(a.Hs);
  T *dAc = static_cast<T *>(a.dAc);
  char *sw = stage + wave * WAVE_STAGE;

  for (int step = 0; step < a.T; ++step) {
    const int t = BACKWARD ? a.T - 1 - step : step;
    const long eidx = (long)t * slot + (long)erow * Hp + ecol;
    f32x4_t xin = {0.f, 0.f, 0.f, 0.f};
    f32x4_t hcur = {0.f, 0.f, 0.f, 0.f};
    if (row_ok) {
      xin = *reinterpret_cast<const f32x4_t *>(a.X + eidx);
      if (BACKWARD) hcur = load4<T>(Hs + slot + eidx);
    }
    f32x16_t acc[UT], acc2[UT];
#pragma unroll
    for (int u = 0; u < UT; ++u)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[u][r] = acc2[u][r] = 0.0f;
    const bool contract = !(BACKWARD && step == 0);
    if (contract) {
      const int soff = (int)((long)(BACKWARD ? t + 1 : t) * slot * 2);
#pragma unroll
      for (int b = 0; b < NBLK; ++b)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned lds_addr = (unsigned)(unsigned long long)(lds_void_ptr)(sw + b * 4096 + i * 1024);
          asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                       :
                       : "s"(lds_addr), "v"(goff[i]), "s"(rsrc), "s"(soff + b * 128)
                       : "memory", "m0");
        }
#pragma unroll
      for (int kk = 0; kk < KS; kk += 2) {
        // block by block as this wave's copies land in LDS (4 loads per block, returned in order)
        if ((kk & 3) == 0) wait_vm_loads<4 * (NBLK - 1)>(4 * (NBLK - 1 - (kk >> 2)));
        const bf16x8_t f0 = *reinterpret_cast<const bf16x8_t *>(sw + (kk >> 2) * 4096 + frag_off[kk & 3]);
        const bf16x8_t f1 = *reinterpret_cast<const bf16x8_t *>(sw + ((kk + 1) >> 2) * 4096 + frag_off[(kk + 1) & 3]);
#pragma unroll
        for (int u = 0; u < UT; ++u) {
          mma16(acc[u], f0, w[u][kk]);
          mma16(acc2[u], f1, w[u][kk + 1]);
        }
      }
#pragma unroll
      for (int u = 0; u < UT; ++u)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[u][r] += acc2[u][r];
    }
    // every fragment this wave read is consumed: its staging memory now carries its partial tiles
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int u = 0; u < UT; ++u) {
      float *red = reinterpret_cast<float *>(sw + u * 4096);
#pragma unroll
      for (int r = 0; r < 16; ++r) red[r * 64 + lane] = acc[u][r];
    }
    __syncthreads();
    f32x4_t s = *reinterpret_cast<const f32x4_t *>(reinterpret_cast<const float *>(stage + eu * 4096) + er * 64 + el);
#pragma unroll
    for (int q = 1; q < NWAVE; ++q) {
      const f32x4_t p = *reinterpret_cast<const f32x4_t *>(
          reinterpret_cast<const float *>(stage + q * WAVE_STAGE + eu * 4096) + er * 64 + el);
#pragma unroll
      for (int e = 0; e < 4; ++e) s[e] += p[e];
    }
    f32x4_t o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool ok = row_ok && (ecol + e) < a.H;
      if (!BACKWARD) {
        o[e] = ok ? sigmoidf_(s[e] + xin[e]) : 0.0f;
      } else {
        o[e] = ok ? (xin[e] + s[e]) * hcur[e] * (1.0f - hcur[e]) : 0.0f;
      }
    }
    if (!BACKWARD) {
      store4_plain(Hs + slot + eidx, o);
      if (a.h_state && step == a.T - 1 && row_ok) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (ecol + e < a.H) a.h_state[(long)erow * a.H + ecol + e] = o[e];
      }
    } else {
      *reinterpret_cast<f32x4_t *>(a.dA32 + eidx) = o;
      store4_plain(dAc + eidx, o);
    }
    if (step + 1 < a.T) xcd_barrier(counter, (unsigned)(step + 1) * nwg, a.spin_limit, a.flags);
  }
#endif
}

// Records which XCD each workgroup of the launch runs on.
__global__ void xcd_probe_kernel(int32_t *out) {
  if (threadIdx.x == 0) out[blockIdx.x] = xcc_id();
}

}  // namespace rnnlm_dev
