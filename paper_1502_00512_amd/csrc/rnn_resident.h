// Recurrent kernel for the widest hidden layer (Hp = 4096, 256 streams, bf16): all T dependent timesteps of a
// window in ONE launch that fills the chip, with the 32 MB state-to-state matrix spread over the register
// files of all 256 compute units for the whole window (Sec. 4.2 marshals the state-to-state work into one
// large matrix product per step; here only the B x H state and partial sums travel between steps).
//
// Decomposition.  XCD x (its own L2, 32 compute units, one workgroup each) owns the 512 hidden units
// [512 x, +512).  Workgroup j of an XCD (a ticket from a per-XCD counter, so placement does not rely on the
// dispatch order) is (kc, uc, sh) = (j / 8, (j / 2) % 4, j % 2): contraction range [1024 kc, +1024), units
// [512 x + 128 uc, +128), streams [128 sh, +128).  Its eight waves (kh, uq) each keep 32 units x 512 values of
// the contraction dimension as MFMA operand fragments in registers (128 per lane) and run 128 streams through
// them: the state arrives by direct global->LDS loads in eight chunks of 2 x [128 streams][64 k] through a ring
// of four 32 KB stages (one [32 streams][64 k] block per wave and chunk).
//
// Per step: (A) the contraction; (B) the two halves of the workgroup's contraction range are added through
// LDS and the workgroup's partial [128 streams][128 units] goes to a partial-sum buffer that only its XCD
// reads; XCD barrier; (C) workgroup j sums the four partials of streams [8 j, +8) x the XCD's 512 units in
// fixed order, applies the elementwise part and stores the new state; chip-wide barrier.  The elementwise
// part's other operands (the step's rows of X / dHs and, backward, of h) are copied into LDS a step ahead.
//
// Coherence.  Partial sums stay inside one XCD, whose L2 is the one cache its compute units share: plain stores
// (the vector L1 is write-through; every wave waits for their acknowledgement before the workgroup signals)
// and loads with the agent-scope policy, which bypass the L1 (the buffer is reused every step, so the L1 may
// still hold last step's lines).  The state crosses XCDs: agent-scope stores (written through to the memory
// side), read only after the chip-wide barrier by agent-scope loads of addresses no compute unit has touched
// since they were written.
//
// Barriers.  Every counter sits on a line of its own (sync_word) and is polled by at most the 32 workgroups of
// one XCD.  The chip-wide barrier counts arrivals per XCD; the last workgroup of an XCD adds one to every XCD's
// copy of the count of XCDs that have arrived, and a workgroup polls its own XCD's copy.
// Every wait is bounded: on expiry flags[2] is raised and every workgroup still runs to its end.
#pragma once
#include "rnn_persistent.h"

namespace rnnlm_dev {

constexpr int RES_HP = 4096;    // padded hidden size this kernel is built for
constexpr int RES_BP = 256;     // padded streams
constexpr long RES_PART_XCD = 4L * RES_BP * (RES_HP / 8);  // floats of partial sums per XCD and step
constexpr long RES_PART_STEP = 8 * RES_PART_XCD;           // floats per step (16 MB)

struct RnnResidentArgs {
  RnnPersistArgs p;
  float *part;  // [8 XCDs][4 kc][256 streams][512 units], reused by every step
};

template <bool BACKWARD>
__global__ void __launch_bounds__(512) rnn_resident_kernel(const RnnResidentArgs ra) {
#if defined(__HIP_DEVICE_COMPILE__)
  typedef bf16_t T;
  const RnnPersistArgs &a = ra.p;
  constexpr int HP = RES_HP, BP = RES_BP;
  constexpr int NSTAGE = 4, STAGE = 32768, NCHUNK = 8;
  constexpr long slot = (long)BP * HP;
  __shared__ __attribute__((aligned(1024))) char stage[NSTAGE * STAGE];
  __shared__ __attribute__((aligned(1024))) char xstage[8 * 3072];  // per wave: 2 KB of X (dHs), 1 KB of h (backward)
  __shared__ int s_ticket;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int x = xcc_id();
  if (tid == 0)
    s_ticket = (int)__hip_atomic_fetch_add(a.counter + sync_word(2, x), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  const int j = s_ticket;
  if (j >= 32) return;  // surplus workgroup
  const int kc = j >> 3, uc = (j >> 1) & 3, sh = j & 1;
  const int kh = wave >> 2, uq = wave & 3;
  const int lr = lane & 31, lk = (lane >> 5) * 8;
  const int n0 = x * 512 + uc * 128 + uq * 32;  // first unit of this wave (global index)
  const int k0 = kc * 1024 + kh * 512;          // first contraction index of this wave
  unsigned *xcounter = a.counter + sync_word(1, x);
  unsigned *garrive = a.counter + sync_word(3, x);
  unsigned *ggo = a.counter + sync_word(4, x);

  // this wave's slice of the matrix, resident for all T steps: row n of W holds the k-contiguous operand
  bf16x8_t w[32];
  {
    const T *Wp = static_cast<const T *>(a.W) + (long)(n0 + lr) * HP + k0 + lk;
#pragma unroll
    for (int kk = 0; kk < 32; ++kk) w[kk] = *reinterpret_cast<const bf16x8_t *>(Wp + kk * 16);
    // (a wait the compiler's counter bookkeeping sees: otherwise it re-waits for these loads inside the step loop,
    // where its counts would also drain the state copies in flight)
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
  }

  // state copies: this wave brings in, per chunk, one [32 streams][64 k] block of its own half of the
  // contraction range (stream block uq of the workgroup's 128 streams); block (half, sbk) of a stage sits at
  // (half * 4 + sbk) * 4 KB in the swizzled layout of the contraction kernels' K-contiguous tile
  typedef int i32x4_t __attribute__((ext_vector_type(4)));
  i32x4_t rsrc;
  int goff[4];
  {
    const unsigned long long base = reinterpret_cast<unsigned long long>(BACKWARD ? a.dAc : a.Hs);
    rsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)base);
    rsrc[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((base >> 32) & 0xffffu));
    rsrc[2] = __builtin_amdgcn_readfirstlane((int)((long)(a.T + 1) * slot * 2));
    rsrc[3] = 0x00020000;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = i * 8 + (lane >> 3), pch = lane & 7;
      goff[i] = (int)(((long)(sh * 128 + uq * 32 + r) * HP + k0) * 2 + ((pch ^ rowk_swz(r)) << 4));
    }
  }
  // partial-sum stores go through a buffer resource over the whole partial buffer
  __amdgpu_buffer_rsrc_t prsrc = __builtin_amdgcn_make_buffer_rsrc(ra.part, 0, (int)(RES_PART_STEP * 4), 0x00020000);
  const int pvoff = ((((lane >> 5) << 2) * 512) + lr) * 4;
  char *const copy_dst = stage + (kh * 4 + uq) * 4096;
  auto copy_chunk = [&](int c, int soff) {  // chunk c of the step whose state starts soff bytes into the buffer
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const unsigned lds_addr =
          (unsigned)(unsigned long long)(lds_void_ptr)(copy_dst + (c & (NSTAGE - 1)) * STAGE + i * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen sc1 lds"
                   :
                   : "s"(lds_addr), "v"(goff[i]), "s"(rsrc), "s"(soff + c * 128)
                   : "memory", "m0");
    }
  };
  // fragment reads: accumulator tile lb of this wave covers stream block lb ^ (2 kh), so that the two tiles a
  // wave finishes itself (lb = 0, 1) are the ones its partner hands over (lb = 2, 3 there)
  int frag_off[4];
#pragma unroll
  for (int st = 0; st < 4; ++st) frag_off[st] = lr * 128 + (((2 * st + (lane >> 5)) ^ rowk_swz(lr)) << 4);
  const int blk0 = (kh * 4) * 4096;
  const int flip = 2 * kh;

  // step epilogue ownership: stream 8 j + tid / 64, units 8 (tid % 64) .. +7 of the XCD's 512
  const int erow = __builtin_amdgcn_readfirstlane(8 * j + wave);
  const int ecl = lane * 8;
  const int ecol = x * 512 + ecl;
  const bool row_ok = erow < a.B;
  T *Hs = static_cast<T *>(a.Hs);
  T *dAc = static_cast<T *>(a.dAc);
  unsigned xround = 0;  // XCD barriers passed
  // the elementwise part's operands of a step (this wave's row of X / dHs, backward also of h) are copied into LDS
  // one step ahead: issued right after the workgroup's arrival at the chip-wide barrier, so that their latency
  // (first touch of a page of memory every step) passes during the wait
  i32x4_t xrsrc, hrsrc;
  {
    const unsigned long long xb = reinterpret_cast<unsigned long long>(a.X);
    xrsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)xb);
    xrsrc[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((xb >> 32) & 0xffffu));
    xrsrc[2] = __builtin_amdgcn_readfirstlane((int)((long)a.T * slot * 4));
    xrsrc[3] = 0x00020000;
    const unsigned long long hb = reinterpret_cast<unsigned long long>(a.Hs);
    hrsrc[0] = __builtin_amdgcn_readfirstlane((int)(unsigned)hb);
    hrsrc[1] = __builtin_amdgcn_readfirstlane((int)(unsigned)((hb >> 32) & 0xffffu));
    hrsrc[2] = __builtin_amdgcn_readfirstlane((int)((long)(a.T + 1) * slot * 2));
    hrsrc[3] = 0x00020000;
  }
  char *const xs = xstage + wave * 3072;
  const int lane16 = lane * 16;
  auto copy_x = [&](int tt) {  // operands of the elementwise part of the step at window position tt
    const int xoff = (int)(((long)tt * slot + (long)erow * HP + x * 512) * 4);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const unsigned lds_addr = (unsigned)(unsigned long long)(lds_void_ptr)(xs + i * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :
                   : "s"(lds_addr), "v"(lane16), "s"(xrsrc), "s"(xoff + i * 1024)
                   : "memory", "m0");
    }
    if (BACKWARD) {
      const unsigned lds_addr = (unsigned)(unsigned long long)(lds_void_ptr)(xs + 2048);
      const int hoff = (int)(((long)(tt + 1) * slot + (long)erow * HP + x * 512) * 2);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :
                   : "s"(lds_addr), "v"(lane16), "s"(hrsrc), "s"(hoff)
                   : "memory", "m0");
    }
  };
  copy_x(BACKWARD ? a.T - 1 : 0);

  for (int step = 0; step < a.T; ++step) {
    const int t = BACKWARD ? a.T - 1 - step : step;
    const bool contract = !(BACKWARD && step == 0);  // nothing flows into the window's last position
    // nothing is in flight here (the step barrier drained this wave's accesses); saying so in a form the compiler's
    // counter bookkeeping sees keeps it from adding waits of its own between the state copies below
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    if (contract) {
      // ---- (A) contraction ----
      const int soff = (int)((long)(BACKWARD ? t + 1 : t) * slot * 2);
      f32x16_t acc[4];
#pragma unroll
      for (int lb = 0; lb < 4; ++lb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[lb][r] = 0.0f;
      copy_chunk(0, soff);
      copy_chunk(1, soff);
      copy_chunk(2, soff);
#pragma unroll
      for (int c = 0; c < NCHUNK; ++c) {
        // this wave's copies of chunk c have landed (4 loads per chunk; chunks up to c + 2 are in flight)
        if (c + 2 < NCHUNK) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else if (c + 1 < NCHUNK) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // ... and so have the other waves'; everyone is done with chunk c - 1
        if (c + 3 < NCHUNK) copy_chunk(c + 3, soff);
        const char *sb = stage + (c & (NSTAGE - 1)) * STAGE + blk0;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          bf16x8_t f[4];
#pragma unroll
          for (int lb = 0; lb < 4; ++lb)
            f[lb] = *reinterpret_cast<const bf16x8_t *>(sb + ((lb ^ flip) * 4096) + frag_off[st]);
#pragma unroll
          for (int lb = 0; lb < 4; ++lb) mma16(acc[lb], f[lb], w[c * 4 + st]);
        }
      }
      // ---- (B) add the two halves of the contraction range through LDS, store the workgroup's partial ----
      __syncthreads();  // every wave is done reading the stages
      {
        float *give = reinterpret_cast<float *>(stage + wave * 8192);
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
          for (int r = 0; r < 16; ++r) give[q * 1024 + r * 64 + lane] = acc[2 + q][r];
      }
      __syncthreads();
      {
        const float *take = reinterpret_cast<const float *>(stage + (wave ^ 4) * 8192);
        // buffer stores: one register of per-lane addressing, the rest of the address is wave-uniform
        const int pbase = (int)((long)x * RES_PART_XCD * 4) + ((kc * BP + sh * 128) * 512 + uc * 128 + uq * 32) * 4;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
          const int sbk = q ^ flip;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int row = ((r >> 2) << 3) + (r & 3);  // + 4 (lane >> 5), part of pvoff
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, acc[q][r] + take[q * 1024 + r * 64 + lane]),
                                                  prsrc, pvoff, pbase + ((sbk * 32 + row) * 512) * 4, 0);
          }
        }
      }
      // arrival at the XCD barrier: own stores acknowledged, then the workgroup's
      wait_own_stores();
      __syncthreads();
      if (tid == 0) __hip_atomic_fetch_add(xcounter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ++xround;
    }
    const long eidx = (long)t * slot + (long)erow * HP + ecol;
    constexpr int NV = 2;  // float4 groups per thread
    f32x4_t s[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) s[v] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (contract) {
      if (tid == 0) {
        unsigned spins = 0;
        while (__hip_atomic_fetch_or(xcounter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < xround * 32u) {
          __builtin_amdgcn_s_sleep(1);
          if (++spins >= a.spin_limit) {
            a.flags[2] = 1;
            break;
          }
        }
      }
      __syncthreads();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
      // ---- (C) sum of the four partials in fixed order ----
      // (agent-scope policy on the loads: the partial buffer is reused every step, and a plain load could hit the
      // line this compute unit's L1 kept from the step before; the XCD's L2 holds the new values)
      const int cbase = (int)((long)x * RES_PART_XCD * 4);
      const int cvoff = (erow * 512 + ecl) * 4;
      f32x4_t pv[4][NV];
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < NV; ++v)
          pv[q][v] = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(prsrc, cvoff + 16 * v,
                                                                                         cbase + q * (BP * 512 * 4), 16));
#pragma unroll
      for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int e = 0; e < 4; ++e) s[v][e] = ((pv[0][v][e] + pv[1][v][e]) + pv[2][v][e]) + pv[3][v][e];
    }
    // this wave's row of X (dHs) and h: its own copies, landed long ago (every wait since was for all accesses)
    if (!contract) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // (only the very first step can get here early)
    f32x4_t xin[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) xin[v] = *reinterpret_cast<const f32x4_t *>(xs + lane * 32 + 16 * v);
    bf16x8_t hcur;
    if (BACKWARD) hcur = *reinterpret_cast<const bf16x8_t *>(xs + 2048 + lane16);
    float o[4 * NV];
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = v * 4 + e;
        const bool ok = row_ok && (ecol + i) < a.H;
        if (!BACKWARD) {
          o[i] = ok ? sigmoidf_(s[v][e] + xin[v][e]) : 0.0f;
        } else {
          const float hc = (float)hcur[i];
          o[i] = ok ? (xin[v][e] + s[v][e]) * hc * (1.0f - hc) : 0.0f;
        }
      }
    {
      T *dstc = BACKWARD ? dAc + eidx : Hs + slot + eidx;
#pragma unroll
      for (int v = 0; v < NV; ++v) {
        const f32x4_t ov = {o[4 * v], o[4 * v + 1], o[4 * v + 2], o[4 * v + 3]};
        store4<T>(dstc + 4 * v, ov);  // agent scope: other XCDs read it in the next step
        if (BACKWARD) *reinterpret_cast<f32x4_t *>(a.dA32 + eidx + 4 * v) = ov;
      }
      if (!BACKWARD && a.h_state && step == a.T - 1 && row_ok) {
#pragma unroll
        for (int i = 0; i < 4 * NV; ++i)
          if (ecol + i < a.H) a.h_state[(long)erow * a.H + ecol + i] = o[i];
      }
    }
    if (step + 1 < a.T) {
      // chip-wide barrier, with the next step's operand copies started between arrival and wait
      wait_own_stores();  // this wave's agent-scope state stores have been acknowledged
      __syncthreads();
      // arrival in two levels: the XCD's own counter, and the last workgroup of an XCD tells all eight XCDs
      if (tid == 0) {
        const unsigned old = __hip_atomic_fetch_add(garrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old + 1 == (unsigned)(step + 1) * 32u) {
#pragma unroll
          for (int y = 0; y < 8; ++y)
            __hip_atomic_fetch_add(a.counter + sync_word(4, y), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      copy_x(BACKWARD ? t - 1 : t + 1);
      if (tid == 0) {
        unsigned spins = 0;
        while (__hip_atomic_load(ggo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)(step + 1) * 8u) {
          __builtin_amdgcn_s_sleep(1);
          if (++spins >= a.spin_limit) {
            a.flags[2] = 1;
            break;
          }
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the copies have landed (they precede the state copies anyway)
      __syncthreads();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    }
  }
#endif
}

}  // namespace rnnlm_dev
