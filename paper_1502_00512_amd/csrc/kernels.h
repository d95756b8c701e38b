// Non-contraction kernels of the RNNLM step: stream indexing, token checks, embedding gather,
// softmax statistics merge, fused softmax-gradient pass, split-K reduction, sort/segment helpers
// and the segmented embedding update.
#pragma once
#include "common.h"

namespace rnnlm_dev {

// ---- a0: data-offset stream indexing (Sec. 4.2) ------------------------------------------------
__global__ void stream_chunk_kernel(const int32_t *__restrict__ tok, long L, long k, int T, int B,
                                    int32_t *__restrict__ x, int32_t *__restrict__ y) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= T * B) return;
  const int t = i / B, s = i % B;
  const long p = (long)s * L + k * T + t;
  x[i] = tok[p];
  y[i] = tok[p + 1];
}

// First kernel of a window, two kinds of workgroups:
// blockIdx.x < prep_blocks: token check + re-layout into the padded window: xp/yp[t*Bp + s]; padding rows
//   get -1.  Ids outside [0, V) are clamped and raise flags[0].  Also marks padded positions with
//   lse = +inf so that the softmax-gradient pass produces exact zeros there, copies the carried state into
//   slot 0 of the hidden-state buffer (compute type, padded with zeros) and clears the barrier / ticket
//   counters of the persistent recurrent kernel that follows (slot / counters == nullptr: tokens only).
//   prep_blocks covers max(Mp, Bp*Hp) threads.
// blockIdx.x >= prep_blocks (present when X or Xc != nullptr): a1, embedding gather of padded row
//   r = blockIdx.x - prep_blocks: X[r][:] = E[x of that position][:] (fp32), zero on padding.  Compressed
//   architecture (Xc != nullptr): the row is an operand of the contraction through the layer below the
//   state, so it is copied in the compute type from the tile-padded compute copy Ec[.][ldc] into Xc[r][ldc].
template <typename T>
__global__ void __launch_bounds__(256) prep_tokens_kernel(const int32_t *__restrict__ x, const int32_t *__restrict__ y,
                                                          int Tn, int B, int Bp, int Mp, int V,
                                                          int32_t *__restrict__ xp, int32_t *__restrict__ yp,
                                                          float *__restrict__ lse, int32_t *__restrict__ flags,
                                                          const float *__restrict__ h_state, int H, int Hp,
                                                          T *__restrict__ slot, unsigned *__restrict__ counters,
                                                          int prep_blocks, const float *__restrict__ E,
                                                          float *__restrict__ X, const T *__restrict__ Ec = nullptr,
                                                          int ldc = 0, T *__restrict__ Xc = nullptr) {
  if ((int)blockIdx.x >= prep_blocks) {
    const int row = blockIdx.x - prep_blocks;
    const int t = row / Bp, s = row % Bp;
    int w = -1;
    if (t < Tn && s < B) w = min(max(x[t * B + s], 0), V - 1);
    if (Xc) {
      const u32x4_t *src16 = reinterpret_cast<const u32x4_t *>(Ec + (long)max(w, 0) * ldc);
      u32x4_t *dst16 = reinterpret_cast<u32x4_t *>(Xc + (long)row * ldc);
      const int n16 = ldc * (int)sizeof(T) / 16;
      const u32x4_t zero = {0u, 0u, 0u, 0u};
      for (int c = threadIdx.x; c < n16; c += 256) dst16[c] = (w >= 0) ? src16[c] : zero;
      return;
    }
    const float *src = E + (long)max(w, 0) * H;
    float *dst = X + (long)row * Hp;
    if ((H & 3) == 0) {
      for (int c = threadIdx.x * 4; c < Hp; c += 256 * 4) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (w >= 0 && c < H) v = *reinterpret_cast<const float4 *>(src + c);
        *reinterpret_cast<float4 *>(dst + c) = v;
      }
    } else {
      for (int c = threadIdx.x; c < Hp; c += 256) dst[c] = (w >= 0 && c < H) ? src[c] : 0.0f;
    }
    return;
  }
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (counters && i < SYNC_WORDS) counters[i] = 0u;
  if (slot && i < (long)Bp * Hp) {
    const int s = (int)(i / Hp), c = (int)(i % Hp);
    slot[i] = from_f32<T>((s < B && c < H) ? h_state[(long)s * H + c] : 0.0f);
  }
  if (i >= Mp) return;
  const int t = (int)i / Bp, s = (int)i % Bp;
  int xv = -1, yv = -1;
  if (t < Tn && s < B) {
    xv = x[t * B + s];
    yv = y ? y[t * B + s] : 0;
    if (xv < 0 || xv >= V || yv < 0 || yv >= V) {
      flags[0] = 1;
      xv = min(max(xv, 0), V - 1);
      yv = min(max(yv, 0), V - 1);
    }
  } else {
    lse[i] = INFINITY;
  }
  xp[i] = xv;
  if (yp) yp[i] = yv;
}

template <typename T>
__global__ void fill_kernel(T *__restrict__ p, long n, T v) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long stride = (long)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = v;
}

// fp32 master -> padded compute copy.
template <typename T>
__global__ void to_compute_copy_kernel(const float *__restrict__ W, int R, int C, int Cp, long n,
                                       T *__restrict__ Wc) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long stride = (long)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const long r = i / Cp;
    const int c = (int)(i % Cp);
    Wc[i] = from_f32<T>((r < R && c < C) ? W[r * C + c] : 0.0f);
  }
}

// Square transpose of a compute-type matrix (n x n, n a multiple of 32): dst[c][r] = src[r][c].
template <typename T>
__global__ void __launch_bounds__(256) transpose_kernel(const T *__restrict__ src, int n, T *__restrict__ dst) {
  __shared__ T tile[32][33];
  const int bx = blockIdx.x * 32, by = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
  for (int r = ty; r < 32; r += 8) tile[r][tx] = src[(long)(by + r) * n + bx + tx];
  __syncthreads();
  for (int r = ty; r < 32; r += 8) dst[(long)(bx + r) * n + by + tx] = tile[tx][r];
}

// ---- a2 / a8, per-step path for hidden sizes beyond the persistent kernel: the step's contraction runs
// split over the contraction dimension (so that every compute unit gets a workgroup and each operand panel
// is fetched by few of them); these kernels sum the partial products in a fixed order and apply the step's
// elementwise part.  n4 = Bp*Hp/4 groups of 4 columns; part[split][Bp][Hp].
template <typename T>
__global__ void rnn_step_fwd_kernel(const float *__restrict__ part, long split_stride, int splits,
                                    const float *__restrict__ X, int B, int H, int Hp, long n4,
                                    T *__restrict__ Hnext, float *__restrict__ h_state) {
  const long i4 = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i4 >= n4) return;
  const long i = i4 * 4;
  const int row = (int)(i / Hp), col = (int)(i % Hp);
  f32x4_t a = *reinterpret_cast<const f32x4_t *>(part + i);
  for (int s = 1; s < splits; ++s) a += *reinterpret_cast<const f32x4_t *>(part + (long)s * split_stride + i);
  const f32x4_t x = *reinterpret_cast<const f32x4_t *>(X + i);
  f32x4_t hv;
#pragma unroll
  for (int e = 0; e < 4; ++e) hv[e] = (row < B && col + e < H) ? sigmoidf_(a[e] + x[e]) : 0.0f;
  if constexpr (sizeof(T) == 2) {
    bf16x4_t o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16_t)hv[e];
    *reinterpret_cast<bf16x4_t *>(Hnext + i) = o;
  } else {
    *reinterpret_cast<f32x4_t *>(Hnext + i) = hv;
  }
  if (h_state && row < B)
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (col + e < H) h_state[(long)row * H + col + e] = hv[e];
}

template <typename T>
__global__ void rnn_step_bwd_kernel(const float *__restrict__ part, long split_stride, int splits,
                                    const float *__restrict__ dHs, const T *__restrict__ Hs, int B, int H, int Hp,
                                    long n4, float *__restrict__ dA32, T *__restrict__ dAc) {
  const long i4 = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i4 >= n4) return;
  const long i = i4 * 4;
  const int row = (int)(i / Hp), col = (int)(i % Hp);
  f32x4_t a = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int s = 0; s < splits; ++s) a += *reinterpret_cast<const f32x4_t *>(part + (long)s * split_stride + i);
  const f32x4_t g = *reinterpret_cast<const f32x4_t *>(dHs + i);
  f32x4_t d;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float hv = to_f32(Hs[i + e]);
    d[e] = (row < B && col + e < H) ? (g[e] + a[e]) * hv * (1.0f - hv) : 0.0f;
  }
  *reinterpret_cast<f32x4_t *>(dA32 + i) = d;
  if constexpr (sizeof(T) == 2) {
    bf16x4_t o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (bf16_t)d[e];
    *reinterpret_cast<bf16x4_t *>(dAc + i) = o;
  } else {
    *reinterpret_cast<f32x4_t *>(dAc + i) = d;
  }
}

// ---- a4 (part 1): merge the per-row-block (max, sum exp) partials of each position into the log
// normaliser, and form log P(target) = z_target - lse (Sec. 4.2: explicitly normalised output).
// Block = 64 positions x 16 groups of partials; each group is merged sequentially in a fixed order, then
// the 16 group results are merged in order by the group-0 thread.
__global__ void __launch_bounds__(1024) merge_stats_kernel(const float2 *__restrict__ part, int nPart, long ldz, int T,
                                                           int B, int Bp, const float *__restrict__ zy,
                                                           float *__restrict__ lse, float *__restrict__ logp_int,
                                                           float *__restrict__ logp_out) {
  __shared__ float2 sh[16][64];
  const int lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int m = blockIdx.x * 64 + lane;
  const bool valid = m < T * Bp;
  float mx = -INFINITY, sum = 0.0f;
  if (valid) {
    auto merge = [&](const float2 q) {
      if (q.y > 0.0f) {
        const float nmx = fmaxf(mx, q.x);
        sum = sum * __expf(mx - nmx) + q.y * __expf(q.x - nmx);
        mx = nmx;
      }
    };
    int p = grp;
    for (; p + 48 < nPart; p += 64) {  // four partials per round: their loads are independent
      float2 q[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) q[u] = part[(long)(p + 16 * u) * ldz + m];
#pragma unroll
      for (int u = 0; u < 4; ++u) merge(q[u]);
    }
    for (; p < nPart; p += 16) merge(part[(long)p * ldz + m]);
  }
  sh[grp][lane] = make_float2(mx, sum);
  __syncthreads();
  if (grp != 0 || !valid) return;
  const int t = m / Bp, s = m % Bp;
  if (s >= B) return;  // padding keeps lse = +inf
  for (int g = 1; g < 16; ++g) {
    const float2 q = sh[g][lane];
    if (q.y > 0.0f) {
      const float nmx = fmaxf(mx, q.x);
      sum = sum * __expf(mx - nmx) + q.y * __expf(q.x - nmx);
      mx = nmx;
    }
  }
  const float l = mx + __logf(sum);
  lse[m] = l;
  const float lp = zy[m] - l;
  logp_int[t * B + s] = lp;
  if (logp_out) logp_out[t * B + s] = lp;
}

// Sum of the window's log-probabilities in fp64 with a fixed reduction tree; raises flags[1] when the
// result is not finite.  counters != nullptr: also clears the barrier / ticket counters of the
// persistent recurrent kernel (this kernel sits between its forward and its backward launch).
__global__ void sum_logp_kernel(const float *__restrict__ logp, int n, double *__restrict__ out,
                                double *__restrict__ running, int32_t *__restrict__ flags,
                                unsigned *__restrict__ counters) {
  __shared__ double sh[1024];
  if (counters)  // for the backward recurrent kernel
    for (int i = threadIdx.x; i < SYNC_WORDS; i += 1024) counters[i] = 0u;
  double a = 0.0;
  for (int i = threadIdx.x; i < n; i += 1024) a += (double)logp[i];
  sh[threadIdx.x] = a;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) sh[threadIdx.x] += sh[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const double s = sh[0];
    if (out) *out = s;
    if (running) *running += s;
    if (!(s == s) || s - s != 0.0) flags[1] = 1;
  }
}

// ---- a4 (part 2) + a5: fused softmax gradient, in place on the vocabulary-major logits ----------
//   dz[v][m] = (exp(z[v][m] - lse[m]) - [v == y[m]]) / M      (gradient of the mean NLL)
//   db[v]    = sum_m dz[v][m];   b_out[v] = alpha*b[v] - lr*db[v]
// One wavefront owns ROWS_PER_WAVE vocabulary rows and walks the window positions once, so the
// per-position lse / target id loaded for a 16-byte column chunk serve all of its rows and several row
// loads are in flight per lane.  Rows v >= V and padded positions (lse = +inf) become zero.  Workgroups take the
// vocabulary from its top down, so that what this pass writes last is what the contraction over the vocabulary
// that follows reads first (still in the memory-side cache: 1-3 % on that contraction).
template <typename T>
__global__ void __launch_bounds__(256) softmax_grad_kernel(T *__restrict__ ZT, long ldz, int Mp, int V, int Vp,
                                                           const float *__restrict__ lse,
                                                           const int32_t *__restrict__ yp, float invM,
                                                           const float *__restrict__ b, float *__restrict__ b_out,
                                                           float alpha, float lr) {
  constexpr int VEC = Elem<T>::VEC;
  constexpr int R = 4;  // rows per wave
  const int lane = threadIdx.x & 63;
  const int v0 = ((gridDim.x - 1 - blockIdx.x) * 4 + (threadIdx.x >> 6)) * R;
  if (v0 >= Vp) return;
  T *row = ZT + (long)v0 * ldz;
  float db[R];
#pragma unroll
  for (int r = 0; r < R; ++r) db[r] = 0.0f;
  for (int c = lane * VEC; c < Mp; c += 64 * VEC) {
    u32x4_t raw[R];
#pragma unroll
    for (int r = 0; r < R; ++r) raw[r] = *reinterpret_cast<const u32x4_t *>(row + (long)r * ldz + c);
    float l[VEC];
    int y[VEC];
#pragma unroll
    for (int e = 0; e < VEC; e += 4) {
      const f32x4_t lv = *reinterpret_cast<const f32x4_t *>(lse + c + e);
      const u32x4_t yv = *reinterpret_cast<const u32x4_t *>(yp + c + e);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        l[e + q] = lv[q];
        y[e + q] = (int)yv[q];
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      union {
        u32x4_t u;
        T t[VEC];
      } in, o;
      in.u = raw[r];
      const int v = v0 + r;
#pragma unroll
      for (int e = 0; e < VEC; ++e) {
        float p = __expf(to_f32(in.t[e]) - l[e]);
        if (y[e] == v) p -= 1.0f;
        p = (v < V) ? p * invM : 0.0f;
        db[r] += p;
        o.t[e] = from_f32<T>(p);
      }
      *reinterpret_cast<u32x4_t *>(row + (long)r * ldz + c) = o.u;
    }
  }
#pragma unroll
  for (int r = 0; r < R; ++r) {
    float d = db[r];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) d += __shfl_xor(d, o, 64);
    const int v = v0 + r;
    if (lane == 0 && v < V) b_out[v] = ((alpha != 0.0f) ? alpha * b[v] : 0.0f) - lr * d;
  }
}

// ---- a6: fixed-order reduction of the split-K partial sums -------------------------------------
__global__ void splitk_reduce_kernel(const float *__restrict__ part, long n, long split_stride, int splits,
                                     float *__restrict__ out) {
  const long i = ((long)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (i >= n) return;
  float4 a = *reinterpret_cast<const float4 *>(part + i);
  for (int s = 1; s < splits; ++s) {
    const float4 q = *reinterpret_cast<const float4 *>(part + (long)s * split_stride + i);
    a.x += q.x;
    a.y += q.y;
    a.z += q.z;
    a.w += q.w;
  }
  *reinterpret_cast<float4 *>(out + i) = a;
}

// ---- a10 helpers (integer-exact): stable order of window positions by input id ------------------
// rank[m] = #{m' : (x[m'], m') < (x[m], m)};  perm[rank[m]] = m.
// Block = 64 positions x 16 slices of the key array (1024 threads).
__global__ void __launch_bounds__(1024) rank_sort_kernel(const int32_t *__restrict__ xp, int M, int B, int Bp,
                                                         int32_t *__restrict__ perm) {
  __shared__ int32_t keys[4096];
  __shared__ int32_t cnt[16][64];
  const int lane = threadIdx.x & 63, slice = threadIdx.x >> 6;
  const int m = blockIdx.x * 64 + lane;
  const int mykey = (m < M) ? xp[(m / B) * Bp + (m % B)] : 0;
  int rank = 0;
  for (int base = 0; base < M; base += 4096) {
    const int n = min(4096, M - base);
    for (int i = threadIdx.x; i < n; i += 1024) {
      const int mm = base + i;
      keys[i] = xp[(mm / B) * Bp + (mm % B)];
    }
    __syncthreads();
    for (int i = slice; i < n; i += 16) {
      const int k = keys[i];
      rank += (k < mykey) || (k == mykey && base + i < m);
    }
    __syncthreads();
  }
  cnt[slice][lane] = rank;
  __syncthreads();
  if (slice == 0 && m < M) {
    int r = 0;
    for (int g = 0; g < 16; ++g) r += cnt[g][lane];
    perm[r] = m;
  }
}

// Run starts of equal ids in sorted order; single workgroup of 1024 threads, fixed scan order.
__global__ void segment_kernel(const int32_t *__restrict__ xp, const int32_t *__restrict__ perm, int M, int B,
                               int Bp, int32_t *__restrict__ seg_start, int32_t *__restrict__ nseg) {
  __shared__ int32_t sc[1024];
  __shared__ int32_t carry;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int base = 0; base < M; base += 1024) {
    const int r = base + threadIdx.x;
    int head = 0;
    if (r < M) {
      const int m = perm[r];
      const int k = xp[(m / B) * Bp + (m % B)];
      if (r == 0) {
        head = 1;
      } else {
        const int mq = perm[r - 1];
        head = xp[(mq / B) * Bp + (mq % B)] != k;
      }
    }
    sc[threadIdx.x] = head;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
      int add = 0;
      if ((int)threadIdx.x >= off) add = sc[threadIdx.x - off];
      __syncthreads();
      sc[threadIdx.x] += add;
      __syncthreads();
    }
    const int incl = sc[threadIdx.x];
    const int c0 = carry;
    if (head) seg_start[c0 + incl - 1] = r;
    __syncthreads();
    if (threadIdx.x == 1023) carry = c0 + incl;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    seg_start[carry] = M;
    *nseg = carry;
  }
}

// ---- a10: segmented embedding update, atomic-free and order-fixed -------------------------------
//   out[w][:] = alpha*E[w][:] - lr * sum_{m in run of w} dA[m][:]
// blockIdx.x = run index (exits when >= *nseg), blockIdx.y = block of 256*VEC columns; a thread owns VEC
// consecutive columns.  The run's members are dealt round-robin to PARTS partial sums (member i of the run goes
// to sum i mod PARTS, each sum accumulated in ascending m), which are then added in order 0..PARTS-1: a fixed
// summation tree, so results are bitwise reproducible.  All PARTS sums live in the thread's registers: a group
// of 16 members is 16 independent row loads in flight, and the small workgroups (no LDS, no barrier) leave
// eight of them resident per compute unit, which is what a pass made of dependent memory round trips (run
// bounds -> position -> rows) needs: it is bound by latency times occupancy, not by bandwidth.
// VEC = 4: H % 4 == 0; VEC = 1: any H.
// Ec (may be nullptr): compute copy [.][ldc] of the updated matrix, refreshed with the new row (the tied word
// matrix of the compressed architecture is an operand of the output layer as well).
template <int VEC, typename T>
__global__ void __launch_bounds__(256) scatter_update_kernel(const float *__restrict__ dA, int Hp, int H, int B,
                                                             int Bp, const int32_t *__restrict__ xp,
                                                             const int32_t *__restrict__ perm,
                                                             const int32_t *__restrict__ seg_start,
                                                             const int32_t *__restrict__ nseg,
                                                             const float *__restrict__ E, float *__restrict__ out,
                                                             float alpha, float lr, int compact_ld,
                                                             T *__restrict__ Ec, int ldc) {
  constexpr int PARTS = 4, GROUP = 4 * PARTS;
  const int g = blockIdx.x;
  if (g >= *nseg) return;
  const int col = (blockIdx.y * 256 + threadIdx.x) * VEC;
  if (col >= H) return;
  const int r0 = seg_start[g], r1 = seg_start[g + 1];
  const int m0 = perm[r0];
  const int w = xp[(m0 / B) * Bp + (m0 % B)];
  const long idx = (long)w * H + col;
  // the row being updated does not depend on the sum: ask for it first
  float old[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) old[e] = 0.0f;
  if (alpha != 0.0f) {
    if (VEC == 4) {
      const f32x4_t t = *reinterpret_cast<const f32x4_t *>(E + idx);
#pragma unroll
      for (int e = 0; e < VEC; ++e) old[e] = t[e];
    } else {
      old[0] = E[idx];
    }
  }
  auto row_of = [&](int r) {
    const int m = perm[r];
    return ((long)(m / B) * Bp + (m % B)) * Hp + col;
  };
  auto load_row = [&](long at, float (&v)[VEC]) {
    if (VEC == 4) {
      const f32x4_t t = *reinterpret_cast<const f32x4_t *>(dA + at);
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[e] = t[e];
    } else {
      v[0] = dA[at];
    }
  };
  float acc[PARTS][VEC];
#pragma unroll
  for (int p = 0; p < PARTS; ++p)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[p][e] = 0.0f;
  int r = r0;
  for (; r + GROUP <= r1; r += GROUP) {
    long at[GROUP];
#pragma unroll
    for (int k = 0; k < GROUP; ++k) at[k] = row_of(r + k);
    float v[GROUP][VEC];
#pragma unroll
    for (int k = 0; k < GROUP; ++k) load_row(at[k], v[k]);
#pragma unroll
    for (int k = 0; k < GROUP; ++k)  // member r + k belongs to sum k % PARTS (r - r0 is a multiple of GROUP)
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[k % PARTS][e] += v[k][e];
  }
  for (; r < r1; r += PARTS) {
    float v[PARTS][VEC];
#pragma unroll
    for (int p = 0; p < PARTS; ++p) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[p][e] = 0.0f;
      if (r + p < r1) load_row(row_of(r + p), v[p]);
    }
#pragma unroll
    for (int p = 0; p < PARTS; ++p)
      if (r + p < r1) {
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[p][e] += v[p][e];
      }
  }
#pragma unroll
  for (int p = 1; p < PARTS; ++p)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[0][e] += acc[p][e];
  // compact_ld > 0: the run's result goes to row g of a compact [runs][compact_ld] buffer instead of row w
  const long oidx = compact_ld > 0 ? (long)g * compact_ld + col : idx;
  float nv[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) nv[e] = ((alpha != 0.0f) ? alpha * old[e] : 0.0f) - lr * acc[0][e];
  if (VEC == 4) {
    f32x4_t t;
#pragma unroll
    for (int e = 0; e < VEC; ++e) t[e] = nv[e];
    *reinterpret_cast<f32x4_t *>(out + oidx) = t;
  } else {
    out[oidx] = nv[0];
  }
  if (Ec) {
#pragma unroll
    for (int e = 0; e < VEC; ++e) Ec[(long)w * ldc + col + e] = from_f32<T>(nv[e]);
  }
}

// fp32 -> compute type, element by element (n elements).
template <typename T>
__global__ void to_compute_kernel(const float *__restrict__ src, long n, T *__restrict__ dst) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long stride = (long)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = from_f32<T>(src[i]);
}

// 8-bit row-wise quantisation (Sec. 5.4 quantises all the weights; the scheme is a reading): one workgroup
// per row r of W[R][C]: scale = max|row| / 127 (1 for an all-zero row), code = round-half-to-even(w / scale)
// clipped to [-127, 127], all in fp32 with correctly rounded division; the compute copy Wc[r][ldc] receives
// code * scale.  max is order-independent, so the result does not depend on the reduction tree.
template <typename T>
__global__ void __launch_bounds__(256) quantize_rows_kernel(const float *__restrict__ W, int C,
                                                            int8_t *__restrict__ codes, float *__restrict__ scale,
                                                            T *__restrict__ Wc, int ldc) {
  __shared__ float red[256];
  const int r = blockIdx.x;
  const float *row = W + (long)r * C;
  float amax = 0.0f;
  for (int c = threadIdx.x; c < C; c += 256) amax = fmaxf(amax, fabsf(row[c]));
  red[threadIdx.x] = amax;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
    __syncthreads();
  }
  amax = red[0];
  const float sc = amax > 0.0f ? amax / 127.0f : 1.0f;
  if (threadIdx.x == 0) scale[r] = sc;
  for (int c = threadIdx.x; c < C; c += 256) {
    float q = rintf(row[c] / sc);
    q = fminf(fmaxf(q, -127.0f), 127.0f);
    codes[(long)r * C + c] = (int8_t)q;
    Wc[(long)r * ldc + c] = from_f32<T>(q * sc);
  }
}

// ---- measured peaks of the box (reported next to the published ones) -----------------------------
// Register-resident MFMA loop: 8 independent 32x32x16 bf16 accumulations per iteration and wave, operands
// rotated every iteration.  RANDOM = operand bits drawn from a hash (the sustained rate with realistic
// data: power management lowers the clock when operands toggle); otherwise constant operands.
template <bool RANDOM>
__global__ void __launch_bounds__(512) mfma_rate_kernel(float *out, int iters) {
  auto hashu = [](unsigned x) {
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
  };
  bf16x8_t a[4], b[2];
  for (int q = 0; q < 4; ++q)
    for (int e = 0; e < 8; ++e) {
      const unsigned hsh = hashu(threadIdx.x * 131 + q * 17 + e + blockIdx.x * 7919);
      a[q][e] = RANDOM ? (bf16_t)(((int)(hsh & 0xffff) - 32768) / 65536.0f) : (bf16_t)0.5f;
    }
  for (int q = 0; q < 2; ++q)
    for (int e = 0; e < 8; ++e) {
      const unsigned hsh = hashu(threadIdx.x * 733 + q * 29 + e + 1234567);
      b[q][e] = RANDOM ? (bf16_t)(((int)(hsh & 0xffff) - 32768) / 65536.0f) : (bf16_t)0.25f;
    }
  f32x16_t acc[8];
  for (int i = 0; i < 8; ++i)
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i * 2 + j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i * 2 + j], 0, 0, 0);
    bf16x8_t t = a[0];
    a[0] = a[1];
    a[1] = a[2];
    a[2] = a[3];
    a[3] = t;
    t = b[0];
    b[0] = b[1];
    b[1] = t;
  }
  float sum = 0;
  for (int i = 0; i < 8; ++i)
    for (int r = 0; r < 16; ++r) sum += acc[i][r];
  out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

// Plain device copy, 16 bytes per lane, grid-stride.
__global__ void __launch_bounds__(256) copy_kernel(const u32x4_t *__restrict__ src, u32x4_t *__restrict__ dst, long n16) {
  long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long stride = (long)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) dst[i] = src[i];
}

}  // namespace rnnlm_dev
