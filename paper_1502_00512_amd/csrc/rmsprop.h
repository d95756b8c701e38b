// rmsprop scaling of the SGD step (Sec. 4.2 of the paper: SGD with rmsprop, smoothing constant 0.9995, and
// for the input-to-state and state-to-output matrices one statistic per word, averaged over the hidden
// units, instead of one per weight).  With r the running mean of squared gradients:
//   r <- rho*r + (1-rho)*s ;  theta <- theta - lr * g / (sqrt(r) + eps)
// s = g^2 per element (U, b) or the mean over the row of g^2 (E, Wo).  The gradients are produced by the
// same kernels as the plain step with their update epilogues redirected into gradient buffers; the kernels
// here apply them.  A zero gradient moves nothing (also when the denominator is zero).
#pragma once
#include "common.h"

namespace rnnlm_dev {

// r[i] *= rho: decay of a per-word statistic; the words touched in this window add (1-rho)*s afterwards.
__global__ void rms_decay_kernel(float *__restrict__ r, long n, float rho) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) r[i] *= rho;
}

// One statistic per word; one workgroup per gradient row.
//   dense (perm == nullptr):   row w = blockIdx.x of G[.][ldg], r[w] <- rho*r[w] + (1-rho)*ms
//   compact (perm != nullptr): row i = blockIdx.x < *nseg of G belongs to the word of the i-th run of the
//                              sorted window positions; r[w] was decayed already: r[w] <- r[w] + (1-rho)*ms
// then W[w][:] -= lr / (sqrt(r[w]) + eps) * g[:] on the fp32 master (leading dimension H) and, when
// Wc != nullptr, the compute copy (leading dimension Hp) is refreshed.  The mean of squares is reduced
// in a fixed order (per-lane strided sums, butterfly, then the four waves in order).
template <typename T>
__global__ void __launch_bounds__(256) rms_row_apply_kernel(const float *__restrict__ G, long ldg,
                                                            const int32_t *__restrict__ xp,
                                                            const int32_t *__restrict__ perm,
                                                            const int32_t *__restrict__ seg_start,
                                                            const int32_t *__restrict__ nseg, int B, int Bp, int H,
                                                            int Hp, float *__restrict__ W, T *__restrict__ Wc,
                                                            float *__restrict__ r, float rho, float lr, float eps) {
  __shared__ float red[4];
  int w = blockIdx.x;
  if (perm) {
    if ((int)blockIdx.x >= *nseg) return;
    const int m0 = perm[seg_start[blockIdx.x]];
    w = xp[(m0 / B) * Bp + (m0 % B)];
  }
  const float *g = G + (long)blockIdx.x * ldg;
  float *wrow = W + (long)w * H;
  const bool vec = (H & 3) == 0;  // 16-byte accesses; the first 4096 columns of the gradient row stay in registers
  f32x4_t gc[4];
  float ss = 0.0f;
  if (vec) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int c = (it * 256 + threadIdx.x) * 4;
      gc[it] = f32x4_t{0.0f, 0.0f, 0.0f, 0.0f};
      if (c < H) gc[it] = *reinterpret_cast<const f32x4_t *>(g + c);
#pragma unroll
      for (int e = 0; e < 4; ++e) ss = fmaf(gc[it][e], gc[it][e], ss);
    }
    for (int c = (1024 + threadIdx.x) * 4; c < H; c += 1024) {
      const f32x4_t v = *reinterpret_cast<const f32x4_t *>(g + c);
#pragma unroll
      for (int e = 0; e < 4; ++e) ss = fmaf(v[e], v[e], ss);
    }
  } else {
    for (int c = threadIdx.x; c < H; c += 256) ss = fmaf(g[c], g[c], ss);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) ss += __shfl_xor(ss, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float ms = ((red[0] + red[1]) + (red[2] + red[3])) / (float)H;
  const float rold = r[w];
  const float rnew = (perm ? rold : rho * rold) + (1.0f - rho) * ms;
  const float scale = lr / (sqrtf(rnew) + eps);
  __syncthreads();  // every thread has read r[w] before it is overwritten
  if (threadIdx.x == 0) r[w] = rnew;
  auto apply4 = [&](int c, const f32x4_t &gv) {
    f32x4_t v = *reinterpret_cast<const f32x4_t *>(wrow + c);
    bool moved = false;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (gv[e] != 0.0f) {
        v[e] -= scale * gv[e];
        moved = true;
      }
    if (moved) *reinterpret_cast<f32x4_t *>(wrow + c) = v;
    if (Wc) {
      if constexpr (sizeof(T) == 2) {
        bf16x4_t hv;
#pragma unroll
        for (int e = 0; e < 4; ++e) hv[e] = (bf16_t)v[e];
        *reinterpret_cast<bf16x4_t *>(Wc + (long)w * Hp + c) = hv;
      } else {
        *reinterpret_cast<f32x4_t *>(Wc + (long)w * Hp + c) = v;
      }
    }
  };
  if (vec) {
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int c = (it * 256 + threadIdx.x) * 4;
      if (c < H) apply4(c, gc[it]);
    }
    for (int c = (1024 + threadIdx.x) * 4; c < H; c += 1024) apply4(c, *reinterpret_cast<const f32x4_t *>(g + c));
  } else {
    for (int c = threadIdx.x; c < H; c += 256) {
      const float gv = g[c];
      float v = wrow[c];
      if (gv != 0.0f) {
        v -= scale * gv;
        wrow[c] = v;
      }
      if (Wc) Wc[(long)w * Hp + c] = from_f32<T>(v);
    }
  }
}

// Per-element statistic on a compact list (the output bias under the noise-contrastive criterion): entry i
// < *nseg holds the gradient of the word of the i-th run of the sorted update list; rb was decayed already.
__global__ void rms_bias_compact_kernel(const float *__restrict__ g, const int32_t *__restrict__ ids,
                                        const int32_t *__restrict__ perm, const int32_t *__restrict__ seg_start,
                                        const int32_t *__restrict__ nseg, float *__restrict__ b,
                                        float *__restrict__ rb, float rho, float lr, float eps) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= *nseg) return;
  const int w = ids[perm[seg_start[i]]];
  const float gv = g[i];
  const float rnew = rb[w] + (1.0f - rho) * gv * gv;
  rb[w] = rnew;
  if (gv != 0.0f) b[w] -= lr * gv / (sqrtf(rnew) + eps);
}

// One statistic per element (U: R x C with a compute copy of leading dimension ldc; b: 1 x V, no copy).
template <typename T>
__global__ void rms_elem_apply_kernel(const float *__restrict__ G, int R, int C, float *__restrict__ W,
                                      T *__restrict__ Wc, int ldc, float *__restrict__ r, float rho, float lr,
                                      float eps) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (long)R * C) return;
  const float gv = G[i];
  const float rnew = rho * r[i] + (1.0f - rho) * gv * gv;
  r[i] = rnew;
  float v = W[i];
  if (gv != 0.0f) {
    v -= lr * gv / (sqrtf(rnew) + eps);
    W[i] = v;
  }
  if (Wc) Wc[(i / C) * ldc + (i % C)] = from_f32<T>(v);
}

}  // namespace rnnlm_dev
