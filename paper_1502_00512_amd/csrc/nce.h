// Kernels of the noise-contrastive training criterion (Sec. 4.2 of the paper names it; the estimator
// is Gutmann & Hyvarinen's, in the form Mnih & Teh use for language models).
//
// For window position m with hidden state h_m and target y_m, and K noise words n_0..n_{K-1} shared by
// the whole window, with scores z_m(w) = Wo[w].h_m + b[w] and D_m(w) = z_m(w) - lnZ - ln(K q(w)):
//   J_m = softplus(-D_m(y_m)) + sum_j softplus(D_m(n_j)),        softplus(d) = ln(1 + e^d)
//   dJ_m/dz_m(y_m) = -(1 - sigmoid(D_m(y_m))),  dJ_m/dz_m(n_j) = sigmoid(D_m(n_j)),
// window loss = mean of J_m.  The dense parts (all positions x all noise words) run on the contraction
// kernels over a gathered panel of Wo rows; the kernels here do the gathers, the elementwise pass, the
// per-target terms and the order-fixed, atomic-free update of the touched rows of Wo and b.
//
// Index conventions: "row" = t*Bp + s is a padded window position; "m" = t*B + s the compact one; entry
// e of the update list is noise word e for e < K and the target of compact position e - K otherwise.
#pragma once
#include "common.h"

namespace rnnlm_dev {

constexpr int NCE_COLSUM_PARTS = 16;  // row-block partials of the noise words' bias gradient

__device__ inline float softplusf_(float d) { return fmaxf(d, 0.0f) + log1pf(__expf(-fabsf(d))); }
__device__ inline float logisticf_(float d) {
  const float e = __expf(-fabsf(d));
  return (d >= 0.0f) ? 1.0f / (1.0f + e) : e / (1.0f + e);
}

// Preparation of a window's noise words, one workgroup per (padded) noise slot j < Kp plus ceil(M/256)
// workgroups for the targets:
//   noise id checked (flags[0] on an id outside [0,V), clamped); offset off[j] = b[n_j] - lnZ - ln K - lnq[n_j]
//   (0 for the padding j >= K); panel row Wn[j][:] = Wo_c[n_j][:] (zero rows for the padding; Hp is a multiple
//   of 256); update list ids[0..K) = noise words, ids[K + m] = target of compact position m.
template <typename T>
__global__ void __launch_bounds__(256) nce_prep_kernel(const int32_t *__restrict__ noise, int K, int Kp, int V,
                                                       const float *__restrict__ lnq, const float *__restrict__ b,
                                                       float lnZ_lnK, const int32_t *__restrict__ yp, int M, int B,
                                                       int Bp, const T *__restrict__ Wo_c, int Hp,
                                                       T *__restrict__ Wn, float *__restrict__ off,
                                                       int32_t *__restrict__ ids, int32_t *__restrict__ flags) {
  constexpr int VEC = 16 / (int)sizeof(T);
  const int j = blockIdx.x;
  if (j >= Kp) {  // target part of the update list
    const int m = (j - Kp) * 256 + threadIdx.x;
    if (m < M) ids[K + m] = yp[(m / B) * Bp + (m % B)];
    return;
  }
  int w = 0;
  if (j < K) {
    w = noise[j];
    const bool bad = w < 0 || w >= V;
    w = min(max(w, 0), V - 1);
    if (threadIdx.x == 0) {
      if (bad) flags[0] = 1;
      off[j] = b[w] - lnZ_lnK - lnq[w];
      ids[j] = w;
    }
  } else if (threadIdx.x == 0) {
    off[j] = 0.0f;
  }
  const u32x4_t *src = reinterpret_cast<const u32x4_t *>(Wo_c + (long)w * Hp);
  u32x4_t *dst = reinterpret_cast<u32x4_t *>(Wn + (long)j * Hp);
  const u32x4_t zero = {0u, 0u, 0u, 0u};
  for (int c = threadIdx.x; c < Hp / VEC; c += 256) dst[c] = (j < K) ? src[c] : zero;
}

// Score of the target word of every position: dt[row] = Wo_c[y].Hs[row] + b[y] - shift - lnq[y]
// (lnq == nullptr: no noise term).  One wave per padded position (4 per workgroup); lanes stride the
// row, then a butterfly sum.  out (may be nullptr) receives the valid positions in compact order t*B + s.
template <typename T>
__global__ void __launch_bounds__(256) nce_target_score_kernel(const T *__restrict__ Hs1, const T *__restrict__ Wo_c,
                                                               int Hp, const int32_t *__restrict__ yp,
                                                               const float *__restrict__ b,
                                                               const float *__restrict__ lnq, float shift, int rows,
                                                               int B, int Bp, float *__restrict__ dt,
                                                               float *__restrict__ out) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  const int y = yp[row];
  if (y < 0) {
    if (lane == 0) dt[row] = 0.0f;
    return;
  }
  const T *hrow = Hs1 + (long)row * Hp, *wrow = Wo_c + (long)y * Hp;
  float acc = 0.0f;
  for (int c = lane; c < Hp; c += 64) acc = fmaf(to_f32(hrow[c]), to_f32(wrow[c]), acc);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) {
    const float v = acc + b[y] - shift - (lnq ? lnq[y] : 0.0f);
    dt[row] = v;
    if (out) out[(row / Bp) * B + (row % Bp)] = v;
  }
}

// Scores of a shortlist of C candidate words per position (Sec. 5.4 ranks a shortlist of candidates):
// out[(t*B + s)*C + c] = Wc[cand].F[row] + b[cand] - shift, F = what the output layer reads (ld = width
// Dp).  One wave per (position, candidate); ids outside [0, V) are clamped and raise flags[0].
template <typename T>
__global__ void __launch_bounds__(256) score_candidates_kernel(const T *__restrict__ F, const T *__restrict__ Wc, int Dp,
                                                               const int32_t *__restrict__ cand, int C, int V,
                                                               const float *__restrict__ b, float shift, long total,
                                                               int B, int Bp, int32_t *__restrict__ flags,
                                                               float *__restrict__ out) {
  const long item = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (item >= total) return;
  const long pos = item / C;  // compact position index t*B + s
  const long row = (pos / B) * Bp + (pos % B);
  int w = cand[item];
  if (w < 0 || w >= V) {
    if (lane == 0) flags[0] = 1;
    w = min(max(w, 0), V - 1);
  }
  const T *frow = F + row * Dp, *wrow = Wc + (long)w * Dp;
  float acc = 0.0f;
  for (int c = lane; c < Dp; c += 64) acc = fmaf(to_f32(frow[c]), to_f32(wrow[c]), acc);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) out[item] = acc + b[w] - shift;
}

// Elementwise pass over one padded position (one workgroup per row of the score matrix S[Mp][Kp]):
// dS[row][j] = sigmoid(S + off[j]) * scale in the contraction operand type (0 for padding rows and
// columns), the position's loss J, and the target coefficient ct[row] = -(1 - sigmoid(dt)) * scale.
template <typename T>
__global__ void __launch_bounds__(256) nce_grad_kernel(const float *__restrict__ S, int Kp, int K,
                                                       const float *__restrict__ off, const float *__restrict__ dt,
                                                       int Tn, int B, int Bp, float scale, T *__restrict__ dS,
                                                       float *__restrict__ ct, float *__restrict__ J_int,
                                                       float *__restrict__ J_out) {
  __shared__ float red[4];
  const int row = blockIdx.x, t = row / Bp, s = row % Bp;
  const bool valid = t < Tn && s < B;
  const float *srow = S + (long)row * Kp;
  T *drow = dS + (long)row * Kp;
  float cost = 0.0f;
  for (int j = threadIdx.x; j < Kp; j += 256) {
    float g = 0.0f;
    if (valid && j < K) {
      const float d = srow[j] + off[j];
      g = logisticf_(d) * scale;
      cost += softplusf_(d);
    }
    drow[j] = from_f32<T>(g);
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) cost += __shfl_xor(cost, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = cost;
  __syncthreads();
  if (threadIdx.x != 0) return;
  if (!valid) {
    ct[row] = 0.0f;
    return;
  }
  const float d = dt[row];
  const float total = ((red[0] + red[1]) + (red[2] + red[3])) + softplusf_(-d);
  ct[row] = -logisticf_(-d) * scale;
  const int m = t * B + s;
  J_int[m] = total;
  if (J_out) J_out[m] = total;
}

// Bias gradient of noise word j: gcol[j] = sum over valid positions of sigmoid(S[row][j] + off[j]) * scale,
// in two fixed-order levels.  Level 1: workgroup (column block x, row block y) = 64 columns x 16 row
// groups over the positions m = y, y + gridDim.y, ...; each group sums its positions in ascending order,
// the 16 group sums are added in order into part[y][j].  Level 2 (the row blocks, in order) is done by the
// consumer, nce_row_update_kernel, when it forms the word's bias gradient.
__global__ void __launch_bounds__(1024) nce_colsum_kernel(const float *__restrict__ S, int Kp, int K,
                                                          const float *__restrict__ off, int Tn, int B, int Bp,
                                                          float scale, float *__restrict__ part) {
  __shared__ float sh[16][64];
  const int c = threadIdx.x & 63, grp = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + c;
  float acc = 0.0f;
  if (j < K) {
    const float o = off[j];
    const int M = Tn * B;
    for (int m = blockIdx.y * 16 + grp; m < M; m += 16 * gridDim.y) {
      const long row = (long)(m / B) * Bp + (m % B);
      acc += logisticf_(S[row * Kp + j] + o) * scale;
    }
  }
  sh[grp][c] = acc;
  __syncthreads();
  if (grp != 0) return;
  float tot = 0.0f;
  for (int g = 0; g < 16; ++g) tot += sh[g][c];
  part[(long)blockIdx.y * Kp + j] = tot;
}

// dHs[row][:] += ct[row] * Wo_c[y_row][:]: the target word's share of what the output layer sends back.
template <typename T>
__global__ void __launch_bounds__(256) nce_target_dhs_kernel(const T *__restrict__ Wo_c, int Hp,
                                                             const int32_t *__restrict__ yp,
                                                             const float *__restrict__ ct,
                                                             float *__restrict__ dHs) {
  const int row = blockIdx.x;
  const int y = yp[row];
  if (y < 0) return;
  const float c = ct[row];
  const T *w = Wo_c + (long)y * Hp;
  float *d = dHs + (long)row * Hp;
  for (int col = threadIdx.x; col < Hp; col += 256) d[col] = fmaf(c, to_f32(w[col]), d[col]);
}

// Update of the touched rows of Wo, atomic-free and order-fixed:
//   out[w][:] = alpha*Wo[w][:] - lr * ( sum_{noise entries e of w} G[e][:] + sum_{target entries} ct*Hs[row][:] )
// blockIdx.x = run of equal ids in the sorted update list (exits when >= *nseg), blockIdx.y = block of
// 64*VEC columns.  The run's members are dealt round-robin to 16 partial sums (each in ascending list
// order) which are then added in order.  Also refreshes the compute copy of the row when Wc != nullptr.
// compact_ld > 0 redirects the results to compact per-run buffers (see below).
// The first column block also updates the word's bias the same way:
//   b_out[w] = alpha*b[w] - lr * (sum over w's noise entries of their column sums + sum of ct over its target
//   entries); a noise entry's column sum is the sum, in order, of the NCE_COLSUM_PARTS row-block partials
//   gpart[y][Kp].
template <typename T, int VEC>
__global__ void __launch_bounds__(1024) nce_row_update_kernel(const float *__restrict__ G, const T *__restrict__ Hs1,
                                                              int Hp, int H, int K, int B, int Bp,
                                                              const float *__restrict__ ct,
                                                              const int32_t *__restrict__ ids,
                                                              const int32_t *__restrict__ perm,
                                                              const int32_t *__restrict__ seg_start,
                                                              const int32_t *__restrict__ nseg,
                                                              const float *__restrict__ W, float *__restrict__ out,
                                                              T *__restrict__ Wc, const float *__restrict__ gpart,
                                                              int Kp,
                                                              const float *__restrict__ b, float *__restrict__ b_out,
                                                              float alpha, float lr, int compact_ld) {
  constexpr int PARTS = 16, LANES = 64;
  __shared__ float sh[PARTS][LANES * VEC];
  __shared__ float shb[PARTS];
  const int g = blockIdx.x;
  if (g >= *nseg) return;
  const int lane = threadIdx.x % LANES, partn = threadIdx.x / LANES;
  const int col = (blockIdx.y * LANES + lane) * VEC;
  const int r0 = seg_start[g], r1 = seg_start[g + 1];
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = 0.0f;
  float bacc = 0.0f;  // bias sum of the part (meaningful in its first lane)
  const bool live = col < H;
  // one member: its row (times its coefficient) and its bias term
  auto fetch = [&](int r, float (&v)[VEC], float &bv) {
    const int ent = perm[r];
    if (ent < K) {
      bv = 0.0f;
      if (lane == 0) {  // the part's bias sum is kept by its first lane only
        float pv[NCE_COLSUM_PARTS];  // all partials requested before any is added
#pragma unroll
        for (int y = 0; y < NCE_COLSUM_PARTS; ++y) pv[y] = gpart[(long)y * Kp + ent];
        bv = pv[0];
#pragma unroll
        for (int y = 1; y < NCE_COLSUM_PARTS; ++y) bv += pv[y];
      }
      if (live) {
        const float *src = G + (long)ent * Hp + col;
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = src[e];
      }
    } else {
      const int m = ent - K;
      const long row = (long)(m / B) * Bp + (m % B);
      const float c = ct[row];
      bv = c;
      if (live) {
        const T *src = Hs1 + row * Hp + col;
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = c * to_f32(src[e]);
      }
    }
  };
  int r = r0 + partn;
  for (; r + 3 * PARTS < r1; r += 4 * PARTS) {  // four members at a time: their loads are independent
    float v[4][VEC], bv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
#pragma unroll
      for (int e = 0; e < VEC; ++e) v[q][e] = 0.0f;
      fetch(r + q * PARTS, v[q], bv[q]);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      bacc += bv[q];
#pragma unroll
      for (int e = 0; e < VEC; ++e) acc[e] += v[q][e];
    }
  }
  for (; r < r1; r += PARTS) {
    float v[VEC], bv;
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] = 0.0f;
    fetch(r, v, bv);
    bacc += bv;
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] += v[e];
  }
#pragma unroll
  for (int e = 0; e < VEC; ++e) sh[partn][lane * VEC + e] = acc[e];
  if (lane == 0) shb[partn] = bacc;
  __syncthreads();
  if (blockIdx.y == 0 && threadIdx.x == 0) {
    const int wb = ids[perm[r0]];
    float tot = shb[0];
    for (int q = 1; q < PARTS; ++q) tot += shb[q];
    b_out[compact_ld > 0 ? g : wb] = ((alpha != 0.0f) ? alpha * b[wb] : 0.0f) - lr * tot;
  }
  if (partn != 0 || !live) return;
#pragma unroll
  for (int q = 1; q < PARTS; ++q)
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] += sh[q][lane * VEC + e];
  const int w = ids[perm[r0]];
  const long idx = (long)w * H + col;
  // compact_ld > 0: the run's result goes to row g of a compact [runs][compact_ld] buffer (and its bias
  // term to entry g of b_out) instead of the word's own row
  const long oidx = compact_ld > 0 ? (long)g * compact_ld + col : idx;
  if constexpr (VEC == 4) {  // H % 4 == 0: 16-byte accesses to the master row
    f32x4_t v = {0.0f, 0.0f, 0.0f, 0.0f};
    if (alpha != 0.0f) v = *reinterpret_cast<const f32x4_t *>(W + idx) * alpha;
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] -= lr * acc[e];
    *reinterpret_cast<f32x4_t *>(out + oidx) = v;
    if (Wc) {
      if constexpr (sizeof(T) == 2) {
        bf16x4_t hv;
#pragma unroll
        for (int e = 0; e < 4; ++e) hv[e] = (bf16_t)v[e];
        *reinterpret_cast<bf16x4_t *>(Wc + (long)w * Hp + col) = hv;
      } else {
        *reinterpret_cast<f32x4_t *>(Wc + (long)w * Hp + col) = v;
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
      const float v = ((alpha != 0.0f) ? alpha * W[idx + e] : 0.0f) - lr * acc[e];
      out[oidx + e] = v;
      if (Wc) Wc[(long)w * Hp + col + e] = from_f32<T>(v);
    }
  }
}

}  // namespace rnnlm_dev