/*
 * fp64 CPU oracle for the minibatched Elman RNN language-model step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker the HIP path is judged
 * against; it is never part of the product path.  It shares no code, header,
 * table or helper with the HIP library, and neither includes the other.
 *
 * What it computes (plain definitions, loops only, no blocking or fusion):
 *   - the plain Elman recurrent network without hidden bias units of Sec. 4.1:
 *       a_t = E[w_t] + U h_{t-1},  h_t = 1/(1+exp(-a_t)),
 *     whose output is a probability for every word of the vocabulary given h_t (Sec. 4.1),
 *     explicitly normalised as Sec. 4.2 does when reporting perplexity:
 *       z = Wo h_t + b,  log P(w | history) = z_w - log sum_v exp(z_v);
 *   - noffset = B token streams read from B different points of one corpus, each
 *     with its own carried hidden state (Sec. 4.2 data-offset scheme); the state is
 *     never reset at sentence markers (Sec. 2.3 keeps between-sentence context);
 *   - one update per window of T positions (the "minibatch" of Sec. 4.2): the
 *     gradient of the mean negative log-likelihood of the B*T tokens of the window,
 *     back-propagated through time to the window start and no further, followed by
 *     one plain SGD step (Sec. 4.2 names stochastic gradient descent);
 *   - perplexity = exp(-mean log P) (Sec. 1 names it the primary metric);
 *   - the same step with the noise-contrastive criterion Sec. 4.2 trains with (the
 *     oracle_nce_* functions further down state the estimator and the readings taken).
 *
 * Layouts: row-major; E[V][H], U[H][H] (a_i = sum_j U[i][j] h_j), Wo[V][H], b[V],
 * h[B][H]; token windows are time-major x[T][B], y[T][B].
 *
 * Readings where the paper is silent: sigmoid hidden units, zero initial state,
 * an output bias b (trained), mean (not summed) loss over the window, natural log.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)
#define ORACLE_ERR_TOKEN (-2)
#define ORACLE_ERR_NOMEM (-3)

static int check_tokens(const int32_t *a, long n, int V) {
  for (long i = 0; i < n; ++i)
    if (a[i] < 0 || a[i] >= V) return ORACLE_ERR_TOKEN;
  return ORACLE_OK;
}

/* Stream indexing of window k (Sec. 4.2 data-offset scheme): L = floor((N-1)/B)
 * positions per stream; stream s reads inputs tok[s*L + k*T + t] and predicts the
 * next token of the corpus. Returns the number of full windows floor(L/T). */
long oracle_stream_chunk(const int32_t *tok, long N, int B, int T, long k, int32_t *x, int32_t *y) {
  if (!tok || B <= 0 || T <= 0 || N < 2) return ORACLE_ERR_ARG;
  long L = (N - 1) / B;
  long nchunks = L / T;
  if (x && y) {
    if (k < 0 || k >= nchunks) return ORACLE_ERR_ARG;
    for (int t = 0; t < T; ++t)
      for (int s = 0; s < B; ++s) {
        long p = (long)s * L + k * T + t;
        x[(long)t * B + s] = tok[p];
        y[(long)t * B + s] = tok[p + 1];
      }
  }
  return nchunks;
}

/* Forward pass of one window from state h0.  Fills Hs[T][B][H], logp[T][B] and,
 * when P != NULL, the full normalised distributions P[T][B][V]. */
static int forward_window(int V, int H, int B, int T, const double *E, const double *U, const double *Wo,
                          const double *b, const double *h0, const int32_t *x, const int32_t *y, double *Hs,
                          double *P, double *logp) {
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = 0; s < B; ++s) {
    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    if (!z) {
#pragma omp atomic write
      err = 1;
      continue;
    }
    const double *hprev = h0 + (size_t)s * H;
    for (int t = 0; t < T; ++t) {
      const size_t m = (size_t)t * B + s;
      const double *e = E + (size_t)x[m] * H;
      double *h = Hs + m * H;
      for (int i = 0; i < H; ++i) {
        const double *u = U + (size_t)i * H;
        double a = 0.0;
#pragma omp simd reduction(+ : a)
        for (int j = 0; j < H; ++j) a += u[j] * hprev[j];
        a += e[i];
        h[i] = 1.0 / (1.0 + exp(-a));
      }
      double mx = -INFINITY;
      for (int v = 0; v < V; ++v) {
        const double *w = Wo + (size_t)v * H;
        double acc = 0.0;
#pragma omp simd reduction(+ : acc)
        for (int j = 0; j < H; ++j) acc += w[j] * h[j];
        z[v] = acc + b[v];
        if (z[v] > mx) mx = z[v];
      }
      double sum = 0.0;
      for (int v = 0; v < V; ++v) sum += exp(z[v] - mx);
      const double lse = mx + log(sum);
      logp[m] = z[y[m]] - lse;
      if (P) {
        double *p = P + m * V;
        for (int v = 0; v < V; ++v) p[v] = exp(z[v] - lse);
      }
      hprev = h;
    }
    free(z);
  }
  return err ? ORACLE_ERR_NOMEM : ORACLE_OK;
}

/* log P(y | history) for one window; advances h in place. Optional outputs
 * (may be NULL): Hs_out[T][B][H] hidden states, P_out[T][B][V] distributions. */
int oracle_forward_logprob(int V, int H, int B, int T, const double *E, const double *U, const double *Wo,
                           const double *b, double *h, const int32_t *x, const int32_t *y, double *logp,
                           double *Hs_out, double *P_out) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0 || !E || !U || !Wo || !b || !h || !x || !y || !logp) return ORACLE_ERR_ARG;
  if (check_tokens(x, (long)B * T, V) || check_tokens(y, (long)B * T, V)) return ORACLE_ERR_TOKEN;
  double *Hs = Hs_out ? Hs_out : (double *)malloc(sizeof(double) * (size_t)T * B * H);
  if (!Hs) return ORACLE_ERR_NOMEM;
  int rc = forward_window(V, H, B, T, E, U, Wo, b, h, x, y, Hs, P_out, logp);
  if (rc == ORACLE_OK) memcpy(h, Hs + (size_t)(T - 1) * B * H, sizeof(double) * (size_t)B * H);
  if (!Hs_out) free(Hs);
  return rc;
}

/* Truncated back-propagation through time over one window (the "minibatch" of Sec. 4.2), given
 * dHs[T][B][H] = the derivative of the window loss with respect to each hidden state through the
 * output layer alone.  Per stream, backwards in time:
 *   dh_j = dHs_j + sum_i U[i][j] da_next_i ;  da = dh * h * (1-h)   (da_next = 0 at the last position)
 * the carried state h0 is a constant, so the chain stops at the window start.  Fills dA[T][B][H]
 * (= dLoss/da), gU[H][H] and gE[V][H]. */
static void backprop_through_time(int V, int H, int B, int T, const double *U, const double *h0, const int32_t *x,
                                  const double *Hs, const double *dHs, double *dA, double *gU, double *gE) {
  const size_t M = (size_t)B * T;
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = 0; s < B; ++s) {
    for (int t = T - 1; t >= 0; --t) {
      const size_t m = (size_t)t * B + s;
      const double *dh = dHs + m * H;
      double *da = dA + m * H;
      const double *h = Hs + m * H;
      if (t == T - 1) {
        for (int j = 0; j < H; ++j) da[j] = dh[j] * h[j] * (1.0 - h[j]);
      } else {
        const double *dan = dA + ((size_t)(t + 1) * B + s) * H;
        for (int j = 0; j < H; ++j) da[j] = dh[j];
        for (int i = 0; i < H; ++i) {
          const double *u = U + (size_t)i * H;
          const double di = dan[i];
          for (int j = 0; j < H; ++j) da[j] += u[j] * di;
        }
        for (int j = 0; j < H; ++j) da[j] *= h[j] * (1.0 - h[j]);
      }
    }
  }
  /* gU[i][j] = sum_{t,s} da[t][s][i] * hprev[t][s][j], hprev = h0 at t = 0 */
#pragma omp parallel for schedule(static)
  for (int i = 0; i < H; ++i) {
    double *g = gU + (size_t)i * H;
    for (int j = 0; j < H; ++j) g[j] = 0.0;
    for (int t = 0; t < T; ++t)
      for (int s = 0; s < B; ++s) {
        const size_t m = (size_t)t * B + s;
        const double *hp = (t > 0) ? Hs + ((size_t)(t - 1) * B + s) * H : h0 + (size_t)s * H;
        const double di = dA[m * H + i];
        for (int j = 0; j < H; ++j) g[j] += di * hp[j];
      }
  }
  /* gE[w] = sum over window positions whose input id is w of da */
  memset(gE, 0, sizeof(double) * (size_t)V * H);
  for (size_t m = 0; m < M; ++m) {
    double *g = gE + (size_t)x[m] * H;
    const double *da = dA + m * H;
    for (int j = 0; j < H; ++j) g[j] += da[j];
  }
}

/* Gradient of the window's mean negative log-likelihood
 *   Loss = -(1/(B*T)) * sum_{t,s} log P(y[t][s] | ...)
 * with respect to E, U, Wo, b, all evaluated at the given parameters; the carried
 * state h0 is a constant (truncated back-propagation through time: the gradient
 * stops at the window start).  h0 is not modified; h_out (may be NULL) receives the
 * state after the window.  Optional debug outputs (may be NULL): Hs[T][B][H],
 * dZ[T][B][V] (= dLoss/dz), dHs[T][B][H] (= Wo^T dz only), dA[T][B][H] (= dLoss/da). */
int oracle_grad_chunk(int V, int H, int B, int T, const double *E, const double *U, const double *Wo,
                      const double *b, const double *h0, const int32_t *x, const int32_t *y, double *logp,
                      double *gE, double *gU, double *gWo, double *gb, double *h_out, double *Hs_out,
                      double *dZ_out, double *dHs_out, double *dA_out) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0 || !E || !U || !Wo || !b || !h0 || !x || !y || !logp || !gE || !gU ||
      !gWo || !gb)
    return ORACLE_ERR_ARG;
  const size_t M = (size_t)B * T;
  if (check_tokens(x, (long)M, V) || check_tokens(y, (long)M, V)) return ORACLE_ERR_TOKEN;
  double *Hs = Hs_out ? Hs_out : (double *)malloc(sizeof(double) * M * H);
  double *dZ = dZ_out ? dZ_out : (double *)malloc(sizeof(double) * M * V);
  double *dHs = dHs_out ? dHs_out : (double *)malloc(sizeof(double) * M * H);
  double *dA = dA_out ? dA_out : (double *)malloc(sizeof(double) * M * H);
  int rc = ORACLE_ERR_NOMEM;
  if (Hs && dZ && dHs && dA) {
    rc = forward_window(V, H, B, T, E, U, Wo, b, h0, x, y, Hs, dZ, logp);
  }
  if (rc == ORACLE_OK) {
    const double scale = 1.0 / (double)M;
    /* dz = (p - onehot(y)) / (B*T) */
#pragma omp parallel for schedule(static)
    for (long m = 0; m < (long)M; ++m) {
      double *d = dZ + (size_t)m * V;
      d[y[m]] -= 1.0;
      for (int v = 0; v < V; ++v) d[v] *= scale;
    }
    /* gWo[v][j] = sum_m dz[m][v] Hs[m][j];  gb[v] = sum_m dz[m][v] */
#pragma omp parallel for schedule(static)
    for (int v = 0; v < V; ++v) {
      double *g = gWo + (size_t)v * H;
      for (int j = 0; j < H; ++j) g[j] = 0.0;
      double sb = 0.0;
      for (size_t m = 0; m < M; ++m) {
        const double d = dZ[m * V + v];
        const double *h = Hs + m * H;
        sb += d;
        for (int j = 0; j < H; ++j) g[j] += d * h[j];
      }
      gb[v] = sb;
    }
    /* dHs[m][j] = sum_v Wo[v][j] dz[m][v]: what the output layer sends back to each hidden state */
#pragma omp parallel for schedule(static)
    for (long m = 0; m < (long)M; ++m) {
      double *dh = dHs + (size_t)m * H;
      for (int j = 0; j < H; ++j) dh[j] = 0.0;
      const double *d = dZ + (size_t)m * V;
      for (int v = 0; v < V; ++v) {
        const double dv = d[v];
        const double *w = Wo + (size_t)v * H;
        for (int j = 0; j < H; ++j) dh[j] += w[j] * dv;
      }
    }
    backprop_through_time(V, H, B, T, U, h0, x, Hs, dHs, dA, gU, gE);
    if (h_out) memcpy(h_out, Hs + (size_t)(T - 1) * B * H, sizeof(double) * (size_t)B * H);
  }
  if (!Hs_out) free(Hs);
  if (!dZ_out) free(dZ);
  if (!dHs_out) free(dHs);
  if (!dA_out) free(dA);
  return rc;
}

/* One training step on one window: gradients at the current parameters, then
 * theta <- theta - lr * g for E, U, Wo, b; h <- state after the window (computed with
 * the pre-update parameters).  logp[T][B]; *sum_logp (may be NULL) = sum of logp. */
int oracle_train_chunk(int V, int H, int B, int T, double *E, double *U, double *Wo, double *b, double *h,
                       const int32_t *x, const int32_t *y, double lr, double *logp, double *sum_logp) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0) return ORACLE_ERR_ARG;
  const size_t nVH = (size_t)V * H, nHH = (size_t)H * H;
  double *gE = (double *)malloc(sizeof(double) * nVH);
  double *gWo = (double *)malloc(sizeof(double) * nVH);
  double *gU = (double *)malloc(sizeof(double) * nHH);
  double *gb = (double *)malloc(sizeof(double) * (size_t)V);
  double *hn = (double *)malloc(sizeof(double) * (size_t)B * H);
  int rc = ORACLE_ERR_NOMEM;
  if (gE && gWo && gU && gb && hn)
    rc = oracle_grad_chunk(V, H, B, T, E, U, Wo, b, h, x, y, logp, gE, gU, gWo, gb, hn, NULL, NULL, NULL, NULL);
  if (rc == ORACLE_OK) {
    for (size_t i = 0; i < nVH; ++i) E[i] -= lr * gE[i];
    for (size_t i = 0; i < nVH; ++i) Wo[i] -= lr * gWo[i];
    for (size_t i = 0; i < nHH; ++i) U[i] -= lr * gU[i];
    for (int v = 0; v < V; ++v) b[v] -= lr * gb[v];
    memcpy(h, hn, sizeof(double) * (size_t)B * H);
    if (sum_logp) {
      double sacc = 0.0;
      for (size_t m = 0; m < (size_t)B * T; ++m) sacc += logp[m];
      *sum_logp = sacc;
    }
  }
  free(gE); free(gWo); free(gU); free(gb); free(hn);
  return rc;
}

/* ---- rmsprop (Sec. 4.2: the paper trains with SGD and rmsprop, smoothing constant 0.9995) -----------
 *
 * One training step on one window with the rmsprop scaling of the SGD step.  Readings where the paper
 * is silent: a running mean of squared gradients  r <- rho*r + (1-rho)*s  is updated first and the step
 * is  theta <- theta - lr * g / (sqrt(r) + eps);  for the state-to-state matrix U and the output bias
 * b, s = g^2 element by element (rU[H][H], rb[V]); for the input-to-state and state-to-output matrices
 * E and Wo each WORD has a single value, s = the mean over the H units of the squared gradient of that
 * word's row (rE[V], rWo[V]: Sec. 4.2 averages over the nstate units so that each word has one value).
 * Rows whose gradient is zero (words not in the window) keep their weights and their value decays by
 * rho like any other.  The statistics are caller-initialised state, updated in place. */
/* The rmsprop-scaled step itself, given the gradients (see oracle_train_chunk_rmsprop for the readings). */
static void rmsprop_apply(int V, int H, double *E, double *U, double *Wo, double *b, const double *gE,
                          const double *gU, const double *gWo, const double *gb, double lr, double rho, double eps,
                          double *rE, double *rU, double *rWo, double *rb) {
  const size_t nHH = (size_t)H * H;
  /* one value per word for E and Wo */
  for (int w = 0; w < V; ++w) {
    double sE = 0.0, sW = 0.0;
    for (int j = 0; j < H; ++j) {
      sE += gE[(size_t)w * H + j] * gE[(size_t)w * H + j];
      sW += gWo[(size_t)w * H + j] * gWo[(size_t)w * H + j];
    }
    rE[w] = rho * rE[w] + (1.0 - rho) * (sE / H);
    rWo[w] = rho * rWo[w] + (1.0 - rho) * (sW / H);
    const double dE = sqrt(rE[w]) + eps, dW = sqrt(rWo[w]) + eps;
    for (int j = 0; j < H; ++j) {
      /* a zero gradient moves nothing (also when the denominator is zero) */
      if (gE[(size_t)w * H + j] != 0.0) E[(size_t)w * H + j] -= lr * gE[(size_t)w * H + j] / dE;
      if (gWo[(size_t)w * H + j] != 0.0) Wo[(size_t)w * H + j] -= lr * gWo[(size_t)w * H + j] / dW;
    }
  }
  /* one value per element for U and b */
  for (size_t i = 0; i < nHH; ++i) {
    rU[i] = rho * rU[i] + (1.0 - rho) * gU[i] * gU[i];
    if (gU[i] != 0.0) U[i] -= lr * gU[i] / (sqrt(rU[i]) + eps);
  }
  for (int v = 0; v < V; ++v) {
    rb[v] = rho * rb[v] + (1.0 - rho) * gb[v] * gb[v];
    if (gb[v] != 0.0) b[v] -= lr * gb[v] / (sqrt(rb[v]) + eps);
  }
}

int oracle_train_chunk_rmsprop(int V, int H, int B, int T, double *E, double *U, double *Wo, double *b, double *h,
                               const int32_t *x, const int32_t *y, double lr, double rho, double eps, double *rE,
                               double *rU, double *rWo, double *rb, double *logp, double *sum_logp) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0 || !rE || !rU || !rWo || !rb) return ORACLE_ERR_ARG;
  const size_t nVH = (size_t)V * H, nHH = (size_t)H * H;
  double *gE = (double *)malloc(sizeof(double) * nVH);
  double *gWo = (double *)malloc(sizeof(double) * nVH);
  double *gU = (double *)malloc(sizeof(double) * nHH);
  double *gb = (double *)malloc(sizeof(double) * (size_t)V);
  double *hn = (double *)malloc(sizeof(double) * (size_t)B * H);
  int rc = ORACLE_ERR_NOMEM;
  if (gE && gWo && gU && gb && hn)
    rc = oracle_grad_chunk(V, H, B, T, E, U, Wo, b, h, x, y, logp, gE, gU, gWo, gb, hn, NULL, NULL, NULL, NULL);
  if (rc == ORACLE_OK) {
    rmsprop_apply(V, H, E, U, Wo, b, gE, gU, gWo, gb, lr, rho, eps, rE, rU, rWo, rb);
    memcpy(h, hn, sizeof(double) * (size_t)B * H);
    if (sum_logp) {
      double sacc = 0.0;
      for (size_t m = 0; m < (size_t)B * T; ++m) sacc += logp[m];
      *sum_logp = sacc;
    }
  }
  free(gE); free(gWo); free(gU); free(gb); free(hn);
  return rc;
}

/* ---- Noise-contrastive estimation (Sec. 4.2 names it as the training criterion) -------------------
 *
 * The paper gives no formula, noise distribution, sample count or normaliser; this follows the
 * published estimator (Gutmann & Hyvarinen; for language models Mnih & Teh) under these readings:
 *   - the unnormalised score of word w at window position m is z_m(w) = Wo[w].h_m + b[w], read as
 *     log P up to the constant lnZ (a parameter; 0 = self-normalised);
 *   - K noise words n_0..n_{K-1}, drawn by the caller from a noise distribution q (log-probabilities
 *     lnq[V]) and SHARED by all B*T positions of the window;
 *   - with D_m(w) = z_m(w) - lnZ - ln(K q(w)) and sigma the logistic function, position m costs
 *       J_m = -ln sigma(D_m(y_m)) - sum_j ln(1 - sigma(D_m(n_j)))
 *     (each noise word is its own term, also when it repeats or equals the target);
 *   - window loss = mean of J_m over the B*T positions; its gradient is back-propagated through time
 *     exactly as for the normalised criterion.
 * ln sigma(d) = -softplus(-d), ln(1 - sigma(d)) = -softplus(d), softplus(d) = ln(1 + e^d). */
static double softplus(double d) { return d > 0.0 ? d + log1p(exp(-d)) : log1p(exp(d)); }
static double logistic(double d) { return d >= 0.0 ? 1.0 / (1.0 + exp(-d)) : exp(d) / (1.0 + exp(d)); }

/* The recurrence alone: Hs[T][B][H] from state h0 (a_t = E[w_t] + U h_{t-1}, h_t = sigmoid(a_t)). */
static void hidden_forward(int H, int B, int T, const double *E, const double *U, const double *h0,
                           const int32_t *x, double *Hs) {
#pragma omp parallel for schedule(dynamic, 1)
  for (int s = 0; s < B; ++s) {
    const double *hprev = h0 + (size_t)s * H;
    for (int t = 0; t < T; ++t) {
      const size_t m = (size_t)t * B + s;
      const double *e = E + (size_t)x[m] * H;
      double *h = Hs + m * H;
      for (int i = 0; i < H; ++i) {
        const double *u = U + (size_t)i * H;
        double a = 0.0;
#pragma omp simd reduction(+ : a)
        for (int j = 0; j < H; ++j) a += u[j] * hprev[j];
        a += e[i];
        h[i] = 1.0 / (1.0 + exp(-a));
      }
      hprev = h;
    }
  }
}

/* Gradient of the window's mean NCE loss with respect to E, U, Wo, b at the given parameters.
 * noise[K] ids in [0,V); lnq[V]; J[T][B] receives the per-position losses.  h0 is not modified;
 * h_out (may be NULL) receives the state after the window.  Optional debug outputs (may be NULL):
 * ct[T][B] = dLoss/dz_m(y_m), dS[T][B][K] = dLoss/dz_m(n_j) (one entry per noise draw), dHs[T][B][H],
 * dA[T][B][H]. */
int oracle_nce_grad_chunk(int V, int H, int B, int T, const double *E, const double *U, const double *Wo,
                          const double *b, const double *h0, const int32_t *x, const int32_t *y, int K,
                          const int32_t *noise, const double *lnq, double lnZ, double *J, double *gE, double *gU,
                          double *gWo, double *gb, double *h_out, double *ct_out, double *dS_out, double *dHs_out,
                          double *dA_out) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0 || K <= 0 || !E || !U || !Wo || !b || !h0 || !x || !y || !noise ||
      !lnq || !J || !gE || !gU || !gWo || !gb)
    return ORACLE_ERR_ARG;
  const size_t M = (size_t)B * T;
  if (check_tokens(x, (long)M, V) || check_tokens(y, (long)M, V) || check_tokens(noise, K, V)) return ORACLE_ERR_TOKEN;
  double *Hs = (double *)malloc(sizeof(double) * M * H);
  double *dHs = dHs_out ? dHs_out : (double *)malloc(sizeof(double) * M * H);
  double *dA = dA_out ? dA_out : (double *)malloc(sizeof(double) * M * H);
  int rc = (Hs && dHs && dA) ? ORACLE_OK : ORACLE_ERR_NOMEM;
  if (rc == ORACLE_OK) {
    hidden_forward(H, B, T, E, U, h0, x, Hs);
    const double lnK = log((double)K), scale = 1.0 / (double)M;
    memset(gWo, 0, sizeof(double) * (size_t)V * H);
    memset(gb, 0, sizeof(double) * (size_t)V);
    memset(dHs, 0, sizeof(double) * M * H);
    /* positions one after the other: every scored word w with coefficient c = dLoss/dz_m(w) adds
     * c*h_m to gWo[w], c to gb[w] and c*Wo[w] to dHs[m] */
    for (size_t m = 0; m < M; ++m) {
      const double *h = Hs + m * H;
      double *dh = dHs + m * H;
      double cost = 0.0;
      for (int j = -1; j < K; ++j) { /* j = -1: the target word, j >= 0: noise word j */
        const int w = (j < 0) ? y[m] : noise[j];
        const double *wo = Wo + (size_t)w * H;
        double z = b[w];
        for (int i = 0; i < H; ++i) z += wo[i] * h[i];
        const double d = z - lnZ - (lnK + lnq[w]);
        double c;
        if (j < 0) {
          cost += softplus(-d);         /* -ln sigma(d) */
          c = -(1.0 - logistic(d)) * scale;
          if (ct_out) ct_out[m] = c;
        } else {
          cost += softplus(d);          /* -ln(1 - sigma(d)) */
          c = logistic(d) * scale;
          if (dS_out) dS_out[m * K + j] = c;
        }
        double *g = gWo + (size_t)w * H;
        for (int i = 0; i < H; ++i) g[i] += c * h[i];
        gb[w] += c;
        for (int i = 0; i < H; ++i) dh[i] += c * wo[i];
      }
      J[m] = cost;
    }
    backprop_through_time(V, H, B, T, U, h0, x, Hs, dHs, dA, gU, gE);
    if (h_out) memcpy(h_out, Hs + (size_t)(T - 1) * B * H, sizeof(double) * (size_t)B * H);
  }
  free(Hs);
  if (!dHs_out) free(dHs);
  if (!dA_out) free(dA);
  return rc;
}

/* One NCE training step on one window: gradients at the current parameters, then one plain SGD
 * step on E, U, Wo, b; h <- state after the window (pre-update parameters).  J[T][B]; *sum_J (may
 * be NULL) = sum of J. */
int oracle_nce_train_chunk(int V, int H, int B, int T, double *E, double *U, double *Wo, double *b, double *h,
                           const int32_t *x, const int32_t *y, int K, const int32_t *noise, const double *lnq,
                           double lnZ, double lr, double *J, double *sum_J) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0) return ORACLE_ERR_ARG;
  const size_t nVH = (size_t)V * H, nHH = (size_t)H * H;
  double *gE = (double *)malloc(sizeof(double) * nVH);
  double *gWo = (double *)malloc(sizeof(double) * nVH);
  double *gU = (double *)malloc(sizeof(double) * nHH);
  double *gb = (double *)malloc(sizeof(double) * (size_t)V);
  double *hn = (double *)malloc(sizeof(double) * (size_t)B * H);
  int rc = ORACLE_ERR_NOMEM;
  if (gE && gWo && gU && gb && hn)
    rc = oracle_nce_grad_chunk(V, H, B, T, E, U, Wo, b, h, x, y, K, noise, lnq, lnZ, J, gE, gU, gWo, gb, hn, NULL,
                               NULL, NULL, NULL);
  if (rc == ORACLE_OK) {
    for (size_t i = 0; i < nVH; ++i) E[i] -= lr * gE[i];
    for (size_t i = 0; i < nVH; ++i) Wo[i] -= lr * gWo[i];
    for (size_t i = 0; i < nHH; ++i) U[i] -= lr * gU[i];
    for (int v = 0; v < V; ++v) b[v] -= lr * gb[v];
    memcpy(h, hn, sizeof(double) * (size_t)B * H);
    if (sum_J) {
      double sacc = 0.0;
      for (size_t m = 0; m < (size_t)B * T; ++m) sacc += J[m];
      *sum_J = sacc;
    }
  }
  free(gE); free(gWo); free(gU); free(gb); free(hn);
  return rc;
}

/* The noise-contrastive step with the rmsprop scaling: the paper's own combination (Sec. 4.2 trains with
 * noise-contrastive estimation, SGD and rmsprop).  Gradients of oracle_nce_grad_chunk, step of
 * rmsprop_apply; words that are neither target nor noise have a zero row in gWo and a zero entry in gb. */
int oracle_nce_train_chunk_rmsprop(int V, int H, int B, int T, double *E, double *U, double *Wo, double *b, double *h,
                                   const int32_t *x, const int32_t *y, int K, const int32_t *noise, const double *lnq,
                                   double lnZ, double lr, double rho, double eps, double *rE, double *rU, double *rWo,
                                   double *rb, double *J, double *sum_J) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0 || !rE || !rU || !rWo || !rb) return ORACLE_ERR_ARG;
  const size_t nVH = (size_t)V * H, nHH = (size_t)H * H;
  double *gE = (double *)malloc(sizeof(double) * nVH);
  double *gWo = (double *)malloc(sizeof(double) * nVH);
  double *gU = (double *)malloc(sizeof(double) * nHH);
  double *gb = (double *)malloc(sizeof(double) * (size_t)V);
  double *hn = (double *)malloc(sizeof(double) * (size_t)B * H);
  int rc = ORACLE_ERR_NOMEM;
  if (gE && gWo && gU && gb && hn)
    rc = oracle_nce_grad_chunk(V, H, B, T, E, U, Wo, b, h, x, y, K, noise, lnq, lnZ, J, gE, gU, gWo, gb, hn, NULL,
                               NULL, NULL, NULL);
  if (rc == ORACLE_OK) {
    rmsprop_apply(V, H, E, U, Wo, b, gE, gU, gWo, gb, lr, rho, eps, rE, rU, rWo, rb);
    memcpy(h, hn, sizeof(double) * (size_t)B * H);
    if (sum_J) {
      double sacc = 0.0;
      for (size_t m = 0; m < (size_t)B * T; ++m) sacc += J[m];
      *sum_J = sacc;
    }
  }
  free(gE); free(gWo); free(gU); free(gb); free(hn);
  return rc;
}

/* Unnormalised scoring, forward only (Sec. 4.2: for rescoring the output is used without the explicit
 * normalisation): score[t][s] = Wo[y].h_t + b[y] - lnZ for the given next words y only, with lnZ the
 * constant a self-normalised (NCE-trained) model is read against.  Advances h in place. */
int oracle_forward_score(int V, int H, int B, int T, const double *E, const double *U, const double *Wo,
                         const double *b, double *h, const int32_t *x, const int32_t *y, double lnZ,
                         double *score) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0 || !E || !U || !Wo || !b || !h || !x || !y || !score) return ORACLE_ERR_ARG;
  const size_t M = (size_t)B * T;
  if (check_tokens(x, (long)M, V) || check_tokens(y, (long)M, V)) return ORACLE_ERR_TOKEN;
  double *Hs = (double *)malloc(sizeof(double) * M * H);
  if (!Hs) return ORACLE_ERR_NOMEM;
  hidden_forward(H, B, T, E, U, h, x, Hs);
  for (size_t m = 0; m < M; ++m) {
    const double *wo = Wo + (size_t)y[m] * H, *hm = Hs + m * H;
    double z = b[y[m]];
    for (int i = 0; i < H; ++i) z += wo[i] * hm[i];
    score[m] = z - lnZ;
  }
  memcpy(h, Hs + (size_t)(T - 1) * B * H, sizeof(double) * (size_t)B * H);
  free(Hs);
  return ORACLE_OK;
}

/* Perplexity of a token array: B streams from a zero state, every full window of T
 * positions scored, PPL = exp(-sum logp / #scored).  The result does not depend on
 * T except through which tail positions are dropped. */
int oracle_perplexity(int V, int H, int B, int T, const double *E, const double *U, const double *Wo,
                      const double *b, const int32_t *tok, long N, double *ppl, long *scored) {
  if (V <= 0 || H <= 0 || B <= 0 || T <= 0 || !tok || !ppl || N < 2) return ORACLE_ERR_ARG;
  long nchunks = oracle_stream_chunk(tok, N, B, T, 0, NULL, NULL);
  if (nchunks < 1) return ORACLE_ERR_ARG;
  const size_t M = (size_t)B * T;
  double *h = (double *)calloc((size_t)B * H, sizeof(double));
  int32_t *x = (int32_t *)malloc(sizeof(int32_t) * M);
  int32_t *y = (int32_t *)malloc(sizeof(int32_t) * M);
  double *lp = (double *)malloc(sizeof(double) * M);
  int rc = (h && x && y && lp) ? ORACLE_OK : ORACLE_ERR_NOMEM;
  double total = 0.0;
  for (long k = 0; k < nchunks && rc == ORACLE_OK; ++k) {
    oracle_stream_chunk(tok, N, B, T, k, x, y);
    rc = oracle_forward_logprob(V, H, B, T, E, U, Wo, b, h, x, y, lp, NULL, NULL);
    for (size_t m = 0; m < M && rc == ORACLE_OK; ++m) total += lp[m];
  }
  if (rc == ORACLE_OK) {
    *ppl = exp(-total / (double)(nchunks * (long)M));
    if (scored) *scored = nchunks * (long)M;
  }
  free(h); free(x); free(y); free(lp);
  return rc;
}

/* Integer helper for the embedding gradient: positions m = 0..M-1 of a window
 * ordered by (x[m], m) (a stable sort by id), and the start of each run of equal
 * ids.  perm[M]; seg_start[M+1] (first nseg+1 entries valid, seg_start[nseg] = M).
 * Returns nseg. */
int oracle_sort_segments(const int32_t *x, int M, int32_t *perm, int32_t *seg_start) {
  if (!x || M <= 0 || !perm || !seg_start) return ORACLE_ERR_ARG;
  for (int m = 0; m < M; ++m) perm[m] = m;
  for (int i = 1; i < M; ++i) { /* insertion sort: stable by construction */
    int32_t p = perm[i];
    int j = i - 1;
    while (j >= 0 && x[perm[j]] > x[p]) {
      perm[j + 1] = perm[j];
      --j;
    }
    perm[j + 1] = p;
  }
  int nseg = 0;
  for (int r = 0; r < M; ++r)
    if (r == 0 || x[perm[r]] != x[perm[r - 1]]) seg_start[nseg++] = r;
  seg_start[nseg] = M;
  return nseg;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
