/*
 * rnnlm.h - C ABI of the MI355X (gfx950) Elman RNN language-model training step.
 *
 * The model is the plain Elman recurrent network without hidden bias units that Sec. 4.1 of the paper
 * on scaling recurrent neural network language models describes:
 *     h_t = sigmoid(E[w_t] + U h_{t-1}),   z_t = Wo h_t + b,
 *     log P(w | history) = z_t[w] - log sum_v exp(z_t[v])   (explicitly normalised, Sec. 4.2)
 * trained on B = "noffset" token streams read from B points of one corpus, each with its
 * own carried hidden state (data-offset scheme, Sec. 4.2), with one update per window of T
 * positions (the "minibatch" of Sec. 4.2): truncated back-propagation through time over the
 * window, then plain stochastic gradient descent (Sec. 4.2).  The hidden state is never reset
 * at sentence markers (Sec. 2.3 keeps between-sentence context).  Perplexity (Sec. 1) is
 * exp(-mean log P).
 *
 * Conventions
 *   - Every array is row-major.  E[V][H], U[H][H] (a_i = sum_j U[i][j] h_j), Wo[V][H], b[V],
 *     h_state[B][H].  Token windows are time-major: x[T][B], y[T][B], logp[T][B]; the row index
 *     of position (t, s) is m = t*B + s.  Log-probabilities are natural logs.
 *   - "dev" pointers are DEVICE pointers of the configured HIP device; "host" pointers are
 *     ordinary host memory.  The library borrows the caller's parameter, state and workspace
 *     buffers (it allocates no device memory itself) and updates E, U, Wo, b, h_state in place.
 *     The buffers must stay alive and must not be written by the caller while a call is in
 *     flight on the stream.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *     work and return without waiting unless stated otherwise.  Calls on one handle must be
 *     issued on one stream at a time (they share the workspace).
 *   - Every function returns RNNLM_OK (0) or a negative rnnlm_status; nothing throws.
 *   - Token ids outside [0, V) never cause an out-of-bounds access: they are clamped on the
 *     device and a sticky flag is raised, reported as RNNLM_ERR_TOKEN_RANGE by the next
 *     synchronising call (rnnlm_perplexity, rnnlm_check).
 *   - Gradients are those of the MEAN negative log-likelihood of the B*T tokens of a window.
 *     All T positions of a window use the same (pre-update) parameters; duplicates of an input
 *     id within a window add up in a fixed order (no atomics), so results are run-to-run bitwise
 *     reproducible.
 */
#ifndef RNNLM_H
#define RNNLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rnnlm rnnlm_t; /* opaque host-side handle */

typedef enum {
  RNNLM_FP32 = 0,            /* fp32 storage, fp32 MFMA contraction */
  RNNLM_BF16_FP32MASTER = 1  /* bf16 operands (round-to-nearest-even), fp32 accumulation, fp32 master weights */
} rnnlm_precision;

typedef enum {
  RNNLM_OK = 0,
  RNNLM_ERR_ARG = -1,         /* null pointer, non-positive size, T > T_max, workspace too small, misaligned */
  RNNLM_ERR_TOKEN_RANGE = -2, /* some token id was outside [0, V) (ids were clamped, results are meaningless) */
  RNNLM_ERR_NONFINITE = -3,   /* a window's sum of log-probabilities was not finite */
  RNNLM_ERR_HIP = -4,         /* a HIP runtime call failed */
  RNNLM_ERR_NOMEM = -5,       /* host allocation failed */
  RNNLM_ERR_TIMEOUT = -6      /* a bounded wait inside a persistent kernel expired (results are meaningless) */
} rnnlm_status;

typedef struct {
  int32_t V;         /* vocabulary size, > 0 */
  int32_t H;         /* hidden units ("nstate"), > 0 */
  int32_t B;         /* parallel token streams ("noffset"), > 0 */
  int32_t T_max;     /* longest window a call may pass, > 0 */
  int32_t precision; /* rnnlm_precision */
  int32_t device;    /* HIP device ordinal */
  int32_t K_max;     /* most noise words per window the noise-contrastive calls may pass; 0 = those calls are
                        not used (no workspace is set aside for them), >= 0, at most 65536 */
  int32_t rmsprop;   /* 1: rnnlm_train_chunk_rmsprop may be called (adds gradient buffers of the size of Wo, U
                        and b to the workspace); 0: it may not */
  int32_t P;         /* 0: the plain architecture above.  > 0: the compressed architecture of Sec. 5.4 with
                        layers of P units below and above the state and tied word matrices (see "Compressed
                        architecture" below); requires K_max = 0 and rmsprop = 0 */
} rnnlm_config;

typedef struct {
  float *E;               /* dev [V][H]  input->state matrix (embedding rows), fp32 master */
  float *U;               /* dev [H][H]  state->state matrix */
  float *Wo;              /* dev [V][H]  state->output matrix */
  float *b;               /* dev [V]     output bias */
  float *h_state;         /* dev [B][H]  carried hidden state */
  void *workspace;        /* dev, 256-byte aligned, >= rnnlm_workspace_bytes(cfg) */
  size_t workspace_bytes;
  /* compressed architecture only (cfg.P > 0; NULL otherwise): then E is dev [V][P] and Wo must be NULL */
  float *A;               /* dev [H][P]  layer below the state -> state */
  float *C;               /* dev [P][H]  state -> layer above the state */
} rnnlm_buffers;

/* Device bytes of workspace the configuration needs (0 if cfg is invalid). */
size_t rnnlm_workspace_bytes(const rnnlm_config *cfg);

/* Validates cfg/buffers, binds the caller's buffers, clears the workspace and h_state (zero initial
 * state), and builds the compute copies of U and Wo (bf16 or fp32, tile-padded) inside the
 * workspace.  *out receives the handle.  Synchronises the device before returning. */
int rnnlm_init(const rnnlm_config *cfg, const rnnlm_buffers *buf, rnnlm_t **out);

/* Releases the host handle (device buffers belong to the caller). NULL is allowed. */
void rnnlm_free(rnnlm_t *h);

/* Stream indexing of window k under the data-offset scheme of Sec. 4.2: with L = floor((N-1)/B),
 * x[t][s] = tok[s*L + k*T + t] and y[t][s] = tok[s*L + k*T + t + 1].  tok: dev int32[N];
 * x, y: dev int32[T][B].  Requires 0 <= k < floor(L/T), 1 <= T <= T_max. Integer-exact. */
int rnnlm_stream_chunk(rnnlm_t *h, const int32_t *tok, int64_t N, int64_t k, int32_t T, int32_t *x, int32_t *y,
                       void *stream);

/* log P(y[t][s] | stream s up to x[t][s]) for one window (Sec. 4.1 / 4.2 normalised output),
 * starting from h_state, which is advanced to the state after the window.
 * x, y: dev int32[T][B]; logp: dev float[T][B]. */
int rnnlm_forward_logprob(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float *logp, void *stream);

/* One training step on one window (Sec. 4.2): forward, truncated BPTT gradients of the mean
 * negative log-likelihood at the current parameters, then theta <- theta - lr*g for E, U, Wo, b, and
 * h_state <- state after the window (computed with the pre-update parameters).
 * logp: dev float[T][B] or NULL; sum_logp: dev double (sum of the window's log-probs) or NULL. */
int rnnlm_train_chunk(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float lr, float *logp,
                      double *sum_logp, void *stream);

/* Running means of squared gradients for rnnlm_train_chunk_rmsprop, caller-owned and caller-initialised
 * device arrays, updated in place: one value per WORD for the input-to-state and state-to-output matrices
 * (Sec. 4.2 averages over the nstate units so that each word has a single value), one per element for U
 * and b. */
typedef struct {
  float *rE;  /* dev [V]    */
  float *rU;  /* dev [H][H] */
  float *rWo; /* dev [V]    */
  float *rb;  /* dev [V]    */
} rnnlm_rmsprop_state;

/* rnnlm_train_chunk with the rmsprop scaling of Sec. 4.2 (the paper trains with SGD and rmsprop, smoothing
 * constant 0.9995).  Readings where the paper is silent: the statistic is updated first,
 * r <- rho*r + (1-rho)*s, then theta <- theta - lr * g / (sqrt(r) + eps); s = g^2 element by element for
 * U and b, and the mean over the H units of the squared gradient of the word's row for E and Wo; words
 * whose row has a zero gradient keep their weights while their statistic decays by rho; a zero gradient
 * moves nothing.  Requires cfg.rmsprop = 1; 0 <= rho <= 1, eps >= 0.  Other arguments as rnnlm_train_chunk. */
int rnnlm_train_chunk_rmsprop(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float lr, float rho,
                              float eps, const rnnlm_rmsprop_state *state, float *logp, double *sum_logp,
                              void *stream);

/* rnnlm_nce_train_chunk with the rmsprop scaling of rnnlm_train_chunk_rmsprop: the combination Sec. 4.2
 * trains with (noise-contrastive estimation, SGD, rmsprop).  Words that are neither target nor noise in
 * the window have a zero gradient row in Wo and entry in b: they keep their weights and their statistics
 * decay by rho.  Requires cfg.K_max >= K and cfg.rmsprop = 1. */
int rnnlm_nce_train_chunk_rmsprop(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, const int32_t *noise,
                                  int32_t K, const float *lnq, float lnZ, float lr, float rho, float eps,
                                  const rnnlm_rmsprop_state *state, float *J, double *sum_J, void *stream);

/* Same kernels as rnnlm_train_chunk but the update epilogues write the gradients (of the mean
 * negative log-likelihood) into caller buffers instead of updating: dE: dev float[V][H] (rows of ids
 * not in x are zero), dU: dev float[H][H], dWo: dev float[V][H], db: dev float[V]; logp as above or
 * NULL.  Parameters and h_state are left unchanged. */
int rnnlm_grad_chunk(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float *dE, float *dU, float *dWo,
                     float *db, float *logp, void *stream);

/* One training step on one window under the noise-contrastive criterion that Sec. 4.2 trains with.
 * The paper gives neither formula nor constants; this is the published estimator (Gutmann & Hyvarinen;
 * Mnih & Teh for language models) with these readings: scores z_m(w) = Wo[w].h_m + b[w] are
 * log-probabilities up to the constant lnZ; K noise words, drawn by the caller from a noise
 * distribution with log-probabilities lnq, are shared by all B*T positions of the window; with
 * D_m(w) = z_m(w) - lnZ - ln(K q(w)) position m costs
 *     J_m = -ln sigmoid(D_m(y_m)) - sum_j ln(1 - sigmoid(D_m(noise[j])))
 * (every noise word is a term of its own, also when it repeats or equals the target); the window
 * loss is the mean of J_m; its gradient goes back through time as in rnnlm_train_chunk and is
 * followed by the same plain SGD step, which here touches only the rows of Wo and entries of b of the
 * target and noise words (contributions to one row add up in a fixed order, no atomics).
 * noise: dev int32[K], 1 <= K <= K_max, ids in [0,V) (checked like token ids); lnq: dev float[V];
 * J: dev float[T][B] or NULL; sum_J: dev double (sum of the window's J) or NULL.  The explicitly
 * normalised output used for perplexity is unchanged (rnnlm_forward_logprob, rnnlm_perplexity). */
int rnnlm_nce_train_chunk(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, const int32_t *noise, int32_t K,
                          const float *lnq, float lnZ, float lr, float *J, double *sum_J, void *stream);

/* Same kernels as rnnlm_nce_train_chunk with the updates redirected: gradients of the mean
 * noise-contrastive loss into dE, dU, dWo: dev float[V][H] / [H][H] / [V][H] and db: dev float[V] (rows
 * and entries of words that are neither input, target nor noise are zero); J as above or NULL.
 * Parameters and h_state are left unchanged. */
int rnnlm_nce_grad_chunk(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, const int32_t *noise, int32_t K,
                         const float *lnq, float lnZ, float *dE, float *dU, float *dWo, float *db, float *J,
                         void *stream);

/* Forward-only unnormalised scoring (Sec. 4.2: for rescoring the output is used without the explicit
 * normalisation, which is what makes it fast): score[t][s] = Wo[y[t][s]].h_t + b[y[t][s]] - lnZ for the
 * given next words only, no pass over the vocabulary; lnZ is the constant a self-normalised
 * (noise-contrastively trained) model is read against.  Starts from h_state and advances it, so calls
 * chain along a stream of text.  x, y: dev int32[T][B]; score: dev float[T][B]. */
int rnnlm_forward_score(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float lnZ, float *score,
                        void *stream);

/* rnnlm_forward_score for a shortlist of C candidate next words per position (Sec. 5.4 predicts the next
 * word from a shortlist of candidates supplied by a pruned n-gram and ranks them by the network's output):
 * score[t][s][c] = Wo[cand[t][s][c]].h_t + b[cand[t][s][c]] - lnZ (compressed architecture: the tied matrix
 * applied to the layer above the state), unnormalised, no pass over the vocabulary.  Starts from h_state and
 * advances it.  x: dev int32[T][B]; cand: dev int32[T][B][C], 1 <= C <= 65536, ids in [0,V) (checked like
 * token ids); score: dev float[T][B][C].  Works for both architectures, as does rnnlm_forward_score. */
int rnnlm_forward_score_shortlist(rnnlm_t *h, const int32_t *x, const int32_t *cand, int32_t C, int32_t T, float lnZ,
                                  float *score, void *stream);

/* ---- Compressed architecture (Sec. 5.4: word prediction under a memory limit) ---------------------------
 * Sec. 5.4 shrinks the network by inserting layers of 512 units below and above the hidden state, tying the
 * input-side and output-side word matrices as each other's transpose, and quantising all weights, trained
 * end to end.  It gives no formulas; the readings taken (cfg.P > 0 selects this model):
 *     x_t = E[w_t] (P values),  h_t = sigmoid(A x_t + U h_{t-1}),  p_t = C h_t,  z_t = E p_t + b
 * - the inserted layers are linear and have no bias (a low-rank factorisation of the two word-sized
 * matrices); E[V][P] is both the table of input rows and the output matrix; b stays a parameter.
 * rnnlm_forward_logprob, rnnlm_train_chunk, rnnlm_perplexity, rnnlm_stream_chunk and the state calls work on
 * this model unchanged (the tied matrix receives the sum of its input-side and output-side gradients; the
 * output-side part is applied first); rnnlm_grad_chunk_compressed exports its gradients.  The
 * noise-contrastive and rmsprop calls and rnnlm_grad_chunk return RNNLM_ERR_ARG; the two scoring calls work. */

/* rnnlm_grad_chunk for the compressed architecture: gradients of the window's mean negative
 * log-likelihood into dE: dev float[V][P] (both roles of the tied matrix added), dA: dev float[H][P],
 * dU: dev float[H][H], dC: dev float[P][H], db: dev float[V] (all 16-byte aligned); logp: dev float[T][B] or
 * NULL.  Parameters and h_state are left unchanged.  Requires cfg.P > 0. */
int rnnlm_grad_chunk_compressed(rnnlm_t *h, const int32_t *x, const int32_t *y, int32_t T, float *dE, float *dA,
                                float *dU, float *dC, float *db, float *logp, void *stream);

/* 8-bit weights of the compressed architecture (Sec. 5.4 quantises all the weights; the scheme is a
 * reading): symmetric, linear, one scale per matrix row, scale = max|row| / 127 (1 for an all-zero row),
 * code = round-half-to-even(w / scale) in [-127, 127], both computed in fp32.  Caller-owned device
 * arrays: codes int8 [rows][cols] of the matrix, scales float [rows]. */
typedef struct {
  int8_t *qE; float *sE; /* dev [V][P], [V] */
  int8_t *qA; float *sA; /* dev [H][P], [H] */
  int8_t *qU; float *sU; /* dev [H][H], [H] */
  int8_t *qC; float *sC; /* dev [P][H], [P] */
} rnnlm_quantized;

/* Quantises E, A, U and C from the fp32 masters into q and makes the model RUN on the quantised values
 * w' = code * scale: the compute copies every forward pass reads are rebuilt from them (the masters and b
 * are not touched, so rnnlm_sync_compute_copies returns to the unquantised model).  Training calls after
 * this update the masters as usual and refresh the copies of what they touch.  Requires cfg.P > 0. */
int rnnlm_quantize_weights(rnnlm_t *h, const rnnlm_quantized *q, void *stream);

/* Perplexity (Sec. 1, Sec. 4.2: normalised output) of tok: dev int32[N]: h_state is reset to zero,
 * the array is split into B streams as in rnnlm_stream_chunk and every full window of T positions
 * is scored; *ppl (HOST) = exp(-sum logp / scored), *scored (HOST, may be NULL) = windows*B*T.
 * Waits for the stream; reports RNNLM_ERR_TOKEN_RANGE / RNNLM_ERR_NONFINITE. */
int rnnlm_perplexity(rnnlm_t *h, const int32_t *tok, int64_t N, int32_t T, double *ppl, int64_t *scored,
                     void *stream);

/* h_state <- 0. */
int rnnlm_reset_state(rnnlm_t *h, void *stream);

/* Rebuilds the compute copies of U and Wo (compressed architecture: of E, A, U and C) from the fp32
 * masters (after the caller overwrote the masters, e.g. when loading a checkpoint). */
int rnnlm_sync_compute_copies(rnnlm_t *h, void *stream);

/* Waits for the stream and returns RNNLM_ERR_TOKEN_RANGE if any call since the last check saw an
 * out-of-range token id, RNNLM_ERR_NONFINITE / RNNLM_ERR_TIMEOUT likewise (the flags are cleared),
 * RNNLM_ERR_HIP on a device error, else RNNLM_OK. */
int rnnlm_check(rnnlm_t *h, void *stream);

/* Integer intermediates of the embedding-gradient step for the window x: dev int32[T][B]:
 * perm: dev int32[B*T] = positions m ordered by (x[m], m) (stable sort by id); seg_start: dev
 * int32[B*T+1] = start of each run of equal ids in that order, followed by B*T; nseg: dev int32 =
 * number of runs.  Integer-exact. */
int rnnlm_sort_segments(rnnlm_t *h, const int32_t *x, int32_t T, int32_t *perm, int32_t *seg_start, int32_t *nseg,
                        void *stream);

/* rnnlm_sort_segments for callers that cannot allocate device memory and hold no handle with a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the
 * padded id list they need in a static device array of the library instead of the caller's workspace.  The
 * call allocates and frees nothing (no handle, no workspace; the static array, about 0.5 MB per GPU, exists
 * from library load to process end) and runs on the CURRENT device, which must be the stream's.
 * x: dev int32[T][B]; V: ids must lie in [0, V) (others are clamped, and *range_flag, dev int32 or NULL, is set
 * to 1, else 0); perm: dev int32[B*T]; seg_start: dev int32[B*T+1]; nseg: dev int32.  Limit: T * round_up(B, 32),
 * rounded up to a multiple of 256, must not exceed 65536 positions, else RNNLM_ERR_ARG.  All calls on one GPU
 * share the one array: calls that overlap in time on the same GPU (different streams or threads) race. */
int rnnlm_sort_segments_static(const int32_t *x, int32_t T, int32_t B, int32_t V, int32_t *perm, int32_t *seg_start,
                               int32_t *nseg, int32_t *range_flag, void *stream);

/* Number of polls a grid-wide barrier of the persistent recurrent kernels waits before it gives up,
 * raises the flag that rnnlm_check reports as RNNLM_ERR_TIMEOUT and lets the kernel run to its end
 * (default 2^18, about a second).  For tests of that error path: polls = 1 makes waits expire at once. */
int rnnlm_set_barrier_spin_limit(rnnlm_t *h, uint32_t polls);

/* How the workgroups of a persistent recurrent kernel hand the state h_t (backward: the gradient dA_t) to one
 * another between the steps of a window (Sec. 4.2: the state-to-state work of all streams is done together).
 * AUTO (default): the XCD-local exchange when the placement probe at init allows it and there are at most 8
 * blocks of 32 streams, else the chip-wide one.  CHIP_WIDE: always agent-scope accesses and one counter for the
 * whole grid.  XCD_LOCAL: like AUTO, but RNNLM_ERR_ARG when the XCD-local exchange is not available for this
 * handle.  Both exchanges compute the same values in the same order: results are bitwise equal (tested).
 * The widest recurrent shape (bf16, H padded to 4096, 256 streams) runs as one launch that keeps the
 * state-to-state matrix in the register files of all compute units; it needs the same placement as the XCD-local
 * exchange, and CHIP_WIDE selects one launch pair per step for it instead (same products, another order of
 * additions: equal to bf16 rounding of the state, not bitwise).  That one-launch kernel occupies every compute
 * unit for its duration: calls on two handles of that shape must not overlap in time on one GPU (their waits
 * would expire: RNNLM_ERR_TIMEOUT).  No effect on other shapes that run one launch per step. */
typedef enum { RNNLM_EXCHANGE_AUTO = 0, RNNLM_EXCHANGE_CHIP_WIDE = 1, RNNLM_EXCHANGE_XCD_LOCAL = 2 } rnnlm_exchange;
int rnnlm_set_recurrent_exchange(rnnlm_t *h, int32_t mode);

/* Measures what this machine sustains, for reports next to the published peaks (HOST outputs): a register-
 * resident bf16 MFMA loop with hash-random operands and with constant operands (TFLOP/s; the two differ
 * because power management lowers the clock when operand bits toggle), and a plain device copy inside
 * the workspace (GB/s, read + write).  Uses the logits area of the workspace as scratch; waits for
 * the stream.  Outputs are 0 when the workspace is too small for a test. */
int rnnlm_measure_peaks(rnnlm_t *h, double *mfma_bf16_random_tflops, double *mfma_bf16_constant_tflops,
                        double *copy_gbs, void *stream);

/* Stage timing with HIP events on the call's stream (for benchmarks; off by default).  Stages of a
 * window, in the order of the kernel sequence: */
typedef enum {
  RNNLM_STAGE_PREP = 0,         /* token check, state load, embedding gather */
  RNNLM_STAGE_RNN_FWD = 1,      /* T recurrent forward steps */
  RNNLM_STAGE_OUT_FWD = 2,      /* output-layer forward contraction (+ fused softmax statistics) */
  RNNLM_STAGE_STATS = 3,        /* statistics merge, log-probabilities, their sum */
  RNNLM_STAGE_SOFTMAX_GRAD = 4, /* fused softmax gradient + bias update */
  RNNLM_STAGE_OUT_BWD_H = 5,    /* gradient w.r.t. the hidden states (contraction over the vocabulary, split-K) */
  RNNLM_STAGE_RNN_BWD = 6,      /* T recurrent backward steps */
  RNNLM_STAGE_OUT_BWD_W = 7,    /* output weight gradient contraction + SGD */
  RNNLM_STAGE_REC_W = 8,        /* recurrent weight gradient contraction + SGD */
  RNNLM_STAGE_EMB = 9,          /* sort/segments + segmented embedding update */
  RNNLM_STAGE_REDUCE = 10,      /* fixed-order sum of the split-K partials of stage 5 */
  /* noise-contrastive calls: stages 2-5 and 7 are replaced by */
  RNNLM_STAGE_NCE_SCORE = 11,   /* noise-row gather, score contraction, target scores */
  RNNLM_STAGE_NCE_GRAD = 12,    /* elementwise pass: coefficients, losses, bias-gradient column sums */
  RNNLM_STAGE_NCE_BWD_H = 13,   /* gradient w.r.t. the hidden states (contraction over the noise words + targets) */
  RNNLM_STAGE_NCE_BWD_W = 14,   /* noise-row weight gradient contraction */
  RNNLM_STAGE_NCE_UPDATE = 15,  /* sort/segments of the touched words + row and bias updates */
  RNNLM_STAGE_RMSPROP = 16,     /* rmsprop calls: statistics + scaled updates from the gradient buffers */
  RNNLM_STAGE_PROJ = 17,        /* compressed architecture: the contractions through the layers below and above
                                   the state (forward, backward and their weight updates) */
  RNNLM_STAGE_COUNT = 18
} rnnlm_stage;

/* Brackets every later execution of the stages whose bit (1u << stage) is set in stage_mask with a
 * pair of HIP events (at most 16384 pairs between two reads; further executions are not recorded).
 * stage_mask = 0 switches timing off. */
int rnnlm_profile_enable(rnnlm_t *h, uint32_t stage_mask);

/* Waits for the recorded events, then returns the stage's accumulated duration in milliseconds and
 * number of executions since the last read of that stage (HOST pointers), and clears them. */
int rnnlm_profile_read(rnnlm_t *h, int32_t stage, double *total_ms, int64_t *executions);

/* Static description of a status code. */
const char *rnnlm_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* RNNLM_H */
