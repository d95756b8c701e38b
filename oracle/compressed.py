"""fp64 numpy oracle of the compressed architecture of Sec. 5.4 (word prediction under a memory limit).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the cpu_baseline leg of the
benchmark.  It shares nothing with the HIP path.

Sec. 5.4 compresses the recurrent network by (1) inserting layers of 512 units below and above the hidden
state, (2) tying the input-side and output-side word matrices as each other's transpose, (3) quantising
all weights, and trains the result end to end.  The section gives no formulas; the readings taken here
(stated again where the HIP path documents them):

  * the inserted layers are LINEAR bottlenecks without bias (a low-rank factorisation of the two
    word-sized matrices; the paper inserts them to shrink the model, not to add depth):
        x_t = E[w_t]                    (P values, P = 512 in the paper)
        a_t = A x_t + U h_{t-1},  h_t = sigmoid(a_t)          (A: H x P)
        p_t = C h_t                                            (C: P x H)
        z_t = E p_t + b,  log P(w | history) = z_t[w] - log sum_v exp(z_t[v])
    i.e. the V x P matrix E is both the table of input rows and the output matrix (tying); the output
    bias b stays a parameter of its own;
  * training is the same window step as for the plain architecture: mean negative log-likelihood of
    the B*T tokens, back-propagation through time to the window start, one plain SGD step; the tied
    matrix receives the sum of its input-side and output-side gradients;
  * quantisation is symmetric, linear, 8 bits, one scale per matrix row: scale = max|row| / 127 (1 for
    an all-zero row), code = round-half-to-even(w / scale) in [-127, 127], both computed in fp32 (the
    codes are integers decided by floating point, so the precision is part of the definition); the
    quantised model uses w' = code * scale for E, A, U and C and keeps b as it is.

Layouts: row-major numpy arrays; token windows are time-major x[T][B], y[T][B].
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class CompressedModel:
    E: np.ndarray  # [V][P]  input rows and output matrix (tied)
    A: np.ndarray  # [H][P]  layer below the state -> state
    U: np.ndarray  # [H][H]  state -> state
    C: np.ndarray  # [P][H]  state -> layer above the state
    b: np.ndarray  # [V]     output bias
    h: np.ndarray  # [B][H]  carried state

    def copy(self) -> "CompressedModel":
        return CompressedModel(*(np.array(a, dtype=np.float64, copy=True) for a in
                                 (self.E, self.A, self.U, self.C, self.b, self.h)))


def _check(m: CompressedModel, x: np.ndarray, y: np.ndarray):
    V = m.E.shape[0]
    if x.shape != y.shape or x.ndim != 2 or x.shape[1] != m.h.shape[0]:
        raise ValueError("oracle: bad argument")
    if x.min() < 0 or x.max() >= V or y.min() < 0 or y.max() >= V:
        raise ValueError("oracle: token id out of range")


def _forward(m: CompressedModel, x: np.ndarray, y: np.ndarray):
    """Hidden states Hs[T][B][H], bottleneck outputs Ps[T][B][P], distributions Pr[T][B][V], logp[T][B]."""
    T, B = x.shape
    H, P = m.A.shape
    V = m.E.shape[0]
    Hs = np.zeros((T, B, H))
    Ps = np.zeros((T, B, P))
    Pr = np.zeros((T, B, V))
    logp = np.zeros((T, B))
    h = m.h
    for t in range(T):
        a = m.E[x[t]] @ m.A.T + h @ m.U.T
        h = 1.0 / (1.0 + np.exp(-a))
        p = h @ m.C.T
        z = p @ m.E.T + m.b
        mx = z.max(axis=1, keepdims=True)
        lse = mx[:, 0] + np.log(np.exp(z - mx).sum(axis=1))
        Hs[t], Ps[t] = h, p
        Pr[t] = np.exp(z - lse[:, None])
        logp[t] = z[np.arange(B), y[t]] - lse
    return Hs, Ps, Pr, logp


def forward_logprob(m: CompressedModel, x: np.ndarray, y: np.ndarray) -> np.ndarray:
    """log P(y | history) for one window; advances m.h."""
    _check(m, x, y)
    Hs, _, _, logp = _forward(m, x, y)
    m.h = Hs[-1].copy()
    return logp


def forward_score_shortlist(m: CompressedModel, x: np.ndarray, cand: np.ndarray, lnZ: float = 0.0) -> np.ndarray:
    """Unnormalised scores E[c].p_t + b[c] - lnZ of the candidate words cand[T][B][C] (Sec. 5.4 ranks a
    shortlist of candidates); advances m.h.  forward_score(m, x, y) is the case of one candidate."""
    T, B = x.shape
    if cand.shape[:2] != (T, B) or cand.min() < 0 or cand.max() >= m.E.shape[0]:
        raise ValueError("oracle: bad argument")
    score = np.zeros(cand.shape)
    h = m.h
    for t in range(T):
        h = 1.0 / (1.0 + np.exp(-(m.E[x[t]] @ m.A.T + h @ m.U.T)))
        p = h @ m.C.T
        for s in range(B):
            score[t, s] = m.E[cand[t, s]] @ p[s] + m.b[cand[t, s]] - lnZ
    m.h = h.copy()
    return score


def forward_score(m: CompressedModel, x: np.ndarray, y: np.ndarray, lnZ: float = 0.0) -> np.ndarray:
    return forward_score_shortlist(m, x, y[:, :, None], lnZ)[:, :, 0]


def grad_chunk(m: CompressedModel, x: np.ndarray, y: np.ndarray):
    """Gradient of the window's mean negative log-likelihood with respect to E, A, U, C, b at the given
    parameters; the carried state is a constant (the chain stops at the window start).  m is not modified.
    Returns a dict with gE, gA, gU, gC, gb, logp and h_out (the state after the window)."""
    _check(m, x, y)
    T, B = x.shape
    H, P = m.A.shape
    Hs, Ps, Pr, logp = _forward(m, x, y)
    gE = np.zeros_like(m.E)
    gA = np.zeros_like(m.A)
    gU = np.zeros_like(m.U)
    gC = np.zeros_like(m.C)
    gb = np.zeros_like(m.b)
    da_next = np.zeros((B, H))
    for t in range(T - 1, -1, -1):
        dz = Pr[t].copy()
        dz[np.arange(B), y[t]] -= 1.0
        dz /= float(B * T)
        gb += dz.sum(axis=0)
        gE += dz.T @ Ps[t]                      # output role of the tied matrix: z = E p + b
        dp = dz @ m.E
        gC += dp.T @ Hs[t]                      # p = C h
        dh = dp @ m.C + da_next @ m.U           # through the layer above and through the next step
        da = dh * Hs[t] * (1.0 - Hs[t])
        hprev = Hs[t - 1] if t > 0 else m.h
        gU += da.T @ hprev
        xt = m.E[x[t]]
        gA += da.T @ xt                         # a = A x + U h
        dx = da @ m.A
        np.add.at(gE, x[t], dx)                 # input role of the tied matrix: x = E[w]
        da_next = da
    return {"gE": gE, "gA": gA, "gU": gU, "gC": gC, "gb": gb, "logp": logp, "h_out": Hs[-1].copy()}


def train_chunk(m: CompressedModel, x: np.ndarray, y: np.ndarray, lr: float) -> np.ndarray:
    """One plain SGD step on one window (in place); returns logp[T][B] of the pre-update parameters."""
    g = grad_chunk(m, x, y)
    m.E -= lr * g["gE"]
    m.A -= lr * g["gA"]
    m.U -= lr * g["gU"]
    m.C -= lr * g["gC"]
    m.b -= lr * g["gb"]
    m.h = g["h_out"]
    return g["logp"]


def perplexity(m: CompressedModel, tok: np.ndarray, T: int):
    """exp(-mean log P) over the full windows of the corpus under the data-offset scheme, from a zero state."""
    B = m.h.shape[0]
    L = (len(tok) - 1) // B
    n = L // T
    mm = m.copy()
    mm.h = np.zeros_like(m.h)
    total = 0.0
    for k in range(n):
        idx = (np.arange(B)[None, :] * L + k * T + np.arange(T)[:, None])
        total += forward_logprob(mm, tok[idx].astype(np.int64), tok[idx + 1].astype(np.int64)).sum()
    return float(np.exp(-total / (n * B * T))), n * B * T


def quantize_rows(W: np.ndarray):
    """Symmetric 8-bit row-wise quantisation, decided in fp32: returns (codes int8 [R][C], scale float32 [R])."""
    W32 = np.asarray(W, dtype=np.float32)
    amax = np.abs(W32).max(axis=1)
    scale = np.where(amax > 0, amax / np.float32(127.0), np.float32(1.0)).astype(np.float32)
    q = np.rint(W32 / scale[:, None])           # fp32 division, round half to even
    codes = np.clip(q, -127, 127).astype(np.int8)
    return codes, scale


def dequantize_rows(codes: np.ndarray, scale: np.ndarray) -> np.ndarray:
    return codes.astype(np.float64) * scale.astype(np.float64)[:, None]


def quantized(m: CompressedModel) -> CompressedModel:
    """The model whose four matrices are replaced by their 8-bit row-wise quantised values (b, h unchanged)."""
    q = m.copy()
    for name in ("E", "A", "U", "C"):
        setattr(q, name, dequantize_rows(*quantize_rows(getattr(m, name))))
    return q
