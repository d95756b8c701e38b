"""ctypes front end of the fp64 CPU oracle (oracle/rnnlm_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of the benchmark.  It shares nothing with the HIP path.
All arrays are numpy, float64 / int32, C-contiguous, row-major:
E[V][H], U[H][H] (a = E[w] + U h), Wo[V][H], b[V], h[B][H], x/y[T][B].
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass

import numpy as np

from .build import build

_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_stream_chunk.restype = C.c_long
        _lib.oracle_forward_logprob.restype = C.c_int
        _lib.oracle_grad_chunk.restype = C.c_int
        _lib.oracle_train_chunk.restype = C.c_int
        _lib.oracle_perplexity.restype = C.c_int
        _lib.oracle_nce_grad_chunk.restype = C.c_int
        _lib.oracle_nce_train_chunk.restype = C.c_int
        _lib.oracle_forward_score.restype = C.c_int
        _lib.oracle_train_chunk_rmsprop.restype = C.c_int
        _lib.oracle_nce_train_chunk_rmsprop.restype = C.c_int
        _lib.oracle_sort_segments.restype = C.c_int
        _lib.oracle_num_threads.restype = C.c_int
    return _lib


def _d(a):
    if a is None:
        return C.POINTER(C.c_double)()
    assert a.dtype == np.float64 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_double))


def _i(a):
    if a is None:
        return C.POINTER(C.c_int32)()
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def _check(rc):
    if rc != 0:
        raise ValueError({-1: "oracle: bad argument", -2: "oracle: token id out of range",
                          -3: "oracle: out of memory"}.get(rc, f"oracle: error {rc}"))


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def stream_chunk(tok: np.ndarray, B: int, T: int, k: int):
    """(x[T][B], y[T][B]) of window k under the data-offset scheme (Sec. 4.2)."""
    x = np.empty((T, B), np.int32)
    y = np.empty((T, B), np.int32)
    n = lib().oracle_stream_chunk(_i(tok), C.c_long(tok.size), B, T, C.c_long(k), _i(x), _i(y))
    if n < 0:
        raise ValueError("oracle: bad stream_chunk arguments")
    return x, y


def num_chunks(N: int, B: int, T: int) -> int:
    return ((N - 1) // B) // T


@dataclass
class Model:
    E: np.ndarray
    U: np.ndarray
    Wo: np.ndarray
    b: np.ndarray
    h: np.ndarray

    @classmethod
    def from_weights(cls, E, U, Wo, b, B):
        E = np.ascontiguousarray(E, dtype=np.float64).copy()
        return cls(E, np.ascontiguousarray(U, np.float64).copy(), np.ascontiguousarray(Wo, np.float64).copy(),
                   np.ascontiguousarray(b, np.float64).copy(), np.zeros((B, E.shape[1]), np.float64))

    @property
    def V(self):
        return self.E.shape[0]

    @property
    def H(self):
        return self.E.shape[1]

    @property
    def B(self):
        return self.h.shape[0]

    def copy(self):
        return Model(self.E.copy(), self.U.copy(), self.Wo.copy(), self.b.copy(), self.h.copy())


def forward_logprob(m: Model, x, y, want_states=False, want_probs=False):
    """logp[T][B]; advances m.h. Optionally also Hs[T][B][H] and P[T][B][V]."""
    T = x.shape[0]
    logp = np.empty((T, m.B), np.float64)
    Hs = np.empty((T, m.B, m.H), np.float64) if want_states else None
    P = np.empty((T, m.B, m.V), np.float64) if want_probs else None
    _check(lib().oracle_forward_logprob(m.V, m.H, m.B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _d(m.h),
                                        _i(np.ascontiguousarray(x, np.int32)), _i(np.ascontiguousarray(y, np.int32)),
                                        _d(logp), _d(Hs), _d(P)))
    out = [logp]
    if want_states:
        out.append(Hs)
    if want_probs:
        out.append(P)
    return out[0] if len(out) == 1 else tuple(out)


def grad_chunk(m: Model, x, y, debug=False):
    """Gradients of the window's MEAN negative log-likelihood at m's parameters.

    Returns dict(logp, gE, gU, gWo, gb, h_next[, Hs, dZ, dHs, dA]); m is not modified.
    """
    T = x.shape[0]
    V, H, B = m.V, m.H, m.B
    r = dict(logp=np.empty((T, B)), gE=np.empty((V, H)), gU=np.empty((H, H)), gWo=np.empty((V, H)),
             gb=np.empty(V), h_next=np.empty((B, H)))
    dbg = dict(Hs=np.empty((T, B, H)), dZ=np.empty((T, B, V)), dHs=np.empty((T, B, H)), dA=np.empty((T, B, H))) \
        if debug else dict(Hs=None, dZ=None, dHs=None, dA=None)
    _check(lib().oracle_grad_chunk(V, H, B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _d(m.h),
                                   _i(np.ascontiguousarray(x, np.int32)), _i(np.ascontiguousarray(y, np.int32)),
                                   _d(r["logp"]), _d(r["gE"]), _d(r["gU"]), _d(r["gWo"]), _d(r["gb"]),
                                   _d(r["h_next"]), _d(dbg["Hs"]), _d(dbg["dZ"]), _d(dbg["dHs"]), _d(dbg["dA"])))
    if debug:
        r.update(dbg)
    return r


def train_chunk(m: Model, x, y, lr: float):
    """One SGD step on one window, in place. Returns (logp[T][B], sum_logp)."""
    T = x.shape[0]
    logp = np.empty((T, m.B), np.float64)
    s = C.c_double(0.0)
    _check(lib().oracle_train_chunk(m.V, m.H, m.B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _d(m.h),
                                    _i(np.ascontiguousarray(x, np.int32)), _i(np.ascontiguousarray(y, np.int32)),
                                    C.c_double(lr), _d(logp), C.byref(s)))
    return logp, s.value


@dataclass
class RmspropState:
    """Running means of squared gradients (Sec. 4.2 rmsprop): one value per word for E and Wo
    (rE[V], rWo[V]), one per element for U and b (rU[H][H], rb[V])."""
    rE: np.ndarray
    rU: np.ndarray
    rWo: np.ndarray
    rb: np.ndarray

    @classmethod
    def filled(cls, V, H, value):
        return cls(np.full(V, value, np.float64), np.full((H, H), value, np.float64), np.full(V, value, np.float64),
                   np.full(V, value, np.float64))

    def copy(self):
        return RmspropState(self.rE.copy(), self.rU.copy(), self.rWo.copy(), self.rb.copy())


def train_chunk_rmsprop(m: Model, st: RmspropState, x, y, lr: float, rho: float, eps: float):
    """One rmsprop-scaled SGD step on one window, in place (model and statistics).
    Returns (logp[T][B], sum_logp)."""
    T = x.shape[0]
    logp = np.empty((T, m.B), np.float64)
    s = C.c_double(0.0)
    _check(lib().oracle_train_chunk_rmsprop(m.V, m.H, m.B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _d(m.h),
                                            _i(np.ascontiguousarray(x, np.int32)),
                                            _i(np.ascontiguousarray(y, np.int32)), C.c_double(lr), C.c_double(rho),
                                            C.c_double(eps), _d(st.rE), _d(st.rU), _d(st.rWo), _d(st.rb), _d(logp),
                                            C.byref(s)))
    return logp, s.value


def nce_grad_chunk(m: Model, x, y, noise, lnq, lnZ=0.0, debug=False):
    """Gradients of the window's MEAN noise-contrastive loss (Sec. 4.2 criterion; K = len(noise) noise
    words shared by the window, noise log-probabilities lnq[V], constant normaliser lnZ).

    Returns dict(J[T][B], gE, gU, gWo, gb, h_next[, ct[T][B], dS[T][B][K], dHs, dA]); m is not modified.
    """
    T = x.shape[0]
    V, H, B = m.V, m.H, m.B
    noise = np.ascontiguousarray(noise, np.int32).reshape(-1)
    K = noise.size
    lnq = np.ascontiguousarray(lnq, np.float64)
    assert lnq.shape == (V,)
    r = dict(J=np.empty((T, B)), gE=np.empty((V, H)), gU=np.empty((H, H)), gWo=np.empty((V, H)),
             gb=np.empty(V), h_next=np.empty((B, H)))
    dbg = dict(ct=np.empty((T, B)), dS=np.empty((T, B, K)), dHs=np.empty((T, B, H)), dA=np.empty((T, B, H))) \
        if debug else dict(ct=None, dS=None, dHs=None, dA=None)
    _check(lib().oracle_nce_grad_chunk(V, H, B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _d(m.h),
                                       _i(np.ascontiguousarray(x, np.int32)), _i(np.ascontiguousarray(y, np.int32)),
                                       K, _i(noise), _d(lnq), C.c_double(lnZ), _d(r["J"]), _d(r["gE"]), _d(r["gU"]),
                                       _d(r["gWo"]), _d(r["gb"]), _d(r["h_next"]), _d(dbg["ct"]), _d(dbg["dS"]),
                                       _d(dbg["dHs"]), _d(dbg["dA"])))
    if debug:
        r.update(dbg)
    return r


def nce_train_chunk(m: Model, x, y, noise, lnq, lnZ, lr: float):
    """One SGD step on one window under the noise-contrastive criterion, in place.
    Returns (J[T][B], sum_J)."""
    T = x.shape[0]
    noise = np.ascontiguousarray(noise, np.int32).reshape(-1)
    lnq = np.ascontiguousarray(lnq, np.float64)
    assert lnq.shape == (m.V,)
    J = np.empty((T, m.B), np.float64)
    s = C.c_double(0.0)
    _check(lib().oracle_nce_train_chunk(m.V, m.H, m.B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _d(m.h),
                                        _i(np.ascontiguousarray(x, np.int32)), _i(np.ascontiguousarray(y, np.int32)),
                                        noise.size, _i(noise), _d(lnq), C.c_double(lnZ), C.c_double(lr), _d(J),
                                        C.byref(s)))
    return J, s.value


def nce_train_chunk_rmsprop(m: Model, st: RmspropState, x, y, noise, lnq, lnZ, lr: float, rho: float, eps: float):
    """One rmsprop-scaled step on one window under the noise-contrastive criterion (the paper's own
    combination, Sec. 4.2), in place.  Returns (J[T][B], sum_J)."""
    T = x.shape[0]
    noise = np.ascontiguousarray(noise, np.int32).reshape(-1)
    lnq = np.ascontiguousarray(lnq, np.float64)
    assert lnq.shape == (m.V,)
    J = np.empty((T, m.B), np.float64)
    s = C.c_double(0.0)
    _check(lib().oracle_nce_train_chunk_rmsprop(m.V, m.H, m.B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _d(m.h),
                                                _i(np.ascontiguousarray(x, np.int32)),
                                                _i(np.ascontiguousarray(y, np.int32)), noise.size, _i(noise),
                                                _d(lnq), C.c_double(lnZ), C.c_double(lr), C.c_double(rho),
                                                C.c_double(eps), _d(st.rE), _d(st.rU), _d(st.rWo), _d(st.rb), _d(J),
                                                C.byref(s)))
    return J, s.value


def forward_score(m: Model, x, y, lnZ=0.0):
    """Unnormalised scores z[y] - lnZ of the given next words, score[T][B]; advances m.h (Sec. 4.2: the
    output as used for rescoring, without the explicit normalisation)."""
    T = x.shape[0]
    score = np.empty((T, m.B), np.float64)
    _check(lib().oracle_forward_score(m.V, m.H, m.B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _d(m.h),
                                      _i(np.ascontiguousarray(x, np.int32)), _i(np.ascontiguousarray(y, np.int32)),
                                      C.c_double(lnZ), _d(score)))
    return score


def forward_score_shortlist(m: Model, x, cand, lnZ=0.0):
    """Unnormalised scores of a shortlist of candidate next words, score[T][B][C] for cand[T][B][C] (Sec. 5.4
    ranks the candidates a pruned n-gram proposes); one forward_score pass per candidate column from the same
    starting state; advances m.h."""
    T, B, Cn = cand.shape
    score = np.empty((T, B, Cn), np.float64)
    h0 = m.h.copy()
    for c in range(Cn):
        m.h = h0.copy()
        score[:, :, c] = forward_score(m, x, np.ascontiguousarray(cand[:, :, c]), lnZ)
    return score


def perplexity(m: Model, tok: np.ndarray, T: int):
    """(PPL, scored) over all full windows of T positions, B streams from a zero state."""
    ppl = C.c_double(0.0)
    scored = C.c_long(0)
    tok = np.ascontiguousarray(tok, np.int32)
    _check(lib().oracle_perplexity(m.V, m.H, m.B, T, _d(m.E), _d(m.U), _d(m.Wo), _d(m.b), _i(tok),
                                   C.c_long(tok.size), C.byref(ppl), C.byref(scored)))
    return ppl.value, scored.value


def sort_segments(x: np.ndarray):
    """Stable order of window positions by id and run starts: (perm[M], seg_start[nseg+1])."""
    xf = np.ascontiguousarray(x, np.int32).reshape(-1)
    M = xf.size
    perm = np.empty(M, np.int32)
    seg = np.empty(M + 1, np.int32)
    n = lib().oracle_sort_segments(_i(xf), M, _i(perm), _i(seg))
    if n < 0:
        raise ValueError("oracle: bad sort_segments arguments")
    return perm, seg[:n + 1].copy()
