"""Thin ctypes binding of include/rnnlm.h: argument marshalling only.

Every step of the path runs in the HIP library; PyTorch only owns device memory and
streams.  Function names mirror the C ABI.  Importing this module needs the built
librnnlm_hip.so next to it (see build.py) and raises if it is missing: there is no
fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librnnlm_hip.so")

RNNLM_FP32 = 0
RNNLM_BF16_FP32MASTER = 1
RNNLM_EXCHANGE_AUTO, RNNLM_EXCHANGE_CHIP_WIDE, RNNLM_EXCHANGE_XCD_LOCAL = 0, 1, 2

SYMBOLS = [
    "rnnlm_workspace_bytes", "rnnlm_init", "rnnlm_free", "rnnlm_stream_chunk", "rnnlm_forward_logprob",
    "rnnlm_train_chunk", "rnnlm_grad_chunk", "rnnlm_perplexity", "rnnlm_reset_state",
    "rnnlm_sync_compute_copies", "rnnlm_check", "rnnlm_sort_segments", "rnnlm_status_string",
    "rnnlm_profile_enable", "rnnlm_profile_read", "rnnlm_set_barrier_spin_limit", "rnnlm_measure_peaks",
    "rnnlm_nce_train_chunk", "rnnlm_nce_grad_chunk", "rnnlm_forward_score",
    "rnnlm_train_chunk_rmsprop", "rnnlm_nce_train_chunk_rmsprop",
    "rnnlm_grad_chunk_compressed", "rnnlm_quantize_weights", "rnnlm_forward_score_shortlist",
    "rnnlm_set_recurrent_exchange", "rnnlm_sort_segments_static",
]

STAGES = ["prep", "rnn_fwd", "out_fwd", "stats", "softmax_grad", "out_bwd_h", "rnn_bwd", "out_bwd_w", "rec_w", "emb", "reduce",
          "nce_score", "nce_grad", "nce_bwd_h", "nce_bwd_w", "nce_update", "rmsprop", "proj"]


class rnnlm_config(C.Structure):
    _fields_ = [("V", C.c_int32), ("H", C.c_int32), ("B", C.c_int32), ("T_max", C.c_int32),
                ("precision", C.c_int32), ("device", C.c_int32), ("K_max", C.c_int32), ("rmsprop", C.c_int32),
                ("P", C.c_int32)]


class rnnlm_rmsprop_state(C.Structure):
    _fields_ = [("rE", C.c_void_p), ("rU", C.c_void_p), ("rWo", C.c_void_p), ("rb", C.c_void_p)]


class rnnlm_buffers(C.Structure):
    _fields_ = [("E", C.c_void_p), ("U", C.c_void_p), ("Wo", C.c_void_p), ("b", C.c_void_p),
                ("h_state", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("A", C.c_void_p), ("C", C.c_void_p)]


class rnnlm_quantized(C.Structure):
    _fields_ = [("qE", C.c_void_p), ("sE", C.c_void_p), ("qA", C.c_void_p), ("sA", C.c_void_p),
                ("qU", C.c_void_p), ("sU", C.c_void_p), ("qC", C.c_void_p), ("sC", C.c_void_p)]


class RnnlmError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {status_string(status)} ({status})")
        self.status = status


_lib = None


def load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_1502_00512_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.rnnlm_workspace_bytes.restype = C.c_size_t
    lib.rnnlm_workspace_bytes.argtypes = [C.POINTER(rnnlm_config)]
    lib.rnnlm_init.argtypes = [C.POINTER(rnnlm_config), C.POINTER(rnnlm_buffers), C.POINTER(vp)]
    lib.rnnlm_free.argtypes = [vp]
    lib.rnnlm_free.restype = None
    lib.rnnlm_stream_chunk.argtypes = [vp, vp, i64, i64, i32, vp, vp, vp]
    lib.rnnlm_forward_logprob.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.rnnlm_train_chunk.argtypes = [vp, vp, vp, i32, C.c_float, vp, vp, vp]
    lib.rnnlm_grad_chunk.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp]
    lib.rnnlm_perplexity.argtypes = [vp, vp, i64, i32, C.POINTER(C.c_double), C.POINTER(i64), vp]
    lib.rnnlm_reset_state.argtypes = [vp, vp]
    lib.rnnlm_sync_compute_copies.argtypes = [vp, vp]
    lib.rnnlm_check.argtypes = [vp, vp]
    lib.rnnlm_sort_segments.argtypes = [vp, vp, i32, vp, vp, vp, vp]
    lib.rnnlm_set_barrier_spin_limit.argtypes = [vp, C.c_uint32]
    lib.rnnlm_set_recurrent_exchange.argtypes = [vp, i32]
    lib.rnnlm_sort_segments_static.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp]
    lib.rnnlm_measure_peaks.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), vp]
    f32 = C.c_float
    lib.rnnlm_nce_train_chunk.argtypes = [vp, vp, vp, i32, vp, i32, vp, f32, f32, vp, vp, vp]
    lib.rnnlm_nce_grad_chunk.argtypes = [vp, vp, vp, i32, vp, i32, vp, f32, vp, vp, vp, vp, vp, vp]
    lib.rnnlm_train_chunk_rmsprop.argtypes = [vp, vp, vp, i32, f32, f32, f32, C.POINTER(rnnlm_rmsprop_state), vp, vp, vp]
    lib.rnnlm_nce_train_chunk_rmsprop.argtypes = [vp, vp, vp, i32, vp, i32, vp, f32, f32, f32, f32,
                                                  C.POINTER(rnnlm_rmsprop_state), vp, vp, vp]
    lib.rnnlm_forward_score.argtypes = [vp, vp, vp, i32, f32, vp, vp]
    lib.rnnlm_forward_score_shortlist.argtypes = [vp, vp, vp, i32, i32, f32, vp, vp]
    lib.rnnlm_grad_chunk_compressed.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, vp]
    lib.rnnlm_quantize_weights.argtypes = [vp, C.POINTER(rnnlm_quantized), vp]
    lib.rnnlm_profile_enable.argtypes = [vp, C.c_uint32]
    lib.rnnlm_profile_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.rnnlm_status_string.argtypes = [C.c_int]
    lib.rnnlm_status_string.restype = C.c_char_p
    for name in SYMBOLS:
        if name not in ("rnnlm_workspace_bytes", "rnnlm_free", "rnnlm_status_string"):
            getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().rnnlm_status_string(int(status)).decode()


def _ok(rc: int, what: str):
    if rc != 0:
        raise RnnlmError(rc, what)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def rnnlm_workspace_bytes(V, H, B, T_max, precision, device=0, K_max=0, rmsprop=0, P=0) -> int:
    cfg = rnnlm_config(V, H, B, T_max, precision, device, K_max, rmsprop, P)
    return int(load().rnnlm_workspace_bytes(C.byref(cfg)))


def rnnlm_sort_segments_static(x, V: int, perm, seg_start, nseg, range_flag=None, stream=None):
    """The handle-free call: x int32[T][B] and the three outputs are device tensors the caller allocated."""
    _ok(load().rnnlm_sort_segments_static(_ptr(x), x.shape[0], x.shape[1], V, _ptr(perm), _ptr(seg_start), _ptr(nseg),
                                          _ptr(range_flag), _stream(stream)), "rnnlm_sort_segments_static")


class Rnnlm:
    """Owns the torch tensors (masters, state, workspace) and the library handle.

    Plain architecture: E[V][H], U, Wo[V][H], b.  Compressed architecture (Sec. 5.4): pass Wo=None and
    A[H][P], C[P][H]; then E is the tied word matrix [V][P]."""

    def __init__(self, E, U, Wo, b, B: int, T_max: int, precision: int, device: int = 0, K_max: int = 0,
                 rmsprop: bool = False, r_init: float = 1.0, A=None, C_=None):
        import torch
        self.lib = load()
        dev = torch.device("cuda", device)
        f = lambda a: torch.as_tensor(a, dtype=torch.float32).contiguous().to(dev).clone()
        self.E, self.U, self.b = f(E), f(U), f(b)
        self.H = self.U.shape[0]
        self.V = self.E.shape[0]
        self.P = 0
        self.Wo = self.A = self.C = None
        if A is not None:
            assert Wo is None and C_ is not None
            self.A, self.C = f(A), f(C_)
            self.P = self.E.shape[1]
            assert self.A.shape == (self.H, self.P) and self.C.shape == (self.P, self.H)
        else:
            self.Wo = f(Wo)
            assert self.E.shape == (self.V, self.H) and self.Wo.shape == (self.V, self.H)
        self.B, self.T_max, self.precision, self.device = int(B), int(T_max), int(precision), dev
        assert self.U.shape == (self.H, self.H) and self.b.shape == (self.V,)
        self.h_state = torch.zeros(self.B, self.H, dtype=torch.float32, device=dev)
        self.K_max = int(K_max)
        cfg = rnnlm_config(self.V, self.H, self.B, self.T_max, self.precision, device, self.K_max, int(bool(rmsprop)),
                           self.P)
        if rmsprop:  # the caller-owned statistics, all starting at r_init
            fill = lambda *shp: torch.full(shp, float(r_init), dtype=torch.float32, device=dev)
            self.rE, self.rU, self.rWo, self.rb = fill(self.V), fill(self.H, self.H), fill(self.V), fill(self.V)
            self.rms_state = rnnlm_rmsprop_state(self.rE.data_ptr(), self.rU.data_ptr(), self.rWo.data_ptr(),
                                                 self.rb.data_ptr())
        nbytes = int(self.lib.rnnlm_workspace_bytes(C.byref(cfg)))
        if nbytes == 0:
            raise RnnlmError(-1, "rnnlm_workspace_bytes")
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)
        opt = lambda t: None if t is None else t.data_ptr()
        buf = rnnlm_buffers(self.E.data_ptr(), self.U.data_ptr(), opt(self.Wo), self.b.data_ptr(),
                            self.h_state.data_ptr(), self.workspace.data_ptr(), nbytes, opt(self.A), opt(self.C))
        self.handle = C.c_void_p()
        torch.cuda.synchronize(dev)
        _ok(self.lib.rnnlm_init(C.byref(cfg), C.byref(buf), C.byref(self.handle)), "rnnlm_init")

    def close(self):
        if getattr(self, "handle", None):
            import torch
            torch.cuda.synchronize(self.device)
            self.lib.rnnlm_free(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the calls of the C ABI, same names ----------------------------------------------------
    def rnnlm_stream_chunk(self, tok, k: int, T: int, x=None, y=None, stream=None):
        import torch
        if x is None:
            x = torch.empty(T, self.B, dtype=torch.int32, device=self.device)
            y = torch.empty(T, self.B, dtype=torch.int32, device=self.device)
        _ok(self.lib.rnnlm_stream_chunk(self.handle, _ptr(tok), tok.numel(), k, T, _ptr(x), _ptr(y), _stream(stream)),
            "rnnlm_stream_chunk")
        return x, y

    def rnnlm_forward_logprob(self, x, y, logp=None, stream=None):
        import torch
        T = x.shape[0]
        if logp is None:
            logp = torch.empty(T, self.B, dtype=torch.float32, device=self.device)
        _ok(self.lib.rnnlm_forward_logprob(self.handle, _ptr(x), _ptr(y), T, _ptr(logp), _stream(stream)),
            "rnnlm_forward_logprob")
        return logp

    def rnnlm_train_chunk(self, x, y, lr: float, logp=None, sum_logp=None, stream=None):
        _ok(self.lib.rnnlm_train_chunk(self.handle, _ptr(x), _ptr(y), x.shape[0], lr, _ptr(logp), _ptr(sum_logp),
                                       _stream(stream)), "rnnlm_train_chunk")

    def rnnlm_grad_chunk(self, x, y, want_logp=True, stream=None):
        import torch
        z = lambda *s: torch.empty(*s, dtype=torch.float32, device=self.device)
        dE, dU, dWo, db = z(self.V, self.H), z(self.H, self.H), z(self.V, self.H), z(self.V)
        logp = z(x.shape[0], self.B) if want_logp else None
        _ok(self.lib.rnnlm_grad_chunk(self.handle, _ptr(x), _ptr(y), x.shape[0], _ptr(dE), _ptr(dU), _ptr(dWo),
                                      _ptr(db), _ptr(logp), _stream(stream)), "rnnlm_grad_chunk")
        return dict(gE=dE, gU=dU, gWo=dWo, gb=db, logp=logp)

    def rnnlm_grad_chunk_compressed(self, x, y, want_logp=True, stream=None):
        import torch
        z = lambda *s: torch.empty(*s, dtype=torch.float32, device=self.device)
        dE, dA, dU, dC, db = z(self.V, self.P), z(self.H, self.P), z(self.H, self.H), z(self.P, self.H), z(self.V)
        logp = z(x.shape[0], self.B) if want_logp else None
        _ok(self.lib.rnnlm_grad_chunk_compressed(self.handle, _ptr(x), _ptr(y), x.shape[0], _ptr(dE), _ptr(dA),
                                                 _ptr(dU), _ptr(dC), _ptr(db), _ptr(logp), _stream(stream)),
            "rnnlm_grad_chunk_compressed")
        return dict(gE=dE, gA=dA, gU=dU, gC=dC, gb=db, logp=logp)

    def rnnlm_quantize_weights(self, stream=None):
        """Returns dict name -> (codes int8 tensor, scale float tensor); the model then runs on the quantised values."""
        import torch
        out = {}
        ptrs = []
        for name, W in (("E", self.E), ("A", self.A), ("U", self.U), ("C", self.C)):
            q = torch.empty(W.shape, dtype=torch.int8, device=self.device)
            s = torch.empty(W.shape[0], dtype=torch.float32, device=self.device)
            out[name] = (q, s)
            ptrs += [q.data_ptr(), s.data_ptr()]
        qs = rnnlm_quantized(*ptrs)
        _ok(self.lib.rnnlm_quantize_weights(self.handle, C.byref(qs), _stream(stream)), "rnnlm_quantize_weights")
        return out

    def rnnlm_perplexity(self, tok, T: int, stream=None):
        ppl = C.c_double(0.0)
        scored = C.c_int64(0)
        _ok(self.lib.rnnlm_perplexity(self.handle, _ptr(tok), tok.numel(), T, C.byref(ppl), C.byref(scored),
                                      _stream(stream)), "rnnlm_perplexity")
        return ppl.value, scored.value

    def rnnlm_train_chunk_rmsprop(self, x, y, lr: float, rho: float, eps: float, logp=None, sum_logp=None,
                                  stream=None):
        state = getattr(self, "rms_state", None)
        _ok(self.lib.rnnlm_train_chunk_rmsprop(self.handle, _ptr(x), _ptr(y), x.shape[0], lr, rho, eps,
                                               C.byref(state) if state is not None else None, _ptr(logp),
                                               _ptr(sum_logp), _stream(stream)), "rnnlm_train_chunk_rmsprop")

    def rnnlm_nce_train_chunk_rmsprop(self, x, y, noise, lnq, lnZ: float, lr: float, rho: float, eps: float, J=None,
                                      sum_J=None, stream=None):
        state = getattr(self, "rms_state", None)
        _ok(self.lib.rnnlm_nce_train_chunk_rmsprop(self.handle, _ptr(x), _ptr(y), x.shape[0], _ptr(noise),
                                                   noise.numel(), _ptr(lnq), lnZ, lr, rho, eps,
                                                   C.byref(state) if state is not None else None, _ptr(J),
                                                   _ptr(sum_J), _stream(stream)), "rnnlm_nce_train_chunk_rmsprop")

    def rnnlm_forward_score(self, x, y, lnZ: float = 0.0, score=None, stream=None):
        import torch
        T = x.shape[0]
        if score is None:
            score = torch.empty(T, self.B, dtype=torch.float32, device=self.device)
        _ok(self.lib.rnnlm_forward_score(self.handle, _ptr(x), _ptr(y), T, lnZ, _ptr(score), _stream(stream)),
            "rnnlm_forward_score")
        return score

    def rnnlm_forward_score_shortlist(self, x, cand, lnZ: float = 0.0, score=None, stream=None):
        import torch
        T, C_ = x.shape[0], cand.shape[2]
        if score is None:
            score = torch.empty(T, self.B, C_, dtype=torch.float32, device=self.device)
        _ok(self.lib.rnnlm_forward_score_shortlist(self.handle, _ptr(x), _ptr(cand), C_, T, lnZ, _ptr(score),
                                                   _stream(stream)), "rnnlm_forward_score_shortlist")
        return score

    def rnnlm_nce_train_chunk(self, x, y, noise, lnq, lnZ: float, lr: float, J=None, sum_J=None, stream=None):
        _ok(self.lib.rnnlm_nce_train_chunk(self.handle, _ptr(x), _ptr(y), x.shape[0], _ptr(noise), noise.numel(),
                                           _ptr(lnq), lnZ, lr, _ptr(J), _ptr(sum_J), _stream(stream)),
            "rnnlm_nce_train_chunk")

    def rnnlm_nce_grad_chunk(self, x, y, noise, lnq, lnZ: float, want_J=True, stream=None):
        import torch
        z = lambda *s: torch.empty(*s, dtype=torch.float32, device=self.device)
        dE, dU, dWo, db = z(self.V, self.H), z(self.H, self.H), z(self.V, self.H), z(self.V)
        J = z(x.shape[0], self.B) if want_J else None
        _ok(self.lib.rnnlm_nce_grad_chunk(self.handle, _ptr(x), _ptr(y), x.shape[0], _ptr(noise), noise.numel(),
                                          _ptr(lnq), lnZ, _ptr(dE), _ptr(dU), _ptr(dWo), _ptr(db), _ptr(J),
                                          _stream(stream)), "rnnlm_nce_grad_chunk")
        return dict(gE=dE, gU=dU, gWo=dWo, gb=db, J=J)

    def rnnlm_reset_state(self, stream=None):
        _ok(self.lib.rnnlm_reset_state(self.handle, _stream(stream)), "rnnlm_reset_state")

    def rnnlm_sync_compute_copies(self, stream=None):
        _ok(self.lib.rnnlm_sync_compute_copies(self.handle, _stream(stream)), "rnnlm_sync_compute_copies")

    def rnnlm_check(self, stream=None):
        _ok(self.lib.rnnlm_check(self.handle, _stream(stream)), "rnnlm_check")

    def rnnlm_set_barrier_spin_limit(self, polls: int):
        _ok(self.lib.rnnlm_set_barrier_spin_limit(self.handle, polls), "rnnlm_set_barrier_spin_limit")

    def rnnlm_set_recurrent_exchange(self, mode: int):
        _ok(self.lib.rnnlm_set_recurrent_exchange(self.handle, mode), "rnnlm_set_recurrent_exchange")

    def rnnlm_measure_peaks(self, stream=None):
        r, c, g = C.c_double(0), C.c_double(0), C.c_double(0)
        _ok(self.lib.rnnlm_measure_peaks(self.handle, C.byref(r), C.byref(c), C.byref(g), _stream(stream)),
            "rnnlm_measure_peaks")
        return dict(mfma_bf16_random_tflops=r.value, mfma_bf16_constant_tflops=c.value, copy_gbs=g.value)

    def rnnlm_profile_enable(self, stage_mask: int):
        _ok(self.lib.rnnlm_profile_enable(self.handle, stage_mask), "rnnlm_profile_enable")

    def rnnlm_profile_read(self, stage: int):
        ms = C.c_double(0.0)
        n = C.c_int64(0)
        _ok(self.lib.rnnlm_profile_read(self.handle, stage, C.byref(ms), C.byref(n)), "rnnlm_profile_read")
        return ms.value, n.value

    def rnnlm_sort_segments(self, x, stream=None):
        import torch
        M = x.numel()
        perm = torch.empty(M, dtype=torch.int32, device=self.device)
        seg = torch.empty(M + 1, dtype=torch.int32, device=self.device)
        nseg = torch.zeros(1, dtype=torch.int32, device=self.device)
        _ok(self.lib.rnnlm_sort_segments(self.handle, _ptr(x), x.shape[0], _ptr(perm), _ptr(seg), _ptr(nseg),
                                         _stream(stream)), "rnnlm_sort_segments")
        n = int(nseg.item())
        return perm, seg[:n + 1]
