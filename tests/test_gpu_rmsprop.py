"""GPU parity of the rmsprop-scaled training step (Sec. 4.2: SGD with rmsprop, one statistic per word for
E and Wo) against the fp64 oracle, through the C ABI, on the same seeded inputs.  fp32 path: log-probs
|d| <= 2e-4*|ref| + 1e-6, parameters after several windows within 1e-4*max(1, |theta|), statistics within
1e-3 relative; bf16 path: window perplexity within 1e-2 relative while both sides train."""
import math

import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_1502_00512_amd import binding, synth

pytestmark = pytest.mark.gpu

FP32, BF16 = binding.RNNLM_FP32, binding.RNNLM_BF16_FP32MASTER


def dev(a):
    return torch.as_tensor(np.ascontiguousarray(a)).cuda()


def make(V, H, B, T, precision, seed, r0, scale=0.1):
    E, U, Wo, b = synth.make_weights(V, H, "uniform", scale, seed)
    g = binding.Rnnlm(E, U, Wo, b, B, T, precision, rmsprop=True, r_init=r0)
    o = O.Model.from_weights(E, U, Wo, b, B)
    st = O.RmspropState.filled(V, H, r0)
    return g, o, st


@pytest.mark.parametrize("V,H,B,T,W,r0,rho,eps", [
    (1000, 64, 4, 8, 10, 1.0, 0.9, 1e-6),        # cfg1 shape
    (777, 50, 5, 7, 6, 1e-2, 0.9995, 1e-4),      # ragged everything, the paper's smoothing constant
    (2500, 160, 20, 5, 5, 1e-4, 0.95, 1e-3),     # several tiles, small statistics
    (400, 1100, 6, 3, 3, 1.0, 0.9, 1e-6),        # H > 1024: per-step recurrent launches, multi-block rows
])
def test_rmsprop_train_chunks_fp32(V, H, B, T, W, r0, rho, eps):
    lr = 0.02
    g, o, st = make(V, H, B, T, FP32, seed=V + H, r0=r0)
    tok = synth.zipf_tokens(W * B * T + B + 1, V, 1.1, 8)
    dtok = dev(tok)
    logp = torch.empty(T, B, device="cuda")
    s = torch.zeros(1, dtype=torch.float64, device="cuda")
    for k in range(W):
        x, y = g.rnnlm_stream_chunk(dtok, k, T)
        g.rnnlm_train_chunk_rmsprop(x, y, lr, rho, eps, logp, s)
        ref, sref = O.train_chunk_rmsprop(o, st, *O.stream_chunk(tok, B, T, k), lr, rho, eps)
        got = logp.cpu().numpy().astype(np.float64)
        assert (np.abs(got - ref) <= 2e-4 * np.abs(ref) + 1e-6).all(), (k, np.abs(got - ref).max())
        assert abs(s.item() - sref) <= 2e-4 * abs(sref)
    for name, a, c in (("E", g.E, o.E), ("U", g.U, o.U), ("Wo", g.Wo, o.Wo), ("b", g.b, o.b), ("h", g.h_state, o.h)):
        d = np.abs(a.cpu().numpy() - c).max()
        assert d <= 1e-4 * max(1.0, np.abs(c).max()), (name, d)
    for name, a, c in (("rE", g.rE, st.rE), ("rU", g.rU, st.rU), ("rWo", g.rWo, st.rWo), ("rb", g.rb, st.rb)):
        a = a.cpu().numpy().astype(np.float64)
        assert (np.abs(a - c) <= 1e-3 * np.abs(c) + 1e-12).all(), (name, np.abs(a / c - 1).max())
    # the evaluation path sees the trained weights (compute copies were refreshed)
    xe, ye = O.stream_chunk(tok, B, T, 0)
    lp = g.rnnlm_forward_logprob(dev(xe), dev(ye)).cpu().numpy().astype(np.float64)
    lr_ = O.forward_logprob(o, xe, ye)
    assert (np.abs(lp - lr_) <= 2e-4 * np.abs(lr_) + 1e-6).all()
    g.rnnlm_check()


def test_rmsprop_untouched_words_keep_weights_and_decay():
    V, H, B, T, rho = 500, 32, 4, 4, 0.9
    g, o, st = make(V, H, B, T, FP32, seed=3, r0=0.5)
    tok = synth.zipf_tokens(B * T + B + 1, V, 1.1, 4)
    x, y = O.stream_chunk(tok, B, T, 0)
    E0 = g.E.clone()
    g.rnnlm_train_chunk_rmsprop(dev(x), dev(y), 0.1, rho, 1e-6)
    unseen = torch.ones(V, dtype=torch.bool, device="cuda")
    unseen[dev(x).long().flatten()] = False
    assert torch.equal(g.E[unseen], E0[unseen])
    assert torch.allclose(g.rE[unseen], torch.full_like(g.rE[unseen], 0.5 * rho), rtol=1e-6)
    assert (g.rE[~unseen] > 0.5 * rho).all()
    g.rnnlm_check()


def test_rmsprop_frozen_unit_statistics_equal_plain_sgd_bitwise():
    """rho = 1, r = 1, eps = 0: every denominator is exactly 1, so the step must equal the fused SGD step
    of rnnlm_train_chunk bit for bit (same gradient kernels, same rounding of the update)."""
    V, H, B, T = 1500, 96, 8, 5
    E, U, Wo, b = synth.make_weights(V, H, "uniform", 0.1, 5)
    g1 = binding.Rnnlm(E, U, Wo, b, B, T, FP32, rmsprop=True, r_init=1.0)
    g2 = binding.Rnnlm(E, U, Wo, b, B, T, FP32)
    tok = synth.zipf_tokens(3 * B * T + B + 1, V, 1.1, 6)
    for k in range(3):
        x, y = O.stream_chunk(tok, B, T, k)
        g1.rnnlm_train_chunk_rmsprop(dev(x), dev(y), 0.25, 1.0, 0.0)
        g2.rnnlm_train_chunk(dev(x), dev(y), 0.25)
    for a, c in ((g1.E, g2.E), (g1.U, g2.U), (g1.Wo, g2.Wo), (g1.b, g2.b), (g1.h_state, g2.h_state)):
        assert torch.equal(a, c)


@pytest.mark.parametrize("precision", [FP32, BF16])
def test_rmsprop_bitwise_determinism(precision):
    outs = []
    for _ in range(2):
        g, o, st = make(2000, 128, 16, 6, precision, seed=9, r0=1e-2)
        tok = synth.zipf_tokens(3 * 16 * 6 + 17, 2000, 1.1, 10)
        for k in range(3):
            x, y = O.stream_chunk(tok, 16, 6, k)
            g.rnnlm_train_chunk_rmsprop(dev(x), dev(y), 0.01, 0.9995, 1e-4)
        g.rnnlm_check()
        outs.append([t.clone() for t in (g.E, g.U, g.Wo, g.b, g.h_state, g.rE, g.rU, g.rWo, g.rb)])
    for a, c in zip(*outs):
        assert torch.equal(a, c)


def test_rmsprop_bf16_training_tracks_oracle():
    V, H, B, T, W = 4000, 256, 32, 10, 30
    lr, rho, eps, r0 = 0.002, 0.9995, 1e-4, 1e-4
    g, o, st = make(V, H, B, T, BF16, seed=41, r0=r0)
    tok = synth.zipf_tokens(W * B * T + B + 1, V, 1.1, 42)
    dtok = dev(tok)
    logp = torch.empty(T, B, device="cuda")
    ratios = []
    for k in range(W):
        x, y = g.rnnlm_stream_chunk(dtok, k, T)
        g.rnnlm_train_chunk_rmsprop(x, y, lr, rho, eps, logp)
        ref, _ = O.train_chunk_rmsprop(o, st, *O.stream_chunk(tok, B, T, k), lr, rho, eps)
        ratios.append(math.exp(-logp.double().mean().item()) / math.exp(-ref.mean()))
    assert abs(ratios[0] - 1) < 1e-2 and max(abs(r - 1) for r in ratios) < 2e-2, (ratios[0], ratios[-1])
    assert ratios[-1] == ratios[-1]
    g.rnnlm_check()


def test_rmsprop_needs_the_configuration_flag():
    E, U, Wo, b = synth.make_weights(300, 32, "uniform", 0.1, 1)
    g = binding.Rnnlm(E, U, Wo, b, 2, 4, FP32)
    tok = synth.zipf_tokens(20, 300, 1.1, 2)
    x, y = O.stream_chunk(tok, 2, 4, 0)
    with pytest.raises(binding.RnnlmError):
        g.rnnlm_train_chunk_rmsprop(dev(x), dev(y), 0.1, 0.9, 1e-6)


# ---- the paper's own combination: noise-contrastive criterion + rmsprop -----------------------------------

def make_nce(V, H, B, T, K, precision, seed, r0, scale=0.1):
    E, U, Wo, b = synth.make_weights(V, H, "uniform", scale, seed)
    g = binding.Rnnlm(E, U, Wo, b, B, T, precision, K_max=K, rmsprop=True, r_init=r0)
    o = O.Model.from_weights(E, U, Wo, b, B)
    return g, o, O.RmspropState.filled(V, H, r0)


@pytest.mark.parametrize("V,H,B,T,K,W,r0,rho,eps", [
    (1000, 64, 4, 8, 16, 8, 1.0, 0.9, 1e-6),
    (777, 50, 5, 7, 13, 5, 1e-2, 0.9995, 1e-4),
    (2500, 160, 20, 5, 300, 4, 1e-3, 0.95, 1e-3),
])
def test_nce_rmsprop_train_chunks_fp32(V, H, B, T, K, W, r0, rho, eps):
    lr, lnZ = 0.02, 0.5 * math.log(V)
    g, o, st = make_nce(V, H, B, T, K, FP32, seed=V + K, r0=r0)
    tok = synth.zipf_tokens(W * B * T + B + 1, V, 1.1, 8)
    lnq, thr = synth.unigram_noise(tok, V)
    dtok, dlnq = dev(tok), dev(lnq)
    J = torch.empty(T, B, device="cuda")
    s = torch.zeros(1, dtype=torch.float64, device="cuda")
    for k in range(W):
        x, y = g.rnnlm_stream_chunk(dtok, k, T)
        noise = synth.noise_words(thr, K, 19, k)
        g.rnnlm_nce_train_chunk_rmsprop(x, y, dev(noise), dlnq, lnZ, lr, rho, eps, J, s)
        ref, sref = O.nce_train_chunk_rmsprop(o, st, *O.stream_chunk(tok, B, T, k), noise, lnq.astype(np.float64), lnZ,
                                              lr, rho, eps)
        got = J.cpu().numpy().astype(np.float64)
        assert (np.abs(got - ref) <= 2e-4 * np.abs(ref) + 1e-6).all(), (k, np.abs(got - ref).max())
        assert abs(s.item() - sref) <= 2e-4 * abs(sref)
    for name, a, c in (("E", g.E, o.E), ("U", g.U, o.U), ("Wo", g.Wo, o.Wo), ("b", g.b, o.b), ("h", g.h_state, o.h)):
        d = np.abs(a.cpu().numpy() - c).max()
        assert d <= 1e-4 * max(1.0, np.abs(c).max()), (name, d)
    for name, a, c in (("rE", g.rE, st.rE), ("rU", g.rU, st.rU), ("rWo", g.rWo, st.rWo), ("rb", g.rb, st.rb)):
        a = a.cpu().numpy().astype(np.float64)
        assert (np.abs(a - c) <= 1e-3 * np.abs(c) + 1e-12).all(), (name, np.abs(a / c - 1).max())
    xe, ye = O.stream_chunk(tok, B, T, 0)
    lp = g.rnnlm_forward_logprob(dev(xe), dev(ye)).cpu().numpy().astype(np.float64)
    lr_ = O.forward_logprob(o, xe, ye)
    assert (np.abs(lp - lr_) <= 2e-4 * np.abs(lr_) + 1e-6).all()     # compute copies of the touched rows refreshed
    g.rnnlm_check()


def test_nce_rmsprop_frozen_unit_statistics_equal_nce_sgd_bitwise():
    V, H, B, T, K = 1500, 96, 8, 5, 64
    E, U, Wo, b = synth.make_weights(V, H, "uniform", 0.1, 5)
    g1 = binding.Rnnlm(E, U, Wo, b, B, T, FP32, K_max=K, rmsprop=True, r_init=1.0)
    g2 = binding.Rnnlm(E, U, Wo, b, B, T, FP32, K_max=K)
    tok = synth.zipf_tokens(3 * B * T + B + 1, V, 1.1, 6)
    lnq, thr = synth.unigram_noise(tok, V)
    for k in range(3):
        x, y = O.stream_chunk(tok, B, T, k)
        noise = dev(synth.noise_words(thr, K, 7, k))
        g1.rnnlm_nce_train_chunk_rmsprop(dev(x), dev(y), noise, dev(lnq), 1.0, 0.25, 1.0, 0.0)
        g2.rnnlm_nce_train_chunk(dev(x), dev(y), noise, dev(lnq), 1.0, 0.25)
    for a, c in ((g1.E, g2.E), (g1.U, g2.U), (g1.Wo, g2.Wo), (g1.b, g2.b), (g1.h_state, g2.h_state)):
        assert torch.equal(a, c)


def test_nce_rmsprop_bf16_training_tracks_oracle():
    V, H, B, T, K, W = 4000, 256, 32, 10, 256, 30
    lr, rho, eps, r0 = 0.002, 0.9995, 1e-4, 1e-4
    g, o, st = make_nce(V, H, B, T, K, BF16, seed=41, r0=r0)
    tok = synth.zipf_tokens(W * B * T + B + 1, V, 1.1, 42)
    lnq, thr = synth.unigram_noise(tok, V)
    dtok, dlnq = dev(tok), dev(lnq)
    lnZ = 0.5 * math.log(V)
    s = torch.zeros(1, dtype=torch.float64, device="cuda")
    ratios = []
    for k in range(W):
        x, y = g.rnnlm_stream_chunk(dtok, k, T)
        noise = synth.noise_words(thr, K, 43, k)
        g.rnnlm_nce_train_chunk_rmsprop(x, y, dev(noise), dlnq, lnZ, lr, rho, eps, None, s)
        _, sref = O.nce_train_chunk_rmsprop(o, st, *O.stream_chunk(tok, B, T, k), noise, lnq.astype(np.float64), lnZ,
                                            lr, rho, eps)
        ratios.append(s.item() / sref)
    assert max(abs(r - 1) for r in ratios) < 2e-2, (ratios[0], ratios[-1])
    g.rnnlm_check()
