"""GPU parity of the noise-contrastive training calls (Sec. 4.2 criterion) against the fp64 oracle,
through the C ABI, on the same seeded inputs.  Tolerances as for the normalised criterion: fp32 path
per-position losses |d| <= 1e-4*|ref| + 1e-6 and gradients per tensor 1e-3 (max and l2); bf16 path mean
loss within 1e-2 relative and gradients within 2e-2 of each tensor's scale."""
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


def setup(V, H, B, T, K, precision, seed, scale=0.3, bias_scale=0.5, K_max=None, init="uniform"):
    E, U, Wo, b = synth.make_weights(V, H, init, scale, seed)
    if bias_scale:
        b = synth.uniform_weights((V,), -bias_scale, bias_scale, seed + 99)
    g = binding.Rnnlm(E, U, Wo, b, B, T, precision, K_max=K if K_max is None else K_max)
    o = O.Model.from_weights(E, U, Wo, b, B)
    tok = synth.zipf_tokens(3 * B * T + B + 1, V, 1.1, seed + 5)
    lnq, thr = synth.unigram_noise(tok, V)
    return g, o, tok, lnq, thr


def check_rel(got, ref, rel=1e-4, abs_=1e-6):
    got = got.detach().cpu().numpy().astype(np.float64)
    bad = np.abs(got - ref) > rel * np.abs(ref) + abs_
    assert not bad.any(), f"max |d| = {np.abs(got - ref).max():.3e}"


def check_grad(name, got, ref, rel=1e-3):
    got = got.detach().cpu().numpy().astype(np.float64)
    d = got - ref
    assert np.isfinite(got).all(), name
    assert np.abs(d).max() <= rel * np.abs(ref).max(), f"{name}: max {np.abs(d).max():.3e} vs {np.abs(ref).max():.3e}"
    assert np.linalg.norm(d) <= rel * np.linalg.norm(ref), f"{name}: l2 {np.linalg.norm(d):.3e} vs {np.linalg.norm(ref):.3e}"


SHAPES = [
    # V, H, B, T, K   (cfg1 shape; ragged everything; several tiles + ragged tails; K = 1; K > 256; T = 1)
    (1000, 64, 4, 8, 16),
    (777, 50, 5, 7, 13),
    (3001, 200, 33, 3, 300),
    (10000, 256, 32, 10, 128),
    (300, 130, 3, 1, 1),
    (520, 96, 70, 2, 257),
]


@pytest.mark.parametrize("V,H,B,T,K", SHAPES)
def test_nce_grad_chunk_fp32(V, H, B, T, K):
    g, o, tok, lnq, thr = setup(V, H, B, T, K, FP32, seed=3 * V + H)
    lnZ = 0.4
    x, y = O.stream_chunk(tok, B, T, 0)
    g.rnnlm_forward_logprob(dev(x), dev(y))      # non-zero carried state on both sides
    O.forward_logprob(o, x, y)
    x, y = O.stream_chunk(tok, B, T, 1)
    noise = synth.noise_words(thr, K, 77, 1)
    noise[0] = y[0, 0]                           # a noise word equal to a target
    if K > 2:
        noise[-1] = noise[1]                     # a repeated noise word
    before = [t.clone() for t in (g.E, g.U, g.Wo, g.b, g.h_state)]
    r = g.rnnlm_nce_grad_chunk(dev(x), dev(y), dev(noise), dev(lnq), lnZ)
    ref = O.nce_grad_chunk(o, x, y, noise, lnq.astype(np.float64), lnZ)
    check_rel(r["J"], ref["J"])
    for k in ("gE", "gU", "gWo", "gb"):
        check_grad(k, r[k], ref[k])
    for a, c in zip(before, (g.E, g.U, g.Wo, g.b, g.h_state)):
        assert torch.equal(a, c)
    untouched = np.setdiff1d(np.arange(V), np.concatenate([y.ravel(), noise]))
    assert not r["gWo"].cpu().numpy()[untouched].any() and not r["gb"].cpu().numpy()[untouched].any()
    g.rnnlm_check()


@pytest.mark.parametrize("V,H,B,T,K,W", [(1000, 64, 4, 8, 16, 10), (2500, 160, 20, 5, 100, 6)])
def test_nce_train_chunks_fp32(V, H, B, T, K, W):
    lr, lnZ = 0.1, math.log(V) * 0.5
    g, o, tok, lnq, thr = setup(V, H, B, T, K, FP32, seed=17, scale=0.1, bias_scale=0.0)
    tok = synth.zipf_tokens(W * B * T + B + 1, V, 1.1, 18)
    dtok, dlnq = dev(tok), dev(lnq)
    J = torch.empty(T, B, device="cuda")
    s = torch.zeros(1, dtype=torch.float64, device="cuda")
    for k in range(W):
        x, y = g.rnnlm_stream_chunk(dtok, k, T)
        noise = synth.noise_words(thr, K, 19, k)
        g.rnnlm_nce_train_chunk(x, y, dev(noise), dlnq, lnZ, lr, J, s)
        xr, yr = O.stream_chunk(tok, B, T, k)
        ref, sref = O.nce_train_chunk(o, xr, yr, noise, lnq.astype(np.float64), lnZ, lr)
        check_rel(J, ref, rel=1e-4)
        assert abs(s.item() - sref) <= 1e-4 * abs(sref)
    for name, a, c in (("E", g.E, o.E), ("U", g.U, o.U), ("Wo", g.Wo, o.Wo), ("b", g.b, o.b), ("h", g.h_state, o.h)):
        d = np.abs(a.cpu().numpy() - c).max()
        assert d <= 1e-4 * max(1.0, np.abs(c).max()), (name, d)
    # the normalised evaluation path sees the trained weights (compute copies were refreshed)
    xe, ye = O.stream_chunk(tok, B, T, 0)
    lp = g.rnnlm_forward_logprob(dev(xe), dev(ye))
    check_rel(lp, O.forward_logprob(o, xe, ye), rel=1e-4)
    g.rnnlm_check()


@pytest.mark.parametrize("precision", [FP32, BF16])
def test_nce_bitwise_determinism(precision):
    V, H, B, T, K = 2000, 128, 16, 6, 200
    outs = []
    for _ in range(2):
        g, o, tok, lnq, thr = setup(V, H, B, T, K, precision, seed=23, scale=0.1)
        dtok, dlnq = dev(tok), dev(lnq)
        for k in range(3):
            x, y = g.rnnlm_stream_chunk(dtok, k, T)
            g.rnnlm_nce_train_chunk(x, y, dev(synth.noise_words(thr, K, 29, k)), dlnq, 1.0, 0.1)
        g.rnnlm_check()
        outs.append([t.clone() for t in (g.E, g.U, g.Wo, g.b, g.h_state)])
    for a, c in zip(*outs):
        assert torch.equal(a, c)


BF16_SHAPES = [(3000, 256, 32, 8, 256), (1000, 1100, 8, 3, 100), (5000, 512, 64, 10, 1000)]


@pytest.mark.parametrize("V,H,B,T,K", BF16_SHAPES)
def test_nce_bf16_loss_and_gradients(V, H, B, T, K):
    g, o, tok, lnq, thr = setup(V, H, B, T, K, BF16, seed=V + K, scale=0.1, bias_scale=0.2)
    lnZ = 2.0
    x, y = O.stream_chunk(tok, B, T, 0)
    noise = synth.noise_words(thr, K, 31, 0)
    r = g.rnnlm_nce_grad_chunk(dev(x), dev(y), dev(noise), dev(lnq), lnZ)
    ref = O.nce_grad_chunk(o, x, y, noise, lnq.astype(np.float64), lnZ)
    assert abs(r["J"].double().mean().item() / ref["J"].mean() - 1) < 1e-2
    for k in ("gE", "gU", "gWo", "gb"):
        check_grad(k, r[k], ref[k], rel=2e-2)
    g.rnnlm_check()


def test_nce_bf16_training_tracks_oracle():
    V, H, B, T, K, W, lr = 4000, 256, 32, 10, 256, 30, 0.2
    g, o, tok, lnq, thr = setup(V, H, B, T, K, BF16, seed=41, scale=0.1, bias_scale=0.0)
    tok = synth.zipf_tokens(W * B * T + B + 1, V, 1.1, 42)
    dtok, dlnq = dev(tok), dev(lnq)
    lnZ = math.log(V) * 0.5
    s = torch.zeros(1, dtype=torch.float64, device="cuda")
    ratios = []
    for k in range(W):
        x, y = g.rnnlm_stream_chunk(dtok, k, T)
        noise = synth.noise_words(thr, K, 43, k)
        g.rnnlm_nce_train_chunk(x, y, dev(noise), dlnq, lnZ, lr, None, s)
        _, sref = O.nce_train_chunk(o, *O.stream_chunk(tok, B, T, k), noise, lnq.astype(np.float64), lnZ, lr)
        ratios.append(s.item() / sref)
    assert max(abs(r - 1) for r in ratios) < 1e-2, (ratios[0], ratios[-1])
    g.rnnlm_check()


def test_nce_arguments_are_validated():
    g, o, tok, lnq, thr = setup(500, 32, 4, 4, 8, FP32, seed=51)
    x, y = O.stream_chunk(tok, 4, 4, 0)
    noise = synth.noise_words(thr, 8, 1, 0)
    with pytest.raises(binding.RnnlmError):   # more noise words than the handle was configured for
        g.rnnlm_nce_train_chunk(dev(x), dev(y), dev(np.concatenate([noise, noise])), dev(lnq), 0.0, 0.1)
    g0 = binding.Rnnlm(*synth.make_weights(500, 32, "uniform", 0.1, 3), 4, 4, FP32)   # K_max = 0
    with pytest.raises(binding.RnnlmError):
        g0.rnnlm_nce_train_chunk(dev(x), dev(y), dev(noise), dev(lnq), 0.0, 0.1)
    bad = noise.copy()
    bad[3] = 500                               # out-of-range noise id: clamped, reported, never a fault
    g.rnnlm_nce_train_chunk(dev(x), dev(y), dev(bad), dev(lnq), 0.0, 0.1)
    with pytest.raises(binding.RnnlmError) as e:
        g.rnnlm_check()
    assert e.value.status == -2


# ---- full-size checks, in the launch configuration bench.py --criterion nce times -----------------------

def _cfg_setup(name, K, weights="config"):
    cfg = synth.CONFIGS[name]
    if weights == "config":
        E, U, Wo, b = synth.make_weights(cfg.V, cfg.H, cfg.init, cfg.init_scale, cfg.weight_seed)
    else:  # cheaper generator for the largest shapes, same scale
        E, U, Wo, b = synth.make_weights(cfg.V, cfg.H, "uniform", cfg.init_scale * 1.7, cfg.weight_seed)
    g = binding.Rnnlm(E, U, Wo, b, cfg.B, cfg.T, BF16 if cfg.precision == "bf16" else FP32, K_max=K)
    return cfg, g, (E, U, Wo, b)


def test_cfg3_full_size_nce_window():
    """cfg3 (V=64,000 H=1024 B=128 T=20, bf16 operands, 1024 noise words): one whole window against the
    oracle: mean loss within 1e-2, every position's loss within 2e-2 relative, every gradient tensor within
    2e-2 of its scale, then the SGD step itself on the touched rows and the untouched rows left alone."""
    K = 1024
    cfg, g, (E, U, Wo, b) = _cfg_setup("cfg3", K)
    o = O.Model.from_weights(E, U, Wo, b, cfg.B)
    tok = synth.make_tokens(cfg, 2_000_000)
    lnq, thr = synth.unigram_noise(tok, cfg.V)
    noise = synth.noise_words(thr, K, cfg.data_seed + 7, 0)
    lnZ = math.log(cfg.V)
    x, y = O.stream_chunk(tok, cfg.B, cfg.T, 0)
    r = g.rnnlm_nce_grad_chunk(dev(x), dev(y), dev(noise), dev(lnq), lnZ)
    ref = O.nce_grad_chunk(o, x, y, noise, lnq.astype(np.float64), lnZ)
    J = r["J"].cpu().numpy().astype(np.float64)
    assert abs(J.mean() / ref["J"].mean() - 1) < 1e-2
    assert (np.abs(J - ref["J"]) <= 2e-2 * np.abs(ref["J"])).all()
    for kk in ("gE", "gU", "gWo", "gb"):
        check_grad(kk, r[kk], ref[kk], rel=2e-2)
    Wo0, b0 = g.Wo.clone(), g.b.clone()
    g.rnnlm_nce_train_chunk(dev(x), dev(y), dev(noise), dev(lnq), lnZ, cfg.lr)
    assert torch.allclose(g.Wo, Wo0 - cfg.lr * r["gWo"], rtol=0, atol=1e-7)
    assert torch.allclose(g.b, b0 - cfg.lr * r["gb"], rtol=0, atol=1e-7)
    touched = torch.zeros(cfg.V, dtype=torch.bool, device="cuda")
    touched[dev(np.concatenate([y.ravel(), noise])).long()] = True
    assert torch.equal(g.Wo[~touched], Wo0[~touched]) and torch.equal(g.b[~touched], b0[~touched])
    g.rnnlm_check()


def test_cfg5_nce_sampled_streams():
    """cfg5 at full shape (V=100,000 H=4096 B=256 T=32, 1024 noise words): the oracle runs three whole
    streams of the first window one by one (the forward pass and the per-position losses of a stream do not
    depend on the other streams); the GPU's losses for those streams must agree within 2e-2 per position
    and 1e-2 in the mean.  Size-independent properties: finite results, rows of dWo and entries of db of
    words that are neither target nor noise are exactly zero."""
    K = 1024
    cfg, g, (E, U, Wo, b) = _cfg_setup("cfg5", K, weights="uniform")
    tok = synth.make_tokens(cfg, 4_000_000)
    lnq, thr = synth.unigram_noise(tok, cfg.V)
    noise = synth.noise_words(thr, K, cfg.data_seed + 7, 0)
    lnZ = math.log(cfg.V)
    x, y = O.stream_chunk(tok, cfg.B, cfg.T, 0)
    r = g.rnnlm_nce_grad_chunk(dev(x), dev(y), dev(noise), dev(lnq), lnZ)
    J = r["J"].cpu().numpy().astype(np.float64)
    assert np.isfinite(J).all()
    E64, U64, Wo64, b64 = (np.asarray(a, np.float64) for a in (E, U, Wo, b))
    for s in (0, 200, 255):
        o1 = O.Model(E64, U64, Wo64, b64, np.zeros((1, cfg.H)))
        ref = O.nce_grad_chunk(o1, np.ascontiguousarray(x[:, s:s + 1]), np.ascontiguousarray(y[:, s:s + 1]), noise,
                               lnq.astype(np.float64), lnZ)["J"][:, 0]
        assert abs(J[:, s].mean() / ref.mean() - 1) < 1e-2
        assert (np.abs(J[:, s] - ref) <= 2e-2 * np.abs(ref)).all()
    for kk in ("gE", "gU", "gWo", "gb"):
        assert torch.isfinite(r[kk]).all()
    touched = torch.zeros(cfg.V, dtype=torch.bool, device="cuda")
    touched[dev(np.concatenate([y.ravel(), noise])).long()] = True
    assert not r["gWo"][~touched].any() and not r["gb"][~touched].any()
    assert r["gWo"][touched].abs().sum() > 0
    g.rnnlm_check()


# ---- forward-only unnormalised scoring (Sec. 4.2: the output as used for rescoring) ----------------------

@pytest.mark.parametrize("V,H,B,T,precision,tol", [(1000, 64, 1, 8, FP32, 1e-4), (3001, 200, 5, 7, FP32, 1e-4),
                                                   (10000, 256, 16, 10, FP32, 1e-4), (520, 96, 70, 2, FP32, 1e-4),
                                                   (5000, 512, 8, 12, BF16, 2e-2), (4000, 1100, 3, 4, BF16, 2e-2)])
def test_forward_score(V, H, B, T, precision, tol):
    """Small-batch scoring of given next words against the oracle, two chained windows (carried state)."""
    E, U, Wo, b = synth.make_weights(V, H, "uniform", 0.3, V + H)
    b = synth.uniform_weights((V,), -0.5, 0.5, 7)
    g = binding.Rnnlm(E, U, Wo, b, B, T, precision)
    o = O.Model.from_weights(E, U, Wo, b, B)
    tok = synth.zipf_tokens(2 * B * T + B + 1, V, 1.1, 3)
    lnZ = 1.25
    for k in range(2):
        x, y = O.stream_chunk(tok, B, T, k)
        got = g.rnnlm_forward_score(dev(x), dev(y), lnZ).cpu().numpy().astype(np.float64)
        ref = O.forward_score(o, x, y, lnZ)
        scale = max(1.0, np.abs(ref).max())
        assert np.abs(got - ref).max() <= tol * scale, (k, np.abs(got - ref).max())
    assert np.abs(g.h_state.cpu().numpy() - o.h).max() < (1e-5 if precision == FP32 else 2e-2)
    g.rnnlm_check()


def test_forward_score_matches_the_normalised_path_up_to_the_log_partition():
    """score + lnZ - logp is the same for every next word asked for at a position (it is the position's
    log-partition): two calls with different targets from the same state."""
    V, H, B, T = 2000, 128, 4, 6
    E, U, Wo, b = synth.make_weights(V, H, "uniform", 0.3, 5)
    g = binding.Rnnlm(E, U, Wo, b, B, T, FP32)
    tok = synth.zipf_tokens(4 * B * T + 1, V, 1.1, 6)
    x, y1 = O.stream_chunk(tok, B, T, 0)
    _, y2 = O.stream_chunk(tok, B, T, 1)
    parts = []
    for y in (y1, y2):
        g.rnnlm_reset_state()
        s = g.rnnlm_forward_score(dev(x), dev(y), 0.0)
        g.rnnlm_reset_state()
        lp = g.rnnlm_forward_logprob(dev(x), dev(y))
        parts.append((s - lp).cpu().numpy())
    assert np.abs(parts[0] - parts[1]).max() < 1e-4


def test_forward_score_shortlist_plain_architecture():
    """Scores of a shortlist of candidate next words per position on the plain architecture, fp32 and bf16,
    against one oracle scoring pass per candidate column."""
    V, H, B, T, Cn = 1200, 96, 6, 5, 19
    E, U, Wo, b = synth.make_weights(V, H, "uniform", 0.3, 17)
    b = synth.uniform_weights((V,), -0.2, 0.2, 18)
    tok = synth.zipf_tokens(B * T + B + 1, V, 1.1, 19)
    x, y = O.stream_chunk(tok, B, T, 0)
    cand = np.random.default_rng(5).integers(0, V, (T, B, Cn)).astype(np.int32)
    cand[:, :, 3] = y
    ref = O.forward_score_shortlist(O.Model.from_weights(E, U, Wo, b, B), x, cand, 1.1)
    for precision, tol in ((binding.RNNLM_FP32, 1e-4), (binding.RNNLM_BF16_FP32MASTER, 2e-2)):
        g = binding.Rnnlm(E, U, Wo, b, B, T, precision)
        got = g.rnnlm_forward_score_shortlist(torch.as_tensor(x).cuda(), torch.as_tensor(cand).cuda(), 1.1)
        single = binding.Rnnlm(E, U, Wo, b, B, T, precision).rnnlm_forward_score(
            torch.as_tensor(x).cuda(), torch.as_tensor(y).cuda(), 1.1)
        g.rnnlm_check()
        assert np.abs(got.cpu().numpy() - ref).max() <= tol * max(1.0, np.abs(ref).max())
        assert torch.equal(got[:, :, 3], single)

