"""Pins of the fp64 oracle against things other than itself (CPU only).

Each test states what fixes the expected value: a closed form, an invariant of the
model of Sec. 4.1/4.2, a special case that reduces to a textbook routine, central
finite differences, or an independent autograd evaluation of the same loss.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden", "worked_example_v3_h2.txt")
LN2, LN3 = math.log(2.0), math.log(3.0)


def rand_model(V, H, B, seed, scale=0.5, h_scale=0.0):
    r = np.random.default_rng(seed)
    m = O.Model(r.uniform(-scale, scale, (V, H)), r.uniform(-scale, scale, (H, H)),
                r.uniform(-scale, scale, (V, H)), r.uniform(-scale, scale, V),
                r.uniform(0, 1, (B, H)) * h_scale)
    return m


def rand_tokens(V, T, B, seed):
    r = np.random.default_rng(seed)
    return r.integers(0, V, (T, B)).astype(np.int32), r.integers(0, V, (T, B)).astype(np.int32)


def worked_model():
    E = np.array([[0, LN3], [-LN3, LN3], [0, 0]], float)
    U = np.array([[0, 8 / 3 * LN3], [-4 * LN3, 0]], float)
    Wo = np.array([[4 * LN2, 0], [0, 4 * LN3], [0, 0]], float)
    b = np.array([0, 0, LN2], float)
    return O.Model(E, U, Wo, b, np.zeros((1, 2)))


def read_golden():
    g = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        if k == "gE":
            g.setdefault("gE", {})[int(v[0])] = [float(t) for t in v[1:]]
        else:
            g[k] = [float(t) for t in v]
    return g


def test_golden_file_matches_closed_forms():
    """The fixture's numbers re-derived with exact rationals and logs of small integers."""
    g = read_golden()
    assert g["logp"] == pytest.approx([math.log(9 / 11), math.log(2 / 13)], abs=1e-11)
    assert g["ppl"][0] == pytest.approx(math.sqrt(143 / 18), abs=1e-11)
    dz0 = [Fraction(4, 33), Fraction(27, 33) - 1, Fraction(2, 33)]
    dz1 = [Fraction(8, 13), Fraction(3, 13), Fraction(2, 13) - 1]
    h0 = [Fraction(1, 2), Fraction(3, 4)]
    h1 = [Fraction(3, 4), Fraction(1, 4)]
    gb = [float(a + c) for a, c in zip(dz0, dz1)]
    assert g["gb"] == pytest.approx(gb, abs=1e-11)
    gWo = [float(dz0[v] * h0[j] + dz1[v] * h1[j]) for v in range(3) for j in range(2)]
    assert g["gWo"] == pytest.approx(gWo, abs=1e-11)
    dh1 = [4 * LN2 * float(dz1[0]), 4 * LN3 * float(dz1[1])]
    da1 = [dh1[j] * float(h1[j] * (1 - h1[j])) for j in range(2)]
    assert g["da1"] == pytest.approx(da1, abs=1e-11)
    # dh0_j = sum_v Wo[v][j] dz0_v + sum_i U[i][j] da1_i
    dh0 = [4 * LN2 * float(dz0[0]) + (-4 * LN3) * da1[1], 4 * LN3 * float(dz0[1]) + (8 / 3 * LN3) * da1[0]]
    da0 = [dh0[j] * float(h0[j] * (1 - h0[j])) for j in range(2)]
    assert g["da0"] == pytest.approx(da0, abs=1e-11)
    gU = [da1[i] * float(h0[j]) for i in range(2) for j in range(2)]
    assert g["gU"] == pytest.approx(gU, abs=1e-11)
    assert g["gE"][0] == pytest.approx(da0, abs=1e-11) and g["gE"][1] == pytest.approx(da1, abs=1e-11)


def test_worked_example():
    g = read_golden()
    m = worked_model()
    x = np.array([[0], [1]], np.int32)
    y = np.array([[1], [2]], np.int32)
    r = O.grad_chunk(m, x, y, debug=True)
    assert r["logp"].ravel() == pytest.approx(g["logp"], abs=1e-11)
    assert r["Hs"].ravel() == pytest.approx([0.5, 0.75, 0.75, 0.25], abs=1e-13)
    two = 2.0  # the oracle returns gradients of the mean loss over B*T = 2 tokens
    assert (two * r["gb"]) == pytest.approx(g["gb"], abs=1e-11)
    assert (two * r["gWo"]).ravel() == pytest.approx(g["gWo"], abs=1e-11)
    assert (two * r["gU"]).ravel() == pytest.approx(g["gU"], abs=1e-11)
    assert (two * r["dA"][1, 0]) == pytest.approx(g["da1"], abs=1e-11)
    assert (two * r["dA"][0, 0]) == pytest.approx(g["da0"], abs=1e-11)
    for w in range(3):
        assert (two * r["gE"][w]) == pytest.approx(g["gE"][w], abs=1e-11)
    ppl, scored = O.perplexity(m, np.array([0, 1, 2], np.int32), T=2)
    assert scored == 2 and ppl == pytest.approx(g["ppl"][0], abs=1e-11)


def test_uniform_model_perplexity_is_V():
    """Wo = 0, b = 0: every distribution is uniform, so logp = -ln V and PPL = V."""
    V, H, B, T = 37, 5, 3, 4
    m = rand_model(V, H, B, 1)
    m.Wo[:] = 0
    m.b[:] = 0
    tok = np.random.default_rng(2).integers(0, V, 200).astype(np.int32)
    ppl, scored = O.perplexity(m, tok, T)
    assert scored == ((200 - 1) // B // T) * B * T
    assert ppl == pytest.approx(V, rel=1e-12)
    x, y = O.stream_chunk(tok, B, T, 0)
    assert O.forward_logprob(m, x, y) == pytest.approx(-math.log(V), rel=1e-12)


def test_softmax_sums_to_one_and_logp_consistent():
    V, H, B, T = 50, 6, 3, 5
    m = rand_model(V, H, B, 3, scale=2.0)
    x, y = rand_tokens(V, T, B, 4)
    logp, P = O.forward_logprob(m, x, y, want_probs=True)
    assert P.sum(-1) == pytest.approx(1.0, abs=1e-12)
    picked = np.take_along_axis(P, y[..., None].astype(np.int64), -1)[..., 0]
    assert np.log(picked) == pytest.approx(logp, abs=1e-12)


def _loss(m, x, y):
    mm = m.copy()
    return -O.forward_logprob(mm, x, y).mean()


@pytest.mark.parametrize("V,H,B,T,seed", [(7, 4, 2, 4, 0), (5, 3, 1, 3, 1), (6, 2, 2, 1, 2)])
def test_finite_differences(V, H, B, T, seed):
    """Central differences of the mean NLL for EVERY entry of E, U, Wo, b; repeated ids inside
    the window and a non-zero carried state."""
    m = rand_model(V, H, B, seed, scale=0.8, h_scale=1.0)
    x, y = rand_tokens(V, T, B, seed + 10)
    x[0, :] = x[-1, :]  # force duplicates of an input id within the window
    r = O.grad_chunk(m, x, y)
    eps = 1e-5
    for name, g in (("E", r["gE"]), ("U", r["gU"]), ("Wo", r["gWo"]), ("b", r["gb"])):
        p = getattr(m, name)
        fd = np.zeros_like(p)
        it = np.nditer(p, flags=["multi_index"])
        for _ in it:
            idx = it.multi_index
            old = p[idx]
            p[idx] = old + eps
            lp = _loss(m, x, y)
            p[idx] = old - eps
            lm = _loss(m, x, y)
            p[idx] = old
            fd[idx] = (lp - lm) / (2 * eps)
        assert np.abs(fd - g).max() <= 1e-6 * max(1.0, np.abs(g).max()) * 1e-1 + 1e-9, name


def _torch_grads(m, x, y):
    E, U, Wo, b = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (m.E, m.U, m.Wo, m.b))
    h = torch.tensor(m.h, dtype=torch.float64)
    xt = torch.tensor(x, dtype=torch.long)
    yt = torch.tensor(y, dtype=torch.long)
    lps = []
    for t in range(x.shape[0]):
        h = torch.sigmoid(E[xt[t]] + h @ U.T)
        z = h @ Wo.T + b
        lps.append(torch.log_softmax(z, -1).gather(1, yt[t][:, None])[:, 0])
    lp = torch.stack(lps)
    (-lp.mean()).backward()
    return lp.detach().numpy(), E.grad.numpy(), U.grad.numpy(), Wo.grad.numpy(), b.grad.numpy(), h.detach().numpy()


@pytest.mark.parametrize("V,H,B,T,seed", [(23, 8, 3, 6, 5), (40, 16, 4, 9, 6), (11, 5, 1, 12, 7)])
def test_against_autograd(V, H, B, T, seed):
    """Same loss written with library ops (fp64 CPU tensors) and differentiated by autograd:
    the oracle's hand-derived BPTT must agree for all gradients, log-probs and the carried state."""
    m = rand_model(V, H, B, seed, scale=0.7, h_scale=1.0)
    x, y = rand_tokens(V, T, B, seed + 1)
    x[1 % T, :] = x[0, :]
    r = O.grad_chunk(m, x, y)
    lp, gE, gU, gWo, gb, hT = _torch_grads(m, x, y)
    assert r["logp"] == pytest.approx(lp, abs=1e-12)
    for a, c in ((r["gE"], gE), (r["gU"], gU), (r["gWo"], gWo), (r["gb"], gb), (r["h_next"], hT)):
        assert np.abs(a - c).max() <= 1e-12 * max(1.0, np.abs(c).max())


def test_parameter_count_matches_table1():
    """No hidden bias (Sec. 4.1): parameters besides b number 2VH + H^2; with V = 64,000 this gives
    the model sizes of Table 1 (in millions)."""
    table1 = {128: 16.4, 256: 32.8, 512: 65.8, 1024: 132, 2048: 266, 4096: 541}
    for H, millions in table1.items():
        n = 2 * 64000 * H + H * H
        assert abs(n / 1e6 - millions) < (0.06 if millions < 100 else 0.6)
    m = rand_model(9, 4, 2, 0)
    assert m.E.size + m.U.size + m.Wo.size == 2 * 9 * 4 + 16


def test_chunking_invariance_and_state_carry():
    """The state is carried across windows and never reset (Sec. 2.3, Sec. 4.2): one window of T
    gives the same log-probs as T windows of 1, or any other split."""
    V, H, B, T = 19, 6, 3, 12
    m = rand_model(V, H, B, 11, scale=0.9)
    x, y = rand_tokens(V, T, B, 12)
    whole = O.forward_logprob(m.copy(), x, y)
    for split in (1, 3, 4):
        mm = m.copy()
        parts = [O.forward_logprob(mm, x[a:a + split], y[a:a + split]) for a in range(0, T, split)]
        assert np.concatenate(parts) == pytest.approx(whole, abs=1e-13)


def test_stream_independence():
    V, H, B, T = 17, 5, 4, 6
    m = rand_model(V, H, B, 13, scale=0.9, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 14)
    r = O.grad_chunk(m, x, y)
    acc = {k: 0.0 for k in ("gE", "gU", "gWo", "gb")}
    for s in range(B):
        ms = O.Model(m.E, m.U, m.Wo, m.b, m.h[s:s + 1].copy())
        rs = O.grad_chunk(ms, x[:, s:s + 1].copy(), y[:, s:s + 1].copy())
        assert rs["logp"][:, 0] == pytest.approx(r["logp"][:, s], abs=1e-13)
        assert rs["h_next"][0] == pytest.approx(r["h_next"][s], abs=1e-14)
        for k in acc:
            acc[k] = acc[k] + rs[k] / B
    for k in acc:
        assert np.abs(acc[k] - r[k]).max() < 1e-13


def test_softmax_gradient_identities():
    V, H, B, T = 29, 7, 3, 5
    m = rand_model(V, H, B, 15, scale=1.0, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 16)
    r = O.grad_chunk(m, x, y, debug=True)
    assert abs(r["gb"].sum()) < 1e-14
    assert np.abs(r["gWo"].sum(0)).max() < 1e-14
    assert np.abs(r["dZ"].sum(-1)).max() < 1e-15
    m2 = m.copy()
    m2.b += 3.25
    assert O.forward_logprob(m2, x, y) == pytest.approx(r["logp"], abs=1e-12)


def test_U_zero_is_softmax_regression():
    """U = 0: h_t = sigmoid(E[w_t]) has no history, so the model is multinomial logistic regression
    on those features; log-probs and output-layer gradients from the textbook formula."""
    V, H, B, T = 31, 6, 3, 7
    m = rand_model(V, H, B, 17, scale=1.0, h_scale=1.0)
    m.U[:] = 0
    x, y = rand_tokens(V, T, B, 18)
    r = O.grad_chunk(m, x, y)
    F = 1 / (1 + np.exp(-m.E[x.ravel()]))
    Z = F @ m.Wo.T + m.b
    LP = Z - logsumexp(Z, axis=1, keepdims=True)
    n = x.size
    assert r["logp"].ravel() == pytest.approx(LP[np.arange(n), y.ravel()], abs=1e-12)
    D = np.exp(LP)
    D[np.arange(n), y.ravel()] -= 1
    D /= n
    assert np.abs(D.T @ F - r["gWo"]).max() < 1e-14
    assert np.abs(D.sum(0) - r["gb"]).max() < 1e-14
    assert np.abs(r["gU"]).max() > 0  # gU itself need not vanish: it is a derivative AT U = 0


def test_unigram_special_case():
    """E = 0, U = 0, Wo = 0, b_v = ln f_v: the model is the unigram distribution f; scoring targets
    whose empirical distribution is f gives PPL = exp(entropy(f)) and a zero bias gradient."""
    V, B, T, H = 6, 2, 30, 3
    counts = np.array([20, 14, 10, 8, 5, 3])
    yflat = np.repeat(np.arange(V), counts)
    np.random.default_rng(0).shuffle(yflat)
    y = yflat.reshape(T, B).astype(np.int32)
    x = np.random.default_rng(1).integers(0, V, (T, B)).astype(np.int32)
    f = counts / counts.sum()
    m = O.Model(np.zeros((V, H)), np.zeros((H, H)), np.zeros((V, H)), np.log(f), np.zeros((B, H)))
    r = O.grad_chunk(m, x, y, debug=True)
    assert r["Hs"] == pytest.approx(0.5, abs=0)
    assert math.exp(-r["logp"].mean()) == pytest.approx(math.exp(-(f * np.log(f)).sum()), rel=1e-13)
    assert np.abs(r["gb"]).max() < 1e-15


def test_T1_is_feedforward_net():
    """T = 1: nothing flows back through U, the gradients are those of a one-hidden-layer net with
    input (onehot(w), h_prev) written out directly."""
    V, H, B = 13, 5, 4
    m = rand_model(V, H, B, 19, scale=0.9, h_scale=1.0)
    x, y = rand_tokens(V, 1, B, 20)
    r = O.grad_chunk(m, x, y)
    a = m.E[x[0]] + m.h @ m.U.T
    h = 1 / (1 + np.exp(-a))
    z = h @ m.Wo.T + m.b
    p = np.exp(z - logsumexp(z, 1, keepdims=True))
    dz = p.copy()
    dz[np.arange(B), y[0]] -= 1
    dz /= B
    da = (dz @ m.Wo) * h * (1 - h)
    assert np.abs(da.T @ m.h - r["gU"]).max() < 1e-14
    gE = np.zeros_like(m.E)
    np.add.at(gE, x[0], da)
    assert np.abs(gE - r["gE"]).max() < 1e-14
    assert np.abs(dz.T @ h - r["gWo"]).max() < 1e-14


def test_vocabulary_relabelling():
    V, H, B, T = 21, 6, 2, 8
    m = rand_model(V, H, B, 21, scale=0.9)
    x, y = rand_tokens(V, T, B, 22)
    base = O.forward_logprob(m.copy(), x, y)
    perm = np.random.default_rng(23).permutation(V)  # new id of old id w is perm[w]
    inv = np.argsort(perm)
    m2 = O.Model(m.E[inv].copy(), m.U.copy(), m.Wo[inv].copy(), m.b[inv].copy(), m.h.copy())
    assert O.forward_logprob(m2, perm[x].astype(np.int32), perm[y].astype(np.int32)) == pytest.approx(base, abs=1e-13)


def test_sgd_step():
    V, H, B, T = 15, 4, 3, 5
    m = rand_model(V, H, B, 24, scale=0.8, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 25)
    r = O.grad_chunk(m, x, y)
    m1 = m.copy()
    lr = 0.37
    logp, s = O.train_chunk(m1, x, y, lr)
    assert logp == pytest.approx(r["logp"], abs=0) and s == pytest.approx(r["logp"].sum(), abs=1e-12)
    for k, g in (("E", "gE"), ("U", "gU"), ("Wo", "gWo"), ("b", "gb")):
        assert np.array_equal(getattr(m1, k), getattr(m, k) - lr * r[g])
    assert np.array_equal(m1.h, r["h_next"])
    m0 = m.copy()
    O.train_chunk(m0, x, y, 0.0)
    for k in ("E", "U", "Wo", "b"):
        assert np.array_equal(getattr(m0, k), getattr(m, k))
    assert np.array_equal(m0.h, r["h_next"]) and not np.array_equal(m0.h, m.h)


def test_sgd_decreases_loss_on_repeated_window():
    V, H, B, T = 30, 8, 4, 6
    m = rand_model(V, H, B, 26, scale=0.1)
    x, y = rand_tokens(V, T, B, 27)
    h0 = m.h.copy()
    losses = []
    for _ in range(30):
        m.h[:] = h0
        logp, _ = O.train_chunk(m, x, y, 1.0)
        losses.append(-logp.mean())
    assert losses[-1] < 0.85 * losses[0] and all(b < a for a, b in zip(losses, losses[1:]))


def test_stream_chunk_indexing():
    N, B, T = 103, 4, 5
    tok = np.arange(N, dtype=np.int32) * 3 % 50
    L = (N - 1) // B
    assert O.num_chunks(N, B, T) == L // T == 5
    for k in range(L // T):
        x, y = O.stream_chunk(tok, B, T, k)
        for t in range(T):
            for s in range(B):
                assert x[t, s] == tok[s * L + k * T + t] and y[t, s] == tok[s * L + k * T + t + 1]
    with pytest.raises(ValueError):
        O.stream_chunk(tok, B, T, L // T)


def test_sort_segments_is_stable_sort():
    r = np.random.default_rng(3)
    for M, V in ((1, 5), (17, 4), (200, 30), (64, 1)):
        x = r.integers(0, V, M).astype(np.int32)
        perm, seg = O.sort_segments(x)
        assert np.array_equal(perm, np.argsort(x, kind="stable"))
        xs = x[perm]
        starts = np.flatnonzero(np.r_[True, xs[1:] != xs[:-1]])
        assert np.array_equal(seg, np.r_[starts, M])


def test_token_range_is_an_error():
    m = rand_model(5, 3, 1, 0)
    x = np.array([[5]], np.int32)
    y = np.array([[0]], np.int32)
    with pytest.raises(ValueError):
        O.forward_logprob(m, x, y)
    with pytest.raises(ValueError):
        O.grad_chunk(m, y, np.array([[-1]], np.int32))
