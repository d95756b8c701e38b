"""Pins of the oracle's noise-contrastive step (Sec. 4.2 criterion) against things other than itself
(CPU only): a hand-computed example, closed forms, central finite differences, an independent
autograd evaluation, the limit in which the estimator becomes maximum likelihood (checked against the
already pinned normalised criterion), and invariances."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import oracle as O
from test_oracle_pins import rand_model, rand_tokens, worked_model

GOLD = os.path.join(os.path.dirname(__file__), "golden", "nce_worked_example_v3_h2.txt")
LN2, LN3 = math.log(2.0), math.log(3.0)


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


def rand_q(V, seed):
    q = np.random.default_rng(seed).uniform(0.2, 1.0, V)
    return q / q.sum()


def test_golden_file_matches_closed_forms():
    g = read_golden()
    assert g["J"] == pytest.approx([math.log(55 / 54) + 2 * math.log(5), math.log(5 / 4) + math.log(9) + math.log(5)],
                                   abs=1e-11)
    h0, h1 = [Fraction(1, 2), Fraction(3, 4)], [Fraction(3, 4), Fraction(1, 4)]
    # coefficients dJ/dz: target -(1 - sigma), noise +sigma
    c0 = {1: -(1 - Fraction(54, 55)), 0: Fraction(4, 5), 2: Fraction(4, 5)}
    c1 = {2: -(1 - Fraction(4, 5)) + Fraction(4, 5), 0: Fraction(8, 9)}
    gb = [float(c0.get(w, 0) + c1.get(w, 0)) for w in range(3)]
    assert g["gb"] == pytest.approx(gb, abs=1e-11)
    gWo = [float(c0.get(w, 0) * h0[j] + c1.get(w, 0) * h1[j]) for w in range(3) for j in range(2)]
    assert g["gWo"] == pytest.approx(gWo, abs=1e-11)
    # dh = sum_w c_w Wo[w], Wo = [[4ln2,0],[0,4ln3],[0,0]]
    dh1 = [4 * LN2 * float(c1[0]), 0.0]
    da1 = [dh1[j] * float(h1[j] * (1 - h1[j])) for j in range(2)]
    assert g["da1"] == pytest.approx(da1, abs=1e-11)
    # dh0_j = sum_w c_w Wo[w][j] + sum_i U[i][j] da1_i, U = [[0,(8/3)ln3],[-4ln3,0]]
    dh0 = [4 * LN2 * float(c0[0]) + (-4 * LN3) * da1[1], 4 * LN3 * float(c0[1]) + (8 / 3 * LN3) * da1[0]]
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
    lnq = np.log(np.array([0.5, 0.25, 0.25]))
    r = O.nce_grad_chunk(m, x, y, np.array([0, 2], np.int32), lnq, 0.0, debug=True)
    assert r["J"].ravel() == pytest.approx(g["J"], abs=1e-11)
    two = 2.0  # gradients of the mean over B*T = 2 positions
    assert two * r["ct"].ravel() == pytest.approx([-1 / 55, -1 / 5], abs=1e-12)
    assert two * r["dS"].ravel() == pytest.approx([4 / 5, 4 / 5, 8 / 9, 4 / 5], abs=1e-12)
    assert (two * r["gb"]) == pytest.approx(g["gb"], abs=1e-11)
    assert (two * r["gWo"]).ravel() == pytest.approx(g["gWo"], abs=1e-11)
    assert (two * r["gU"]).ravel() == pytest.approx(g["gU"], abs=1e-11)
    assert (two * r["dA"][1, 0]) == pytest.approx(g["da1"], abs=1e-11)
    assert (two * r["dA"][0, 0]) == pytest.approx(g["da0"], abs=1e-11)
    for w in range(3):
        assert (two * r["gE"][w]) == pytest.approx(g["gE"][w], abs=1e-11)
    assert r["h_next"].ravel() == pytest.approx([0.75, 0.25], abs=1e-13)


def test_zero_output_weights_closed_form():
    """Wo = 0, b = 0, lnZ = 0: D(w) = -ln(K q(w)) whatever the history, so
    J_m = ln(1 + K q(y_m)) + sum_j ln(1 + 1/(K q(n_j)))."""
    V, H, B, T, K = 11, 4, 3, 5, 7
    m = rand_model(V, H, B, 3, h_scale=1.0)
    m.Wo[:] = 0
    m.b[:] = 0
    x, y = rand_tokens(V, T, B, 4)
    q = rand_q(V, 5)
    noise = np.random.default_rng(6).integers(0, V, K).astype(np.int32)
    r = O.nce_grad_chunk(m, x, y, noise, np.log(q))
    want = np.log1p(K * q[y]) + np.log1p(1.0 / (K * q[noise])).sum()
    assert r["J"] == pytest.approx(want, rel=1e-12)
    assert np.abs(r["gE"]).max() == 0 and np.abs(r["gU"]).max() == 0  # nothing flows back through Wo = 0


def nce_loss(m, x, y, noise, lnq, lnZ):
    return O.nce_grad_chunk(m, x, y, noise, lnq, lnZ)["J"].mean()


@pytest.mark.parametrize("V,H,B,T,K,lnZ,seed", [(5, 3, 2, 3, 4, 0.0, 1), (4, 2, 1, 4, 6, 0.7, 2), (7, 4, 2, 2, 3, -0.4, 3)])
def test_finite_differences(V, H, B, T, K, lnZ, seed):
    """Central differences of the mean loss for every entry of E, U, Wo, b; windows with repeated
    input ids, repeated noise words, a noise word equal to a target, and a non-zero carried state."""
    m = rand_model(V, H, B, seed, scale=0.8, h_scale=1.0)
    x, y = rand_tokens(V, T, B, seed + 10)
    x[-1] = x[0]
    noise = np.random.default_rng(seed + 20).integers(0, V, K).astype(np.int32)
    noise[0] = y[0, 0]
    noise[-1] = noise[1]
    lnq = np.log(rand_q(V, seed + 30))
    r = O.nce_grad_chunk(m, x, y, noise, lnq, lnZ)
    eps = 1e-5
    for name, g in (("E", r["gE"]), ("U", r["gU"]), ("Wo", r["gWo"]), ("b", r["gb"])):
        P = getattr(m, name)
        num = np.empty_like(P)
        it = np.nditer(P, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = P[i]
            P[i] = old + eps
            lp = nce_loss(m, x, y, noise, lnq, lnZ)
            P[i] = old - eps
            lm = nce_loss(m, x, y, noise, lnq, lnZ)
            P[i] = old
            num[i] = (lp - lm) / (2 * eps)
        assert g == pytest.approx(num, rel=1e-6, abs=1e-9), name


def test_autograd_of_the_same_loss():
    """The criterion written with fp64 library ops (logsigmoid) and differentiated by autograd."""
    V, H, B, T, K, lnZ = 9, 5, 3, 4, 6, 0.3
    m = rand_model(V, H, B, 7, scale=0.7, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 8)
    noise = np.random.default_rng(9).integers(0, V, K).astype(np.int32)
    lnq = np.log(rand_q(V, 10))
    r = O.nce_grad_chunk(m, x, y, noise, lnq, lnZ)
    E, U, Wo, b = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (m.E, m.U, m.Wo, m.b))
    h = torch.tensor(m.h)
    off = torch.tensor(lnZ + math.log(K) + lnq)
    nz = torch.tensor(noise, dtype=torch.long)
    tot = 0.0
    for t in range(T):
        h = torch.sigmoid(E[torch.tensor(x[t], dtype=torch.long)] + h @ U.T)
        D = h @ Wo.T + b - off                      # [B][V]
        yt = torch.tensor(y[t], dtype=torch.long)
        pos = torch.nn.functional.logsigmoid(D.gather(1, yt[:, None])[:, 0])
        neg = torch.nn.functional.logsigmoid(-D[:, nz]).sum(1)
        tot = tot - (pos + neg).sum()
    (tot / (B * T)).backward()
    assert r["J"].sum() == pytest.approx(tot.item(), rel=1e-12)
    for name, p in (("gE", E), ("gU", U), ("gWo", Wo), ("gb", b)):
        assert r[name] == pytest.approx(p.grad.numpy(), rel=1e-9, abs=1e-12), name


def proportional_noise(q_frac, reps):
    """A noise list in which word w appears exactly K q(w) times: its noise sum equals its expectation."""
    den = np.lcm.reduce([f.denominator for f in q_frac])
    base = np.concatenate([np.full(int(f * den), w, np.int32) for w, f in enumerate(q_frac)])
    return np.tile(base, reps)


def test_large_K_limit_is_maximum_likelihood_single_position():
    """With the model normalised (lnZ = the position's log-partition) and noise counts proportional
    to q, the estimator's gradient tends to the gradient of the normalised criterion as K grows
    (error of order p(w)/(K q(w))): compared with the already pinned full-softmax gradient, all four
    parameter groups, non-zero carried state."""
    V, H = 4, 3
    qf = [Fraction(1, 2), Fraction(1, 4), Fraction(1, 8), Fraction(1, 8)]
    lnq = np.log(np.array([float(f) for f in qf]))
    m = rand_model(V, H, 1, 21, scale=0.9, h_scale=1.0)
    x = np.array([[2]], np.int32)
    y = np.array([[1]], np.int32)
    ref = O.grad_chunk(m, x, y, debug=True)
    z = ref["Hs"][0, 0] @ m.Wo.T + m.b
    lnZ = ref["logp"][0, 0] * -1 + z[1]          # log-partition = z_y - log p(y)
    errs = []
    for reps in (2 ** 8, 2 ** 14):
        noise = proportional_noise(qf, reps)
        r = O.nce_grad_chunk(m, x, y, noise, lnq, lnZ)
        errs.append(max(np.abs(r[k] - ref[k]).max() / np.abs(ref[k]).max() for k in ("gE", "gU", "gWo", "gb")))
    assert errs[1] < 2e-4 and errs[1] < errs[0] / 30   # first-order convergence in 1/K


def test_large_K_limit_is_maximum_likelihood_whole_window():
    """Wo = 0 and b = ln p with sum p = 1: every position is normalised with lnZ = 0, so the same limit
    holds for a whole multi-stream window (gWo and gb are non-zero, nothing flows into E and U)."""
    V, H, B, T = 4, 3, 2, 3
    qf = [Fraction(1, 4), Fraction(1, 4), Fraction(3, 8), Fraction(1, 8)]
    lnq = np.log(np.array([float(f) for f in qf]))
    m = rand_model(V, H, B, 22, h_scale=1.0)
    m.Wo[:] = 0
    m.b[:] = np.log(np.array([0.1, 0.2, 0.3, 0.4]))
    x, y = rand_tokens(V, T, B, 23)
    ref = O.grad_chunk(m, x, y)
    r = O.nce_grad_chunk(m, x, y, proportional_noise(qf, 2 ** 14), lnq, 0.0)
    for k in ("gWo", "gb"):
        assert np.abs(r[k] - ref[k]).max() < 2e-4 * np.abs(ref[k]).max(), k


def test_shift_of_bias_and_normaliser_cancels():
    V, H, B, T, K = 8, 4, 2, 3, 5
    m = rand_model(V, H, B, 31, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 32)
    noise = np.random.default_rng(33).integers(0, V, K).astype(np.int32)
    lnq = np.log(rand_q(V, 34))
    a = O.nce_grad_chunk(m, x, y, noise, lnq, 0.25)
    m2 = m.copy()
    m2.b += 1.5
    b_ = O.nce_grad_chunk(m2, x, y, noise, lnq, 1.75)
    for k in ("J", "gE", "gU", "gWo", "gb"):
        assert a[k] == pytest.approx(b_[k], rel=1e-12, abs=1e-14), k


def test_noise_order_and_relabelling_do_not_matter():
    V, H, B, T, K = 9, 4, 2, 3, 6
    m = rand_model(V, H, B, 41, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 42)
    noise = np.random.default_rng(43).integers(0, V, K).astype(np.int32)
    lnq = np.log(rand_q(V, 44))
    a = O.nce_grad_chunk(m, x, y, noise, lnq, 0.1)
    b_ = O.nce_grad_chunk(m, x, y, noise[::-1].copy(), lnq, 0.1)
    for k in ("J", "gE", "gU", "gWo", "gb"):
        assert a[k] == pytest.approx(b_[k], rel=1e-12, abs=1e-14), k
    perm = np.random.default_rng(45).permutation(V)           # new id of word w is perm[w]
    inv = np.argsort(perm)
    m2 = O.Model(m.E[inv].copy(), m.U.copy(), m.Wo[inv].copy(), m.b[inv].copy(), m.h.copy())
    c = O.nce_grad_chunk(m2, perm[x].astype(np.int32), perm[y].astype(np.int32), perm[noise].astype(np.int32),
                         lnq[inv].copy(), 0.1)
    assert a["J"] == pytest.approx(c["J"], rel=1e-12)
    assert a["gWo"] == pytest.approx(c["gWo"][perm], rel=1e-12, abs=1e-14)
    assert a["gU"] == pytest.approx(c["gU"], rel=1e-12, abs=1e-14)


def test_streams_are_independent():
    V, H, B, T, K = 8, 3, 3, 4, 5
    m = rand_model(V, H, B, 51, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 52)
    noise = np.random.default_rng(53).integers(0, V, K).astype(np.int32)
    lnq = np.log(rand_q(V, 54))
    full = O.nce_grad_chunk(m, x, y, noise, lnq, 0.0)
    acc = {k: 0.0 for k in ("gE", "gU", "gWo", "gb")}
    for s in range(B):
        ms = O.Model(m.E, m.U, m.Wo, m.b, m.h[s:s + 1].copy())
        one = O.nce_grad_chunk(ms, x[:, s:s + 1].copy(), y[:, s:s + 1].copy(), noise, lnq, 0.0)
        assert one["J"][:, 0] == pytest.approx(full["J"][:, s], rel=1e-12)
        for k in acc:
            acc[k] = acc[k] + one[k] / B
    for k in acc:
        assert full[k] == pytest.approx(acc[k], rel=1e-11, abs=1e-14), k


def test_sgd_identity_and_state_advance():
    V, H, B, T, K, lr = 10, 4, 2, 3, 5, 0.3
    m = rand_model(V, H, B, 61, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 62)
    noise = np.random.default_rng(63).integers(0, V, K).astype(np.int32)
    lnq = np.log(rand_q(V, 64))
    g = O.nce_grad_chunk(m, x, y, noise, lnq, 0.2)
    m1 = m.copy()
    J, sJ = O.nce_train_chunk(m1, x, y, noise, lnq, 0.2, lr)
    assert J == pytest.approx(g["J"], rel=1e-14) and sJ == pytest.approx(g["J"].sum(), rel=1e-13)
    for name, gn in (("E", "gE"), ("U", "gU"), ("Wo", "gWo"), ("b", "gb")):
        assert np.array_equal(getattr(m1, name), getattr(m, name) - lr * g[gn]), name
    assert np.array_equal(m1.h, g["h_next"])
    m0 = m.copy()
    O.nce_train_chunk(m0, x, y, noise, lnq, 0.2, 0.0)
    assert all(np.array_equal(getattr(m0, n), getattr(m, n)) for n in ("E", "U", "Wo", "b"))
    assert np.array_equal(m0.h, g["h_next"])


def test_out_of_range_noise_is_rejected():
    m = rand_model(5, 2, 1, 71)
    x, y = rand_tokens(5, 2, 1, 72)
    with pytest.raises(ValueError):
        O.nce_grad_chunk(m, x, y, np.array([0, 5], np.int32), np.log(rand_q(5, 73)))


# ---- unnormalised forward scoring (Sec. 4.2: the output as used for rescoring) -------------------------

def test_score_worked_example():
    """On the hand-computed model the scores are logs of small integers: z0 = [ln4, ln27, ln2],
    z1 = [ln8, ln3, ln2]."""
    x = np.array([[0], [1]], np.int32)
    for y, want in (([1, 2], [math.log(27), math.log(2)]), ([0, 0], [math.log(4), math.log(8)]),
                    ([2, 1], [math.log(2), math.log(3)])):
        m = worked_model()
        s = O.forward_score(m, x, np.array(y, np.int32).reshape(2, 1), lnZ=0.5)
        assert s.ravel() == pytest.approx([w - 0.5 for w in want], abs=1e-12)
        assert m.h.ravel() == pytest.approx([0.75, 0.25], abs=1e-13)


def test_score_differs_from_log_probability_by_the_log_partition():
    """score + lnZ - logp is the position's log-partition, the same whatever next word is asked for; it
    equals logsumexp of the scores of all words."""
    V, H, B, T = 13, 5, 3, 4
    m = rand_model(V, H, B, 81, h_scale=1.0)
    x, _ = rand_tokens(V, T, B, 82)
    allz = np.empty((V, T, B))
    lses = []
    for w in range(V):
        y = np.full((T, B), w, np.int32)
        s = O.forward_score(m.copy(), x, y, lnZ=0.0)
        lp = O.forward_logprob(m.copy(), x, y)
        allz[w] = s
        lses.append(s - lp)
    for w in range(1, V):
        assert lses[w] == pytest.approx(lses[0], rel=1e-12, abs=1e-12)
    from scipy.special import logsumexp
    assert lses[0] == pytest.approx(logsumexp(allz, axis=0), rel=1e-12)


def test_score_advances_state_like_the_normalised_pass_and_chains():
    V, H, B, T = 9, 4, 2, 6
    m = rand_model(V, H, B, 91, h_scale=1.0)
    x, y = rand_tokens(V, T, B, 92)
    a, b_ = m.copy(), m.copy()
    whole = O.forward_score(a, x, y, 0.3)
    O.forward_logprob(b_, x, y)
    assert np.array_equal(a.h, b_.h)
    c = m.copy()
    parts = np.concatenate([O.forward_score(c, x[t:t + 1], y[t:t + 1], 0.3) for t in range(T)])
    assert parts == pytest.approx(whole, rel=1e-13)


def test_shortlist_scores_normalise_to_the_pinned_distribution():
    """With every word on the shortlist, score - logsumexp(score) is the pinned normalised log-probability,
    whatever lnZ; the order of the candidates does not matter; the state advances as in a forward pass."""
    m = rand_model(8, 4, 2, 91, scale=0.6, h_scale=1.0)
    x, y = rand_tokens(8, 5, 2, 92)
    allw = np.ascontiguousarray(np.broadcast_to(np.arange(8, dtype=np.int32), (5, 2, 8)))
    a, b_ = m.copy(), m.copy()
    sc = O.forward_score_shortlist(a, x, allw, lnZ=0.9)
    lp = O.forward_logprob(b_, x, y)
    mx = sc.max(axis=2, keepdims=True)
    lse = mx[:, :, 0] + np.log(np.exp(sc - mx).sum(axis=2))
    picked = np.take_along_axis(sc, y[:, :, None].astype(np.int64), axis=2)[:, :, 0]
    assert picked - lse == pytest.approx(lp, rel=1e-12, abs=1e-13)
    assert np.array_equal(a.h, b_.h)
    perm = np.random.default_rng(4).permutation(8)
    sc2 = O.forward_score_shortlist(m.copy(), x, np.ascontiguousarray(allw[:, :, perm]), lnZ=0.9)
    assert sc2 == pytest.approx(sc[:, :, perm], rel=1e-14)

