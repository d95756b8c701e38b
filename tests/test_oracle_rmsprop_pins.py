"""Pins of the oracle's rmsprop step (Sec. 4.2: SGD with rmsprop, one statistic per word for the
input-to-state and state-to-output matrices) against things other than itself (CPU only).  The gradients
it scales come from the already pinned oracle.grad_chunk; what is pinned here is the scaling: special
cases that reduce to the pinned plain SGD step, closed forms of the first step and of the running mean,
and which parameters share a statistic."""
import math

import numpy as np
import pytest

from oracle import oracle as O
from test_oracle_pins import rand_model, rand_tokens


def setup(seed=1, V=9, H=4, B=2, T=3):
    m = rand_model(V, H, B, seed, scale=0.7, h_scale=1.0)
    x, y = rand_tokens(V, T, B, seed + 1)
    x[:, 0] = [0, 1, 0][:T]           # a repeated input id; ids V-1, V-2 never occur as inputs
    x[x >= V - 2] = 2
    return m, x, y


def test_frozen_unit_statistics_give_plain_sgd():
    """rho = 1 freezes the statistics; with r = 1 and eps = 0 every denominator is 1: the step is the
    pinned plain SGD step, for all four parameter groups."""
    m, x, y = setup()
    a, b_ = m.copy(), m.copy()
    st = O.RmspropState.filled(m.V, m.H, 1.0)
    lp1, s1 = O.train_chunk_rmsprop(a, st, x, y, 0.3, 1.0, 0.0)
    lp2, s2 = O.train_chunk(b_, x, y, 0.3)
    assert np.array_equal(lp1, lp2) and s1 == s2
    for n in ("E", "U", "Wo", "b", "h"):
        assert getattr(a, n) == pytest.approx(getattr(b_, n), rel=1e-15, abs=1e-18), n
    assert all((getattr(st, n) == 1.0).all() for n in ("rE", "rU", "rWo", "rb"))


def test_frozen_statistics_rescale_the_learning_rate():
    """rho = 1, r = c^2, eps = e: the step is plain SGD with rate lr / (c + e) (pins the square root and
    where eps sits)."""
    m, x, y = setup(3)
    c, e, lr = 0.37, 0.05, 0.2
    a, b_ = m.copy(), m.copy()
    st = O.RmspropState.filled(m.V, m.H, c * c)
    O.train_chunk_rmsprop(a, st, x, y, lr, 1.0, e)
    O.train_chunk(b_, x, y, lr / (c + e))
    for n in ("E", "U", "Wo", "b"):
        assert getattr(a, n) == pytest.approx(getattr(b_, n), rel=1e-13, abs=1e-16), n


def test_first_step_from_zero_statistics_has_a_closed_form():
    """r = 0, eps = 0: element-wise groups (U, b) move every entry by exactly lr / sqrt(1 - rho) against the
    sign of its gradient, whatever its size; word-wise groups (E, Wo) move each touched row along its
    gradient with Euclidean length lr * sqrt(H) / sqrt(1 - rho); untouched rows of E do not move."""
    m, x, y = setup(5)
    lr, rho = 0.01, 0.9
    g = O.grad_chunk(m, x, y)
    a = m.copy()
    st = O.RmspropState.filled(m.V, m.H, 0.0)
    O.train_chunk_rmsprop(a, st, x, y, lr, rho, 0.0)
    step = lr / math.sqrt(1 - rho)
    assert (a.U - m.U) == pytest.approx(-step * np.sign(g["gU"]), rel=1e-12)
    assert (a.b - m.b) == pytest.approx(-step * np.sign(g["gb"]), rel=1e-12)
    for name, gn in (("Wo", "gWo"), ("E", "gE")):
        d = getattr(a, name) - getattr(m, name)
        for w in range(m.V):
            gw = g[gn][w]
            if np.abs(gw).max() == 0:
                assert not d[w].any()
                continue
            assert np.linalg.norm(d[w]) == pytest.approx(step * math.sqrt(m.H), rel=1e-12)
            cos = -(d[w] @ gw) / (np.linalg.norm(d[w]) * np.linalg.norm(gw))
            assert cos == pytest.approx(1.0, abs=1e-12)
    unseen = np.setdiff1d(np.arange(m.V), x.ravel())
    assert unseen.size >= 2 and not (a.E[unseen] - m.E[unseen]).any()


def test_running_mean_is_a_geometric_series():
    """With lr = 0 and the carried state put back, every step sees the same gradient g, so after n steps
    r_n = rho^n r_0 + (1 - rho^n) s with s = g^2 (U, b) or the row mean of g^2 (E, Wo); for words with a
    zero gradient row the statistic just decays: r_n = rho^n r_0."""
    m, x, y = setup(7)
    rho, r0 = 0.8, 0.3
    g = O.grad_chunk(m, x, y)
    st = O.RmspropState.filled(m.V, m.H, r0)
    a = m.copy()
    for n in range(1, 5):
        a.h[:] = m.h
        O.train_chunk_rmsprop(a, st, x, y, 0.0, rho, 1e-3)
        f = rho ** n
        assert st.rU == pytest.approx(f * r0 + (1 - f) * g["gU"] ** 2, rel=1e-12)
        assert st.rb == pytest.approx(f * r0 + (1 - f) * g["gb"] ** 2, rel=1e-12)
        assert st.rWo == pytest.approx(f * r0 + (1 - f) * (g["gWo"] ** 2).mean(axis=1), rel=1e-12)
        assert st.rE == pytest.approx(f * r0 + (1 - f) * (g["gE"] ** 2).mean(axis=1), rel=1e-12)
    for n in ("E", "U", "Wo", "b"):
        assert np.array_equal(getattr(a, n), getattr(m, n))      # lr = 0 moves nothing
    unseen = np.setdiff1d(np.arange(m.V), x.ravel())
    assert st.rE[unseen] == pytest.approx(rho ** 4 * r0, rel=1e-13)


def test_statistic_is_updated_before_it_is_used():
    """One step from r_0 with the smoothing constant of Sec. 4.2 (0.9995): the denominator is
    sqrt(rho r_0 + (1 - rho) g^2) + eps, not sqrt(r_0) + eps — checked on the bias, whose gradient and
    update are scalars per word."""
    m, x, y = setup(9)
    lr, rho, eps, r0 = 0.05, 0.9995, 1e-4, 2e-4
    g = O.grad_chunk(m, x, y)["gb"]
    a = m.copy()
    st = O.RmspropState.filled(m.V, m.H, r0)
    O.train_chunk_rmsprop(a, st, x, y, lr, rho, eps)
    want_new = m.b - lr * g / (np.sqrt(rho * r0 + (1 - rho) * g * g) + eps)
    want_old = m.b - lr * g / (math.sqrt(r0) + eps)
    assert a.b == pytest.approx(want_new, rel=1e-13)
    assert np.abs(a.b - want_old).max() > 1e-6      # the two orders are distinguishable here


def test_training_with_rmsprop_lowers_the_loss():
    V, H, B, T = 30, 8, 4, 5
    m = rand_model(V, H, B, 11, scale=0.3)
    st = O.RmspropState.filled(V, H, 1e-4)
    tok = np.random.default_rng(12).integers(0, V, 400).astype(np.int32)
    first = last = None
    for ep in range(6):
        m.h[:] = 0
        tot = 0.0
        for k in range(O.num_chunks(tok.size, B, T)):
            x, y = O.stream_chunk(tok, B, T, k)
            tot += O.train_chunk_rmsprop(m, st, x, y, 0.003, 0.95, 1e-6)[1]
        first = tot if first is None else first
        last = tot
    assert last > first   # summed log-probability of the training text rises


# ---- the paper's own combination: noise-contrastive criterion + rmsprop (Sec. 4.2) ----------------------

def nce_inputs(m, seed):
    r = np.random.default_rng(seed)
    q = r.uniform(0.2, 1.0, m.V)
    return r.integers(0, m.V - 2, 5).astype(np.int32), np.log(q / q.sum())


def test_nce_rmsprop_with_frozen_unit_statistics_is_the_pinned_nce_sgd_step():
    m, x, y = setup(21)
    noise, lnq = nce_inputs(m, 22)
    a, b_ = m.copy(), m.copy()
    st = O.RmspropState.filled(m.V, m.H, 1.0)
    J1, s1 = O.nce_train_chunk_rmsprop(a, st, x, y, noise, lnq, 0.3, 0.2, 1.0, 0.0)
    J2, s2 = O.nce_train_chunk(b_, x, y, noise, lnq, 0.3, 0.2)
    assert np.array_equal(J1, J2) and s1 == s2
    for n in ("E", "U", "Wo", "b", "h"):
        assert getattr(a, n) == pytest.approx(getattr(b_, n), rel=1e-15, abs=1e-18), n


def test_nce_rmsprop_scales_the_pinned_nce_gradient():
    """First step from r = 0, eps = 0: touched rows of Wo move along the NCE gradient with length
    lr*sqrt(H)/sqrt(1-rho), touched biases by lr/sqrt(1-rho) against the gradient's sign; words that are
    neither target nor noise keep row, bias, and a statistic that only decays."""
    m, x, y = setup(23)
    noise, lnq = nce_inputs(m, 24)
    lr, rho = 0.01, 0.9
    g = O.nce_grad_chunk(m, x, y, noise, lnq, 0.1)
    a = m.copy()
    st = O.RmspropState.filled(m.V, m.H, 0.0)
    st.rWo[:] = 0.5
    st.rb[:] = 0.5
    touched = np.zeros(m.V, bool)
    touched[np.concatenate([y.ravel(), noise])] = True
    st.rWo[touched] = 0.0
    st.rb[touched] = 0.0
    O.nce_train_chunk_rmsprop(a, st, x, y, noise, lnq, 0.1, lr, rho, 0.0)
    step = lr / math.sqrt(1 - rho)
    for w in range(m.V):
        d = a.Wo[w] - m.Wo[w]
        if not touched[w]:
            assert not d.any() and a.b[w] == m.b[w]
            assert st.rWo[w] == pytest.approx(0.5 * rho) and st.rb[w] == pytest.approx(0.5 * rho)
            continue
        assert np.linalg.norm(d) == pytest.approx(step * math.sqrt(m.H), rel=1e-12)
        assert -(d @ g["gWo"][w]) / (np.linalg.norm(d) * np.linalg.norm(g["gWo"][w])) == pytest.approx(1.0, abs=1e-12)
        assert a.b[w] - m.b[w] == pytest.approx(-step * np.sign(g["gb"][w]), rel=1e-12)
    assert (~touched).sum() >= 1
