"""Pins of the compressed-architecture oracle (Sec. 5.4: 512-unit layers below and above the state, tied
word matrices, quantised weights) against things other than itself (CPU only): the already pinned plain
oracle through the exact factorisation E' = E A^T, Wo' = E C, a hand-computed example, finite differences,
library autograd on an independently written forward pass, and hand-picked rows for the quantiser."""
import math

import numpy as np
import pytest

from oracle import compressed as Cq
from oracle import oracle as O


def rand_cmodel(V, H, P, B, seed, scale=0.6, h_scale=1.0):
    r = np.random.default_rng(seed)
    return Cq.CompressedModel(E=r.normal(0, scale, (V, P)), A=r.normal(0, scale, (H, P)),
                              U=r.normal(0, scale, (H, H)), C=r.normal(0, scale, (P, H)),
                              b=r.normal(0, scale, V), h=h_scale * r.uniform(0, 1, (B, H)))


def rand_tokens(V, T, B, seed):
    r = np.random.default_rng(seed)
    return r.integers(0, V, (T, B)), r.integers(0, V, (T, B))


def plain_equivalent(m):
    """The plain Elman model computing the same function: E' = E A^T, Wo' = E C."""
    p = O.Model(np.ascontiguousarray(m.E @ m.A.T), m.U.copy(), np.ascontiguousarray(m.E @ m.C), m.b.copy(),
                m.h.copy())
    return p


def test_forward_equals_the_plain_oracle_on_the_factorised_matrices():
    m = rand_cmodel(11, 5, 3, 2, 1)
    x, y = rand_tokens(11, 4, 2, 2)
    p = plain_equivalent(m)
    lp_plain = O.forward_logprob(p, x, y)
    lp = Cq.forward_logprob(m, x, y)
    assert lp == pytest.approx(lp_plain, rel=1e-12, abs=1e-13)
    assert m.h == pytest.approx(p.h, rel=1e-12)


def test_gradients_are_the_plain_oracles_pushed_through_the_factorisation():
    """Chain rule on E' = E A^T and Wo' = E C: gA = gE'^T E, gC = E^T gWo', gE = gE' A + gWo' C^T; U and b are
    shared.  The plain gradients come from the pinned oracle.grad_chunk."""
    m = rand_cmodel(13, 6, 4, 3, 3)
    x, y = rand_tokens(13, 5, 3, 4)
    x[0, 0] = x[1, 0] = 7                    # a repeated input id
    y[2, 1] = x[2, 1]                        # a word that is input and target at once
    gp = O.grad_chunk(plain_equivalent(m), x, y)
    g = Cq.grad_chunk(m, x, y)
    assert g["logp"] == pytest.approx(gp["logp"], rel=1e-12, abs=1e-13)
    assert g["gU"] == pytest.approx(gp["gU"], rel=1e-10, abs=1e-14)
    assert g["gb"] == pytest.approx(gp["gb"], rel=1e-10, abs=1e-14)
    assert g["gA"] == pytest.approx(gp["gE"].T @ m.E, rel=1e-10, abs=1e-14)
    assert g["gC"] == pytest.approx(m.E.T @ gp["gWo"], rel=1e-10, abs=1e-14)
    assert g["gE"] == pytest.approx(gp["gE"] @ m.A + gp["gWo"] @ m.C.T, rel=1e-10, abs=1e-14)
    assert g["h_out"] == pytest.approx(gp["h_next"], rel=1e-12)


def test_hand_computed_example():
    """V = 2, P = H = 1, one position, input word 0, target word 0, zero carried state.
    E = [[ln 2], [0]], A = 0, C = 2: h = 1/2, p = 1, z = (ln 2, 0), so P = (2/3, 1/3).
    Loss = -ln(2/3); dz = (-1/3, 1/3); output-role gE = dz * p; dp = dz.E = -ln2/3; gC = dp*h = -ln2/6;
    dh = dp*C = -2 ln2/3; da = dh/4 = -ln2/6; gA = da * x = -(ln2)^2/6; gU = 0 (zero state); dx = da*A = 0."""
    ln2 = math.log(2.0)
    m = Cq.CompressedModel(E=np.array([[ln2], [0.0]]), A=np.array([[0.0]]), U=np.array([[0.3]]),
                           C=np.array([[2.0]]), b=np.zeros(2), h=np.zeros((1, 1)))
    x = np.array([[0]])
    g = Cq.grad_chunk(m, x, np.array([[0]]))
    assert g["logp"][0, 0] == pytest.approx(math.log(2 / 3), rel=1e-14)
    assert Cq.grad_chunk(m, x, np.array([[1]]))["logp"][0, 0] == pytest.approx(math.log(1 / 3), rel=1e-14)
    assert g["gb"] == pytest.approx([-1 / 3, 1 / 3], rel=1e-14)
    assert g["gE"][:, 0] == pytest.approx([-1 / 3, 1 / 3], rel=1e-14)
    assert g["gC"][0, 0] == pytest.approx(-ln2 / 6, rel=1e-14)
    assert g["gA"][0, 0] == pytest.approx(-ln2 * ln2 / 6, rel=1e-14)
    assert g["gU"][0, 0] == 0.0
    assert g["h_out"][0, 0] == 0.5


def window_loss(m, x, y):
    return -Cq.forward_logprob(m.copy(), x, y).mean()


@pytest.mark.parametrize("name", ["E", "A", "U", "C", "b"])
def test_finite_differences(name):
    m = rand_cmodel(7, 4, 3, 2, 11, scale=0.5)
    x, y = rand_tokens(7, 4, 2, 12)
    x[0, 0] = x[2, 0] = 3
    y[1, 1] = 3                              # word 3 is an input (twice) and a target
    g = Cq.grad_chunk(m, x, y)["g" + name]
    eps = 1e-6
    W = getattr(m, name)
    num = np.zeros_like(W)
    it = np.nditer(W, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        old = W[idx]
        W[idx] = old + eps
        lp = window_loss(m, x, y)
        W[idx] = old - eps
        lm = window_loss(m, x, y)
        W[idx] = old
        num[idx] = (lp - lm) / (2 * eps)
    assert g == pytest.approx(num, rel=2e-6, abs=2e-9)


def test_autograd_on_an_independent_forward():
    torch = pytest.importorskip("torch")
    m = rand_cmodel(9, 5, 3, 2, 21)
    x, y = rand_tokens(9, 4, 2, 22)
    x[0, 1] = x[3, 1] = 2
    ps = {n: torch.tensor(getattr(m, n), dtype=torch.float64, requires_grad=True) for n in "EAUCb"}
    h = torch.tensor(m.h, dtype=torch.float64)
    nll = torch.zeros((), dtype=torch.float64)
    for t in range(x.shape[0]):
        emb = torch.nn.functional.embedding(torch.tensor(x[t]), ps["E"])
        h = torch.sigmoid(torch.nn.functional.linear(emb, ps["A"]) + torch.nn.functional.linear(h, ps["U"]))
        logits = torch.nn.functional.linear(torch.nn.functional.linear(h, ps["C"]), ps["E"], ps["b"])
        nll = nll + torch.nn.functional.cross_entropy(logits, torch.tensor(y[t]), reduction="sum")
    (nll / x.size).backward()
    g = Cq.grad_chunk(m, x, y)
    for n in "EAUCb":
        assert g["g" + n] == pytest.approx(ps[n].grad.numpy(), rel=1e-10, abs=1e-14), n


def test_streams_are_independent_and_the_state_carries():
    m = rand_cmodel(8, 4, 3, 3, 31)
    x, y = rand_tokens(8, 6, 3, 32)
    whole = Cq.forward_logprob(m.copy(), x, y)
    a = m.copy()
    two = np.concatenate([Cq.forward_logprob(a, x[:2], y[:2]), Cq.forward_logprob(a, x[2:], y[2:])])
    assert two == pytest.approx(whole, rel=1e-13)
    single = Cq.CompressedModel(m.E, m.A, m.U, m.C, m.b, m.h[1:2].copy())
    assert Cq.forward_logprob(single, x[:, 1:2], y[:, 1:2])[:, 0] == pytest.approx(whole[:, 1], rel=1e-13)


def test_sgd_step_identity_and_training_lowers_the_loss():
    m = rand_cmodel(10, 6, 4, 2, 41, scale=0.3)
    x, y = rand_tokens(10, 5, 2, 42)
    g = Cq.grad_chunk(m, x, y)
    a = m.copy()
    lp = Cq.train_chunk(a, x, y, 0.25)
    assert np.array_equal(lp, g["logp"])
    for n in "EAUCb":
        assert getattr(a, n) == pytest.approx(getattr(m, n) - 0.25 * g["g" + n], rel=1e-15, abs=1e-18), n
    assert np.array_equal(a.h, g["h_out"])
    first = -lp.mean()
    for _ in range(30):
        a.h = m.h.copy()
        last = -Cq.train_chunk(a, x, y, 0.25).mean()
    assert last < 0.7 * first


def test_zero_word_matrix_gives_the_uniform_distribution():
    m = rand_cmodel(12, 4, 3, 2, 51)
    m.E[:] = 0.0
    m.b[:] = 0.0
    tok = np.random.default_rng(5).integers(0, 12, 101)
    ppl, n = Cq.perplexity(m, tok, 5)
    assert n == 100 and ppl == pytest.approx(12.0, rel=1e-13)


def test_shortlist_scores_normalise_to_the_pinned_distribution():
    """With every word on the shortlist, score - logsumexp(score) is the normalised log-probability of the
    pinned forward pass, whatever lnZ; a single candidate is the scoring call of one word."""
    m = rand_cmodel(9, 5, 3, 2, 81)
    x, y = rand_tokens(9, 4, 2, 82)
    allw = np.broadcast_to(np.arange(9), (4, 2, 9)).copy()
    a, b_ = m.copy(), m.copy()
    sc = Cq.forward_score_shortlist(a, x, allw, lnZ=1.7)
    lp = Cq.forward_logprob(b_, x, y)
    mx = sc.max(axis=2, keepdims=True)
    lse = mx[:, :, 0] + np.log(np.exp(sc - mx).sum(axis=2))
    picked = np.take_along_axis(sc, y[:, :, None], axis=2)[:, :, 0]
    assert picked - lse == pytest.approx(lp, rel=1e-12, abs=1e-13)
    assert np.array_equal(a.h, b_.h)
    assert Cq.forward_score(m.copy(), x, y, 1.7) == pytest.approx(picked, rel=1e-14)
    perm = np.random.default_rng(3).permutation(9)           # the order of the candidates does not matter
    sc2 = Cq.forward_score_shortlist(m.copy(), x, allw[:, :, perm], lnZ=1.7)
    assert sc2 == pytest.approx(sc[:, :, perm], rel=1e-14)


# ---- quantiser -------------------------------------------------------------------------------------

def test_quantiser_on_hand_picked_rows():
    """Rows whose largest magnitude is 127 * 2^k have a scale that is an exact power of two, so the codes are
    plain roundings: ties go to the even integer, the sign is kept, zero rows get scale 1 and zero codes."""
    row = np.array([127.0, -63.5, 31.75, 0.5, -0.5, 1.5, 2.5, -2.5, 0.0, 126.49])
    W = np.stack([row, row * 2.0 ** -10, np.zeros_like(row), -row])
    codes, scale = Cq.quantize_rows(W)
    want = np.array([127, -64, 32, 0, 0, 2, 2, -2, 0, 126], np.int8)
    assert scale.dtype == np.float32 and codes.dtype == np.int8
    assert scale.tolist() == [1.0, 2.0 ** -10, 1.0, 1.0]
    assert codes[0].tolist() == want.tolist()
    assert codes[1].tolist() == want.tolist()
    assert codes[2].tolist() == [0] * row.size
    assert codes[3].tolist() == (-want).tolist()


def test_quantiser_error_bound_range_and_stability():
    r = np.random.default_rng(61)
    W = r.normal(0, 0.2, (50, 37)) * r.uniform(0.01, 10, (50, 1))
    codes, scale = Cq.quantize_rows(W)
    assert np.abs(codes.astype(int)).max(axis=1).tolist() == [127] * 50      # the largest entry of a row is +-127
    err = np.abs(Cq.dequantize_rows(codes, scale) - W.astype(np.float32))
    assert (err <= 0.5 * scale[:, None] * (1 + 1e-5)).all()
    codes2, scale2 = Cq.quantize_rows(Cq.dequantize_rows(codes, scale))
    assert np.array_equal(codes2, codes)
    assert scale2 == pytest.approx(scale, rel=2e-7)


def test_quantised_model_of_the_papers_shape_fits_the_stated_size():
    """Sec. 5.4: vocabulary 10K, nstate 1024, 512-unit layers, tied word matrices, at 10 MB.  One byte per
    weight plus one fp32 scale per row plus the fp32 bias."""
    V, H, P = 10_000, 1024, 512
    weights = V * P + H * P + H * H + P * H
    total = weights + 4 * (V + H + H + P) + 4 * V
    assert 7e6 < total < 10e6
    assert 2 * V * H + H * H > 2 * 10e6      # the plain architecture does not fit even at one byte per weight


def test_quantised_model_stays_close_to_the_original():
    m = rand_cmodel(40, 16, 8, 2, 71, scale=0.4)
    x, y = rand_tokens(40, 6, 2, 72)
    q = Cq.quantized(m)
    assert np.abs(q.E - m.E).max() <= np.abs(m.E).max() / 254 * 1.001
    lp = Cq.forward_logprob(m.copy(), x, y)
    lq = Cq.forward_logprob(q, x, y)
    assert np.abs(lp - lq).max() < 0.1 and not np.array_equal(lp, lq)
