"""Seeded generators: determinism and the statistics the workload recipe promises."""
import numpy as np

from paper_1502_00512_amd import synth


def test_counter_rng_is_a_pure_function_of_seed_and_index():
    a = synth.counter_u64(7, 0, 1000)
    b = np.concatenate([synth.counter_u64(7, 0, 400), synth.counter_u64(7, 400, 600)])
    assert np.array_equal(a, b)
    assert not np.array_equal(a, synth.counter_u64(8, 0, 1000))
    assert len(np.unique(a)) == 1000


def test_tokens_deterministic_and_in_range():
    c = synth.CONFIGS["cfg1"]
    t1 = synth.make_tokens(c)
    t2 = synth.make_tokens(c)
    assert t1.dtype == np.int32 and t1.size == c.N
    assert synth.sha256_of(t1) == synth.sha256_of(t2)
    assert t1.min() >= 0 and t1.max() < c.V


def test_zipf_rank_frequency_slope():
    s = 1.1
    tok = synth.zipf_tokens(400_000, 5000, s, 123)
    cnt = np.bincount(tok, minlength=5000).astype(float)
    r = np.arange(1, 51)
    slope = np.polyfit(np.log(r), np.log(cnt[:50]), 1)[0]
    assert abs(slope + s) < 0.05


def test_sentence_marker_rate():
    lam = 20.0
    tok = synth.zipf_tokens(500_000, 10_000, 1.1, 5, sentence_lambda=lam)
    rate = (tok == 0).mean()
    assert abs(rate - 1.0 / (lam + 1.0)) < 0.002
    gaps = np.diff(np.flatnonzero(tok == 0)) - 1
    assert gaps.min() >= 1 and abs(gaps.mean() - lam) < 0.3


def test_markov_variant_keeps_range_and_adds_structure():
    V = 2000
    plain = synth.zipf_tokens(100_000, V, 1.0, 9)
    mk = synth.zipf_tokens(100_000, V, 1.0, 9, markov_contexts=64)
    assert mk.min() >= 0 and mk.max() < V and not np.array_equal(plain, mk)
    assert 0.4 < (plain == mk).mean() < 0.6


def test_weights():
    E, U, Wo, b = synth.make_weights(300, 32, "uniform", 0.1, 77)
    assert E.shape == (300, 32) and U.shape == (32, 32) and Wo.shape == (300, 32) and b.shape == (300,)
    assert E.dtype == np.float32 and abs(E).max() <= 0.1 and not b.any()
    assert not np.array_equal(E, Wo)
    Wn = synth.normal_weights((400, 100), 0.02, 3)
    assert abs(Wn.std() - 0.02) < 5e-4 and abs(Wn.mean()) < 5e-4
    assert np.array_equal(Wn, synth.normal_weights((400, 100), 0.02, 3))
