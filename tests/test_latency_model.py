"""Latency model and can_schedule (CPU): planted coefficients come back, can_schedule is the
brute-force answer."""
import numpy as np

from paper_2410_01228_amd.latency_model import LatencyModel, features, fit


def test_features_are_per_request_sums():
    # one chunk of 4 tokens on 10 cached, one decode on 7 cached
    f = features([(4, 10), (1, 7)])
    assert f.tolist() == [5.0, 4 * 14 + 1 * 8, 14 + 8, 1.0]


def test_fit_recovers_planted_coefficients():
    true = LatencyModel(k_p=2e-8, k2=3e-12, k4=5e-10, k5=8e-6)
    rng = np.random.default_rng(1)
    samples = []
    for _ in range(60):
        batch = [(int(rng.integers(1, 2048)), int(rng.integers(0, 30000))) for _ in range(int(rng.integers(1, 6)))]
        samples.append((batch, true.predict(batch)))
    m, rel = fit(samples)
    np.testing.assert_allclose(m.coef, true.coef, rtol=1e-6)
    assert rel.max() < 1e-9


def test_can_schedule_matches_brute_force():
    m = LatencyModel(k_p=2e-8, k2=3e-12, k4=5e-10, k5=8e-6)
    batch = [(1, 4000)] * 64                                   # online decodes already in the batch
    for budget in (1e-5, 5e-5, 2e-4, 1e-3):
        for req_tokens, ctx in ((2048, 0), (2048, 16000), (10, 500)):
            got = m.can_schedule(batch, req_tokens, ctx, budget)
            brute = 0
            for n in range(1, req_tokens + 1):
                if m.predict(batch + [(n, ctx)]) <= budget:
                    brute = n
            assert got == brute
    # more context -> fewer tokens fit (the point of a context-aware model)
    assert m.can_schedule(batch, 2048, 30000, 2e-4) < m.can_schedule(batch, 2048, 0, 2e-4)
    assert m.can_schedule(batch, 2048, 0, 1e-9) == 0


def test_fit_never_returns_a_negative_coefficient():
    """Timings in which the per-token term is not identifiable (noise larger than its effect) must
    come back with that term at zero, not negative -- an unconstrained fit of these samples trades
    it against the constant -- and can_schedule on the result stays monotone in context."""
    import pytest
    true = LatencyModel(k_p=0.0, k2=1.5e-11, k4=6e-10, k5=2.2e-5)
    rng = np.random.default_rng(8)
    samples = []
    for _ in range(40):
        batch = [(int(rng.integers(1, 2048)), int(rng.integers(0, 30000))) for _ in range(int(rng.integers(1, 4)))]
        samples.append((batch, true.predict(batch) * float(1 + 0.05 * rng.standard_normal())))
    A = np.stack([features(b) for b, _ in samples])
    y = np.array([t for _, t in samples])
    free, *_ = np.linalg.lstsq(A / y[:, None], np.ones(len(y)), rcond=None)
    assert free.min() < 0, "the planted case must be one where the unconstrained fit goes negative"
    m, rel = fit(samples)
    assert m.coef.min() >= 0 and rel.mean() < 0.06
    batch = [(1, 4000)] * 64
    fits = [m.can_schedule(batch, 2048, ctx, 5e-4) for ctx in (0, 4000, 16000, 32000)]
    assert fits == sorted(fits, reverse=True) and fits[0] > fits[-1] >= 0
    with pytest.raises(ValueError):
        LatencyModel(k_p=-1e-9, k2=1e-11, k4=1e-10, k5=1e-5).can_schedule(batch, 100, 0, 1e-3)
