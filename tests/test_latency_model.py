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
