"""hat_sched_* (host code of the library) against the scheduling oracle on the same seeded sample
streams: moving averages and predictions to rounding, chunk sizes and drafting-step counts exactly.
Runs without a GPU."""
import numpy as np
import pytest

from oracle.chunk_sched import ChunkSched


@pytest.fixture(scope="module")
def HatSched():
    import os
    from paper_2503_18989_amd.binding import lib_path
    if not os.path.exists(lib_path()):
        from paper_2503_18989_amd.build import build
        build(verbose=False)
    from paper_2503_18989_amd import HatSched
    return HatSched


def delay_curve(x):
    """The shape the paper reports (Sec. 2.3): nearly flat below ~32 tokens, linear past ~512."""
    return 4.0 + 0.03 * np.maximum(x - 24.0, 0.0) + 0.0005 * np.minimum(x, 512.0)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_streams_of_observations_and_queries(HatSched, seed):
    rng = np.random.default_rng(seed)
    knots = sorted(set(int(k) for k in rng.choice(np.arange(1, 9000), size=int(rng.integers(1, 12)), replace=False)))
    alpha = float(rng.choice([0.0, 0.5, 0.8, 0.95, 1.0]))
    ref, got = ChunkSched(knots, alpha), HatSched(knots, alpha)
    A = 2 * 4096.0
    for step in range(300):
        # before any observation, and after each one, both answer the same questions identically
        if step:
            mu_hat = float(rng.choice([rng.integers(1, 40), rng.integers(100, 600), rng.integers(600, 9000)]))
            eta_hat = float(delay_curve(mu_hat) * rng.uniform(0.9, 1.1))
            ref.observe(mu_hat, eta_hat); got.observe(mu_hat, eta_hat)
            assert got.mu == pytest.approx(ref.mu, rel=1e-13)
        for x in rng.uniform(0, 12000, 4):
            assert got.predict(x) == pytest.approx(ref.predict(x), rel=1e-12, abs=1e-12)
        beta = float(10 ** rng.uniform(2, 6))
        P = int(rng.choice([1, 2, 4, 8]))
        lo = int(rng.integers(1, 64)); hi = lo + int(rng.integers(0, 8192))
        assert got.chunk_size(A, beta, P, lo, hi) == ref.chunk_size(A, beta, P, lo, hi)
        gamma = float(rng.uniform(2, 60))
        assert got.parallel_draft_steps(5, A, beta, 2 * beta, gamma) == ref.parallel_draft_steps(5, A, beta, 2 * beta, gamma)
    got.close()


def test_non_monotone_table_still_returns_the_first_size_that_satisfies_the_rule(HatSched):
    # a delay table with a dip: the rule's left-most solution, not just any root
    knots = [10, 100, 200, 300, 1000]
    vals = [50.0, 60.0, 10.0, 80.0, 90.0]
    ref, got = ChunkSched(knots, 0.0), HatSched(knots, 0.0)
    for k, v in zip(knots, vals):
        ref.observe(k, v); got.observe(k, v)
    ref.observe(10, 50.0); got.observe(10, 50.0)          # mu = 10
    for beta in (200.0, 500.0, 800.0, 1500.0, 4000.0, 1e5):
        for P in (1, 2):
            assert got.chunk_size(100.0, beta, P, 1, 2000) == ref.chunk_size(100.0, beta, P, 1, 2000)
    got.close()


def test_invalid_arguments_are_refused(HatSched):
    with pytest.raises(ValueError):
        HatSched([], 0.8)
    with pytest.raises(ValueError):
        HatSched([4, 4], 0.8)
    with pytest.raises(ValueError):
        HatSched([1, 2], 1.5)
    s = HatSched([64, 256], 0.8)
    with pytest.raises(ValueError):
        s.observe(float("nan"), 1.0)
    with pytest.raises(ValueError):
        s.chunk_size(8192.0, 0.0, 1, 1, 10)
    with pytest.raises(ValueError):
        s.chunk_size(8192.0, 1.0, 0, 1, 10)
    with pytest.raises(ValueError):
        s.chunk_size(8192.0, 1.0, 1, 5, 4)
    with pytest.raises(ValueError):
        s.parallel_draft_steps(5, 8192.0, 1.0, 1.0, 0.0)
    s.close()
