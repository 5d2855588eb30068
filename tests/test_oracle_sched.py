"""Pins for the scheduling oracle: closed forms and special cases the equations fix
(Sec. 3.2 Eq. 1-2, Sec. 3.3 Eq. 3, Sec. 3.5)."""
import math

import numpy as np
import pytest

from oracle.chunk_sched import ChunkSched


def test_moving_average_closed_form():
    # Eq. 1 unrolled: mu^t = alpha^t mu^0 + (1 - alpha) sum_k alpha^(t-k) mu_hat^k, mu^0 = first sample
    rng = np.random.default_rng(3)
    xs = rng.uniform(10, 500, 25)
    for alpha in (0.0, 0.3, 0.8, 1.0):
        s = ChunkSched([256], alpha)
        for x in xs:
            s.observe(x, 1.0)
        t = len(xs) - 1
        want = alpha ** t * xs[0] + (1 - alpha) * sum(alpha ** (t - k) * xs[k] for k in range(1, t + 1))
        assert s.mu == pytest.approx(want, rel=1e-12)
    # a constant load is a fixed point; alpha = 1 never moves, alpha = 0 follows the last sample
    s = ChunkSched([256], 0.8)
    for _ in range(50):
        s.observe(300, 2.0)
    assert s.mu == pytest.approx(300) and s.predict(300) == pytest.approx(2.0)


def test_g_update_is_the_same_average_at_the_observed_knot_only():
    s = ChunkSched([64, 128, 256, 512], 0.8)
    for k, v in ((64, 1.0), (128, 2.0), (256, 4.0), (512, 8.0)):
        s.observe(k, v)
    before = [s.predict(k) for k in (64, 128, 256, 512)]
    assert before == pytest.approx([1.0, 2.0, 4.0, 8.0])
    s.observe(250, 14.0)           # nearest knot: 256
    after = [s.predict(k) for k in (64, 128, 256, 512)]
    assert after == pytest.approx([1.0, 2.0, 0.8 * 4.0 + 0.2 * 14.0, 8.0])
    s.observe(192, 0.0)            # tie between 128 and 256: the lower knot
    assert s.predict(128) == pytest.approx(0.8 * 2.0) and s.predict(256) == pytest.approx(after[2])


def test_interpolation_and_extrapolation():
    s = ChunkSched([100, 200, 400], 0.5)
    assert s.predict(123) == 0.0                       # nothing observed
    s.observe(200, 3.0)
    assert s.predict(5) == 3.0 and s.predict(1e6) == 3.0   # one knot: a constant
    s.observe(400, 7.0)
    assert s.predict(300) == pytest.approx(5.0)
    assert s.predict(100) == pytest.approx(1.0) and s.predict(600) == pytest.approx(11.0)   # the nearest piece continues
    s.observe(100, 2.0)
    assert s.predict(150) == pytest.approx(2.5) and s.predict(300) == pytest.approx(5.0)


@pytest.mark.parametrize("P", [1, 2, 4])
def test_chunk_size_closed_form_for_an_affine_delay(P):
    # g(x) = a + b x  =>  Eq. 3:  X (A/beta - b/P) = 2 (a + b mu) / P
    a, b = 3.0, 0.02
    A = 8192.0
    for mu, beta in ((1, 2e4), (150, 5e4), (700, 1.2e4)):
        knots = sorted({1, mu, 4096, 16384})          # mu is a knot, so observing it keeps g affine
        s = ChunkSched(knots, 0.0)
        for k in knots:
            s.observe(k, a + b * k)
        s.observe(mu, a + b * mu)                      # alpha = 0: mu becomes the last sample
        assert s.mu == mu
        x_real = 2 * (a + b * mu) / P / (A / beta - b / P)
        got = s.chunk_size(A, beta, P, 1, 8192)
        assert got == min(8192, max(1, math.ceil(x_real - 1e-9)))


def test_chunk_size_limits_and_monotonicity():
    s = ChunkSched([16, 64, 256, 1024, 4096], 0.8)
    for k, v in ((16, 5.0), (64, 5.5), (256, 9.0), (1024, 30.0), (4096, 118.0)):
        s.observe(k, v)
    A = 2 * 4096.0
    # a slow uplink covers the in-cloud delay with a tiny chunk; a very fast one never does within range
    assert s.chunk_size(A, 1.0, 1, 8, 2048) == 8
    assert s.chunk_size(A, 1e12, 1, 8, 2048) == 2048
    # faster uplink -> larger chunk; longer pipeline -> smaller chunk
    xs = [s.chunk_size(A, beta, 1, 1, 4096) for beta in (1e3, 1e4, 1e5, 1e6)]
    assert xs == sorted(xs) and xs[0] < xs[-1]
    ps = [s.chunk_size(A, 1e5, P, 1, 4096) for P in (1, 2, 4, 8)]
    assert ps == sorted(ps, reverse=True) and ps[0] > ps[-1]
    # the returned size satisfies the inequality and its predecessor does not
    X = s.chunk_size(A, 1e5, 2, 1, 4096)
    f = lambda x: x * A / 1e5 - (s.predict(s.mu) + s.predict(s.mu + x)) / 2
    assert f(X) >= 0 > f(X - 1)


def test_parallel_draft_steps_is_the_floor_formula():
    s = ChunkSched([150], 0.8)
    s.observe(150, 40.0)
    # (5*8192/1e3 + 40 + 5*8192/2e3) / 7 = (40.96 + 40 + 20.48) / 7 = 14.49..
    assert s.parallel_draft_steps(5, 8192.0, 1e3, 2e3, 7.0) == 14
    assert s.parallel_draft_steps(5, 8192.0, 1e3, 2e3, 101.44) == 1
    assert s.parallel_draft_steps(5, 8192.0, 1e3, 2e3, 101.45) == 0
    # a table whose continuation is negative at mu: the count stays at 0
    s2 = ChunkSched([100, 200], 0.0)
    s2.observe(100, 1.0); s2.observe(200, 50.0); s2.observe(1, 0.0)   # the last sample moves mu to 1 and the knot at 100 to 0
    assert s2.predict(s2.mu) < 0 and s2.parallel_draft_steps(0, 8192.0, 1e3, 2e3, 5.0) == 0
