"""Oracle for the cloud's state monitor and chunk-size rule (test infrastructure only).

Plain Python, float64, written from the paper's Sec. 3.2 (state monitoring, Eq. 1-2), Sec. 3.3
(prompt chunking, Eq. 3) and Sec. 3.5 (parallel drafting, the lambda equation).  Only tests,
`__graft_entry__.smoke()` and bench.py's cpu_baseline leg may import this module.

What the paper fixes: the two moving averages with weight alpha, the balance equation for
the chunk size, the floor formula for the number of parallel drafting steps.  What it leaves open,
and the reading taken here (the product takes the same readings):

 S1  How g(.) is stored: a table of values at fixed knots (token counts, ascending), evaluated
     by linear interpolation between the knots that have been observed; beyond the first/last
     observed knot the nearest linear piece continues (a single observed knot gives a constant).
 S2  Where Eq. 2 updates g: the delay eta_hat was measured for a batch of mu_hat tokens, so the
     update is applied at x = mu_hat (the equation writes the averaged mu^t; with a steady load
     the two coincide, and a profile built from a sweep of sizes only makes sense this way).
 S3  A point update of a table: the knot nearest to x (ties: the lower one) takes
     g <- alpha * g + (1 - alpha) * eta_hat; a knot that has no history takes eta_hat itself.
     The first mu observation likewise initialises mu.
 S4  The chunk size is an integer in [x_min, x_max]: the smallest X whose upload time X*A/beta_up
     is at least (g(mu) + g(mu + X)) / P -- the first size at which the upload of the next chunk
     covers the in-cloud delay of this one (Eq. 3 holds with equality between X-1 and X);
     x_max if no size in the range does.
 S5  The linear continuation of S1 can dip below zero far from the observed knots; lambda_i is a
     number of inference steps, so the floor formula is clamped at 0.
"""
import math


class ChunkSched:
    def __init__(self, knots, alpha):
        self.knots = [int(k) for k in knots]
        assert len(self.knots) >= 1 and all(b > a for a, b in zip(self.knots, self.knots[1:]))
        assert 0.0 <= alpha <= 1.0
        self.alpha = float(alpha)
        self.g = [None] * len(self.knots)
        self.mu = None

    # ---- Sec. 3.2, Eq. 1 and Eq. 2
    def observe(self, mu_hat, eta_hat):
        a = self.alpha
        self.mu = float(mu_hat) if self.mu is None else a * self.mu + (1.0 - a) * float(mu_hat)
        best = 0
        for k in range(1, len(self.knots)):
            if abs(self.knots[k] - mu_hat) < abs(self.knots[best] - mu_hat):
                best = k
        old = self.g[best]
        self.g[best] = float(eta_hat) if old is None else a * old + (1.0 - a) * float(eta_hat)

    # ---- g(x), reading S1
    def predict(self, x):
        pts = [(k, v) for k, v in zip(self.knots, self.g) if v is not None]
        if not pts:
            return 0.0
        if len(pts) == 1:
            return pts[0][1]
        j = 0
        while j + 2 < len(pts) and x > pts[j + 1][0]:
            j += 1
        (x0, y0), (x1, y1) = pts[j], pts[j + 1]
        return y0 + (y1 - y0) * (x - x0) / (x1 - x0)

    # ---- Sec. 3.3, Eq. 3 (reading S4): brute force over the integers
    def chunk_size(self, bytes_per_token, beta_up, pipeline_len, x_min, x_max):
        mu = 0.0 if self.mu is None else self.mu
        wait = self.predict(mu)
        for X in range(x_min, x_max + 1):
            upload = X * bytes_per_token / beta_up
            in_cloud = (wait + self.predict(mu + X)) / pipeline_len
            if upload >= in_cloud:
                return X
        return x_max

    # ---- Sec. 3.5, the lambda equation
    def parallel_draft_steps(self, draft_len, bytes_per_token, beta_up, beta_down, gamma):
        mu = 0.0 if self.mu is None else self.mu
        t = draft_len * bytes_per_token / beta_up + self.predict(mu) + draft_len * bytes_per_token / beta_down
        return max(0, int(math.floor(t / gamma)))   # a number of steps: not below zero (reading S5)
