"""Plain reference of the adaptive-control formulas (Section 4: Eq. 1-6, Algorithm 1; Appendix Table 5).

TEST INFRASTRUCTURE ONLY: imported by tests; the product (the C library behind include/tide_control.h)
shares no code with it.  Everything is the definition written out in Python floats (IEEE double).
Readings where the paper is silent: T(n) between profiled points is interpolated linearly in n and is
undefined outside the profiled range; D_train is the oldest floor(N_threshold * train_fraction) stored
samples; the first N_init requests only initialise the averages; the store is emptied after a round; the
decay rates, epsilon and the N's are inputs (the paper gives no values).  Pinned in tests/test_control_pins.py.
"""
import math

import numpy as np


def expected_accept_length(alpha, gamma):
    """Eq. 2, as the sum it abbreviates: sum_{i=0..gamma} alpha^i."""
    return float(sum(alpha ** i for i in range(gamma + 1)))


def sd_latency(alpha, gamma, d_b, t_verify):
    """Eq. 3."""
    return (gamma * d_b + t_verify) / expected_accept_length(alpha, gamma)


def theoretical_speedup(alpha, gamma, c):
    """Eq. 1."""
    return expected_accept_length(alpha, gamma) / (c * gamma + 1.0)


def speedup(alpha, gamma, d_b, t_b, t_verify):
    """Eq. 4, first line: T(b) / SD(b)."""
    return t_b / sd_latency(alpha, gamma, d_b, t_verify)


def profile_latency(ns, ts, x):
    """T(x): profiled value, linear in n between profiled points, None outside the range."""
    if x < ns[0] or x > ns[-1]:
        return None
    return float(np.interp(x, np.asarray(ns, float), np.asarray(ts, float)))


def practical_speedup(ns, ts, d0, alpha, gamma, batch):
    """Eq. 5 with c(b) = D_0 / T(b), beta(b) = T(b (gamma+1)) / T(b)."""
    tb = profile_latency(ns, ts, batch)
    tv = profile_latency(ns, ts, batch * (gamma + 1))
    if tb is None or tv is None:
        return None
    c, beta = d0 / tb, tv / tb
    return expected_accept_length(alpha, gamma) / (c * gamma + beta)


def min_acceptance(ns, ts, d0, gamma, batch):
    """alpha at which Eq. 5 equals 1: the root in [0,1] of 1 + a + ... + a^gamma = c gamma + beta,
    from the polynomial's roots (numpy.roots).  0 if it already holds at alpha = 0, 2.0 if not even at 1."""
    tb = profile_latency(ns, ts, batch)
    tv = profile_latency(ns, ts, batch * (gamma + 1))
    if tb is None or tv is None:
        return None
    den = (d0 / tb) * gamma + tv / tb
    if den <= 1.0:
        return 0.0
    if den > gamma + 1:
        return 2.0
    coeffs = [1.0] * gamma + [1.0 - den]          # a^gamma + ... + a + (1 - den)
    roots = np.roots(coeffs)
    real = [r.real for r in roots if abs(r.imag) < 1e-9 and -1e-12 <= r.real <= 1.0 + 1e-12]
    return float(min(max(min(real), 0.0), 1.0))


class Controller:
    """Algorithm 1, statement by statement.  observe() returns (store, train_now)."""

    def __init__(self, lambda_short, lambda_long, epsilon, n_init, n_threshold, train_fraction):
        self.ls, self.ll, self.eps = lambda_short, lambda_long, epsilon
        self.n_init, self.n_threshold = n_init, n_threshold
        self.n_train = min(max(int(math.floor(n_threshold * train_fraction)), 1), n_threshold - 1)
        self.first = []               # acceptance rates of the first N_init requests
        self.short = self.long = None
        self.collection_enabled = False
        self.stored = []              # alpha of every stored sample, oldest first
        self.awaiting = False

    def observe(self, alpha):
        if self.short is None:
            self.first.append(alpha)
            if len(self.first) == self.n_init:
                self.short = self.long = sum(self.first) / self.n_init
            return False, False
        self.short = self.ls * self.short + (1 - self.ls) * alpha       # Eq. 6, short time scale
        self.long = self.ll * self.long + (1 - self.ll) * alpha         # Eq. 6, long time scale
        if self.short < self.long - self.eps:
            self.collection_enabled = True
        store = train = False
        if self.collection_enabled and not self.awaiting:
            self.stored.append(alpha)
            store = True
            if len(self.stored) >= self.n_threshold:
                train = True
                self.awaiting = True
        return store, train

    def train_alpha(self):
        d_train = self.stored[:self.n_train]
        return sum(d_train) / len(d_train) if d_train else None

    def report(self, alpha_eval):
        """Deploy gate: 'deploy' if eval > train, 'stop' (collection off) if eval < train, else 'keep'."""
        assert self.awaiting
        a_train = self.train_alpha()
        if alpha_eval > a_train:
            out = "deploy"
        elif alpha_eval < a_train:
            out = "stop"
            self.collection_enabled = False
        else:
            out = "keep"
        self.stored = []
        self.awaiting = False
        return out
