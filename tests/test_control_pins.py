"""Pins of the adaptive-control oracle (oracle/control_oracle.py) against what the paper and the mathematics fix.

Golden numbers: tests/golden/table5_latency.txt (the paper's Appendix Table 5).  The break-even acceptance
rates and the speedup below were worked out by hand from those printed values with Eq. 5 (gamma = 3,
gpt-oss-120b column): b=1: beta = 4.341/3.416, c = 0.393/3.416; b=16: beta = 9.345/6.123, c = 0.393/6.123;
b=128: beta = 21.50/11.79, c = 0.393/11.79.
"""
import math
import os

import numpy as np
import pytest

from oracle import control_oracle as CO

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table5_latency.txt")


def load_table5():
    ns, cols, d0 = [], [[], [], [], []], None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "D0":
            d0 = [float(v) for v in f[1:]]
            continue
        ns.append(int(f[0]))
        for j in range(4):
            cols[j].append(None if f[1 + j] == "-" else float(f[1 + j]))
    return ns, cols, d0


def column(j):
    ns, cols, d0 = load_table5()
    keep = [i for i, v in enumerate(cols[j]) if v is not None]
    return [ns[i] for i in keep], [cols[j][i] for i in keep], d0[j]


def test_table5_file_shape():
    ns, cols, d0 = load_table5()
    assert ns == [1, 2, 4, 8, 16, 32, 64, 128, 256, 512]
    assert cols[0][0] == 3.416 and cols[0][-1] == 21.50 and cols[1][-1] is None and d0 == [0.393, 0.137, 0.330, 0.843]
    for j in range(4):      # latency grows with the number of tokens in every column
        v = [x for x in cols[j] if x is not None]
        assert all(b > a for a, b in zip(v, v[1:]))


def test_expected_length_closed_form_and_limits():
    # Eq. 2's closed form against the sum, its limits, and the textbook value for alpha = 1/2
    for gamma in range(0, 9):
        for alpha in (0.0, 0.1, 0.37, 0.5, 0.8, 0.999):
            closed = (1 - alpha ** (gamma + 1)) / (1 - alpha)
            assert CO.expected_accept_length(alpha, gamma) == pytest.approx(closed, rel=1e-13)
        assert CO.expected_accept_length(1.0, gamma) == gamma + 1        # every candidate accepted (+ bonus token)
        assert CO.expected_accept_length(0.0, gamma) == 1.0              # only the target's own token
    assert CO.expected_accept_length(0.5, 3) == 1.875                    # 1 + 1/2 + 1/4 + 1/8
    # strictly increasing in alpha and in gamma
    a = [CO.expected_accept_length(x, 3) for x in np.linspace(0, 1, 21)]
    assert all(y > x for x, y in zip(a, a[1:]))
    assert CO.expected_accept_length(0.7, 4) > CO.expected_accept_length(0.7, 3)


def test_speedup_relations():
    # Eq. 4 is T(b)/SD(b); with T(b(gamma+1)) = T(b) it is Eq. 1 with c = D/T (the paper's own derivation)
    for alpha, gamma, d, t in ((0.6, 3, 0.4, 3.4), (0.8, 5, 1.0, 10.0), (0.3, 1, 0.05, 7.0)):
        assert CO.speedup(alpha, gamma, d, t, t) == pytest.approx(CO.theoretical_speedup(alpha, gamma, d / t), rel=1e-13)
        assert CO.speedup(alpha, gamma, d, t, 1.5 * t) < CO.speedup(alpha, gamma, d, t, t)   # costlier verification hurts
        assert CO.sd_latency(alpha, gamma, d, t) * CO.speedup(alpha, gamma, d, t, t) == pytest.approx(t, rel=1e-13)
    # a free draft that is always right: gamma + 1 tokens per target step
    assert CO.theoretical_speedup(1.0, 3, 0.0) == 4.0
    # a draft that is never right only adds cost
    assert CO.theoretical_speedup(0.0, 3, 0.1) == pytest.approx(1 / 1.3)


def test_practical_speedup_on_table5_worked_values():
    ns, ts, d0 = column(0)          # gpt-oss-120b
    assert CO.practical_speedup(ns, ts, d0, 0.6, 3, 1) == pytest.approx(1.3466, abs(5e-4))
    # hand-computed denominators c*gamma + beta
    for b, den in ((1, 1.6159), (16, 1.7188), (128, 1.9236)):
        e = CO.expected_accept_length(0.5, 3)
        assert e / CO.practical_speedup(ns, ts, d0, 0.5, 3, b) == pytest.approx(den, abs=2e-4)
    # break-even acceptance rates, and that they ARE break-even points
    for b, a0 in ((1, 0.396), (16, 0.440), (128, 0.517)):
        a = CO.min_acceptance(ns, ts, d0, 3, b)
        assert a == pytest.approx(a0, abs=1.5e-3)
        assert CO.practical_speedup(ns, ts, d0, a, 3, b) == pytest.approx(1.0, abs=1e-9)
    # the paper's point: large batches need a better draft (verification gets compute-bound); on the printed
    # numbers the requirement is lowest at b = 1 and highest at b = 128 (it is not monotone in between: 16 vs 32)
    req = [CO.min_acceptance(ns, ts, d0, 3, b) for b in (1, 2, 4, 8, 16, 32, 64, 128)]
    assert min(req) == req[0] and max(req) == req[-1] and req[-1] - req[0] > 0.1
    # Eq. 5 with a flat T(n) (memory-bound: beta = 1) is Eq. 1
    flat = [5.0] * len(ns)
    assert CO.practical_speedup(ns, flat, 0.25, 0.7, 3, 8) == pytest.approx(CO.theoretical_speedup(0.7, 3, 0.25 / 5.0), rel=1e-13)
    # outside the profiled range there is no estimate: b(gamma+1) = 1024 > 512
    assert CO.practical_speedup(ns, ts, d0, 0.7, 3, 256) is None
    assert CO.min_acceptance(ns, ts, d0, 3, 256) is None
    # Qwen3 column stops at 128: b = 32 is the last batch size with gamma = 3
    ns2, ts2, d02 = column(1)
    assert CO.practical_speedup(ns2, ts2, d02, 0.7, 3, 32) is not None and CO.practical_speedup(ns2, ts2, d02, 0.7, 3, 33) is None


def test_profile_interpolation():
    ns, ts, _ = column(0)
    assert CO.profile_latency(ns, ts, 8) == 5.236
    assert CO.profile_latency(ns, ts, 12) == pytest.approx(0.5 * (5.236 + 6.123))
    assert CO.profile_latency(ns, ts, 3) == pytest.approx(0.5 * (3.844 + 4.341))
    assert CO.profile_latency(ns, ts, 0.5) is None and CO.profile_latency(ns, ts, 513) is None
    # break-even where even perfect drafts do not pay / always pay
    assert CO.min_acceptance([1, 4], [1.0, 5.0], 0.1, 3, 1) == 2.0        # beta = 5 > gamma + 1
    assert CO.min_acceptance([1, 4], [1.0, 0.9], 0.01, 3, 1) == 0.0       # c*gamma + beta < 1


def test_controller_hand_traced_run():
    # lambda_short = 1/2, lambda_long = 3/4, epsilon = 0.05, N_init = 2, N_threshold = 4, half of the store trains
    c = CO.Controller(0.5, 0.75, 0.05, 2, 4, 0.5)
    assert c.observe(0.8) == (False, False) and c.short is None
    assert c.observe(0.6) == (False, False)
    assert c.short == pytest.approx(0.7) and c.long == pytest.approx(0.7)            # mean of the first two
    assert c.observe(0.7) == (False, False)                                          # no shift: 0.7 !< 0.65
    assert (c.short, c.long) == (pytest.approx(0.7), pytest.approx(0.7))
    assert c.observe(0.3) == (True, False)     # short 0.5 < long 0.6 - 0.05 -> collection on, this sample stored
    assert (c.short, c.long) == (pytest.approx(0.5), pytest.approx(0.6))
    assert c.collection_enabled
    assert c.observe(0.5) == (True, False)     # short 0.5, long 0.575
    assert c.observe(0.9) == (True, False)     # collection stays on although short 0.7 > long 0.65625
    assert (c.short, c.long) == (pytest.approx(0.7), pytest.approx(0.65625))
    assert c.observe(0.1) == (True, True)      # fourth stored sample: training round
    assert c.train_alpha() == pytest.approx(0.4)                                     # D_train = {0.3, 0.5}
    assert c.observe(0.2) == (False, False)    # nothing is stored while the round runs; the averages still move
    assert c.short == pytest.approx(0.5 * (0.5 * 0.7 + 0.5 * 0.1) + 0.5 * 0.2)
    assert c.report(0.45) == "deploy" and c.collection_enabled and c.stored == []
    # next round: four more samples, evaluation below the training average -> collection off
    flags = [c.observe(a) for a in (0.6, 0.6, 0.2, 0.2)]
    assert flags == [(True, False)] * 3 + [(True, True)]
    assert c.train_alpha() == pytest.approx(0.6)
    assert c.report(0.5) == "stop" and not c.collection_enabled
    assert c.observe(0.6)[0] is False          # off until the next shift
    # equal -> keep, collection unchanged
    c2 = CO.Controller(0.5, 0.75, 0.0, 1, 2, 0.5)
    c2.observe(0.9); c2.observe(0.1); c2.observe(0.1)
    assert c2.awaiting and c2.report(c2.train_alpha()) == "keep" and c2.collection_enabled


def test_controller_no_shift_no_collection():
    rng = np.random.default_rng(7)
    c = CO.Controller(0.8, 0.98, 0.5, 4, 8, 0.75)        # epsilon so large that no shift is ever seen
    assert not any(c.observe(float(a))[0] for a in rng.random(500))
    # a constant stream keeps both averages at that constant
    c = CO.Controller(0.8, 0.98, 0.01, 4, 8, 0.75)
    for _ in range(100):
        c.observe(0.625)
    assert c.short == pytest.approx(0.625, rel=1e-14) and c.long == pytest.approx(0.625, rel=1e-14) and not c.collection_enabled
    # a sustained drop is detected after a few requests, and the EMA obeys Eq. 6's closed form
    for k in range(1, 6):
        c.observe(0.125)
        assert c.short == pytest.approx(0.125 + 0.5 * 0.8 ** k, rel=1e-12)
    assert c.collection_enabled
