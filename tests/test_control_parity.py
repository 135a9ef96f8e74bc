"""The C adaptive-control library (include/tide_control.h) against the Python oracle, through the C ABI.
Host-only code on both sides, so these run without a GPU."""
import math
import os
import re

import numpy as np
import pytest

from oracle import control_oracle as CO
from tests.test_control_pins import column

ctl = pytest.importorskip("paper_2602_05145_amd.control")

HDR = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "tide_control.h")


def test_library_exports_every_declared_symbol():
    text = re.sub(r"/\*.*?\*/", "", open(HDR).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(tide_[a-z_0-9]+)\s*\(", text)))
    assert names and set(names) == set(ctl.EXPORTED)
    for n in names:
        assert hasattr(ctl.lib(), n), n


def test_closed_forms_match_oracle():
    rng = np.random.default_rng(11)
    for _ in range(300):
        alpha, gamma = float(rng.random()), int(rng.integers(0, 9))
        d, t, tv = float(rng.uniform(0.01, 2)), float(rng.uniform(1, 30)), float(rng.uniform(1, 90))
        c = d / t
        assert ctl.tide_expected_accept_length(alpha, gamma) == pytest.approx(CO.expected_accept_length(alpha, gamma), rel=1e-14)
        assert ctl.tide_sd_latency(alpha, gamma, d, tv) == pytest.approx(CO.sd_latency(alpha, gamma, d, tv), rel=1e-14)
        assert ctl.tide_theoretical_speedup(alpha, gamma, c) == pytest.approx(CO.theoretical_speedup(alpha, gamma, c), rel=1e-14)
        assert ctl.tide_speedup(alpha, gamma, d, t, tv) == pytest.approx(CO.speedup(alpha, gamma, d, t, tv), rel=1e-14)
    for gamma in range(6):
        assert ctl.tide_expected_accept_length(1.0, gamma) == gamma + 1
        assert ctl.tide_expected_accept_length(0.0, gamma) == 1.0
    for bad in ((-0.1, 3), (1.1, 3), (0.5, -1), (float("nan"), 3)):
        assert math.isnan(ctl.tide_expected_accept_length(*bad))
    assert math.isnan(ctl.tide_sd_latency(0.5, 3, 0.1, 0.0)) and math.isnan(ctl.tide_speedup(0.5, 3, 0.1, 0.0, 1.0))
    assert math.isnan(ctl.tide_theoretical_speedup(0.5, 3, -1.0))


@pytest.mark.parametrize("col", [0, 1, 2, 3])
def test_profiled_model_matches_oracle_on_table5(col):
    ns, ts, d0 = column(col)
    p, keep = ctl.make_profile(ns, ts, d0)
    for x in [1, 1.5, 2, 3, 7, 8, 100, ns[-1], ns[-1] - 0.25]:
        assert ctl.tide_profile_latency(p, x) == pytest.approx(CO.profile_latency(ns, ts, x), rel=1e-14)
    for x in (0, 0.99, ns[-1] + 1):
        assert math.isnan(ctl.tide_profile_latency(p, x)) and CO.profile_latency(ns, ts, x) is None
    for gamma in (1, 3, 5, 7):
        for b in (1, 2, 3, 5, 8, 16, 31, 32, 33, 64, 100, 128, 256, 512, 513):
            want = CO.practical_speedup(ns, ts, d0, 0.65, gamma, b)
            got = ctl.tide_practical_speedup(p, 0.65, gamma, b)
            wmin, gmin = CO.min_acceptance(ns, ts, d0, gamma, b), ctl.tide_min_acceptance(p, gamma, b)
            if want is None:
                assert math.isnan(got) and math.isnan(gmin) and wmin is None
                assert ctl.tide_should_speculate(p, 0.65, gamma, b) == 0
                continue
            assert got == pytest.approx(want, rel=1e-13)
            assert gmin == pytest.approx(wmin, abs=1e-9)
            assert ctl.tide_should_speculate(p, 0.65, gamma, b) == int(want > 1.0)
            if 0.0 < wmin < 1.0:       # just above / below break-even
                assert ctl.tide_should_speculate(p, min(1.0, wmin + 1e-6), gamma, b) == 1
                assert ctl.tide_should_speculate(p, max(0.0, wmin - 1e-6), gamma, b) == 0


def test_profile_and_argument_validation():
    good, keep = ctl.make_profile([1, 4, 16], [1.0, 2.0, 4.0], 0.1)
    assert ctl.tide_should_speculate(None, 0.5, 3, 1) == -1
    assert ctl.tide_should_speculate(good, 1.5, 3, 1) == -2 and ctl.tide_should_speculate(good, 0.5, 3, 0) == -2
    assert ctl.tide_should_speculate(good, 0.5, 3, 1, margin=0.0) == -2
    for ns, ts, d0 in (([4, 1], [1.0, 2.0], 0.1), ([1, 4], [1.0, -2.0], 0.1), ([1, 4], [1.0, 2.0], 0.0), ([0, 4], [1.0, 2.0], 0.1)):
        bad, k2 = ctl.make_profile(ns, ts, d0)
        assert math.isnan(ctl.tide_profile_latency(bad, 2)) and math.isnan(ctl.tide_practical_speedup(bad, 0.5, 1, 1))
        assert ctl.tide_should_speculate(bad, 0.5, 1, 1) == -2
    assert math.isnan(ctl.tide_profile_latency(None, 2))
    assert ctl.tide_min_acceptance(*[ctl.make_profile([1, 4], [1.0, 5.0], 0.1)[0]], 3, 1) == 2.0
    assert ctl.tide_min_acceptance(*[ctl.make_profile([1, 4], [1.0, 0.9], 0.01)[0]], 3, 1) == 0.0


def run_both(params, alphas, evals):
    """Feeds the same stream to both controllers; on every training round reports the next value of `evals`
    (or exactly the training average when that value is None).  Returns the C side's trace."""
    ls, ll, eps, n_init, n_thr, frac = params
    o = CO.Controller(ls, ll, eps, n_init, n_thr, frac)
    c = ctl.Controller()
    prm = ctl.ControllerParams(ls, ll, eps, n_init, n_thr, frac)
    assert ctl.tide_controller_init(c, prm) == 0
    assert c.n_train == o.n_train
    trace, ev = [], iter(evals)
    names = {ctl.DEPLOY: "deploy", ctl.STOP_COLLECTING: "stop", ctl.KEEP: "keep"}
    for a in alphas:
        flags = ctl.tide_controller_observe(c, a)
        store, train = o.observe(a)
        assert flags == (ctl.STORE if store else 0) | (ctl.TRAIN if train else 0)
        assert bool(c.collection_enabled) == o.collection_enabled and c.n_stored == len(o.stored)
        if o.short is not None:
            assert c.ema_short == pytest.approx(o.short, rel=1e-14) and c.ema_long == pytest.approx(o.long, rel=1e-14)
        trace.append(flags)
        if train:
            ta = ctl.tide_controller_train_alpha(c)
            assert ta == pytest.approx(o.train_alpha(), rel=1e-14)
            e = next(ev)
            e = ta if e is None else e
            # the oracle gets the same number the C side compares against
            want = o.report(e if e != ta else o.train_alpha())
            got = ctl.tide_controller_report(c, e)
            assert names[got] == want
            trace.append(("round", names[got]))
    return trace


def test_controller_matches_oracle_on_random_streams():
    rng = np.random.default_rng(2026)
    for trial in range(40):
        ls = float(rng.uniform(0.0, 0.9))
        ll = float(rng.uniform(ls + 0.01, 0.995))
        params = (ls, ll, float(rng.uniform(0, 0.08)), int(rng.integers(1, 20)), int(rng.integers(2, 40)), float(rng.uniform(0.05, 0.95)))
        # acceptance rates with a few level shifts, as a change of workload would cause
        levels = rng.uniform(0.2, 0.9, size=6)
        alphas = np.clip(np.repeat(levels, 150) + rng.normal(0, 0.05, 900), 0, 1).tolist()
        evals = [None if rng.random() < 0.15 else float(rng.random()) for _ in range(900)]
        trace = run_both(params, alphas, evals)
        if trial == 0:
            assert any(isinstance(t, tuple) for t in trace)      # at least one training round happened


def test_controller_hand_traced_run_through_c_abi():
    c = ctl.Controller()
    assert ctl.tide_controller_init(c, ctl.ControllerParams(0.5, 0.75, 0.05, 2, 4, 0.5)) == 0
    seq = [(0.8, 0), (0.6, 0), (0.7, 0), (0.3, 1), (0.5, 1), (0.9, 1), (0.1, 3), (0.2, 0)]
    for a, flags in seq:
        assert ctl.tide_controller_observe(c, a) == flags
    assert ctl.tide_controller_train_alpha(c) == pytest.approx(0.4)
    assert ctl.tide_controller_report(c, 0.45) == ctl.DEPLOY and c.collection_enabled == 1 and c.n_stored == 0
    assert ctl.tide_controller_report(c, 0.45) == -2                       # no round outstanding


def test_controller_argument_validation():
    c = ctl.Controller()
    ok = dict(lambda_short=0.5, lambda_long=0.9, epsilon=0.02, n_init=4, n_threshold=8, train_fraction=0.8)
    assert ctl.tide_controller_init(None, ctl.ControllerParams(**ok)) == -1
    assert ctl.tide_controller_init(c, None) == -1
    for k, v in (("lambda_short", 0.95), ("lambda_short", -0.1), ("lambda_long", 1.0), ("epsilon", -1e-3), ("n_init", 0),
                 ("n_threshold", 1), ("train_fraction", 0.0), ("train_fraction", 1.0)):
        assert ctl.tide_controller_init(c, ctl.ControllerParams(**{**ok, k: v})) == -2, (k, v)
    assert ctl.tide_controller_init(c, ctl.ControllerParams(**ok)) == 0
    assert ctl.tide_controller_observe(c, 1.5) == -2 and ctl.tide_controller_observe(c, float("nan")) == -2
    assert c.n_seen == 0
    assert math.isnan(ctl.tide_controller_train_alpha(c))
    # n_train stays inside [1, n_threshold - 1]
    assert ctl.tide_controller_init(c, ctl.ControllerParams(**{**ok, "n_threshold": 2, "train_fraction": 0.01})) == 0 and c.n_train == 1
    assert ctl.tide_controller_init(c, ctl.ControllerParams(**{**ok, "n_threshold": 5, "train_fraction": 0.99})) == 0 and c.n_train == 4
