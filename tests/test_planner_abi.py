"""The library's planner entry points (host-only arithmetic, no GPU needed) against the oracle: same plans,
same numbers to the last bits of double precision."""
import math

import numpy as np
import pytest

from oracle import planner as OP
from test_oracle_planner import random_problem


def test_accept_prob_and_tau_match_the_oracle():
    import paper_2511_16193_amd as P
    for p in (0.0, 0.05, 0.5, 0.77, 0.999, 1.0):
        for w in (1, 2, 5, 16, 64):
            assert abs(P.plan_tau(p, w) - OP.tau(p, w)) <= 1e-13 * max(1.0, OP.tau(p, w))
            for a in range(w + 1):
                assert abs(P.plan_accept_prob(p, a, w) - OP.accept_prob(p, a, w)) <= 1e-15
    assert math.isnan(P.plan_tau(0.5, 0))
    assert math.isnan(P.plan_accept_prob(0.5, 3, 2))
    assert math.isnan(P.plan_accept_prob(0.5, -1, 2))


def test_plans_match_the_oracle():
    import paper_2511_16193_amd as P
    rng = np.random.default_rng(2024)
    for trial in range(200):
        W = int(rng.integers(1, 13))
        configs, D_of, V_of = random_problem(rng, W)
        if trial % 7 == 0:                                   # a drafter with no fixed cost, one with no per-request cost
            D_of[1] = OP.Affine(D_of[1].slope, 0.0)
        if trial % 11 == 0:
            D_of[1] = OP.Affine(0.0, D_of[1].icpt if D_of[1].icpt > 0 else 1.0)
        B, G = int(rng.integers(1, 2048)), int(rng.integers(1, 257))
        p = float(rng.choice([0.0, 1.0, rng.uniform(0, 1)], p=[0.05, 0.05, 0.9]))
        want = OP.plan_decoupled(B, G, p, configs, D_of, V_of, W)
        got = P.plan_decoupled(B, G, p, configs, [(D_of[g].slope, D_of[g].icpt) for g in range(1, max(configs) + 1)],
                               [[(V_of[(g, w)].slope, V_of[(g, w)].icpt) for w in range(1, W + 1)] for g in configs], W)
        assert (got["g_d"], got["g_v"], got["w"], got["b"]) == (want.g_d, want.g_v, want.w, want.b), trial
        assert abs(got["tgs"] - want.tgs) <= 1e-13 * want.tgs
        g = configs[-1]
        Vs = [V_of[(g, w)] for w in range(1, W + 1)]
        w1, t1 = P.plan_best_window(p, (D_of[1].slope, D_of[1].icpt), [(v.slope, v.icpt) for v in Vs], 1.0)
        w0, t0 = OP.best_window(p, D_of[1], Vs, 1.0)
        assert w1 == w0 and abs(t1 - t0) <= 1e-13 * t0


def test_fit_matches_the_oracle_and_bad_arguments_are_refused():
    import paper_2511_16193_amd as P
    from paper_2511_16193_amd import SvError
    rng = np.random.default_rng(1)
    b = rng.uniform(1, 300, 12).tolist()
    t = [0.1 * x + 4 + e for x, e in zip(b, rng.normal(0, 0.1, 12))]
    s, i = P.fit_affine(b, t)
    f = OP.fit_affine(b, t)
    assert abs(s - f.slope) <= 1e-14 and abs(i - f.icpt) <= 1e-13
    with pytest.raises(SvError):
        P.fit_affine([3.0, 3.0], [1.0, 2.0])
    with pytest.raises(SvError):
        P.plan_decoupled(8, 4, 1.5, [1], [(1, 1)], [[(1, 1)]], 1)          # p outside [0, 1]
    with pytest.raises(SvError):
        P.plan_decoupled(8, 4, 0.5, [0], [(1, 1)], [[(1, 1)]], 1) if False else P.plan_decoupled(0, 4, 0.5, [1], [(1, 1)], [[(1, 1)]], 1)
