"""Pins of the planner oracle (oracle/planner.py) against what the mathematics fixes, none of which retypes its
formulas: a simulated acceptance process, closed forms of the geometric sums, a plan worked by hand, numpy's
polynomial fit, and invariants of the search."""
import math

import numpy as np
import pytest

from oracle import planner as OP


def simulate_windows(p, w, n, seed):
    """Accepted drafts per window: every draft is accepted with probability p, the window stops at the first
    rejection."""
    rng = np.random.default_rng(seed)
    acc = rng.random((n, w)) < p
    first_rej = np.where(acc.all(axis=1), w, np.argmin(acc, axis=1))
    return first_rej


@pytest.mark.parametrize("p,w", [(0.3, 1), (0.5, 4), (0.8, 7), (0.95, 12)])
def test_accept_prob_is_a_distribution_and_matches_the_simulated_process(p, w):
    probs = [OP.accept_prob(p, a, w) for a in range(w + 1)]
    assert abs(sum(probs) - 1.0) < 1e-12
    n = 400_000
    a = simulate_windows(p, w, n, seed=17 * w)
    counts = np.bincount(a, minlength=w + 1)
    for k in range(w + 1):
        sigma = math.sqrt(n * probs[k] * (1 - probs[k])) + 1.0
        assert abs(counts[k] - n * probs[k]) < 5 * sigma, (k, counts[k], n * probs[k])


@pytest.mark.parametrize("p,w", [(0.3, 1), (0.5, 4), (0.8, 7), (0.95, 12)])
def test_tau_is_the_expectation_over_the_simulated_process(p, w):
    """tau_w = E[(a+1)/2 if a < w else w] over the acceptance process."""
    n = 400_000
    a = simulate_windows(p, w, n, seed=5 + w)
    g = np.where(a < w, (a + 1) / 2.0, float(w))
    se = g.std() / math.sqrt(n)
    assert abs(g.mean() - OP.tau(p, w)) < 5 * se + 1e-9


def test_tau_closed_form_and_special_values():
    # sum_{a<w} (a+1) p^a (1-p) = (1 - p^w)/(1-p) - w p^w  (derivative of the geometric series), hence
    # tau_w = (1 - p^w) / (2 (1-p)) + w p^w / 2
    for p in np.linspace(0.0, 0.99, 34):
        for w in (1, 2, 3, 8, 20):
            closed = (1 - p ** w) / (2 * (1 - p)) + w * p ** w / 2
            assert abs(OP.tau(float(p), w) - closed) < 1e-12 * max(1.0, closed)
    for w in (1, 3, 9):
        assert OP.tau(0.0, w) == 0.5                # always rejected at once: (0+1)/2
        assert OP.tau(1.0, w) == w                  # always fully accepted
    for p in (0.1, 0.6):
        assert abs(OP.tau(p, 1) - (1 + p) / 2) < 1e-15
    # a window yields at most its w drafts, and a very long window tends to the geometric limit 1 / (2 (1 - p))
    # (not monotonically: a window one draft short of a full accept counts half, so at p = 0.2 tau_3 < tau_2)
    for p in (0.2, 0.7, 0.9):
        assert all(OP.tau(p, w) <= w for w in range(1, 30))
        assert abs(OP.tau(p, 400) - 1 / (2 * (1 - p))) < 1e-9
    assert OP.tau(0.2, 3) < OP.tau(0.2, 2)


def test_latency_is_the_slower_of_the_two_sides():
    D, V = OP.Affine(0.5, 1.0), OP.Affine(1.0, 2.0)
    assert OP.iteration_latency(1, D, V, 8) == 10.0          # verify 10 > draft 5
    assert OP.iteration_latency(2, D, V, 8) == 10.0          # equal
    assert OP.iteration_latency(3, D, V, 8) == 15.0          # drafting 3 tokens takes longer
    assert OP.tgs(0.5, 2, D, V, 8) == OP.tau(0.5, 2) / 10.0


def test_plan_worked_by_hand():
    """G = 4 GPUs, B = 8, p = 1/2, verifier configurations {1, 2}, windows 1..2.
    D_1(b) = b + 1, D_2(b) = b/2 + 1; V_{1,w}(b) = 2b + 2, V_{2,w}(b) = b + 2 for both windows.
    tau_1 = 3/4, tau_2 = 1.
      g_v=1, g_d=1: b = ceil(2*8/4) = 4, w_max = max(ceil(2/1), ceil(2/1)) = 2
                    w=1: max(5, 10) = 10 -> 0.075;  w=2: max(10, 10) = 10 -> 0.1
      g_v=2, g_d=1: b = 6, w_max = max(1, 2) = 2;  w=1: max(7, 8) -> 0.09375;  w=2: max(14, 8) -> 1/14
      g_v=2, g_d=2: b = 8, w_max = max(2, 2) = 2;  w=1: max(5, 10) -> 0.075;   w=2: max(10, 10) -> 0.1 (a tie: the first stays)
    """
    D_of = {1: OP.Affine(1.0, 1.0), 2: OP.Affine(0.5, 1.0)}
    V_of = {(1, 1): OP.Affine(2.0, 2.0), (1, 2): OP.Affine(2.0, 2.0), (2, 1): OP.Affine(1.0, 2.0), (2, 2): OP.Affine(1.0, 2.0)}
    plan = OP.plan_decoupled(8, 4, 0.5, [1, 2], D_of, V_of, 2)
    assert (plan.g_d, plan.g_v, plan.w, plan.b) == (1, 1, 2, 4)
    assert plan.tgs == 0.1
    # visiting the configurations in the other order meets (2, 2, 2) first
    plan = OP.plan_decoupled(8, 4, 0.5, [2, 1], D_of, V_of, 2)
    assert (plan.g_d, plan.g_v, plan.w, plan.b) == (2, 2, 2, 8)


def random_problem(rng, W):
    configs = sorted(rng.choice(np.arange(1, 9), size=int(rng.integers(1, 4)), replace=False).tolist())
    D_of = {g: OP.Affine(float(rng.uniform(0.02, 0.3)) / g, float(rng.uniform(0.5, 3.0))) for g in range(1, max(configs) + 1)}
    V_of = {}
    for g in configs:
        s0, i0 = float(rng.uniform(0.05, 0.4)) / g, float(rng.uniform(2.0, 8.0))
        for w in range(1, W + 1):
            V_of[(g, w)] = OP.Affine(s0 * (1 + 0.25 * w), i0 * (1 + 0.02 * w))
    return configs, D_of, V_of


def test_plan_is_the_maximum_of_an_independent_tabulation():
    """The search result equals the argmax of a table built with numpy from the closed form of tau, over the
    same candidate set, with numpy's first-maximum rule standing in for 'strictly larger replaces'."""
    rng = np.random.default_rng(11)
    for trial in range(40):
        W = int(rng.integers(1, 10))
        configs, D_of, V_of = random_problem(rng, W)
        B, G, p = int(rng.integers(8, 512)), int(rng.integers(8, 65)), float(rng.uniform(0.05, 0.97))
        plan = OP.plan_decoupled(B, G, p, configs, D_of, V_of, W)
        cand, val = [], []
        for g_v in configs:
            for g_d in range(1, g_v + 1):
                b = math.ceil((g_d + g_v) * B / G)
                D = D_of[g_d]
                bound = max(math.ceil(V_of[(g_v, W)].slope / D.slope), math.ceil(V_of[(g_v, W)].icpt / D.icpt))
                for w in range(1, min(W, max(1, bound)) + 1):
                    tau = (1 - p ** w) / (2 * (1 - p)) + w * p ** w / 2
                    il = np.maximum(w * (b * D.slope + D.icpt), b * V_of[(g_v, w)].slope + V_of[(g_v, w)].icpt)
                    cand.append((g_d, g_v, w, b))
                    val.append(tau / il)
        val = np.array(val)
        top = val.max()
        assert abs(plan.tgs - top) <= 1e-12 * top
        near = [c for c, v in zip(cand, val) if v >= top * (1 - 1e-12)]
        assert (plan.g_d, plan.g_v, plan.w, plan.b) in near


def test_plan_invariants():
    rng = np.random.default_rng(3)
    W = 6
    configs, D_of, V_of = random_problem(rng, W)
    base = OP.plan_decoupled(256, 32, 0.8, configs, D_of, V_of, W)
    # a clock twice as slow halves TGS and changes no decision
    D2 = {g: OP.Affine(2 * a.slope, 2 * a.icpt) for g, a in D_of.items()}
    V2 = {k: OP.Affine(2 * a.slope, 2 * a.icpt) for k, a in V_of.items()}
    slow = OP.plan_decoupled(256, 32, 0.8, configs, D2, V2, W)
    assert (slow.g_d, slow.g_v, slow.w, slow.b) == (base.g_d, base.g_v, base.w, base.b)
    assert abs(slow.tgs - base.tgs / 2) < 1e-15
    # with drafts that are never accepted a longer window only costs time: the window is 1
    never = OP.plan_decoupled(256, 32, 0.0, configs, D_of, V_of, W)
    assert never.w == 1
    # the best window of a request grows (weakly) with its acceptance rate when verification is the slower side
    D, Vs = OP.Affine(1e-3, 1e-3), [OP.Affine(0.1, 5.0 + 0.05 * w) for w in range(1, 13)]
    ws = [OP.best_window(p, D, Vs, 1.0)[0] for p in (0.1, 0.3, 0.5, 0.7, 0.9, 0.99)]
    assert ws == sorted(ws) and ws[0] >= 1 and ws[-1] == 12


def test_fit_affine_recovers_a_line_and_agrees_with_polyfit():
    f = OP.fit_affine([8, 16, 32, 64], [3.0 + 0.25 * b for b in (8, 16, 32, 64)])
    assert abs(f.slope - 0.25) < 1e-14 and abs(f.icpt - 3.0) < 1e-13
    rng = np.random.default_rng(0)
    b = rng.uniform(1, 300, 25)
    t = 0.116 * b + 3.6 + rng.normal(0, 0.2, 25)
    f = OP.fit_affine(b.tolist(), t.tolist())
    slope, icpt = np.polyfit(b, t, 1)
    assert abs(f.slope - slope) < 1e-10 and abs(f.icpt - icpt) < 1e-9
    with pytest.raises(ValueError):
        OP.fit_affine([4, 4, 4], [1, 2, 3])
