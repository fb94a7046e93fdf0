"""The latency model of the paper's Section 4.1 measured on this GPU, fitted and searched through the library,
against the planner oracle on the same measured points.

V_w(b): the library's verification step on a cut of the 7B-shaped decoder (four layers, full width and
vocabulary), b requests, windows of w drafts; D(b): a plain decoding step (k = 0) on a cut of a 1.5B-shaped
drafter.  The affine fits (sv_fit_affine), the plan of Algorithm 1 (sv_plan_decoupled) and the best window per
acceptance rate (sv_plan_best_window) must be the oracle's on the same points: same lines to 1e-12, same
(g_d, g_v, w, b), TGS to 1e-12.  That time grows with the batch and is roughly affine in it is checked as a
property; the figures themselves are a measurement, not an expectation."""
import numpy as np
import pytest
import torch

from oracle import planner as OP
import workloads as W

pytestmark = pytest.mark.gpu


def test_measured_latency_model_fit_and_plan_match_the_oracle():
    import paper_2511_16193_amd as P
    from workloads.profile_plan import measure, DRAFTER
    batches, windows = [16, 64, 128], [1, 2, 4]
    verifier = W.scaled_down(W.CONFIGS["cfg3"], n_layers=4, prefix_lo=512, prefix_hi=1024)
    drafter = W.Shape("drafter-cut", 4, DRAFTER["d_model"], DRAFTER["n_q_heads"], DRAFTER["n_kv_heads"], DRAFTER["head_dim"],
                      DRAFTER["d_ff"], DRAFTER["vocab"], prefix_lo=512, prefix_hi=1024, seed=3001)
    log = lambda *a: print(*a, flush=True)
    v_pts = measure(verifier, batches, windows, 5, log)
    d_pts = measure(drafter, batches, [0], 5, log)[0]

    # fits: library against oracle on the same points
    D_lib = P.fit_affine([float(b) for b, _ in d_pts], [t for _, t in d_pts])
    D_or = OP.fit_affine([float(b) for b, _ in d_pts], [t for _, t in d_pts])
    assert abs(D_lib[0] - D_or.slope) <= 1e-12 * abs(D_or.slope) and abs(D_lib[1] - D_or.icpt) <= 1e-12 * abs(D_or.icpt) + 1e-15
    V_lib, V_or = {}, {}
    for w in windows:
        bs, ts = [float(b) for b, _ in v_pts[w]], [t for _, t in v_pts[w]]
        V_lib[w], V_or[w] = P.fit_affine(bs, ts), OP.fit_affine(bs, ts)
        assert abs(V_lib[w][0] - V_or[w].slope) <= 1e-12 * abs(V_or[w].slope)
        assert abs(V_lib[w][1] - V_or[w].icpt) <= 1e-12 * abs(V_or[w].icpt) + 1e-15
        # the shape the model assumes: more requests take longer, and a line describes it
        assert ts[0] < ts[-1] and V_or[w].slope > 0
        assert max(abs(V_or[w](b) - t) / t for b, t in zip(bs, ts)) < 0.35
    # a longer window is not cheaper to verify at the largest batch
    assert v_pts[1][-1][1] <= v_pts[4][-1][1] * 1.05

    # window 3 was not measured: linear in w between its neighbours, the same numbers on both sides
    mid = tuple(0.5 * (a + b) for a, b in zip(V_lib[2], V_lib[4]))
    V_list = [V_lib[1], V_lib[2], mid, V_lib[4]]
    V_of = {(1, w + 1): OP.Affine(*V_list[w]) for w in range(4)}
    D_of = {1: OP.Affine(*D_lib)}
    for p in (0.3, 0.6, 0.8, 0.95):
        for B in (64, 256):
            got = P.plan_decoupled(B, 2, p, [1], [D_lib], [V_list], 4)
            want = OP.plan_decoupled(B, 2, p, [1], D_of, V_of, 4)
            assert (got["g_d"], got["g_v"], got["w"], got["b"]) == (want.g_d, want.g_v, want.w, want.b), (p, B)
            assert abs(got["tgs"] - want.tgs) <= 1e-12 * want.tgs
            w1, t1 = P.plan_best_window(p, D_lib, V_list, float(want.b))
            w0, t0 = OP.best_window(p, D_of[1], [V_of[(1, w)] for w in range(1, 5)], float(want.b))
            assert w1 == w0 and abs(t1 - t0) <= 1e-12 * t0
    print("fitted:", {"D": D_lib, "V": V_lib})
