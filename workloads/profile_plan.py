"""Profile the affine latency models of the paper's Section 4.1 on this GPU and run the plan search on them.

    python -m workloads.profile_plan [--verifier cfg3] [--batches 8,16,32,64,128,256]
                                                [--windows 1,2,4,8] [--p 0.8] [--B 256] [--json out.json]

Verification time V_w(b): the library's verification step on the verifier shape (a workload configuration's
model), b requests with seeded prefixes, windows of w target-independent drafts.  Draft time D(b): one plain
decoding step (k = 0) of the same library on a small drafter shape (1.5B-like, head size 128), standing in for a
draft model.  Both are timed as whole steps, inputs resident, median of a few runs.  Least-squares lines through
the points give V'_w, beta_w, D', alpha (sv_fit_affine); windows that were not measured are interpolated
linearly between measured ones.  With one GPU for each role (g_d = g_v = 1, G = 2) Algorithm 1 reduces to the
choice of the window; the script prints that plan, the whole TGS table, and the best window per acceptance rate.
Run from the repository root.
"""
from __future__ import annotations

import argparse
import json
import statistics
import sys
import time

import torch

DRAFTER = dict(name="drafter-1.5b", n_layers=28, d_model=1536, n_q_heads=12, n_kv_heads=2, head_dim=128, d_ff=8960,
               vocab=151936)


def time_steps(fn, reps: int) -> float:
    fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(reps):
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        ts.append((time.perf_counter() - t0) * 1e3)
    return statistics.median(ts)


def measure(shape, batches, windows, reps, log):
    """{w: [(b, ms), ...]} for the given windows (w = 0: plain decoding)."""
    import workloads as W
    from workloads.device_case import DeviceCase
    from workloads import synth
    out = {w: [] for w in windows}
    for b in batches:
        sh = W.scaled_down(shape, batch=b, k=max(max(windows), 1), n_chains=1)
        case = DeviceCase(sh, log=lambda *_: None)
        for w in windows:
            case.k = w
            if w:
                case.independent_drafts(1.0)
            case.uniforms = torch.from_numpy(synth.make_uniforms((b, 1, w + 1), sh.seed, "u")).to(case.device)

            def step():
                case.reset()
                case.step()
            ms = time_steps(step, reps)
            out[w].append((b, ms))
            log(f"  {sh.name}: b = {b:4d}, w = {w}: {ms:8.3f} ms")
        case.close()
        del case
        torch.cuda.empty_cache()
    return out


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--verifier", default="cfg3")
    ap.add_argument("--batches", default="8,16,32,64,128,256")
    ap.add_argument("--windows", default="1,2,4,8")
    ap.add_argument("--p", type=float, default=0.8)
    ap.add_argument("--B", type=int, default=256, help="global batch of the plan")
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--json", default=None)
    args = ap.parse_args(argv)
    import workloads as W
    import paper_2511_16193_amd as P
    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    batches = [int(x) for x in args.batches.split(",")]
    windows = sorted(int(x) for x in args.windows.split(","))
    Wmax = windows[-1]

    vshape = W.CONFIGS[args.verifier]
    log(f"verification steps on {vshape.name} ...")
    v_pts = measure(vshape, batches, windows, args.reps, log)
    dshape = W.Shape(DRAFTER["name"], DRAFTER["n_layers"], DRAFTER["d_model"], DRAFTER["n_q_heads"], DRAFTER["n_kv_heads"],
                     DRAFTER["head_dim"], DRAFTER["d_ff"], DRAFTER["vocab"], prefix_lo=vshape.prefix_lo,
                     prefix_hi=vshape.prefix_hi, seed=vshape.seed + 1)
    log(f"plain decoding steps on {dshape.name} ...")
    d_pts = measure(dshape, batches, [0], args.reps, log)[0]

    fit = lambda pts: P.fit_affine([float(b) for b, _ in pts], [t for _, t in pts])
    D = fit(d_pts)
    V_meas = {w: fit(v_pts[w]) for w in windows}

    def V_of(w):                                            # measured, or linear in w between measured neighbours
        if w in V_meas:
            return V_meas[w]
        lo = max(x for x in windows if x < w) if any(x < w for x in windows) else windows[0]
        hi = min(x for x in windows if x > w)
        f = (w - lo) / (hi - lo)
        return tuple(a + f * (b - a) for a, b in zip(V_meas[lo], V_meas[hi]))
    V = [V_of(w) for w in range(1, Wmax + 1)]

    plan = P.plan_decoupled(args.B, 2, args.p, [1], [D], [V], Wmax)
    res = {"verifier": vshape.name, "drafter": dshape.name, "batches": batches,
           "verify_ms": {str(w): v_pts[w] for w in windows}, "draft_ms": d_pts,
           "D": {"slope_ms_per_request": D[0], "icpt_ms": D[1]},
           "V": {str(w): {"slope_ms_per_request": V[w - 1][0], "icpt_ms": V[w - 1][1], "measured": w in V_meas}
                 for w in range(1, Wmax + 1)},
           "fit_residual_max_rel": {str(w): max(abs(V_meas[w][0] * b + V_meas[w][1] - t) / t for b, t in v_pts[w]) for w in windows},
           "plan": dict(plan, p=args.p, B=args.B, G=2),
           "best_window_by_p": {f"{p:.2f}": P.plan_best_window(p, D, V, float(plan["b"]))[0]
                                for p in (0.3, 0.5, 0.6, 0.7, 0.8, 0.9, 0.95)},
           "tgs_tokens_per_ms": {str(w): P.plan_tau(args.p, w) / max(w * (D[0] * plan["b"] + D[1]), V[w - 1][0] * plan["b"] + V[w - 1][1])
                                 for w in range(1, Wmax + 1)}}
    print(json.dumps(res))
    if args.json:
        with open(args.json, "w") as f:
            json.dump(res, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
