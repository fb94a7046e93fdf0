"""Time the dense projections of a workload configuration's model, one by one, against the vendor library.

    python -m workloads.profile_gemm [--config cfg5] [--rows 800]

For each projection shape of the model (QKV, O, gate/up, down, LM head) at the given number of rows: the
library's own kernel in the launch shape a verification step gives it (sv_op_gemm_bf16_ws with the plan of
sv_op_gemm_plan, packed operands), and torch's matmul on the same bf16 operands (hipBLASLt / rocBLAS), each the
mean of 20 runs after 3 warm-up runs, with seeded N(0,1) activations and N(0,0.02) weights.  The gate/up projection
is timed without the SwiGLU epilogue it carries inside a step.  Prints one JSON line.  Run from the repository root.
"""
from __future__ import annotations

import argparse
import json
import sys

import torch


def mean_us(fn, reps=20, warm=3):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e3


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg5")
    ap.add_argument("--rows", type=int, default=None, help="rows per step (default: the configuration's B * (1 + N k))")
    args = ap.parse_args(argv)
    import workloads as W
    import paper_2511_16193_amd as P
    s = W.CONFIGS[args.config]
    M = args.rows or s.batch * (1 + s.n_chains * s.k)
    qw, kvw = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    shapes = [("qkv", qw + 2 * kvw, s.d_model), ("o", s.d_model, qw)]
    if not s.n_experts:
        shapes += [("gate_up", 2 * s.d_ff, s.d_model), ("down", s.d_model, s.d_ff)]
    shapes.append(("lm_head", s.vocab, s.d_model))
    dev = torch.device("cuda:0")
    g = torch.Generator(device=dev)
    g.manual_seed(s.seed)
    out = {"config": s.name, "rows": M, "projections": {}}
    for name, N, K in shapes:
        a = torch.randn((M, K), generator=g, device=dev).to(torch.bfloat16)
        w = (torch.randn((N, K), generator=g, device=dev) * 0.02).to(torch.bfloat16)
        plan = P.op_gemm_plan(M, N, K)
        ap_, wp = P.op_pack_rows(a), P.op_pack_weight(w)
        ours = mean_us(lambda: P.op_gemm_bf16_ws(ap_, wp, M, splits=plan["splits"], wide=plan["wide"], row_tiles=plan["row_tiles"]))
        lib = mean_us(lambda: a @ w.t())
        flop = 2.0 * M * N * K
        out["projections"][name] = {"N": N, "K": K, "plan": plan, "ours_us": ours, "ours_tflops": flop / ours / 1e6,
                                    "library_us": lib, "library_tflops": flop / lib / 1e6}
        print(f"{name:8s} N={N:6d} K={K:6d} plan {plan}: ours {ours:8.1f} us ({flop / ours / 1e6:7.1f} TFLOP/s), "
              f"library {lib:8.1f} us ({flop / lib / 1e6:7.1f} TFLOP/s)", file=sys.stderr, flush=True)
        del a, w, ap_, wp
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
