#!/usr/bin/env python3
"""Benchmark of the batched speculative-verification step on one MI355X.

One "step" = one whole verification pass over a batch of synthetic requests:
forward of the target over the k drafts (+ x0) of every request against its
paged KV cache, accept/reject + replacement/bonus draw, chain choice, rollback.
The cache is put back to the same saved lengths before every step, so every
step verifies the same drafts against the same state.

Prints ONE JSON line: accepted tokens/s (tokens emitted per verification, the
supplied token included, summed over the batch, per second of step time), the
roofline figures of the kernel class that takes most of the step, and the CPU
oracle timed on a small sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_FP32_TFLOPS = 157.3       # MI355X fp32 vector ALUs

# HBM bytes per launch (read + written) from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs summarised under
# profiles/ (scaled by the copy-kernel calibration stated there), averaged over the launches of a kind in one step.
BRACKET_EVERY = 4          # steps of the timed region between two steps whose dominant-kind launches are bracketed by events

MEASURED_TRAFFIC = {
    # profiles/verify_step_cfg2_hbm_traffic.txt: projections (17994 MiB read + 2660 MiB written) / 113 launches;
    # attention main + merge kernel of one layer (602.5 MiB read + 11.6 MiB written)
    "cfg2-7b-b64-k4": {"gemm": 189.9e6, "attention": 643.9e6},
    # profiles/verify_step_cfg4_hbm_traffic.txt: expert FFN kernels of one layer (1404.9 MiB read + 77.1 MiB
    # written); attention main + merge kernel of one layer (1227.1 MiB read + 20.2 MiB written)
    "cfg4-moe-b128-k4": {"moe": 1397.1e6, "attention": 1307.9e6},
}


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def gemm_flops_per_step(s, T):
    """Flops and launches of the dense projections (QKV, O, dense FFN, LM head) of one step."""
    qw, kvw = s.n_q_heads * s.head_dim, s.n_kv_heads * s.head_dim
    per_layer = s.d_model * (qw + 2 * kvw) + qw * s.d_model + (0 if s.n_experts else 3 * s.d_model * s.d_ff)
    return 2.0 * T * (s.n_layers * per_layer + s.vocab * s.d_model), (2 if s.n_experts else 4) * s.n_layers + 1


def moe_bytes_per_layer(s, T):
    """HBM bytes one mixture-of-experts FFN has to move: every expert's three matrices once (with T * top_k
    assignments far above the expert count every expert has rows), the router matrix, the rows in (bf16) and
    the combined result out (fp32)."""
    return s.n_experts * 3.0 * s.d_model * s.d_expert * 2 + s.n_experts * s.d_model * 2 + T * s.d_model * (2 + 4)


def attention_bytes_per_layer(s, lengths, n):
    es = 4 if s.dtype == "fp32" else 2                              # bytes per cached element
    kv_row = 2 * s.n_kv_heads * s.head_dim * es                     # K and V of one token in one layer
    q_o = 2 * len(lengths) * n * s.n_q_heads * s.head_dim * es      # Q read + output written
    return float(sum(int(L) + n for L in lengths)) * kv_row + q_o


def cpu_baseline(case, n_seqs):
    """Time the oracle, as it stands, on the first n_seqs requests of the same workload."""
    import torch
    from threadpoolctl import threadpool_info
    from oracle import model as M, verify as OV
    import workloads as W
    s = case.shape
    spec = M.ModelSpec(**s.model_fields())
    log(f"cpu baseline: staging weights and the cache of {n_seqs} requests on the host ...")
    wn = W.weights_to_numpy(case.weights)
    n = 1 + case.N * case.k
    caches = []
    for b in range(n_seqs):
        L = int(case.lengths[b])
        c = M.SeqCache(spec, L + n + 1)
        for l in range(s.n_layers):
            k, v = case.kv_block(b, l)
            c.k[l][:L] = k.float().cpu().numpy()
            c.v[l][:L] = v.float().cpu().numpy()
        c.length = L
        caches.append(c)
    x0 = case.x0[:n_seqs].cpu().numpy().astype(np.int64)
    drafts = case.drafts[:n_seqs].cpu().numpy().astype(np.int64)
    q = case.draft_probs[:n_seqs].cpu().numpy()
    u = case.uniforms[:n_seqs].cpu().numpy()
    log("cpu baseline: running the oracle ...")
    t0 = time.perf_counter()
    r = OV.verify_step(spec, wn, caches, x0, drafts, q, u, verify_mode=OV.STOCHASTIC,
                       sample_mode=OV.SAMPLE_EXP_RACE, temperature=1.0)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    emitted = int((r.accepted_len + 1).sum())
    log(f"cpu baseline: {emitted} tokens in {dt:.1f} s on {threads} threads")
    return {"value": emitted / dt, "unit": "accepted tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n_seqs} of {case.B} requests of {s.name}, one step, {dt:.1f} s; weights and cache "
                      f"staged on the host beforehand (not timed)"}, r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--k", type=int, default=None)
    ap.add_argument("--batch", type=int, default=None, help="requests per step (default: the configuration's)")
    ap.add_argument("--sigma", type=float, default=None)
    ap.add_argument("--cpu-seqs", type=int, default=16, help="requests in the oracle sample (0 = skip)")
    ap.add_argument("--gemm-variant", type=int, default=None)
    ap.add_argument("--no-graph", action="store_true", help="skip the extra pass that replays the steps from a HIP graph")
    ap.add_argument("--attn-chunk", type=int, default=None, help="keys per split-KV chunk (tuning)")
    ap.add_argument("--attn-max-row-tiles", type=int, default=None, help="16-row tiles per attention work-group (tuning)")
    ap.add_argument("--drafts", choices=["noisy-target", "independent"], default="noisy-target",
                    help="independent: drafts from q = softmax(N(0,1)) without any device decoding step, so that "
                         "every kernel launch of the process has the timed step's shape (used for profiles)")
    ap.add_argument("--verify", choices=["config", "greedy", "stochastic", "match"], default="config",
                    help="verification rule (default: the configuration's); with `match` the synthetic drafts are "
                         "rarely accepted: use it to time the rule, not for the headline figure")
    ap.add_argument("--drop-row-major", action="store_true",
                    help="free the row-major copy of the weights once they are packed (no oracle baseline then); "
                         "needed for cfg5 at its full batch")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed steps run one plain elementwise pass that reads 1 GiB and writes 1 GiB "
                         "(torch.neg(src, out=dst) on fp32, an op nothing else in the run uses), the known-size kernel against which the HBM byte "
                         "counters of a profiler run are scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs the verification step on ONE GPU (requests shard across workers "
              "with no exchange between them); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as W
    from workloads.device_case import DeviceCase
    import paper_2511_16193_amd as P

    if not torch.cuda.is_available():
        print("bench.py: no GPU", file=sys.stderr)
        sys.exit(1)
    # a stream of its own for everything: the library can only capture its launches into a graph off the null stream
    torch.cuda.set_stream(torch.cuda.Stream())
    shape = W.CONFIGS[args.config]
    if args.batch is not None:
        shape = W.scaled_down(shape, batch=args.batch)
    vmode = {"config": None, "greedy": 0, "stochastic": 1, "match": 2}[args.verify]
    if args.drop_row_major:
        args.cpu_seqs = 0
    case = DeviceCase(shape, k=args.k, verify_mode=vmode, keep_row_major=not args.drop_row_major, log=log)
    if args.gemm_variant is not None:
        case.ver.set_option(P.SV_OPT_GEMM_VARIANT, args.gemm_variant)
    if args.attn_chunk is not None:
        case.ver.set_option(P.SV_OPT_ATTN_CHUNK_KEYS, args.attn_chunk)
    if args.attn_max_row_tiles is not None:
        case.ver.set_option(P.SV_OPT_ATTN_MAX_ROW_TILES, args.attn_max_row_tiles)
    if args.drafts == "independent":
        log("drafting (target-independent q) ...")
        case.independent_drafts(1.0)
    else:
        log("drafting (noisy-target drafts through plain decoding steps) ...")
        case.noisy_target_drafts(None if args.sigma is None else [args.sigma])
    B, N, k = case.B, case.N, case.k
    n = 1 + N * k
    T = B * n
    out = {"accepted_len": torch.empty(B, dtype=torch.int32, device=case.device),
           "out_tokens": torch.empty((B, k + 1), dtype=torch.int32, device=case.device),
           "best_chain": torch.empty(B, dtype=torch.int32, device=case.device)}

    def run(steps):
        for _ in range(steps):
            case.reset()
            case.step(out=out)

    log(f"warm-up {args.warmup} steps ...")
    run(args.warmup)
    torch.cuda.synchronize()
    # un-instrumented pass, for reference in the log; an event between steps (on the stream the library launches
    # on, torch's current one) gives the spread of the single steps
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        marks[i].record()
        run(1)
    marks[args.steps].record()
    torch.cuda.synchronize()
    plain_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    each = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    pick = lambda f: each[min(len(each) - 1, int(round(f * (len(each) - 1))))]
    step_spread = {"p10": pick(0.1), "p50": pick(0.5), "p90": pick(0.9)} if each else None

    # the same steps replayed from a HIP graph (reported beside the contract's figure: the event brackets of the
    # timed region below cannot be recorded inside a graph)
    graph_ms = None
    if not args.no_graph:
        case.ver.set_option(P.SV_OPT_GRAPH, 1)
        run(3)                                     # plain launches, capture, first replay
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        run(args.steps)
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        case.ver.set_option(P.SV_OPT_GRAPH, 0)
        log(f"graph replay: {graph_ms:.3f} ms per step")

    # pre-pass (not timed): every kernel kind bracketed by events, to find the kind that takes most of the step
    # and to time the others
    kinds = {"gemm": P.SV_PROF_GEMM, "attention": P.SV_PROF_ATTENTION, "sampler": P.SV_PROF_SAMPLER, "moe": P.SV_PROF_MOE}
    case.ver.profile_enable(sum(1 << kind for kind in kinds.values()))
    run(1)
    for kind in kinds.values():
        case.ver.profile_read(kind)
    pre_steps = max(3, args.steps // 4)
    run(pre_steps)
    pre = {name: case.ver.profile_read(kind) for name, kind in kinds.items()}    # (total ms, launches)
    dominant_kind = max(("gemm", "attention", "moe"), key=lambda n: pre[n][0])

    # the timed region: K steps, with event brackets around the launches of the dominant kind only, and on every
    # BRACKET_EVERY-th step only (a bracket costs a little pipelining between kernels: ~0.6 ms per step when all
    # ~110 projection launches of every step are bracketed)
    case.ver.profile_enable(1 << kinds[dominant_kind])
    run(1)
    case.ver.profile_read(kinds[dominant_kind])
    case.ver.profile_enable(0)
    torch.cuda.synchronize()
    bracketed_steps = 0
    t0 = time.perf_counter()
    for i in range(args.steps):
        on = i % BRACKET_EVERY == 0
        if on:
            case.ver.profile_enable(1 << kinds[dominant_kind])
            bracketed_steps += 1
        run(1)
        if on:
            case.ver.profile_enable(0)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    timed = case.ver.profile_read(kinds[dominant_kind])

    def per_launch_ms(name):
        tot, n = timed if name == dominant_kind else pre[name]
        return (tot / n if n else 0.0), (n // (bracketed_steps if name == dominant_kind else pre_steps))

    gemm_lms, gemm_lps = per_launch_ms("gemm")
    attn_lms, attn_lps = per_launch_ms("attention")
    moe_lms, moe_lps = per_launch_ms("moe")
    samp_ms = pre["sampler"][0] / pre_steps
    log(f"step {ms_per_step:.3f} ms with event brackets around {dominant_kind} ({plain_ms:.3f} ms without any); per step: "
        f"gemm {gemm_lms * gemm_lps:.3f} ms / {gemm_lps} launches, attention {attn_lms * attn_lps:.3f} ms / {attn_lps}, "
        f"sampler {samp_ms:.3f} ms, moe {moe_lms * moe_lps:.3f} ms / {moe_lps}")

    acc = out["accepted_len"].cpu().numpy()
    emitted = int((acc + 1).sum())
    flops, gemm_launches = gemm_flops_per_step(shape, T)
    abytes = attention_bytes_per_layer(shape, case.lengths, n)
    gemm_tflops = flops / gemm_launches / (gemm_lms * 1e-3) / 1e12
    attn_gbs = abytes / (attn_lms * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC.get(shape.name if args.batch is None and args.k is None else "", {})
    fp32 = shape.dtype == "fp32"     # fp32 models: plain-ALU projections (fp32 vector peak) and the generic attention kernel
    gemm_peak = PEAK_FP32_TFLOPS if fp32 else PEAK_BF16_TFLOPS
    roofs = {
        "gemm": {"kernel": "gemm_f32_kernel (all dense projections + LM head)" if fp32 else "gemm_bf16_ws_kernel (all dense projections + LM head)",
                 "bound": "alu" if fp32 else "mfma", "achieved": gemm_tflops,
                 "peak": gemm_peak, "unit": "TFLOP/s", "frac": gemm_tflops / gemm_peak,
                 "traffic": traffic.get("gemm"), "avg_launch_ms": gemm_lms, "launches_per_step": gemm_lps},
        "attention": {"kernel": "attn_generic_kernel (one layer)" if fp32 else "attn_bf16_regs_kernel or attn_bf16_kernel + attn_merge_kernel (one layer)", "bound": "hbm", "achieved": attn_gbs,
                      "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": attn_gbs / PEAK_HBM_GBS,
                      "traffic": traffic.get("attention"), "avg_launch_ms": attn_lms, "launches_per_step": attn_lps},
    }
    if moe_lps:
        moe_gbs = moe_bytes_per_layer(shape, T) / (moe_lms * 1e-3) / 1e9
        roofs["moe"] = {"kernel": "moe_gemm_kernel<0>, <1> + router, grouping, combine (one layer's expert FFN)",
                        "bound": "hbm", "achieved": moe_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": moe_gbs / PEAK_HBM_GBS, "traffic": traffic.get("moe"), "avg_launch_ms": moe_lms,
                        "launches_per_step": moe_lps}
    dominant = roofs.pop(dominant_kind)
    other = sorted(roofs.values(), key=lambda r: -r["avg_launch_ms"] * r["launches_per_step"])
    for r in other:
        r["timed_in"] = "pre-pass of %d steps with every kind bracketed" % pre_steps

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=case.device)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.neg(src, out=dst)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if args.cpu_seqs > 0:
        cpu, _ = cpu_baseline(case, min(args.cpu_seqs, B))

    res = {
        "metric": "accepted tokens/s of batched spec-verify step", "value": emitted / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": shape.name + (f" at batch {B}" if args.batch is not None else ""), "batch": B, "k": k, "chains": N, "rows_per_step": T,
                   "prefix_tokens": int(case.lengths.sum()), "drafts": args.drafts, "draft_sigma": list(shape.draft_sigma) if args.sigma is None else [args.sigma],
                   "verify": {None: "greedy" if shape.verify_mode == 0 else "stochastic, exponential-race draw, temperature 1.0",
                              0: "greedy", 1: "stochastic, exponential-race draw, temperature 1.0",
                              2: "sampled exact match, exponential-race draw, temperature 1.0"}[vmode]},
        "accepted_drafts_per_step": int(acc.sum()), "emitted_tokens_per_step": emitted,
        "accepted_drafts_tokens_per_s": int(acc.sum()) / (ms_per_step * 1e-3),
        "roofline": dominant, "roofline_other": other,
        "sampler_ms_per_step": samp_ms, "ms_per_step_without_event_brackets": plain_ms,
        "step_ms_without_event_brackets": step_spread,
        "ms_per_step_graph_replay": graph_ms,
        "cpu_baseline": cpu,
    }
    case.close()
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
