#!/usr/bin/env python3
"""Benchmark of the batched speculative-verification step on one MI355X.

One "step" = one whole verification pass over a batch of synthetic requests:
forward of the target over the k drafts (+ x0) of every request against its
paged KV cache, accept/reject + replacement/bonus draw, chain choice, rollback.
The cache is put back to the same saved lengths before every step, so every
step verifies the same drafts against the same state.

Prints ONE JSON line: accepted tokens/s (tokens emitted per verification, the
supplied token included, summed over the batch, per second of step time), the
roofline figures of the kernel class that takes most of the step (against the
published peak and against this GPU's micro-benchmarked one), the other kernel
classes, the sampler and the rollback stage, and the CPU oracle timed on a
small sample of the same workload.

Default workload: the largest configuration, the 32B-shaped decoder in the
long tail of a rollout (B = 32 requests with 16k-32k cached tokens, three
chains of eight drafts: 800 rows per step, 64 GB of weights, 206 GB of cache).
The row-major copy of its weights, which only the oracle leg reads, lives on
the host.  The whole run takes about 80 s, 42 s of which are the oracle on one
request.  --config cfg2 / cfg3 [--k 1|2|4|8] / cfg4 select the other workloads.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_FP32_TFLOPS = 157.3       # MI355X fp32 vector ALUs

DEFAULT_CONFIG = "cfg5"
BRACKET_EVERY = 4          # steps of the timed region between two steps whose dominant-kind launches are bracketed by events
CPU_SEQS = {"cfg1": 4, "cfg2": 16, "cfg3": 8, "cfg4": 2, "cfg5": 1}     # requests in the oracle sample (10-30 s of host work)


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def measured_traffic(tag):
    """HBM bytes per launch of each kind of kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary committed
    for this workload (profiles/verify_step_<tag>_hbm_traffic.txt, lines `bench-traffic <kind> <bytes>`), and the
    file's name.  Nothing is assumed when there is no summary for the workload."""
    path = os.path.join(ROOT, "profiles", f"verify_step_{tag}_hbm_traffic.txt")
    if not os.path.exists(path):
        return {}, None
    out = {}
    for line in open(path):
        m = re.match(r"bench-traffic\s+(\w+)\s+([0-9.eE+]+)", line)
        if m:
            out[m.group(1)] = float(m.group(2))
    return out, os.path.relpath(path, ROOT)


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


def sampler_bytes_per_step(s, B, N, k):
    """One pass over the logits (row statistics) plus, per chain, one logits row and one draft-distribution row for
    the final draw."""
    return (B * (1 + N * k) * s.vocab + B * N * 2 * s.vocab) * 4.0


def cpu_baseline(case, n_seqs, lazy_weights):
    """Time the oracle, as it stands, on the first n_seqs requests of the same workload."""
    from threadpoolctl import threadpool_info
    from oracle import model as M, verify as OV
    import workloads as W
    s = case.shape
    spec = M.ModelSpec(**s.model_fields())
    log(f"cpu baseline: staging {'the cache' if lazy_weights else 'weights and the cache'} of {n_seqs} requests on the host ...")
    wn = W.weights_to_numpy(case.weights, lazy=lazy_weights)
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
    q = None if case.draft_probs is None else case.draft_probs[:n_seqs].cpu().numpy()
    u = case.uniforms[:n_seqs].cpu().numpy()
    log("cpu baseline: running the oracle ...")
    t0 = time.perf_counter()
    r = OV.verify_step(spec, wn, caches, x0, drafts, q, u, verify_mode=OV.STOCHASTIC,
                       sample_mode=OV.SAMPLE_EXP_RACE, temperature=1.0)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    emitted = int((r.accepted_len + 1).sum())
    log(f"cpu baseline: {emitted} tokens in {dt:.1f} s on {threads} threads")
    staged = ("the cache staged on the host beforehand (not timed), each layer's weights widened from their bf16 host copy as "
              "the pass reaches it (timed)") if lazy_weights else "weights and cache staged on the host beforehand (not timed)"
    return {"value": emitted / dt, "unit": "accepted tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"first {n_seqs} of {case.B} requests of {s.name} (k={case.k}), one step, {dt:.1f} s; {staged}"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default=DEFAULT_CONFIG)
    ap.add_argument("--k", type=int, default=None, help="drafts per chain (default: the configuration's)")
    ap.add_argument("--batch", type=int, default=None, help="requests per step (default: the configuration's)")
    ap.add_argument("--sigma", type=float, default=None)
    ap.add_argument("--cpu-seqs", type=int, default=None, help="requests in the oracle sample (0 = skip; default per configuration)")
    ap.add_argument("--no-graph", action="store_true", help="skip the extra pass that replays the steps from a HIP graph")
    ap.add_argument("--attn-chunk", type=int, default=None, help="keys per split-KV chunk (tuning)")
    ap.add_argument("--attn-max-row-tiles", type=int, default=None, help="16-row tiles per attention work-group (tuning)")
    ap.add_argument("--gemm-tile", type=int, default=None, choices=[-1, 0, 1],
                    help="256 x 256 projection kernel: -1 where the plan expects it to pay (default), 0 never, 1 wherever the shape allows (tuning)")
    ap.add_argument("--drafts", choices=["noisy-target", "independent", "one-hot"], default="noisy-target",
                    help="independent: drafts from q = softmax(N(0,1)) without any device decoding step, so that "
                         "every kernel launch of the process has the timed step's shape (used for profiles); "
                         "one-hot: seeded draft ids without a distribution (draft_probs = NULL: what an n-gram drafter sends)")
    ap.add_argument("--verify", choices=["config", "greedy", "stochastic", "match"], default="config",
                    help="verification rule (default: the configuration's); with `match` the synthetic drafts are "
                         "rarely accepted: use it to time the rule, not for the headline figure")
    ap.add_argument("--row-major", choices=["auto", "device", "host", "drop"], default="auto",
                    help="where the row-major copy of the weights, which only the oracle reads, is kept once the library's "
                         "packed copy exists (auto: on the host when both copies and the cache would not fit the device)")
    ap.add_argument("--consecutive", type=int, default=None,
                    help="also time this many consecutive steps, each on the rolled-back cache of the one before, with "
                         "fresh drafts (drafted untimed) every step (default 16 for cfg3, else 0)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed steps run one plain device copy of 1 GiB (probe_copy_kernel), the known-size kernel "
                         "against which the HBM byte counters of a profiler run are scaled")
    ap.add_argument("--calibrate-peaks", action="store_true", help="only measure this GPU's MFMA and copy rates, print them as JSON and exit")
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
    if args.calibrate_peaks:
        peaks = P.probe_peaks()
        peaks["mfma_and_valu_overlap"] = P.probe_mfma_valu()
        print(json.dumps(peaks), flush=True)
        return
    shape = W.CONFIGS[args.config]
    if args.batch is not None:
        shape = W.scaled_down(shape, batch=args.batch)
    if args.consecutive is None:
        args.consecutive = 16 if args.config == "cfg3" else 0
    if args.cpu_seqs is None:
        args.cpu_seqs = CPU_SEQS.get(args.config, 4)
    vmode = {"config": None, "greedy": 0, "stochastic": 1, "match": 2}[args.verify]
    k_eff = shape.k if args.k is None else args.k
    if args.row_major == "auto":
        es = 2 if shape.dtype == "bf16" else 4
        F = shape.n_experts * shape.d_expert if shape.n_experts else shape.d_ff
        qkvo = shape.d_model * (2 * shape.n_q_heads + 2 * shape.n_kv_heads) * shape.head_dim
        w_bytes = es * (shape.n_layers * (qkvo + 3 * shape.d_model * F) + 2 * shape.vocab * shape.d_model)
        kv_bytes = shape.batch * (shape.prefix_lo + shape.prefix_hi) / 2 * shape.n_layers * 2 * shape.n_kv_heads * shape.head_dim * es
        q_bytes = shape.batch * shape.n_chains * k_eff * shape.vocab * 4 * 3
        args.row_major = "host" if 2 * w_bytes + kv_bytes + q_bytes > 250e9 else "device"
    if args.row_major == "drop":
        args.cpu_seqs = 0
    case = DeviceCase(shape, k=args.k, verify_mode=vmode, keep_row_major={"device": True, "host": "host", "drop": False}[args.row_major],
                      max_chains=2, headroom_tokens=(k_eff + 1) * args.consecutive, log=log)
    if args.attn_chunk is not None:
        case.ver.set_option(P.SV_OPT_ATTN_CHUNK_KEYS, args.attn_chunk)
    if args.attn_max_row_tiles is not None:
        case.ver.set_option(P.SV_OPT_ATTN_MAX_ROW_TILES, args.attn_max_row_tiles)
    if args.gemm_tile is not None:
        case.ver.set_option(P.SV_OPT_GEMM_TILE, args.gemm_tile)
    sigmas = None if args.sigma is None else [args.sigma]
    if args.drafts == "independent":
        log("drafting (target-independent q) ...")
        case.independent_drafts(1.0)
    elif args.drafts == "one-hot":
        log("drafting (seeded ids, no draft distribution) ...")
        case.one_hot_drafts()
    else:
        log("drafting (noisy-target drafts through plain decoding steps) ...")
        case.noisy_target_drafts(sigmas)
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
    kinds = {"gemm": P.SV_PROF_GEMM, "attention": P.SV_PROF_ATTENTION, "sampler": P.SV_PROF_SAMPLER, "moe": P.SV_PROF_MOE,
             "rollback": P.SV_PROF_ROLLBACK}
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
        tot, cnt = timed if name == dominant_kind else pre[name]
        return (tot / cnt if cnt else 0.0), (cnt // (bracketed_steps if name == dominant_kind else pre_steps))

    gemm_lms, gemm_lps = per_launch_ms("gemm")
    attn_lms, attn_lps = per_launch_ms("attention")
    moe_lms, moe_lps = per_launch_ms("moe")
    samp_ms = pre["sampler"][0] / pre_steps
    roll_ms = pre["rollback"][0] / pre_steps
    log(f"step {ms_per_step:.3f} ms with event brackets around {dominant_kind} ({plain_ms:.3f} ms without any); per step: "
        f"gemm {gemm_lms * gemm_lps:.3f} ms / {gemm_lps} launches, attention {attn_lms * attn_lps:.3f} ms / {attn_lps}, "
        f"sampler {samp_ms:.3f} ms, rollback {roll_ms:.3f} ms, moe {moe_lms * moe_lps:.3f} ms / {moe_lps}")
    acc = out["accepted_len"].cpu().numpy()
    emitted = int((acc + 1).sum())

    # ---- this GPU's own rooflines ----
    peaks = P.probe_peaks()
    log(f"measured peaks: {peaks}")
    # projections against the MFMA rate on random operands; the read-dominated kernels (attention, expert weights,
    # sampler) against a plain read-only stream; the rollback copy against a plain copy
    mfma_meas, hbm_meas, copy_meas = peaks["mfma_bf16_tflops_random_operands"], peaks["hbm_read_gbs"], peaks["hbm_copy_gbs_read_plus_write"]

    # ---- rollback: the step's own (metadata only unless a chain other than 0 was kept), and a forced-copy variant ----
    es = 4 if shape.dtype == "fp32" else 2
    kv_tok = 2 * shape.n_kv_heads * shape.head_dim * es * shape.n_layers           # bytes of one token's K and V, all layers
    forced = None
    if k > 0:
        Nf = max(N, 2)                                        # the context is sized for two chains at least
        f_acc = torch.full((B,), k, dtype=torch.int32, device=case.device)
        f_best = torch.full((B,), Nf - 1, dtype=torch.int32, device=case.device)
        case.reset()
        case.ver.op_rollback(case.ids, Nf, k, f_acc, f_best, commit=False)        # warm-up
        case.ver.profile_enable(1 << P.SV_PROF_ROLLBACK)
        case.ver.profile_read(P.SV_PROF_ROLLBACK)
        for _ in range(10):
            case.ver.op_rollback(case.ids, Nf, k, f_acc, f_best, commit=False)
        tot, cnt = case.ver.profile_read(P.SV_PROF_ROLLBACK)
        case.ver.profile_enable(0)
        case.reset()
        moved = 2.0 * B * k * kv_tok                           # read + written
        gbs = moved / (tot / cnt * 1e-3) / 1e9
        forced = {"kernel": "compact_kernel, every request's k accepted entries of the last chain moved, all layers in one launch",
                  "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                  "measured_peak": copy_meas, "frac_of_measured_peak": gbs / copy_meas, "bytes_per_launch": moved, "avg_launch_ms": tot / cnt}
    rollback = {"in_step_ms": roll_ms,
                "in_step_note": ("one chain per request: metadata only (the lengths advance, no entry moves)" if N == 1 else
                                 "entries move for requests whose kept chain is not chain 0"),
                "forced_copy": forced}

    # ---- consecutive steps with rollback every step, fresh drafts each time (drafted untimed) ----
    consecutive = None
    if args.consecutive > 0 and args.drafts == "noisy-target" and k > 0:
        log(f"{args.consecutive} consecutive steps ...")
        case.reset()
        saved = (case.x0, case.drafts, case.draft_probs, list(case.cur_lengths))
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.consecutive)]
        tokens, drafts_acc, x0 = 0, 0, case.x0
        for i in range(args.consecutive):
            if i:
                case.noisy_target_drafts(sigmas, x0=x0)       # from the rolled-back state; ends by putting the lengths back
            case.reset()
            torch.cuda.synchronize()
            ev[i][0].record()
            case.step(out=out)
            ev[i][1].record()
            torch.cuda.synchronize()
            a = out["accepted_len"].cpu().numpy()
            tokens += int((a + 1).sum())
            drafts_acc += int(a.sum())
            toks = out["out_tokens"].cpu()
            x0 = toks[torch.arange(B), torch.from_numpy(a).long()].to(torch.int32)   # the supplied token is the next x0
            case.commit(a)
        case.x0, case.drafts, case.draft_probs, case.cur_lengths = saved      # back to the benchmark's own state
        case.reset()
        ms = [e0.elapsed_time(e1) for e0, e1 in ev]
        consecutive = {"steps": args.consecutive, "ms_per_step_mean": float(np.mean(ms)), "ms_per_step_min": float(np.min(ms)),
                       "ms_per_step_max": float(np.max(ms)), "emitted_tokens": tokens, "accepted_drafts": drafts_acc,
                       "tokens_per_s": tokens / (sum(ms) * 1e-3),
                       "note": "each step verifies fresh drafts on the cache the previous step rolled back; drafting is not timed"}
        log(f"consecutive: {consecutive['ms_per_step_mean']:.3f} ms per step, {consecutive['tokens_per_s']:.0f} tokens/s")

    flops, gemm_launches = gemm_flops_per_step(shape, T)
    abytes = attention_bytes_per_layer(shape, case.lengths, n)
    gemm_tflops = flops / gemm_launches / (gemm_lms * 1e-3) / 1e12
    attn_gbs = abytes / (attn_lms * 1e-3) / 1e9
    tag = args.config + (f"_k{k}" if args.config == "cfg3" else "")
    traffic, traffic_src = measured_traffic(tag) if args.batch is None else ({}, None)
    fp32 = shape.dtype == "fp32"     # fp32 models: plain-ALU projections (fp32 vector peak) and the generic attention kernel
    gemm_peak = PEAK_FP32_TFLOPS if fp32 else PEAK_BF16_TFLOPS
    roofs = {
        "gemm": {"kernel": "gemm_f32_kernel (all dense projections + LM head)" if fp32 else "gemm_bf16_ws_kernel (all dense projections + LM head)",
                 "bound": "alu" if fp32 else "mfma", "achieved": gemm_tflops,
                 "peak": gemm_peak, "unit": "TFLOP/s", "frac": gemm_tflops / gemm_peak,
                 "measured_peak": None if fp32 else mfma_meas, "frac_of_measured_peak": None if fp32 else gemm_tflops / mfma_meas,
                 "traffic": traffic.get("gemm"), "avg_launch_ms": gemm_lms, "launches_per_step": gemm_lps},
        "attention": {"kernel": "attn_generic_kernel (one layer)" if fp32 else "attn_bf16_regs_kernel or attn_bf16_kernel + attn_merge_kernel (one layer)", "bound": "hbm", "achieved": attn_gbs,
                      "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": attn_gbs / PEAK_HBM_GBS,
                      "measured_peak": hbm_meas, "frac_of_measured_peak": attn_gbs / hbm_meas,
                      "traffic": traffic.get("attention"), "avg_launch_ms": attn_lms, "launches_per_step": attn_lps},
    }
    if moe_lps:
        moe_gbs = moe_bytes_per_layer(shape, T) / (moe_lms * 1e-3) / 1e9
        roofs["moe"] = {"kernel": "moe_gemm_kernel<0>, <1> + router, grouping, combine (one layer's expert FFN)",
                        "bound": "hbm", "achieved": moe_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": moe_gbs / PEAK_HBM_GBS, "measured_peak": hbm_meas, "frac_of_measured_peak": moe_gbs / hbm_meas,
                        "traffic": traffic.get("moe"), "avg_launch_ms": moe_lms, "launches_per_step": moe_lps}
    for r in roofs.values():
        r["traffic_source"] = traffic_src if r["traffic"] is not None else None
    dominant = roofs.pop(dominant_kind)
    other = sorted(roofs.values(), key=lambda r: -r["avg_launch_ms"] * r["launches_per_step"])
    for r in other:
        r["timed_in"] = "pre-pass of %d steps with every kind bracketed" % pre_steps
    samp_gbs = sampler_bytes_per_step(shape, B, N, k) / (samp_ms * 1e-3) / 1e9 if samp_ms > 0 else 0.0
    sampler = {"kernel": "row_stats, accept, draw (+ merges), select: the whole accept / reject + draw stage of one step",
               "bound": "hbm", "achieved": samp_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": samp_gbs / PEAK_HBM_GBS,
               "frac_of_measured_peak": samp_gbs / hbm_meas, "ms_per_step": samp_ms,
               "bytes_per_step": sampler_bytes_per_step(shape, B, N, k)}

    if args.calibrate_copy:
        P.probe_copy(1 << 30, 1)                           # ten dispatches of probe_copy_kernel, 1 GiB read + 1 GiB written each

    cpu = None
    if args.cpu_seqs > 0 and k > 0 and case.weights is not None:
        cpu = cpu_baseline(case, min(args.cpu_seqs, B), lazy_weights=args.row_major == "host")

    res = {
        "metric": "accepted tokens/s of batched spec-verify step", "value": emitted / (ms_per_step * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": shape.name + (f"-k{k}" if args.config == "cfg3" else "") + (f" at batch {B}" if args.batch is not None else ""),
                   "batch": B, "k": k, "chains": N, "rows_per_step": T,
                   "prefix_tokens": int(case.lengths.sum()), "drafts": args.drafts, "draft_sigma": list(shape.draft_sigma) if args.sigma is None else [args.sigma],
                   "verify": {None: "greedy" if shape.verify_mode == 0 else "stochastic, exponential-race draw, temperature 1.0",
                              0: "greedy", 1: "stochastic, exponential-race draw, temperature 1.0",
                              2: "sampled exact match, exponential-race draw, temperature 1.0"}[vmode]},
        "accepted_drafts_per_step": int(acc.sum()), "emitted_tokens_per_step": emitted,
        "accepted_drafts_tokens_per_s": int(acc.sum()) / (ms_per_step * 1e-3),
        "roofline": dominant, "roofline_other": other, "sampler": sampler, "rollback": rollback,
        "measured_peaks": peaks,
        "sampler_ms_per_step": samp_ms, "ms_per_step_without_event_brackets": plain_ms,
        "step_ms_without_event_brackets": step_spread,
        "ms_per_step_graph_replay": graph_ms,
        "consecutive_steps": consecutive,
        "cpu_baseline": cpu,
    }
    case.close()
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
