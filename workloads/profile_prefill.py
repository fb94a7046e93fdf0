"""Time the prefill entry points on a workload configuration's model.

    python -m workloads.profile_prefill [--config cfg2] [--prompts 64] [--tokens 512] [--rows 5,32]

For each `rows` value a verifier is set up whose steps hold that many rows per request (max_k = rows - 1), and
`prompts` seeded prompts of `tokens` tokens are prefetched together with verify_prefill_batch (`rows` tokens of each
per pass); then one prompt alone with verify_prefill (64-token chunks of a single sequence).  Prints one JSON
line with tokens per second of each.  Run from the repository root.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import torch


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="cfg2")
    ap.add_argument("--prompts", type=int, default=64)
    ap.add_argument("--tokens", type=int, default=512)
    ap.add_argument("--rows", default="5,32")
    args = ap.parse_args(argv)
    import workloads as W
    from workloads import synth
    from paper_2511_16193_amd import Verifier, pack_weights
    shape = W.CONFIGS[args.config]
    dev = torch.device("cuda:0")
    log = lambda *a: print(*a, file=sys.stderr, flush=True)
    log(f"weights for {shape.name} ...")
    weights = pack_weights(synth.make_weights(shape, dev))
    B, n = args.prompts, args.tokens
    prompts = torch.from_numpy(synth.make_tokens((B, n), shape.vocab, shape.seed, "prompt")).to(device=dev, dtype=torch.int32)
    page = 64
    res = {"config": shape.name, "prompts": B, "tokens_per_prompt": n, "batched": {}, "single_sequence": None}
    G = shape.n_q_heads // shape.n_kv_heads
    for rows in [int(x) for x in args.rows.split(",")]:
        pps = (n + rows + page - 1) // page + 2
        ver = Verifier(shape.model_fields(), weights, packed=True, max_batch=B, max_k=rows - 1, max_chains=1, max_seqs=B,
                       page_size=page, num_pages=B * pps + 4, max_pages_per_seq=pps, device="cuda:0")
        ids = list(range(B))
        times = []
        for rep in range(3):
            for b in ids:
                ver.seq_add(b, 0)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ver.prefill_batch(ids, prompts, [n] * B, want_logits=True)
            torch.cuda.synchronize()
            times.append(time.perf_counter() - t0)
            for b in ids:
                ver.seq_remove(b)
        t = min(times[1:])
        per_pass = min(rows, 256 // G)
        res["batched"][str(rows)] = {"rows_per_pass": B * per_pass, "seconds": t, "tokens_per_s": B * n / t}
        log(f"batched, {per_pass} tokens of each of {B} prompts per pass: {t * 1e3:.1f} ms, {B * n / t:.0f} tokens/s")
        if rows == int(args.rows.split(",")[-1]):
            times = []
            for rep in range(3):
                ver.seq_add(0, 0)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                ver.prefill(0, prompts[0], want_logits=True)
                torch.cuda.synchronize()
                times.append(time.perf_counter() - t0)
                ver.seq_remove(0)
            t = min(times[1:])
            res["single_sequence"] = {"seconds": t, "tokens_per_s": n / t}
            log(f"one prompt alone: {t * 1e3:.1f} ms, {n / t:.0f} tokens/s")
        ver.close()
        del ver
        torch.cuda.empty_cache()
    print(json.dumps(res))
    return 0


if __name__ == "__main__":
    sys.exit(main())
