"""Full-size parity: the benchmark workloads at their real shapes, in the launch configuration bench.py times.

 cfg2  7B-shaped dense decoder, 28 layers, B = 64, prefixes 1k-8k, k = 4
 cfg3  the same decoder at the large per-worker batch, B = 256, prefixes 2k-8k, k = 8 and k = 1
 cfg4  mixture-of-experts decoder, 48 layers, 128 experts top-8, B = 128
 cfg5  32B-shaped decoder, 64 layers, three chains of eight drafts over 16k-32k prefixes, B = 32

Requests are independent through the whole step, so parity on a request is exact parity for that request:
the oracle runs on a sample of requests.  What is held to what:

 (a) EVERY LAYER, at the stated tolerance.  The oracle's pass over the sampled requests records the residual
     stream entering every layer.  Each layer is then run on the device alone (sv_op_layer) ON THE ORACLE'S
     INPUT, through the very launches of a step, and its output is pushed through the oracle's final norm and
     LM head beside the oracle's own: the two sets of logits -- what the model would emit if it ended there --
     must agree within 2e-2 (the stated bf16 tolerance; the first layer, whose input is the bare embedding, within
     the one-layer value of the drift law of (c)), the layer's new K/V entries within one bf16 unit (and
     fewer than 1 % of them, over all layers, differ at all).  For the mixture of experts the router and the
     experts of every layer are additionally run on the oracle's own feed-forward input (sv_op_moe_ffn): every
     routing decision whose oracle margin exceeds 1e-4 must pick the same experts with the same weights.
 (b) EVERY DECISION, at the stated margin.  For all requests of the batch the oracle's accept / reject / draw /
     chain rule is applied to the logits the device's step produced: accepted lengths, kept chains and tokens
     must be the device's bit for bit except at margins below 1e-3.
 (c) End to end, the step's logits against the oracle's whole pass.  Two correct implementations drift apart
     over many layers (tests/test_oracle_drift.py shows and quantifies it on the CPU, oracle against a
     float32-accumulating copy of itself), so the bound here is that fixed law, not the per-layer tolerance:
     rms / spread < DRIFT_RMS_PER_SQRT_LAYER * sqrt(layers), maximum < DRIFT_MAX_OVER_RMS times that.  A sampled
     request whose tokens differ from the oracle's must have had an oracle margin below twice that maximum.
     The mixture of experts is chaotic beyond the first routing flip, so its 48-layer pass is held to (a) and
     (b) only and compared end to end on the model cut to two layers.
 (d) Properties that hold for every request whatever the numerics.
"""
import gc

import numpy as np
import pytest
import torch

from oracle import model as M
from oracle import verify as OV
import workloads as W
from harness import LOGIT_TOL, MARGIN, DRIFT_RMS_PER_SQRT_LAYER, DRIFT_MAX_OVER_RMS, decide

pytestmark = pytest.mark.gpu

ROUTE_MARGIN = 1e-4     # relative gap between the last kept and the first dropped expert probability below which the
                        # fp32 router and the float64 router may keep different experts on identical input
ROUTE_CLEAR = 5e-3      # the same on inputs that differ by the rounding flips of an attention block or of a layer or
                        # two (about one rms of the fixed drift law): it decides which rows are compared, not how closely


def spread_samples(lengths, count):
    """The shortest, the longest and requests spread evenly between them by batch index."""
    picks = {int(np.argmin(lengths)), int(np.argmax(lengths))}
    step = max(1, len(lengths) // max(1, count))
    b = step // 2
    while len(picks) < min(count, len(lengths)):
        picks.add(b % len(lengths))
        b += step
    return sorted(picks)


def test_cfg2_full_size_every_layer_every_decision():
    run_full("cfg2", lambda lengths: spread_samples(lengths, 8))


@pytest.mark.parametrize("k", [8, 1])
def test_cfg3_large_batch_full_size(k):
    """B = 256 requests of 2k-8k cached tokens, the per-worker batch of the paper's large-batch regime, at both
    ends of the draft-window sweep (k = 8: 2304 rows per step; k = 1: 512)."""
    run_full("cfg3", lambda lengths: spread_samples(lengths, 3), k=k)


def test_cfg4_moe_full_size_every_layer_every_decision():
    """All 48 layers at full width.  With random weights the router is chaotic end to end: over 48 layers every
    row meets a decision (8th against 9th expert) closer than the drift of the two residual streams, after which
    the row runs through other experts and its logits are unrelated.  Teacher-forced, every one of the 48 layers
    is pinned on its own."""
    run_full("cfg4", lambda lengths: spread_samples(lengths, 2), end_to_end=False)


def test_cfg4_moe_two_layers_full_width_logits_and_decisions():
    run_full("cfg4", lambda lengths: sorted({int(np.argmin(lengths)), int(np.argmax(lengths)), 5, 40, 77, 120}), n_layers=2)


def test_cfg5_32b_three_chains_full_size_every_layer_every_decision():
    """The long-tail configuration at its full size: 64 layers, d 5120, 40/8 heads, B = 32 requests with
    16k-32k cached tokens (206 GB of cache), three chains of eight drafts = 25 new rows per request (125 stacked
    rows per kv head: the skewed attention kernel in two row groups of four tiles, split over many chunks).  The
    row-major copy of the weights, which only the oracle reads, is kept on the host."""
    run_full("cfg5", lambda lengths: sorted({int(np.argmin(lengths)), int(np.argmax(lengths))}), weights_on_host=True)


def run_full(config, pick_sample, n_layers=None, weights_on_host=False, k=None, end_to_end=True):
    from workloads.device_case import DeviceCase
    import paper_2511_16193_amd as P
    shape = W.CONFIGS[config]
    if n_layers is not None:
        shape = W.scaled_down(shape, n_layers=n_layers)
    # the largest case needs nearly the whole device: give back what earlier tests' objects still hold
    gc.collect()
    torch.cuda.empty_cache()
    print(f"[full] building {shape.name} on the device", flush=True)
    case = DeviceCase(shape, k=k, keep_row_major="host" if weights_on_host else True)
    # drafts that do not come from the device path: q = softmax(N(0,1)) independent of the target
    case.independent_drafts(1.0)
    B, N, k, V, layers = case.B, case.N, case.k, shape.vocab, shape.n_layers
    n = 1 + N * k
    print("[full] device step", flush=True)
    out = case.step(want_logits=True)
    torch.cuda.synchronize()
    acc = out["accepted_len"].cpu().numpy()
    toks = out["out_tokens"].cpu().numpy()
    kept = out["best_chain"].cpu().numpy()
    drafts = case.drafts.cpu().numpy().astype(np.int64)

    # ---- (d) properties for all requests ----
    assert acc.min() >= 0 and acc.max() <= k
    assert kept.min() >= 0 and kept.max() < N
    for b in range(B):
        a = int(acc[b])
        assert np.array_equal(toks[b, :a], drafts[b, kept[b], :a])
        assert 0 <= toks[b, a] < V
        assert np.all(toks[b, a + 1:] == -1)
        assert case.ver.seq_len(b) == int(case.lengths[b]) + a + 1
    assert 0 < acc.sum() < B * k                      # both accepts and rejections occur

    # ---- (b) every decision of the batch from the device's own logits, in slices of 16 requests ----
    print("[full] the decision rule on the device's own logits, all requests", flush=True)
    exempt = 0
    for b0 in range(0, B, 16):
        b1 = min(B, b0 + 16)
        a_o, out_o, best_o, margin = decide(out["logits"][b0:b1].cpu().numpy().astype(np.float64), drafts[b0:b1],
                                            case.draft_probs[b0:b1].cpu().numpy(), case.uniforms[b0:b1].cpu().numpy(),
                                            OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 1.0, first_request=b0)
        for i, b in enumerate(range(b0, b1)):
            if acc[b] == a_o[i] and kept[b] == best_o[i] and np.array_equal(toks[b], out_o[i]):
                continue
            assert margin[i] < MARGIN, (b, acc[b], a_o[i], toks[b], out_o[i], kept[b], best_o[i], margin[i])
            exempt += 1
    print(f"[full] decisions identical for {B - exempt} of {B} requests; {exempt} within the 1e-3 margin", flush=True)
    assert exempt <= max(1, B // 8)

    # ---- the oracle's pass over the sample, every layer's input recorded ----
    sample = pick_sample(case.lengths)
    S = len(sample)
    spec = M.ModelSpec(**shape.model_fields())
    wn = W.weights_to_numpy(case.weights, lazy=True)
    caches = []
    for b in sample:
        L = int(case.lengths[b])
        c = M.SeqCache(spec, L + n + 1)
        for l in range(layers):
            kk, vv = case.kv_block(b, l)
            c.k[l][:L] = kk.float().cpu().numpy()
            c.v[l][:L] = vv.float().cpu().numpy()
        c.length = L
        caches.append(c)
    print(f"[full] oracle on requests {sample}", flush=True)
    x0 = case.x0.cpu().numpy().astype(np.int64)[sample]
    _, idx, vis = OV.new_token_layout(k, N)
    tokens = np.concatenate([x0[:, None], drafts[sample].reshape(S, N * k)], axis=1)
    pos = np.array([c.length for c in caches])[:, None] + idx[None]
    trace = {}
    logits = M.forward(spec, wn, caches, tokens, pos, np.broadcast_to(vis, (S, n, n)), trace=trace)
    hidden = trace["hidden"]

    # ---- (a) every layer on the oracle's input ----
    print("[full] every layer on the oracle's input", flush=True)
    case.reset()                                      # lengths back to the prefixes: the layers re-append their rows
    lm64 = np.asarray(wn["lm_head"], dtype=np.float64)
    gain = wn["final_norm"]

    def head_input(h):
        return M.round_to_storage(M.rms_norm(h, gain, spec.rms_eps), spec.dtype)

    worst, unclear_rows, flipped, entries = 0.0, 0, 0, 0
    for l in range(layers):
        h_in = torch.from_numpy(hidden[l].astype(np.float32)).to(case.device)
        res = case.ver.op_layer(sample, n, k, l, h_in, want_routing=True) if shape.n_experts else case.ver.op_layer(sample, n, k, l, h_in)
        h_dev = (res[0] if shape.n_experts else res).cpu().numpy().astype(np.float64)
        rows_ok = np.ones(S * n, dtype=bool)
        if shape.n_experts:
            ids_o, wts_o, margin = trace["routing"][l]
            # (i) the router and the experts on the oracle's own feed-forward input (identical on both sides): every
            # decision with an oracle margin above 1e-4 picks the same experts with the same weights, and the block's
            # output, added to the oracle's residual, gives the same logits within the stated tolerance
            lw = case.weights["layers"][l]
            a_in = torch.from_numpy(trace["ffn_input"][l].astype(np.float32)).to(torch.bfloat16)
            assert np.array_equal(a_in.float().numpy().astype(np.float64), trace["ffn_input"][l])     # already bf16 values
            y_dev, ids_f, wts_f = P.op_moe_ffn(a_in.to(case.device), lw["w_router"].to(case.device), lw["w_gate_up"].to(case.device),
                                               lw["w_down"].to(case.device), shape.top_k)
            ids_f, wts_f = ids_f.cpu().numpy(), wts_f.cpu().numpy()
            clear = margin > ROUTE_MARGIN
            unclear_rows += int((~clear).sum())
            for t in np.nonzero(clear)[0]:
                assert set(ids_f[t]) == set(ids_o[t]), (l, t, ids_f[t], ids_o[t], margin[t])
                got = dict(zip(ids_f[t], wts_f[t]))
                for e, w_ in zip(ids_o[t], wts_o[t]):
                    assert abs(got[e] - w_) < 5e-5, (l, t, e, got[e], w_)
            h_ffn = trace["ffn_residual"][l] + y_dev.cpu().numpy().astype(np.float64)
            dl = M.matmul_wt(head_input(h_ffn)[clear] - head_input(hidden[l + 1])[clear], lm64)
            assert float(np.max(np.abs(dl))) < LOGIT_TOL["bf16"], (l, float(np.max(np.abs(dl))))
            # (ii) the whole layer: its router sees an input that has already passed the layer's attention block on
            # both sides and differs by the rounding flips of that block (router logits move by ~1e-3), so only rows
            # whose decision is clear of that are compared: same experts, weights to 2e-3
            ids_d, wts_d = res[1].cpu().numpy(), res[2].cpu().numpy()
            rows_ok = margin > ROUTE_CLEAR
            for t in np.nonzero(rows_ok)[0]:
                assert set(ids_d[t]) == set(ids_o[t]), (l, t, ids_d[t], ids_o[t], margin[t])
                got = dict(zip(ids_d[t], wts_d[t]))
                for e, w_ in zip(ids_o[t], wts_o[t]):
                    assert abs(got[e] - w_) < 2e-3, (l, t, e, got[e], w_)
        dlogit = M.matmul_wt(head_input(h_dev)[rows_ok] - head_input(hidden[l + 1])[rows_ok], lm64)
        err = float(np.max(np.abs(dlogit))) if rows_ok.any() else 0.0
        worst = max(worst, err if l else 0.0)
        # Every layer is held to the stated tolerance but the first: its input is the bare embedding (spread 0.02), so
        # all it emits is its own output and its logits are a one-layer end-to-end result, which two correct
        # implementations already miss by 2.5e-2 at the 32B shape (tests/test_oracle_drift.py): the first layer is
        # held to the one-layer value of the drift law, never below the stated tolerance.
        bound = max(LOGIT_TOL["bf16"], DRIFT_MAX_OVER_RMS * DRIFT_RMS_PER_SQRT_LAYER * float(logits.std())) if l == 0 else LOGIT_TOL["bf16"]
        assert err < bound, f"layer {l}: logits of the layer's output differ by {err} (bound {bound})"
        for i, b in enumerate(sample):                # the layer's new cache entries
            L = int(case.lengths[b])
            kd, vd = case.ver.kv_read(b, l, L, n)
            kd, vd = kd.float().cpu().numpy(), vd.float().cpu().numpy()
            ko, vo = caches[i].k[l][L:L + n], caches[i].v[l][L:L + n]
            # One bf16 unit is at most 2^-7 of the value.  Besides, where the layer's normalised input itself has an
            # entry that rounds the other way on the two sides (one row in ten), every entry of the row moves by that
            # entry's unit times a weight, in absolute terms: at most 2^-5 (the unit of an input of 4 to 8) x 0.09
            # (a 4.5 sigma weight) = 3e-3, which is several units of the entries that happen to be small.
            assert np.all(np.abs(kd - ko) <= 2.0 ** -7 * np.abs(ko) + 3e-3), (l, b, float(np.max(np.abs(kd - ko) - 2.0 ** -7 * np.abs(ko))))
            assert np.all(np.abs(vd - vo) <= 2.0 ** -7 * np.abs(vo) + 3e-3), (l, b, float(np.max(np.abs(vd - vo) - 2.0 ** -7 * np.abs(vo))))
            flipped += int((kd != ko).sum() + (vd != vo).sum())
            entries += kd.size + vd.size
        if l % 8 == 0 or l == layers - 1:
            print(f"[full]   layer {l}: logit-equivalent error {err:.2e}", flush=True)
    print(f"[full] worst layer after the first: {worst:.2e} (bound {LOGIT_TOL['bf16']}); rows left out for a routing margin below "
          f"{ROUTE_MARGIN}: {unclear_rows} of {layers * S * n}", flush=True)
    assert unclear_rows <= 0.02 * layers * S * n
    # On identical input an entry differs only where the fp32 product sat within ~1e-6 of a rounding boundary, or, for
    # a row whose normalised input has such an entry itself (one row in ten at these widths), in ~2 % of that row's
    # entries: well under 1 % over all rows and layers.  (Every entry was held to one bf16 unit above.)
    print(f"[full] new cache entries that differ by one bf16 unit: {flipped} of {entries} ({flipped / entries:.2e})", flush=True)
    assert flipped < 0.01 * entries

    # ---- (c) end to end ----
    dev_logits = out["logits"][sample].cpu().numpy().astype(np.float64)
    diff = np.abs(dev_logits - logits)
    spread = float(logits.std())
    rms_bound = DRIFT_RMS_PER_SQRT_LAYER * np.sqrt(layers)
    print(f"[full] end to end: max per sampled request {diff.reshape(S, -1).max(axis=1)}, rms/spread "
          f"{float(np.sqrt(np.mean(diff ** 2))) / spread:.2e} (bound {rms_bound:.2e})", flush=True)
    if end_to_end:
        ok_rows = np.ones((S, n), dtype=bool)
        if shape.n_experts:
            per_layer = np.stack([m for (_, _, m) in trace["routing"]]).reshape(layers, S, n)
            # a row stays comparable while its own decisions and those of the rows it attends (the earlier new
            # rows of its request) are clear in every layer
            ok_rows = (np.cumsum(per_layer < ROUTE_CLEAR, axis=2) == 0).all(axis=0)
            print(f"[full] rows with every routing decision clear: {int(ok_rows.sum())} of {ok_rows.size}", flush=True)
            assert ok_rows.sum() >= ok_rows.size // 4
        rms = float(np.sqrt(np.mean(diff[ok_rows] ** 2))) / spread
        assert rms < rms_bound, rms
        max_bound = DRIFT_MAX_OVER_RMS * rms_bound * spread
        assert diff[ok_rows].max() < max_bound, (diff[ok_rows].max(), max_bound)
        # the sampled requests' tokens against the oracle's own decisions
        a_o, out_o, best_o, margin = [], [], [], []
        for i, b in enumerate(sample):
            r = decide(logits[i:i + 1], drafts[b:b + 1], case.draft_probs[b:b + 1].cpu().numpy(),
                       case.uniforms[b:b + 1].cpu().numpy(), OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 1.0, first_request=b)
            a_o.append(r[0][0]); out_o.append(r[1][0]); best_o.append(r[2][0]); margin.append(r[3][0])
        differ = 0
        for i, b in enumerate(sample):
            if acc[b] == a_o[i] and kept[b] == best_o[i] and np.array_equal(toks[b], out_o[i]):
                continue
            if not ok_rows[i].all():
                continue                                      # a routing decision too close to call
            assert margin[i] < 2.0 * max_bound, (b, toks[b], out_o[i], margin[i])
            differ += 1
        print(f"[full] sampled requests whose tokens differ from the oracle's end to end: {differ} of {S} "
              f"(each at an oracle margin below {2.0 * max_bound:.3f})", flush=True)
    case.close()
    del case, out, caches, wn, lm64, hidden, trace
    gc.collect()
    torch.cuda.empty_cache()
