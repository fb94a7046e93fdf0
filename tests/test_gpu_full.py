"""Full-size parity: the benchmark workloads (7B-shaped dense decoder, bf16, B=64, prefixes 1k-8k, k=4; the
mixture-of-experts decoder, 48 layers, 128 experts, B=128; the 32B-shaped decoder with three chains of eight drafts
over 16k-32k prefixes, B=32) with stochastic verification, in the launch
configuration bench.py times, checked against the oracle on a sample of requests (requests are independent
through the whole step, so parity on a request is exact parity for that request) and against properties that
hold for every request."""
import numpy as np
import pytest
import torch

from oracle import model as M
from oracle import verify as OV
import workloads as W
from harness import compare_step, LOGIT_TOL

pytestmark = pytest.mark.gpu


def test_cfg2_full_size_sampled_requests_and_invariants():
    run_full("cfg2", lambda lengths: sorted({int(np.argmin(lengths)), int(np.argmax(lengths)), 7}))


ROUTE_CLEAR = 5e-3      # a router decision with a relative probability gap above this is the same on both sides
                        # (measured: by layer 7 of the 48-layer run a gap between 2e-3 and 5e-3 has flipped)


def test_cfg4_moe_full_size_sampled_request_and_invariants():
    """All 48 layers at full width.  With random weights the router of a mixture-of-experts model is chaotic:
    over 48 layers every row meets a decision (8th against 9th expert) closer than the ~1e-3 by which the
    residual streams of the two sides differ, after which the row runs through other experts and its logits
    are unrelated.  So the 48-layer run is compared, besides the properties that hold for every request, on
    the cache entries of every layer reached before a row's first close decision; logits and decisions are
    compared on the same model cut to two layers."""
    # one request (the shortest prefix): the oracle widens ~40 experts' matrices to float64 per layer
    run_full("cfg4", lambda lengths: [int(np.argmin(lengths))])


def test_cfg4_moe_two_layers_full_width_logits_and_decisions():
    run_full("cfg4", lambda lengths: sorted({int(np.argmin(lengths)), int(np.argmax(lengths)), 5, 40, 77, 120}), n_layers=2)


def test_cfg5_32b_three_chains_full_size_sampled_request_and_invariants():
    """The long-tail configuration at its full size: 64 layers, d 5120, 40/8 heads, B = 32 requests with
    16k-32k cached tokens (206 GB of cache), three chains of eight drafts = 25 new rows per request (125 stacked
    rows per kv head: the skewed attention kernel in two row groups of four tiles, split over many chunks).  The
    row-major copy of the weights, which only the oracle reads, is kept on the host.  Oracle on the request with
    the shortest prefix."""
    run_full("cfg5", lambda lengths: [int(np.argmin(lengths))], weights_on_host=True)


def run_full(config, pick_sample, n_layers=None, weights_on_host=False):
    from workloads.device_case import DeviceCase
    shape = W.CONFIGS[config]
    if n_layers is not None:
        shape = W.scaled_down(shape, n_layers=n_layers)
    # the largest case needs nearly the whole device: give back what earlier tests' objects still hold
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    print(f"[full] building {shape.name} on the device", flush=True)
    case = DeviceCase(shape, keep_row_major="host" if weights_on_host else True)
    # drafts that do not come from the device path: q = softmax(N(0,1)) independent of the target
    case.independent_drafts(1.0)
    B, N, k, V = case.B, case.N, case.k, shape.vocab
    n = 1 + N * k
    print("[full] device step", flush=True)
    out = case.step(want_logits=True)
    torch.cuda.synchronize()
    acc = out["accepted_len"].cpu().numpy()
    toks = out["out_tokens"].cpu().numpy()
    drafts = case.drafts.cpu().numpy()

    # ---- properties for all 64 requests ----
    assert acc.min() >= 0 and acc.max() <= k
    kept = out["best_chain"].cpu().numpy()
    assert kept.min() >= 0 and kept.max() < N
    for b in range(B):
        a = int(acc[b])
        assert np.array_equal(toks[b, :a], drafts[b, kept[b], :a])
        assert 0 <= toks[b, a] < V
        assert np.all(toks[b, a + 1:] == -1)
        assert case.ver.seq_len(b) == int(case.lengths[b]) + a + 1
    assert 0 < acc.sum() < B * k                      # both accepts and rejections occur

    # ---- oracle on a sample (cfg2: the shortest, the longest and one more request) ----
    sample = pick_sample(case.lengths)
    spec = M.ModelSpec(**shape.model_fields())
    wn = W.weights_to_numpy(case.weights, lazy=True)
    caches = []
    for b in sample:
        L = int(case.lengths[b])
        c = M.SeqCache(spec, L + n + 1)
        for l in range(shape.n_layers):
            kk, vv = case.kv_block(b, l)
            c.k[l][:L] = kk.float().cpu().numpy()
            c.v[l][:L] = vv.float().cpu().numpy()
        c.length = L
        caches.append(c)
    print(f"[full] oracle on requests {sample}", flush=True)
    # the exponential-race draw is keyed by the request's index in the batch: run the oracle's sampler
    # with the same keys by placing the sampled requests at their batch positions
    x0 = case.x0.cpu().numpy().astype(np.int64)[sample]
    q = case.draft_probs[sample].cpu().numpy()
    u = case.uniforms[sample].cpu().numpy()
    _, idx, vis = OV.new_token_layout(k, N)
    tokens = np.concatenate([x0[:, None], drafts[sample].reshape(len(sample), N * k)], axis=1)
    pos = np.array([c.length for c in caches])[:, None] + idx[None]
    router_margins = []
    logits = M.forward(spec, wn, caches, tokens, pos, np.broadcast_to(vis, (len(sample), n, n)),
                       router_margins=router_margins)
    # every chain of the sampled requests, then the longest (lowest chain on ties), as the step does
    S = len(sample)
    per_chain = np.empty((S, N, k + 1, V))
    for c in range(N):
        per_chain[:, c, 0] = logits[:, 0]
        per_chain[:, c, 1:] = logits[:, 1 + c * k: 1 + (c + 1) * k]
    stream = (np.array(sample, dtype=np.uint64)[:, None] * np.uint64(N) + np.arange(N, dtype=np.uint64)[None, :]).reshape(-1)
    vc = OV.verify_stochastic(per_chain.reshape(S * N, k + 1, V), drafts[sample].reshape(S * N, k), q.reshape(S * N, k, V),
                              u.reshape(S * N, k + 1), stream, 1.0, OV.SAMPLE_EXP_RACE)
    ch_a = vc.accepted.reshape(S, N)
    want_chain = np.argmax(ch_a, axis=1)

    class v:                                                  # the kept chain's verdict per sampled request
        accepted = ch_a[np.arange(S), want_chain]
        token = vc.token.reshape(S, N)[np.arange(S), want_chain]
        # a decision of any chain can change which chain is kept: the margin is the smallest over the chains
        accept_margin = vc.accept_margin.reshape(S, N).min(axis=1)
        draw_margin = vc.draw_margin.reshape(S, N).min(axis=1)
    dev_logits = out["logits"][sample].cpu().numpy().astype(np.float64)
    diff = np.abs(dev_logits - logits)
    rel_rms = float(np.sqrt(np.mean(diff ** 2)) / logits.std())
    print(f"[full] logit error: max per sampled request {diff.reshape(len(sample), -1).max(axis=1)}, "
          f"mean {diff.mean():.2e}, rms/std {rel_rms:.2e}", flush=True)
    # Tolerance at full depth.  Both sides round activations to bf16 at the same points; a value that
    # sits within the fp32-vs-fp64 difference of a rounding boundary rounds differently on the two
    # sides (one unit = 2^-8 relative), which moves every output of the next projection by ~1e-4
    # relative, which in turn flips a few per cent of the 18944 gated activations ... the difference
    # settles at ~1e-3 of the residual stream per layer whatever the arithmetic, and adds up over the
    # layers as a random walk (measured: max 1.7e-2 after 1 layer, 2.4e-2 after 2, 5.4e-2 after 8,
    # 9.6e-2 after 28 on logits of standard deviation 1.2).  The 2e-2 bound holds per layer, not for 28:
    # here the bound is 2e-2 * sqrt(n_layers) on the maximum and 3 % of the logits' spread on the rms.
    # Mixture-of-experts: a row whose router, in some layer, kept its last expert by a relative margin below
    # the residual stream's ~1e-3 per-layer difference may keep another expert on the device; that row (and,
    # through attention among the new tokens, later rows of its request) then differs by more.  Such rows
    # are left out of the bound and reported.
    ok_rows = np.ones((len(sample), n), dtype=bool)
    if router_margins:
        per_layer = np.stack(router_margins).reshape(shape.n_layers, len(sample), n)
        # a row stays comparable while its own decisions and those of the rows it attends (the earlier new
        # rows of its request) are clear in every layer so far
        clear = np.cumsum(per_layer < ROUTE_CLEAR, axis=2) == 0                   # [layer, request, row]
        clear_upto = np.cumsum(~clear, axis=0) == 0                                # all layers <= l clear
        ok_rows = clear_upto[-1]
        depth = clear_upto.sum(axis=0)                                             # layers passed cleanly
        print(f"[full] layers passed before the first close router decision, per row: {depth.tolist()}; rows "
              f"with all {shape.n_layers} clear: {int(ok_rows.sum())} of {ok_rows.size}", flush=True)
        # cache entries of layer l depend on the decisions of layers < l
        checked = 0
        for i, b in enumerate(sample):
            L = int(case.lengths[b])
            for row in range(1 + int(acc[b])):
                for l in range(min(shape.n_layers, int(depth[i, row]) + 1)):
                    kd, vd = case.ver.kv_read(b, l, L + row, 1)
                    ko, vo = caches[i].k[l][L + row], caches[i].v[l][L + row]
                    kd, vd = kd.float().cpu().numpy()[0], vd.float().cpu().numpy()[0]
                    tol = 0.02 + 0.005 * l          # one bf16 unit at the entries' magnitude, looser with depth
                    assert np.max(np.abs(kd - ko)) < tol and np.max(np.abs(vd - vo)) < tol, (b, row, l)
                    checked += 1
        print(f"[full] cache entries compared at {checked} (row, layer) pairs", flush=True)
        assert checked >= 2 * len(sample)
    if ok_rows.any():
        # The rms bound is the substantive one.  The maximum is taken over millions of logits (25 rows x 152064 at
        # the 32B shape) whose differences are close to Gaussian: it sits 5.5 standard deviations out (measured:
        # 5.6 at the 7B shape, 5.7 at the 32B shape, with the generic attention kernel as with the MFMA ones), so
        # it is held to the larger of the per-layer rule and 6.5 times the rms actually seen.
        rms = float(np.sqrt(np.mean(diff[ok_rows] ** 2)))
        assert rms / logits.std() < 3e-2
        assert diff[ok_rows].max() < max(LOGIT_TOL["bf16"] * np.sqrt(shape.n_layers), 6.5 * rms)
    elif n_layers is not None:
        raise AssertionError("no comparable row in the shallow model")
    beyond = 0
    for i, b in enumerate(sample):
        a = int(v.accepted[i])
        want = list(drafts[b, want_chain[i], :a]) + [int(v.token[i])]
        got = list(toks[b, :acc[b] + 1])
        if a == acc[b] and want == got and kept[b] == want_chain[i]:
            continue
        if not ok_rows[i].all():
            continue                                          # a routing decision too close to call
        margin = min(float(v.accept_margin[i]), float(v.draw_margin[i]))
        allowed = max(1e-3, 2.0 * float(diff[i].max()))
        assert margin < allowed, (b, got, want, margin, float(diff[i].max()))
        beyond += margin >= 1e-3
    print(f"[full] sampled requests beyond the 1e-3 margin: {beyond}", flush=True)
    # the new cache entries of the sampled requests (layer 0: same inputs on both sides)
    for i, b in enumerate(sample):
        L = int(case.lengths[b])
        kd, vd = case.ver.kv_read(b, 0, L, 1 + int(acc[b]))
        # after the rollback the device holds x0 and the kept chain's accepted drafts; the oracle's forward pass
        # left every chain's rows where the pass wrote them
        rows = [L] + [L + 1 + int(kept[b]) * k + j for j in range(int(acc[b]))]
        ko, vo = caches[i].k[0][rows], caches[i].v[0][rows]
        # at most one bf16 unit apart, and only where the fp32 product sat on a rounding boundary (a few per
        # thousand of the entries) -- or, for a row whose normalised input has such an entry itself, a few per cent
        # (measured 2.2 % over the three rows of the 32B-shaped case)
        assert np.max(np.abs(kd.float().cpu().numpy() - ko)) < 0.02
        assert np.mean(kd.float().cpu().numpy() != ko) < 0.05
        assert np.mean(vd.float().cpu().numpy() != vo) < 0.05
    case.close()
    del case, out, caches, wn
    gc.collect()
    torch.cuda.empty_cache()
