"""Device parity of the whole verification step (C ABI) against the oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import model as M
from oracle import verify as OV
import workloads as W
from harness import Case, compare_step, LOGIT_TOL

pytestmark = pytest.mark.gpu


def noisy_greedy_drafts(case, b, x0, k, sigma, rng):
    import copy
    c = copy.deepcopy(case.caches[b])
    d, tok = [], int(x0)
    for _ in range(k):
        lg = M.forward(case.spec, case.wn, [c], np.array([[tok]]), np.array([[c.length]]), np.ones((1, 1, 1), dtype=bool))
        c.length += 1
        tok = int(np.argmax(lg[0, 0] + sigma * rng.standard_normal(case.spec.vocab)))
        d.append(tok)
    return d


def test_cfg1_tiny_fp32_greedy_chained_steps():
    """Workload configuration 1 (cfg1) in full: 2 layers, d 256, 4 heads x 64, vocab 2048, fp32; B=4 prompts of 128
    random ids; real prefill on both sides; k=4 drafts = argmax(target logits + noise) produced one token at
    a time by the oracle; greedy verification; 8 chained steps so that rollback is exercised.  Tokens and
    accepted lengths must be identical, logits within 1e-4, cache contents within 1e-4 after every step."""
    shape = W.CONFIGS["cfg1"]
    B, k = shape.batch, shape.k
    case = Case(shape, [0] * B, verify_mode=OV.GREEDY, synthetic_kv=False, extra_tokens=256)
    prompts = W.make_tokens((B, 128), shape.vocab, shape.seed, "prompt")
    lo, ld = case.prefill(prompts)
    assert np.max(np.abs(lo - ld)) < LOGIT_TOL["fp32"]
    x0 = np.argmax(lo, axis=-1)
    assert np.array_equal(x0, np.argmax(ld, axis=-1))
    rng = np.random.default_rng(shape.seed)
    total = 0
    for step in range(8):
        drafts = np.empty((B, 1, k), dtype=np.int64)
        for b in range(B):
            sigma = 1.0 if step % 4 == 3 else 0.02
            drafts[b, 0] = noisy_greedy_drafts(case, b, x0[b], k, sigma, rng)
        r, g = case.step(x0, drafts, None, None)
        err, exempt, diverged = compare_step(r, g, "fp32", k)
        assert not diverged, f"step {step}: {diverged}"
        x0 = np.array([r.out_tokens[b, r.accepted_len[b]] for b in range(B)])
        total += int(r.accepted_len.sum())
        lens = case.device_lengths()
        assert np.array_equal(lens, [c.length for c in case.caches])
        for b in range(B):
            for l in range(shape.n_layers):
                kd, vd = case.ver.kv_read(b, l, 0, int(lens[b]))
                assert np.max(np.abs(kd.cpu().numpy() - case.caches[b].k[l][:lens[b]])) < 1e-4
                assert np.max(np.abs(vd.cpu().numpy() - case.caches[b].v[l][:lens[b]])) < 1e-4
    assert 0 < total < 8 * B * k
    case.close()


SMALL_BF16 = W.Shape("small-bf16", 3, 256, 8, 2, 128, 512, 2048, dtype="bf16", batch=5, k=4, seed=77)


@pytest.mark.parametrize("k,n_chains,vmode,smode,packed", [
    (4, 1, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, False),
    (4, 1, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, True),
    (4, 1, OV.STOCHASTIC, OV.SAMPLE_INVERSE_CDF, True),
    (1, 1, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, True),
    (8, 1, OV.GREEDY, 0, False),
    (8, 1, OV.GREEDY, 0, True),
    (0, 1, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, True),
    (3, 3, OV.GREEDY, 0, True),
    (3, 3, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, False),
    (3, 3, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, True),
    (6, 3, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, True),     # 76 stacked rows per kv head: two row groups of 3 tiles
    (8, 3, OV.GREEDY, 0, True),                          # 100 stacked rows: two row groups of 4 tiles (the 32B
                                                         # configuration's three chains of eight drafts)
    (-4, 1, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, True),    # k = 4 with ragged draft windows (0..4 per request)
    (3, 3, OV.MATCH, OV.SAMPLE_EXP_RACE, True),          # sampled exact match, three chains
    (4, 1, OV.MATCH, OV.SAMPLE_INVERSE_CDF, True),
    (-4, 2, OV.MATCH, OV.SAMPLE_EXP_RACE, True),         # ... with ragged windows
])
def test_small_bf16_step_with_synthetic_cache(k, n_chains, vmode, smode, packed):
    """bf16 decoder small enough for the oracle (3 layers, d 256, 8 q / 2 kv heads x 128, vocab 2048) over a
    synthetic cache whose lengths are ragged and span several split-KV chunks and a partial tile
    (0, 31, 1024, 2500, 4133 entries), so the MFMA attention's tiling, masking and chunk merge are all hit.
    packed: projection weights (and with them the activations between kernels) in the library's
    streaming order, which selects the weight-streaming projection kernel.
    Drafts come from target-independent q (about half are accepted because random-weight targets are nearly
    flat).  Two consecutive steps: the second runs on the rolled-back cache."""
    ragged = k < 0          # per-request draft windows: the requests of one launch verify different numbers of drafts
    k = abs(k)
    shape = W.scaled_down(SMALL_BF16, k=k, n_chains=n_chains)
    lengths = [0, 31, 1024, 2500, 4133]
    B, V = len(lengths), shape.vocab
    case = Case(shape, lengths, verify_mode=vmode, sample_mode=smode, packed=packed)
    x0 = W.make_tokens((B,), V, shape.seed, "x0")
    alive = np.ones(B, dtype=bool)
    accepted = 0
    for step in range(2):
        if k:
            q = W.make_random_q((B, n_chains, k), V, 1.0, shape.seed + step)
            drafts = W.sample_from(q, shape.seed + step).numpy()
        else:
            q, drafts = None, np.zeros((B, 1, 0), dtype=np.int64)
        if vmode == OV.GREEDY and k:
            # give greedy verification something to accept: the oracle's own greedy continuation for some chains
            import copy
            for b in range(B):
                c = copy.deepcopy(case.caches[b])
                tok = int(x0[b])
                for i in range(k):
                    lg = M.forward(case.spec, case.wn, [c], np.array([[tok]]), np.array([[c.length]]),
                                   np.ones((1, 1, 1), dtype=bool))
                    c.length += 1
                    tok = int(np.argmax(lg[0, 0]))
                    if i < 1 + b % k:
                        drafts[b, (b + step) % n_chains, i] = tok
        u = W.make_uniforms((B, n_chains, k + 1), shape.seed + step)
        if vmode == OV.MATCH and k:
            # ... and match verification: the oracle's own sampled continuation under the (request, slot) keys
            import copy
            for b in range(B):
                c = copy.deepcopy(case.caches[b])
                tok = int(x0[b])
                for i in range(k):
                    lg = M.forward(case.spec, case.wn, [c], np.array([[tok]]), np.array([[c.length]]),
                                   np.ones((1, 1, 1), dtype=bool))
                    c.length += 1
                    p = M.softmax(lg[0, :1], axis=-1)
                    if smode == OV.SAMPLE_INVERSE_CDF:
                        t, _ = OV.draw_inverse_cdf(p, np.array([u[b, 0, i]], dtype=np.float64))
                    else:
                        t, _ = OV.draw_exp_race(p, np.array([u[b, 0, i]], dtype=np.float32), np.array([b], dtype=np.uint64))
                    tok = int(t[0])
                    if i < 1 + b % k:
                        drafts[b, (b + step) % n_chains, i] = tok
        lens = np.array([(b + step) % (k + 1) for b in range(B)], dtype=np.int64) if ragged else None
        r, g = case.step(x0, drafts, q if vmode == OV.STOCHASTIC else None, u if vmode != OV.GREEDY else None,
                         draft_lens=lens)
        if ragged:
            assert np.all(g["accepted_len"] <= lens)
        # rows of requests that diverged earlier (exempt decisions) are no longer comparable
        if not alive.all():
            for key in g:
                g[key][~alive] = {"logits": r.logits, "accepted_len": r.accepted_len, "out_tokens": r.out_tokens,
                                  "best_chain": r.best_chain}[key][~alive]
        err, exempt, diverged = compare_step(r, g, "bf16", k)
        alive[diverged] = False
        accepted += int(r.accepted_len.sum())
        x0 = np.array([r.out_tokens[b, r.accepted_len[b]] for b in range(B)])
        lens = case.device_lengths()
        want = np.array([c.length for c in case.caches])
        assert np.array_equal(lens[alive], want[alive])
        for b in np.nonzero(alive)[0]:
            lo = int(lengths[b])
            if lens[b] > lo:
                # layer 0: inputs are identical on both sides, so the bf16 entries agree except where the
                # fp32 value sat within ~1e-6 of a rounding boundary.  Last layer: the residual stream
                # already differs by ~1e-3 relative, so entries may differ by one or two units.
                for l, frac, atol in ((0, 0.01, 0.02), (shape.n_layers - 1, 1.0, 0.03)):
                    kd, vd = case.ver.kv_read(int(b), l, lo, int(lens[b]) - lo)
                    ko, vo = case.caches[b].k[l][lo:lens[b]], case.caches[b].v[l][lo:lens[b]]
                    kd, vd = kd.float().cpu().numpy(), vd.float().cpu().numpy()
                    assert np.max(np.abs(kd - ko)) < atol and np.max(np.abs(vd - vo)) < atol
                    assert np.mean(kd != ko) <= frac and np.mean(vd != vo) <= frac
    assert alive.sum() >= B - 1
    if k:
        assert accepted > 0
    case.close()


WIDE_FFN = W.Shape("wide-ffn-bf16", 1, 256, 8, 2, 128, 33792, 2048, dtype="bf16", batch=32, k=4, seed=91)


def test_bf16_wide_ffn_gate_up_launch_with_a_short_last_round():
    """One layer whose FFN is 33792 wide under 160 rows (32 requests, k = 4): 264 strips of 128 features for one
    160-row tile, i.e. one full round of 256 work-groups and a last round of 8 strips, which the fused gate/up
    projection hands to 64-row work-groups of half a strip in the same launch.  Logits and decisions against the
    oracle; the down projection that follows reads every feature, so a strip left out or written twice shows."""
    shape = WIDE_FFN
    B, V, k = shape.batch, shape.vocab, shape.k
    lengths = [5 + 7 * b for b in range(B)]
    case = Case(shape, lengths, verify_mode=OV.STOCHASTIC, sample_mode=OV.SAMPLE_EXP_RACE, packed=True)
    x0 = W.make_tokens((B,), V, shape.seed, "x0")
    q = W.make_random_q((B, 1, k), V, 1.0, shape.seed)
    drafts = W.sample_from(q, shape.seed).numpy()
    u = W.make_uniforms((B, 1, k + 1), shape.seed)
    r, g = case.step(x0, drafts, q, u)
    err, exempt, diverged = compare_step(r, g, "bf16", k)
    assert err < LOGIT_TOL["bf16"]
    assert len(diverged) <= 1
    keep = np.array([b not in diverged for b in range(B)])
    assert np.array_equal(case.device_lengths()[keep], np.array([c.length for c in case.caches])[keep])
    case.close()


TALL_BATCH = W.Shape("tall-batch-bf16", 2, 256, 8, 2, 128, 1152, 2048, dtype="bf16", batch=258, k=4, seed=93)


def test_bf16_step_through_the_256_row_projection_kernel():
    """1290 rows (258 requests, k = 4) with the 256 x 256 projection kernel forced on for every projection whose
    output is a multiple of 256 wide (QKV, O, the LM head, and the gated gate/up form with its bf16 epilogue): five
    whole row blocks and one of ten rows, nine gate/up strips, reductions of four and of eighteen fills.  Logits and
    decisions against the oracle; lengths after the rollback."""
    import paper_2511_16193_amd as P
    shape = TALL_BATCH
    B, V, k = shape.batch, shape.vocab, shape.k
    lengths = [3 + (11 * b) % 70 for b in range(B)]
    case = Case(shape, lengths, verify_mode=OV.STOCHASTIC, sample_mode=OV.SAMPLE_EXP_RACE, packed=True)
    case.ver.set_option(P.SV_OPT_GEMM_TILE, 1)
    x0 = W.make_tokens((B,), V, shape.seed, "x0")
    q = W.make_random_q((B, 1, k), V, 1.0, shape.seed)
    drafts = W.sample_from(q, shape.seed).numpy()
    u = W.make_uniforms((B, 1, k + 1), shape.seed)
    r, g = case.step(x0, drafts, q, u)
    err, exempt, diverged = compare_step(r, g, "bf16", k)
    assert err < LOGIT_TOL["bf16"]
    assert len(diverged) <= max(1, B // 8)
    keep = np.array([b not in diverged for b in range(B)])
    assert np.array_equal(case.device_lengths()[keep], np.array([c.length for c in case.caches])[keep])
    case.close()


@pytest.mark.parametrize("packed", [False, True])
def test_bf16_prefill_then_step(packed):
    """Real prefill on both sides (no synthetic cache): prompts of 150 tokens run through verify_prefill in chunks,
    every token cached; then one verification step on top.  Last-row logits of the prefill and the step's results
    against the oracle."""
    shape = W.scaled_down(SMALL_BF16, batch=3, k=4)
    B, k, V = 3, 4, shape.vocab
    case = Case(shape, [0] * B, verify_mode=OV.STOCHASTIC, synthetic_kv=False, extra_tokens=256, packed=packed)
    prompts = W.make_tokens((B, 150), V, shape.seed, "prompt")
    lo, ld = case.prefill(prompts)
    assert np.max(np.abs(lo - ld)) < LOGIT_TOL["bf16"]
    assert np.array_equal(case.device_lengths(), [150] * B)
    for b in range(B):                       # layer 0 entries: same inputs on both sides
        kd, vd = case.ver.kv_read(b, 0, 0, 150)
        assert np.mean(kd.float().cpu().numpy() != case.caches[b].k[0][:150]) < 0.01
        assert np.mean(vd.float().cpu().numpy() != case.caches[b].v[0][:150]) < 0.01
    x0 = np.argmax(lo, axis=-1)
    q = W.make_random_q((B, 1, k), V, 1.0, shape.seed)
    drafts = W.sample_from(q, shape.seed).numpy()
    u = W.make_uniforms((B, 1, k + 1), shape.seed)
    r, g = case.step(x0, drafts, q, u)
    err, exempt, diverged = compare_step(r, g, "bf16", k)
    assert len(diverged) <= 1
    case.close()


@pytest.mark.parametrize("k", [4, 8])
def test_bf16_batched_prefill_of_ragged_prompts(k):
    """Prompts of 1, 3, 5, 37, 150 and 151 tokens prefetched together through verify_prefill_batch (k + 1 tokens
    of each per pass; the short ones drop out, the last pass is ragged), handed over in mixed order; last-token
    logits, lengths and the cache against the oracle's plain causal pass, then one verification step on top."""
    shape = W.scaled_down(SMALL_BF16, batch=6, k=k)
    V = shape.vocab
    lens = [37, 1, 151, 5, 150, 3]
    B = len(lens)
    case = Case(shape, [0] * B, verify_mode=OV.STOCHASTIC, synthetic_kv=False, extra_tokens=256, packed=True)
    prompts = W.make_tokens((B, max(lens)), V, shape.seed + 1, "prompt")
    lo = np.stack([OV.prefill(case.spec, case.wn, case.caches[b], prompts[b, :lens[b]])[-1] for b in range(B)])
    ld = case.ver.prefill_batch(list(range(B)), torch.from_numpy(prompts).to(torch.int32), lens).cpu().numpy()
    assert np.max(np.abs(lo - ld)) < LOGIT_TOL["bf16"]
    assert np.array_equal(case.device_lengths(), lens)
    for b in range(B):                       # layer 0 entries: same inputs on both sides
        kd, vd = case.ver.kv_read(b, 0, 0, lens[b])
        assert np.mean(kd.float().cpu().numpy() != case.caches[b].k[0][:lens[b]]) < 0.01
        assert np.mean(vd.float().cpu().numpy() != case.caches[b].v[0][:lens[b]]) < 0.01
        kd, vd = case.ver.kv_read(b, shape.n_layers - 1, 0, lens[b])
        assert np.max(np.abs(kd.float().cpu().numpy() - case.caches[b].k[shape.n_layers - 1][:lens[b]])) < 0.03
    x0 = np.argmax(lo, axis=-1)
    q = W.make_random_q((B, 1, k), V, 1.0, shape.seed)
    drafts = W.sample_from(q, shape.seed).numpy()
    u = W.make_uniforms((B, 1, k + 1), shape.seed)
    r, g = case.step(x0, drafts, q, u)
    err, exempt, diverged = compare_step(r, g, "bf16", k)
    assert len(diverged) <= 1
    # a second batch of prompts appended to two of the sequences (prefill continues an existing cache)
    more = W.make_tokens((2, 20), V, shape.seed + 2, "more")
    for i, b in enumerate((4, 1)):
        OV.prefill(case.spec, case.wn, case.caches[b], more[i, :20 - 7 * i])
    before = case.device_lengths()
    case.ver.prefill_batch([4, 1], torch.from_numpy(more).to(torch.int32), [20, 13], want_logits=False)
    after = case.device_lengths()
    assert after[4] == before[4] + 20 and after[1] == before[1] + 13 and np.array_equal(np.delete(after, [1, 4]), np.delete(before, [1, 4]))
    assert np.array_equal(after, [c.length for c in case.caches])
    case.close()


def test_batched_prefill_refuses_bad_arguments():
    from paper_2511_16193_amd import SvError
    import ctypes as C
    shape = W.scaled_down(SMALL_BF16, batch=2, k=4)
    case = Case(shape, [0, 0], verify_mode=OV.GREEDY, synthetic_kv=False, packed=True)
    tok = torch.zeros((2, 8), dtype=torch.int32, device="cuda:0")
    lib, ctx = case.ver.lib, case.ver.ctx
    ids, asc, ok = (C.c_int32 * 2)(0, 1), (C.c_int32 * 2)(3, 5), (C.c_int32 * 2)(5, 3)
    assert lib.verify_prefill_batch(ctx, ids, 2, tok.data_ptr(), 8, asc, None) == -1          # not longest first
    assert lib.verify_prefill_batch(ctx, ids, 2, tok.data_ptr(), 4, ok, None) == -1           # longer than the pitch
    assert lib.verify_prefill_batch(ctx, (C.c_int32 * 2)(0, 7), 2, tok.data_ptr(), 8, ok, None) < 0   # no such sequence
    assert np.array_equal(case.device_lengths(), [0, 0])
    assert lib.verify_prefill_batch(ctx, ids, 2, tok.data_ptr(), 8, ok, None) == 0
    assert np.array_equal(case.device_lengths(), [5, 3])
    case.close()
