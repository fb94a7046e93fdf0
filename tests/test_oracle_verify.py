"""Pins of the oracle's accept/reject, samplers, chain choice and rollback
against closed forms, exact enumeration, chi-square statistics and plain
one-token-at-a-time decoding."""
import os

import numpy as np
import pytest
from scipy import stats

from oracle import model as M
from oracle import verify as OV
import workloads as W

HERE = os.path.dirname(os.path.abspath(__file__))
ALPHA = 1e-3
N_TRIALS = 1_000_000
CHUNK = 100_000


def softmax(x):
    return M.softmax(np.asarray(x, dtype=np.float64), axis=-1)


# --------------------------------------------------- counter-based RNG ---

def test_race_generator_reproduces_published_splitmix64_words():
    want = [int(line, 16) for line in open(os.path.join(HERE, "golden", "splitmix64_seed0.txt"))
            if not line.startswith("#") and line.strip()]
    # key 0 = stream 0 and u with an all-zero bit pattern
    U = OV.race_uniforms(np.array([0.0], dtype=np.float32), np.array([0], dtype=np.uint64), 3)[0]
    for v in range(3):
        hi = np.float32(want[v] >> 32)
        assert U[v] == (hi + np.float32(0.5)) * np.float32(2.0 ** -32)


def test_race_uniforms_are_uniform_and_keyed():
    u = np.array([0.25, 0.25, 0.75], dtype=np.float32)
    s = np.array([0, 1, 0], dtype=np.uint64)
    U = OV.race_uniforms(u, s, 200000).astype(np.float64)
    assert U.min() > 0.0 and U.max() <= 1.0
    for r in range(3):
        assert stats.kstest(U[r], "uniform").pvalue > ALPHA
    # different stream or different u -> unrelated rows
    assert abs(np.corrcoef(U[0], U[1])[0, 1]) < 0.01
    assert abs(np.corrcoef(U[0], U[2])[0, 1]) < 0.01
    assert np.array_equal(U, OV.race_uniforms(u, s, 200000).astype(np.float64))


# ------------------------------------------------------------- draws ---

def test_inverse_cdf_against_brute_force():
    rng = np.random.default_rng(0)
    w = rng.random((300, 9))
    w[rng.random((300, 9)) < 0.3] = 0.0
    w[:, 4] += 0.1
    u = rng.random(300)
    tok, _ = OV.draw_inverse_cdf(w, u)
    for s in range(300):
        t, run, want = u[s] * w[s].sum(), 0.0, None
        for v in range(9):
            run += w[s, v]
            if run > t:
                want = v
                break
        assert tok[s] == want
        assert w[s, tok[s]] > 0


@pytest.mark.parametrize("mode", [OV.SAMPLE_INVERSE_CDF, OV.SAMPLE_EXP_RACE])
def test_draw_law_chi_square(mode):
    rng = np.random.default_rng(4)
    w = rng.random(16) ** 3
    w[5] = 0.0
    counts = np.zeros(16)
    seed_rng = np.random.default_rng(40)
    for c in range(N_TRIALS // CHUNK):
        u = seed_rng.random(CHUNK, dtype=np.float32)
        ww = np.broadcast_to(w, (CHUNK, 16))
        if mode == OV.SAMPLE_INVERSE_CDF:
            tok, _ = OV.draw_inverse_cdf(ww, u.astype(np.float64))
        else:
            tok, _ = OV.draw_exp_race(ww, u, np.arange(c * CHUNK, (c + 1) * CHUNK, dtype=np.uint64))
        counts += np.bincount(tok, minlength=16)
    assert counts[5] == 0
    keep = w > 0
    chi2 = np.sum((counts[keep] - N_TRIALS * w[keep] / w.sum()) ** 2 / (N_TRIALS * w[keep] / w.sum()))
    assert chi2 < stats.chi2.ppf(1 - ALPHA, keep.sum() - 1)


# ------------------------------------------ one-token law, enumerated ---

@pytest.mark.parametrize("V", [4, 7, 16])
def test_one_token_law_equals_target_by_enumeration(V):
    """k=1.  The law of the emitted first token, integrating the draft x ~ q and
    both uniforms exactly (acceptance threshold by bisection through the
    oracle, residual law by a dense sorted grid of u through the oracle), must
    equal p."""
    rng = np.random.default_rng(V)
    logits = rng.standard_normal((1, 2, V)) * 1.5
    p = softmax(logits[0, 0])
    q = softmax(rng.standard_normal(V) * 1.5)
    G = 1 << 16
    grid = (np.arange(G) + 0.5) / G
    law = np.zeros(V)
    for x in range(V):
        drafts = np.full((1, 1), x)
        qq = q.reshape(1, 1, V)
        lo, hi = 0.0, 1.0                               # accept iff u < t(x)
        for _ in range(50):
            mid = 0.5 * (lo + hi)
            r = OV.verify_stochastic(logits, drafts, qq, np.array([[mid, 0.5]]), np.zeros(1, np.uint64),
                                     1.0, OV.SAMPLE_INVERSE_CDF)
            if r.accepted[0] == 1:
                lo = mid
            else:
                hi = mid
        t = hi if hi < 1.0 else 1.0
        law[x] += q[x] * t
        if t < 1.0:                                       # residual law: measure of u2 per token
            S = G
            r = OV.verify_stochastic(np.broadcast_to(logits, (S, 2, V)), np.broadcast_to(drafts, (S, 1)),
                                     np.broadcast_to(qq, (S, 1, V)),
                                     np.stack([np.full(S, min(1.0 - 1e-12, t + 1e-9)), grid], axis=1),
                                     np.zeros(S, np.uint64), 1.0, OV.SAMPLE_INVERSE_CDF)
            assert np.all(r.accepted == 0)
            law += q[x] * (1.0 - t) * np.bincount(r.token, minlength=V) / S
    assert np.max(np.abs(law - p)) < 1e-3
    assert abs(law.sum() - 1.0) < 1e-9


# ---------------------------------------------- toy Markov-chain model ---

def toy_tables(seed, V=16, sigma=0.7, context_free=False):
    rng = np.random.default_rng(seed)
    T = rng.standard_normal((V, V)) * 1.5
    if context_free:
        T[:] = T[0]
    noise = rng.standard_normal((V, V)) * sigma
    if context_free:
        noise[:] = noise[0]
    return T, softmax(T + noise)


def run_toy(T, Q, k, n_trials, seed, sample_mode, one_hot=False):
    """Drafts d_i ~ Q[d_{i-1}] (d_0 = x0), target rows T[x0], T[d_1]..T[d_k]."""
    V = T.shape[0]
    rng = np.random.default_rng(seed)
    x0 = rng.integers(0, V, n_trials)
    drafts = np.empty((n_trials, k), dtype=np.int64)
    prev = x0
    cdfQ = np.cumsum(Q, axis=-1)
    for i in range(k):
        r = rng.random(n_trials)
        drafts[:, i] = np.minimum(np.sum(cdfQ[prev] <= r[:, None], axis=-1), V - 1)
        prev = drafts[:, i]
    ctx = np.concatenate([x0[:, None], drafts], axis=1)                # [S, k+1]
    logits = T[ctx]                                                    # [S, k+1, V]
    qrows = None if one_hot else Q[ctx[:, :k]]
    u = rng.random((n_trials, k + 1), dtype=np.float32)
    v = OV.verify_stochastic(logits, drafts, qrows, u, np.arange(n_trials, dtype=np.uint64) + seed * n_trials,
                             1.0, sample_mode)
    return x0, drafts, v


@pytest.mark.parametrize("mode", [OV.SAMPLE_INVERSE_CDF, OV.SAMPLE_EXP_RACE])
def test_output_distribution_matches_target_chi_square(mode):
    """10^6 trials, V=16, k=4, context-dependent tables.  First emitted token
    given x0 follows P[x0]; second emitted token given the first follows
    P[first]; first-slot acceptance rate is 1 - TV(p, q)."""
    T, Q = toy_tables(11)
    P = softmax(T)
    V, k = 16, 4
    c1 = np.zeros((V, V))
    c2 = np.zeros((V, V))
    acc1 = np.zeros(V)
    nx0 = np.zeros(V)
    for c in range(N_TRIALS // CHUNK):
        x0, drafts, v = run_toy(T, Q, k, CHUNK, 100 + c, mode)
        assert v.accepted.max() <= k and v.accepted.min() >= 0
        first = np.where(v.accepted >= 1, drafts[:, 0], v.token)
        np.add.at(c1, (x0, first), 1)
        has2 = v.accepted >= 1
        second = np.where(v.accepted >= 2, drafts[:, 1], v.token)
        np.add.at(c2, (first[has2], second[has2]), 1)
        np.add.at(acc1, x0[has2], 1)
        np.add.at(nx0, x0, 1)
    for counts in (c1, c2):
        exp = counts.sum(axis=1, keepdims=True) * P
        chi2 = np.sum((counts - exp) ** 2 / exp)
        assert chi2 < stats.chi2.ppf(1 - ALPHA, V * (V - 1))
    want = 1.0 - 0.5 * np.sum(np.abs(P - Q), axis=-1)               # sum min(p,q)
    z = (acc1 - nx0 * want) / np.sqrt(nx0 * want * (1 - want))
    assert np.max(np.abs(z)) < 4.5


def test_accepted_length_law_context_free():
    """With the same p and q at every slot, acceptances are i.i.d. with
    probability beta = sum min(p,q), so P(a) = beta^a (1-beta) for a < k and
    beta^k for a = k (Section 4.1 of the paper)."""
    T, Q = toy_tables(12, context_free=True)
    P = softmax(T)
    beta = np.sum(np.minimum(P[0], Q[0]))
    k, n = 4, 400_000
    hist = np.zeros(k + 1)
    for c in range(4):
        _, _, v = run_toy(T, Q, k, n // 4, 200 + c, OV.SAMPLE_INVERSE_CDF)
        hist += np.bincount(v.accepted, minlength=k + 1)
    want = np.array([beta ** a * (1 - beta) for a in range(k)] + [beta ** k]) * n
    chi2 = np.sum((hist - want) ** 2 / want)
    assert chi2 < stats.chi2.ppf(1 - ALPHA, k)


def test_equal_distributions_accept_everything():
    T, _ = toy_tables(13)
    P = softmax(T)
    _, _, v = run_toy(T, P, 4, 50_000, 300, OV.SAMPLE_INVERSE_CDF)
    assert np.all(v.accepted == 4)


@pytest.mark.parametrize("mode", [OV.SAMPLE_INVERSE_CDF, OV.SAMPLE_EXP_RACE])
def test_one_hot_drafts_keep_the_target_law(mode):
    """q = None (one-hot drafts): 'accept with probability p(x), else draw from p
    without x' has the same law as 'draw from p and compare with x': p."""
    T, Q = toy_tables(14)
    P = softmax(T)
    V = 16
    counts = np.zeros((V, V))
    for c in range(5):
        x0, drafts, v = run_toy(T, Q, 2, 100_000, 400 + c, mode, one_hot=True)
        first = np.where(v.accepted >= 1, drafts[:, 0], v.token)
        np.add.at(counts, (x0, first), 1)
    exp = counts.sum(axis=1, keepdims=True) * P
    assert np.sum((counts - exp) ** 2 / exp) < stats.chi2.ppf(1 - ALPHA, V * (V - 1))


def test_zero_temperature_limit_is_greedy():
    rng = np.random.default_rng(6)
    S, k, V = 2000, 3, 16
    logits = rng.standard_normal((S, k + 1, V))
    g = np.argmax(logits, axis=-1)
    drafts = np.where(rng.random((S, k)) < 0.7, g[:, :k], rng.integers(0, V, (S, k)))
    u = rng.random((S, k + 1), dtype=np.float32)
    gr = OV.verify_greedy(logits, drafts)
    st = OV.verify_stochastic(logits, drafts, None, u, np.arange(S, dtype=np.uint64), 1e-4,
                              OV.SAMPLE_INVERSE_CDF)
    sure = gr.accept_margin > 1e-2          # at T=1e-4 a gap of 1e-2 is e^-100
    assert sure.sum() > S // 2
    assert np.array_equal(gr.accepted[sure], st.accepted[sure])
    assert np.array_equal(gr.token[sure], st.token[sure])


def test_greedy_rule_brute_force():
    rng = np.random.default_rng(8)
    S, k, V = 500, 4, 6
    logits = np.round(rng.standard_normal((S, k + 1, V)), 1)      # coarse values -> ties occur
    drafts = rng.integers(0, V, (S, k))
    r = OV.verify_greedy(logits, drafts)
    for s in range(S):
        a = 0
        while a < k and drafts[s, a] == min(v for v in range(V) if logits[s, a, v] == logits[s, a].max()):
            a += 1
        assert r.accepted[s] == a
        assert r.token[s] == min(v for v in range(V) if logits[s, a, v] == logits[s, a].max())


def test_ragged_draft_lengths():
    rng = np.random.default_rng(9)
    S, k, V = 300, 4, 8
    logits = rng.standard_normal((S, k + 1, V))
    g = np.argmax(logits, axis=-1)
    drafts = g[:, :k].copy()                      # every draft would match
    lens = rng.integers(0, k + 1, S)
    r = OV.verify_greedy(logits, drafts, lens)
    assert np.array_equal(r.accepted, lens)
    assert np.array_equal(r.token, g[np.arange(S), lens])
    u = rng.random((S, k + 1), dtype=np.float32)
    q = softmax(logits[:, :k])                    # q == p: accepts all it is allowed to test
    r = OV.verify_stochastic(logits, drafts, q, u, np.arange(S, dtype=np.uint64), 1.0,
                             OV.SAMPLE_INVERSE_CDF, lens)
    assert np.array_equal(r.accepted, lens)


# ---------------------------- whole step: greedy == plain decoding ---

def spec_of(shape):
    return M.ModelSpec(**shape.model_fields())


def autoregressive_greedy(spec, wn, prompt, n_out):
    c = M.SeqCache(spec, len(prompt) + n_out + 2)
    logits = OV.prefill(spec, wn, c, prompt)
    out = [int(np.argmax(logits[-1]))]
    while len(out) < n_out:
        lg = M.forward(spec, wn, [c], np.array([[out[-1]]]), np.array([[c.length]]),
                       np.ones((1, 1, 1), dtype=bool))
        c.length += 1
        out.append(int(np.argmax(lg[0, 0])))
    return out, c


def noisy_greedy_drafts(spec, wn, cache, x0, k, sigma, rng):
    """d_i = argmax(target logits + N(0, sigma^2)), produced one token at a time
    on a copy of the cache."""
    import copy
    c = copy.deepcopy(cache)
    d, tok = [], x0
    for _ in range(k):
        lg = M.forward(spec, wn, [c], np.array([[tok]]), np.array([[c.length]]), np.ones((1, 1, 1), dtype=bool))
        c.length += 1
        tok = int(np.argmax(lg[0, 0] + sigma * rng.standard_normal(spec.vocab)))
        d.append(tok)
    return d


@pytest.mark.parametrize("n_chains", [1, 3])
def test_greedy_verification_reproduces_plain_decoding(n_chains):
    """The tiny fp32 configuration: B=4 prompts of 128 tokens, k=4 noisy-greedy
    drafts, >= 8 chained verification steps with rollback.  The emitted stream
    must equal plain one-token-at-a-time greedy decoding token for token, and
    the cache after each rollback must equal the plain decoder's cache."""
    shape = W.CONFIGS["cfg1"]
    spec = spec_of(shape)
    wn = W.weights_to_numpy(W.make_weights(shape))
    B, k, steps = shape.batch, shape.k, 8
    prompts = W.make_tokens((B, 128), shape.vocab, shape.seed, "prompt")
    rng = np.random.default_rng(shape.seed)
    n_out = steps * (k + 1) + 1
    ref = [autoregressive_greedy(spec, wn, prompts[b], n_out) for b in range(B)]

    caches = [M.SeqCache(spec, 128 + n_out + n_chains * k + 2) for _ in range(B)]
    x0 = np.empty(B, dtype=np.int64)
    for b in range(B):
        x0[b] = int(np.argmax(OV.prefill(spec, wn, caches[b], prompts[b])[-1]))
    streams = [[int(x0[b])] for b in range(B)]
    total_acc = 0
    for step in range(steps):
        drafts = np.empty((B, n_chains, k), dtype=np.int64)
        for b in range(B):
            for c in range(n_chains):
                # The configuration's noise, sigma = 1, dwarfs the spread of random-weight
                # logits (std ~0.3) and gets no draft accepted; it is used on every fourth
                # step, and a sigma at the scale of the top-2 gap on the others.
                sigma = 1.0 if step % 4 == 3 else 0.02 * (1 + c)
                drafts[b, c] = noisy_greedy_drafts(spec, wn, caches[b], int(x0[b]), k, sigma, rng)
        r = OV.verify_step(spec, wn, caches, x0, drafts, None, None, verify_mode=OV.GREEDY)
        for b in range(B):
            a = int(r.accepted_len[b])
            assert 0 <= a <= k
            # a is the longest match over chains
            pos = len(streams[b])
            want_next = ref[b][0][pos: pos + k + 1]
            match = [int(OV.leading_true((drafts[b, c] == np.array(want_next[:k]))[None])[0]) for c in range(n_chains)]
            assert a == max(match)
            assert int(r.best_chain[b]) == int(np.argmax(match))
            emitted = [int(t) for t in r.out_tokens[b, : a + 1]]
            assert np.all(r.out_tokens[b, a + 1:] == -1)
            assert emitted == want_next[: a + 1]
            streams[b] += emitted
            x0[b] = emitted[-1]
            total_acc += a
            # cache == plain decoder's cache over the committed positions
            L = caches[b].length
            assert L == 128 + len(streams[b]) - 1
            for l in range(spec.n_layers):
                assert np.max(np.abs(caches[b].k[l][:L] - ref[b][1].k[l][:L])) < 1e-9
                assert np.max(np.abs(caches[b].v[l][:L] - ref[b][1].v[l][:L])) < 1e-9
    assert total_acc > 0                 # some drafts were accepted, some rejected
    assert total_acc < B * steps * k


# ------------------------- match mode: sampled exact match, lossless for N chains ---

@pytest.mark.parametrize("mode", [OV.SAMPLE_INVERSE_CDF, OV.SAMPLE_EXP_RACE])
def test_match_mode_emits_the_target_law_whatever_the_drafts(mode):
    """V = 16, k = 3, three chains with arbitrary drafts: the first emitted token follows p_1 and, given that
    some chain carried the first token, the second follows that chain's p_2 (chi-square over 4*10^5 windows)."""
    V, k, N, S = 16, 3, 3, 400_000
    rng = np.random.default_rng(77)
    base = rng.standard_normal((k + 1, V)) * 1.5                      # slot i's logits given the sampled path
    other = rng.standard_normal((k + 1, V)) * 1.5                     # what a chain off the path would see
    P = softmax(base)
    drafts = rng.integers(0, V, size=(S, N, k))
    u = rng.random((S, k + 1), dtype=np.float32)
    # the sampled path of every window, by the draw functions on the true slot distributions; a chain sees the
    # path's distribution at slot i+1 only if its first i drafts are on the path (slot 1 is always the true one)
    req = np.arange(S)
    t_path = np.empty((S, k + 1), dtype=np.int64)
    for i in range(k + 1):
        w = np.broadcast_to(P[i], (S, V))
        if mode == OV.SAMPLE_INVERSE_CDF:
            t_path[:, i], _ = OV.draw_inverse_cdf(w, u[:, i].astype(np.float64))
        else:
            t_path[:, i], _ = OV.draw_exp_race(w, u[:, i], req.astype(np.uint64))
    verdicts = []
    for c in range(N):
        on_path = np.cumprod(drafts[:, c] == t_path[:, :k], axis=1).astype(bool)          # [S, k]
        lg = np.empty((S, k + 1, V))
        lg[:, 0] = base[0]
        for i in range(1, k + 1):
            lg[:, i] = np.where(on_path[:, i - 1][:, None], base[i], other[i])
        verdicts.append(OV.verify_match(lg, drafts[:, c], u, req, 1.0, mode))
    acc = np.stack([v.accepted for v in verdicts], axis=1)
    best = np.argmax(acc, axis=1)
    a = acc[req, best]
    y = np.stack([v.token for v in verdicts], axis=1)[req, best]
    out = np.where(np.arange(k + 1)[None, :] < a[:, None], drafts[req, best][:, list(range(k)) + [k - 1]], y[:, None])
    # emitted tokens are the sampled path, as far as they go
    for i in range(k + 1):
        sel = a >= i
        assert np.array_equal(out[sel, i], t_path[sel, i])
    counts = np.bincount(out[:, 0], minlength=V)
    chi2 = np.sum((counts - S * P[0]) ** 2 / (S * P[0]))
    assert chi2 < stats.chi2.ppf(1 - ALPHA, V - 1)
    sel = a >= 1
    counts = np.bincount(out[sel, 1], minlength=V)
    chi2 = np.sum((counts - sel.sum() * P[1]) ** 2 / (sel.sum() * P[1]))
    assert chi2 < stats.chi2.ppf(1 - ALPHA, V - 1)
    # three chains of uniform drafts: the first slot is carried with probability 1 - (1 - 1/V)^3 ... only if the
    # drafts are independent of the path, which they are
    want = 1 - (1 - 1 / V) ** N
    z = (sel.mean() - want) / np.sqrt(want * (1 - want) / S)
    assert abs(z) < 4.5


def plain_sampled_continuation(spec, wn, cache, x0, keys, b, mode, temperature=1.0):
    """One token at a time on a copy of the cache: token i is drawn from the target's distribution after the
    prefix, with key (keys[i], request b)."""
    import copy
    c = copy.deepcopy(cache)
    out, tok = [], int(x0)
    for u in keys:
        lg = M.forward(spec, wn, [c], np.array([[tok]]), np.array([[c.length]]), np.ones((1, 1, 1), dtype=bool))
        c.length += 1
        p = softmax(lg[0, 0] / temperature)[None, :]
        if mode == OV.SAMPLE_INVERSE_CDF:
            t, _ = OV.draw_inverse_cdf(p, np.array([u], dtype=np.float64))
        else:
            t, _ = OV.draw_exp_race(p, np.array([u], dtype=np.float32), np.array([b], dtype=np.uint64))
        tok = int(t[0])
        out.append(tok)
    return out, c


@pytest.mark.parametrize("n_chains,mode", [(1, OV.SAMPLE_EXP_RACE), (3, OV.SAMPLE_EXP_RACE), (3, OV.SAMPLE_INVERSE_CDF)])
def test_match_verification_reproduces_plain_sampling(n_chains, mode):
    """Tiny fp32 model, B = 3 prompts, k = 4, six chained steps with rollback.  Chains agree with the sampled
    path for a random number of tokens and then wander off.  Whatever they hold, the emitted stream equals
    plain sampling with the same (request, slot) keys, the accepted length is the longest agreement, the lowest
    such chain is kept, and the cache equals the plain decoder's."""
    shape = W.scaled_down(W.CONFIGS["cfg1"], batch=3)
    spec = spec_of(shape)
    wn = W.weights_to_numpy(W.make_weights(shape))
    B, k, steps = 3, 4, 6
    prompts = W.make_tokens((B, 40), shape.vocab, shape.seed, "prompt")
    rng = np.random.default_rng(5 + n_chains)
    caches = [M.SeqCache(spec, 40 + steps * (k + 1) + n_chains * k + 4) for _ in range(B)]
    x0 = np.empty(B, dtype=np.int64)
    for b in range(B):
        x0[b] = int(np.argmax(OV.prefill(spec, wn, caches[b], prompts[b])[-1]))
    for step in range(steps):
        u = rng.random((B, n_chains, k + 1), dtype=np.float32)
        path, ref_caches = [], []
        for b in range(B):
            t, c = plain_sampled_continuation(spec, wn, caches[b], x0[b], u[b, 0], b, mode)
            path.append(t)
            ref_caches.append(c)
        drafts = rng.integers(0, shape.vocab, size=(B, n_chains, k))
        agree = rng.integers(0, k + 1, size=(B, n_chains))
        if step == 2:
            agree[:] = k                                              # everything accepted once
        if step == 3:
            agree[:] = 0
        for b in range(B):
            for c in range(n_chains):
                drafts[b, c, :agree[b, c]] = path[b][:agree[b, c]]
                if agree[b, c] < k and drafts[b, c, agree[b, c]] == path[b][agree[b, c]]:
                    drafts[b, c, agree[b, c]] = (drafts[b, c, agree[b, c]] + 1) % shape.vocab
        r = OV.verify_step(spec, wn, caches, x0, drafts, None, u, verify_mode=OV.MATCH, sample_mode=mode)
        for b in range(B):
            a = int(r.accepted_len[b])
            assert a == int(agree[b].max())
            assert int(r.best_chain[b]) == int(np.argmax(agree[b]))
            assert [int(t) for t in r.out_tokens[b, : a + 1]] == path[b][: a + 1]
            assert np.all(r.out_tokens[b, a + 1:] == -1)
            L = caches[b].length
            assert L == ref_caches[b].length - (k + 1) + a + 1
            for l in range(spec.n_layers):
                assert np.max(np.abs(caches[b].k[l][:L] - ref_caches[b].k[l][:L])) < 1e-9
                assert np.max(np.abs(caches[b].v[l][:L] - ref_caches[b].v[l][:L])) < 1e-9
            x0[b] = path[b][a]
