"""Oracle of the verification step proper (test infrastructure only).

What is computed, in the method's order (paper: Introduction "This work";
Section 3 "Opportunity" paragraph for the reject semantics; Section 4.1 for
"acceptance length = output tokens per verification"; Section 5.1 for
temperature 1.0).  For request b with committed-but-uncached token x0 and N
draft chains of k tokens each:

 1. layout     new tokens are [x0, chain0 d_1..d_k, chain1 d_1..d_k, ...]; x0
               sits at position L (the cached length), draft i of any chain at
               position L+i; a draft attends the cache, x0 and the earlier
               drafts of its own chain.
 2. forward    one pass of the target over those rows (model.forward).  The
               row of x0 yields the target's distribution for draft slot 1 of
               every chain; the row of draft i of chain c yields slot i+1.
 3. greedy     g_i = argmax of slot i (lowest id on ties); accept drafts while
               d_i == g_i; emit the accepted drafts and g_{a+1}.
 3' stochastic p_i = softmax(logits_i / temperature); accept draft x = d_i iff
               u_i * q_i(x) < p_i(x) (u in [0,1), so p >= q always accepts);
               at the first rejection r draw the replacement from
               max(p_r - q_r, 0) (renormalised; if that is identically zero,
               from p_r); with no rejection draw a bonus token from p_{k+1}.
               The draw consumes u_{k+1}.  q = None means one-hot drafts.
 4. chains     keep the chain with the largest accepted length (lowest chain
               id on ties).
 5. rollback   the cache keeps x0 and the accepted drafts of the kept chain at
               positions L..L+a; length becomes L+a+1; everything else the pass
               appended is dead.  The emitted last token is NOT cached: it is
               the next step's x0.

 3'' match     (sampled exact match; what the paper's "exact token matching" and
               its Fastest-of-N selection need to stay lossless with several
               chains)  for every slot i the target's own token t_i is drawn from
               p_i = softmax(logits_i / temperature) with randomness keyed by
               (request, slot) only -- uniform u[b, 0, i-1], the same for every
               chain -- and draft d_i is accepted iff d_i == t_i; at the first
               mismatch r the emitted token is t_r, with none it is t_{k+1}.
               Chains that agree with the sampled path see the same p_i and
               hence the same t_i, so whichever chain is kept, the emitted
               tokens are those of plain sampling with the same keys.

Two ways of turning u_{k+1} into a token are defined (the paper fixes none):
 sample_mode 0  inverse CDF over ascending token id: smallest v whose running
                sum of weights exceeds u * total.
 sample_mode 1  exponential race: token v draws e_v = -log1p(-U_v) where U_v is
                a counter-based uniform keyed by (u's bit pattern, b, chain, v);
                the winner is argmax_v (ln w_v - ln e_v).  P(v wins) = w_v/sum w
                because min of independent exponentials with rates w_v lands on
                v with that probability.  The decision is an argmax, so small
                perturbations of the logits matter only when the top-2 gap is
                small, which is what makes token parity checkable at a vocabulary
                of 150k.  The generator (below) is SplitMix64's output function,
                a published algorithm, written here independently of the device
                code.

Pins (tests/test_oracle_verify.py): exact enumeration of the one-token law
(= p); chi-square of 10^6 seeded trials at V=16 against the target chain for
both sample modes; accept rate = 1 - TV(p,q); accepted-length histogram
against p^a(1-p), p^k (Section 4.1); q == p accepts everything; a <= k;
one-hot q == exact-match sampling in law; temperature -> 0 == greedy; greedy
verification == plain one-token-at-a-time decoding over chained steps
including rollback; N chains under greedy: a = max_c match length, tokens
unchanged.
Match mode: the emitted tokens equal plain one-token-at-a-time sampling with
the same keys, for any drafts and any number of chains, over chained steps with
rollback; each emitted token follows the target's distribution (chi-square).
Parity unpinned: which chain stochastic verification keeps when N > 1 (the
longest-chain rule is not distribution preserving; only the greedy case has a
ground truth) and the particular bit-mixing function of sample_mode 1 (pinned
statistically only).
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import model as M

GREEDY = 0
STOCHASTIC = 1
MATCH = 2
SAMPLE_INVERSE_CDF = 0
SAMPLE_EXP_RACE = 1

_MASK64 = (1 << 64) - 1


# ----------------------------------------------------------------- layout ---

def new_token_layout(k: int, n_chains: int):
    """Chain id (-1 for x0), index within chain (0 for x0) and position offset
    of each of the 1 + N*k new rows, plus the [n, n] visibility matrix."""
    n = 1 + n_chains * k
    chain = np.full(n, -1, dtype=np.int64)
    idx = np.zeros(n, dtype=np.int64)
    for c in range(n_chains):
        for i in range(1, k + 1):
            r = 1 + c * k + (i - 1)
            chain[r] = c
            idx[r] = i
    vis = np.zeros((n, n), dtype=bool)
    for i in range(n):
        for j in range(n):
            vis[i, j] = (j == 0) or (chain[j] == chain[i] and idx[j] <= idx[i] and chain[i] >= 0)
    vis[0, :] = False
    vis[0, 0] = True
    return chain, idx, vis


# ------------------------------------------------------ counter-based RNG ---

def race_uniforms(u_last: np.ndarray, stream: np.ndarray, vocab: int) -> np.ndarray:
    """U[s, v] in (0, 1] as float32-exact values, for s over draws, v over ids.

    key = (stream << 32) | bits32(u_last);  z = key + (v+1)*0x9E3779B97F4A7C15;
    z = SplitMix64-finalise(z);  U = (float32(z >> 32) + 0.5) * 2^-32, every
    operation rounded to float32 (so U is reproducible bit for bit anywhere).
    """
    u_bits = np.asarray(u_last, dtype=np.float32).view(np.uint32).astype(np.uint64)
    key = (np.asarray(stream, dtype=np.uint64) << np.uint64(32)) | u_bits            # [S]
    v = np.arange(1, vocab + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = key[:, None] + v[None, :] * np.uint64(0x9E3779B97F4A7C15)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    hi = (z >> np.uint64(32)).astype(np.float32)          # round-to-nearest-even
    return (hi + np.float32(0.5)) * np.float32(2.0 ** -32)


# ------------------------------------------------------------------ draws ---

def draw_inverse_cdf(w: np.ndarray, u: np.ndarray):
    """w [S,V] non-negative weights, u [S].  Token = smallest v with
    cumsum(w)[v] > u*sum(w).  Also returns the relative distance of u*sum(w)
    to the nearest boundary of the winning bucket (a parity margin)."""
    cs = np.cumsum(w, axis=-1)
    total = cs[:, -1]
    t = u * total
    tok = np.sum(cs <= t[:, None], axis=-1)
    tok = np.minimum(tok, w.shape[-1] - 1)
    # weights of zero are never selected except through the clamp above; step back if so
    for s in np.nonzero(np.take_along_axis(w, tok[:, None], -1)[:, 0] == 0)[0]:
        nz = np.nonzero(w[s])[0]
        tok[s] = nz[-1]
    hi = np.take_along_axis(cs, tok[:, None], -1)[:, 0]
    lo = hi - np.take_along_axis(w, tok[:, None], -1)[:, 0]
    margin = np.minimum(hi - t, t - lo) / total
    return tok.astype(np.int64), margin


def draw_exp_race(w: np.ndarray, u: np.ndarray, stream: np.ndarray):
    """Token = argmax_v (ln w_v - ln e_v), e_v = -log1p(-U_v); lowest id wins
    ties; ids with w_v == 0 never win.  Margin = top-2 gap of that score."""
    U = race_uniforms(u, stream, w.shape[-1]).astype(np.float64)
    with np.errstate(divide="ignore"):
        e = -np.log1p(-U)
        score = np.log(w) - np.log(e)
    tok = np.argmax(score, axis=-1)
    part = np.partition(score, -2, axis=-1)
    margin = part[:, -1] - part[:, -2]
    return tok.astype(np.int64), margin


# ------------------------------------------------------- accept / reject ---

@dataclass
class ChainVerdict:
    accepted: np.ndarray        # [S] int, 0..k
    token: np.ndarray           # [S] int, the replacement / bonus token
    accept_margin: np.ndarray   # [S] min over tested slots of |ln p(x) - ln(u q(x))| (greedy: top-2 logit gap)
    draw_margin: np.ndarray     # [S] margin of the final draw (greedy: top-2 logit gap of that row)
    zero_residual: np.ndarray   # [S] bool, residual was identically zero


def leading_true(flags: np.ndarray) -> np.ndarray:
    """Length of the run of True at the start of each row."""
    return np.sum(np.cumprod(flags.astype(np.int64), axis=-1), axis=-1)


def verify_greedy(logits: np.ndarray, drafts: np.ndarray, draft_lens: np.ndarray | None = None) -> ChainVerdict:
    """logits [S, k+1, V] (slot i+1 in row i), drafts [S, k]."""
    S, k1, _ = logits.shape
    k = k1 - 1
    g = np.argmax(logits, axis=-1)                                   # [S, k+1], lowest id on ties
    match = drafts == g[:, :k]
    if draft_lens is not None:
        match = match & (np.arange(k)[None, :] < draft_lens[:, None])
    a = leading_true(match) if k else np.zeros(S, dtype=np.int64)
    top2 = np.partition(logits, -2, axis=-1)[..., -2:]
    gap = top2[..., 1] - top2[..., 0]                                 # [S, k+1]
    tested = np.arange(k1)[None, :] <= a[:, None]                     # rows 0..a decided something
    acc_margin = np.min(np.where(tested, gap, np.inf), axis=-1)
    return ChainVerdict(a, g[np.arange(S), a], acc_margin, gap[np.arange(S), a],
                        np.zeros(S, dtype=bool))


def verify_stochastic(logits: np.ndarray, drafts: np.ndarray, draft_probs: np.ndarray | None,
                      uniforms: np.ndarray, stream: np.ndarray, temperature: float,
                      sample_mode: int, draft_lens: np.ndarray | None = None) -> ChainVerdict:
    """logits [S,k+1,V]; drafts [S,k]; draft_probs [S,k,V] or None (one-hot);
    uniforms [S,k+1]; stream [S] = b*N + chain, keys sample_mode 1."""
    S, k1, V = logits.shape
    k = k1 - 1
    p = M.softmax(np.asarray(logits, dtype=np.float64) / temperature, axis=-1)
    rows = np.arange(S)
    if k:
        p_x = np.take_along_axis(p[:, :k, :], drafts[:, :, None], axis=-1)[:, :, 0]      # p_i(d_i)
        if draft_probs is None:
            q_x = np.ones_like(p_x)
        else:
            q_x = np.take_along_axis(np.asarray(draft_probs, dtype=np.float64),
                                     drafts[:, :, None], axis=-1)[:, :, 0]
        u = np.asarray(uniforms, dtype=np.float64)
        ok = u[:, :k] * q_x < p_x
        if draft_lens is not None:
            ok = ok & (np.arange(k)[None, :] < draft_lens[:, None])
        a = leading_true(ok)
        with np.errstate(divide="ignore"):
            m = np.abs(np.log(p_x) - np.log(u[:, :k] * q_x))
        limit = a + 1 if draft_lens is None else np.minimum(a + 1, draft_lens)
        tested = np.arange(k)[None, :] < limit[:, None]
        acc_margin = np.min(np.where(tested, m, np.inf), axis=-1)
    else:
        a = np.zeros(S, dtype=np.int64)
        acc_margin = np.full(S, np.inf)

    # distribution the final token is drawn from: slot a+1
    w = p[rows, a, :].copy()
    k_eff = np.full(S, k) if draft_lens is None else draft_lens
    rejected = a < k_eff
    zero_res = np.zeros(S, dtype=bool)
    for s in np.nonzero(rejected)[0]:
        if draft_probs is None:
            q_row = np.zeros(V)
            q_row[drafts[s, a[s]]] = 1.0
        else:
            q_row = np.asarray(draft_probs[s, a[s]], dtype=np.float64)
        res = np.maximum(w[s] - q_row, 0.0)
        if np.sum(res) > 0.0:
            w[s] = res
        else:
            zero_res[s] = True
    u_last = np.asarray(uniforms[:, k], dtype=np.float64)
    if sample_mode == SAMPLE_INVERSE_CDF:
        tok, dmargin = draw_inverse_cdf(w, u_last)
    elif sample_mode == SAMPLE_EXP_RACE:
        tok, dmargin = draw_exp_race(w, np.asarray(uniforms[:, k], dtype=np.float32), stream)
    else:
        raise ValueError(sample_mode)
    return ChainVerdict(a, tok, acc_margin, dmargin, zero_res)


def verify_match(logits: np.ndarray, drafts: np.ndarray, slot_uniforms: np.ndarray, request: np.ndarray,
                 temperature: float, sample_mode: int, draft_lens: np.ndarray | None = None) -> ChainVerdict:
    """logits [S,k+1,V]; drafts [S,k]; slot_uniforms [S,k+1] = the (request, slot) keys, equal for the chains
    of a request; request [S] = index of the request in the batch (the stream of sample_mode 1)."""
    S, k1, V = logits.shape
    k = k1 - 1
    p = M.softmax(np.asarray(logits, dtype=np.float64) / temperature, axis=-1)
    if sample_mode == SAMPLE_INVERSE_CDF:
        t, tm = draw_inverse_cdf(p.reshape(S * k1, V), np.asarray(slot_uniforms, dtype=np.float64).reshape(-1))
    elif sample_mode == SAMPLE_EXP_RACE:
        t, tm = draw_exp_race(p.reshape(S * k1, V), np.asarray(slot_uniforms, dtype=np.float32).reshape(-1),
                              np.repeat(np.asarray(request, dtype=np.uint64), k1))
    else:
        raise ValueError(sample_mode)
    t, tm = t.reshape(S, k1), tm.reshape(S, k1)
    match = drafts == t[:, :k]
    if draft_lens is not None:
        match = match & (np.arange(k)[None, :] < draft_lens[:, None])
    a = leading_true(match) if k else np.zeros(S, dtype=np.int64)
    tested = np.arange(k1)[None, :] <= a[:, None]                     # the draws of slots 1..a+1 decided something
    acc_margin = np.min(np.where(tested, tm, np.inf), axis=-1)
    rows = np.arange(S)
    return ChainVerdict(a, t[rows, a], acc_margin, tm[rows, a], np.zeros(S, dtype=bool))


# ------------------------------------------------------------- whole step ---

@dataclass
class StepResult:
    accepted_len: np.ndarray            # [B]
    out_tokens: np.ndarray              # [B, k+1], entries beyond a+1 are -1
    best_chain: np.ndarray              # [B]
    logits: np.ndarray                  # [B, n, V] float64
    chain_accepted: np.ndarray          # [B, N]
    chain_token: np.ndarray             # [B, N]
    accept_margin: np.ndarray           # [B, N]
    draw_margin: np.ndarray             # [B, N]
    zero_residual: np.ndarray           # [B, N]
    router_margins: list = field(default_factory=list)


def verify_step(spec: M.ModelSpec, weights: dict, caches, x0: np.ndarray, drafts: np.ndarray,
                draft_probs: np.ndarray | None, uniforms: np.ndarray | None, *,
                verify_mode: int, sample_mode: int = SAMPLE_INVERSE_CDF, temperature: float = 1.0,
                draft_lens: np.ndarray | None = None) -> StepResult:
    """x0 [B]; drafts [B,N,k]; draft_probs [B,N,k,V] or None; uniforms
    [B,N,k+1].  Advances every cache by a+1 entries (steps 1-5 above)."""
    B, N, k = drafts.shape
    chain, idx, vis = new_token_layout(k, N)
    n = 1 + N * k
    tokens = np.concatenate([np.asarray(x0).reshape(B, 1), drafts.reshape(B, N * k)], axis=1)
    lengths = np.array([c.length for c in caches], dtype=np.int64)
    positions = lengths[:, None] + idx[None, :]
    margins: list = []
    logits = M.forward(spec, weights, caches, tokens, positions,
                       np.broadcast_to(vis, (B, n, n)), router_margins=margins)

    # per (request, chain): rows [x0, chain's drafts] -> slots 1..k+1
    per_chain = np.empty((B, N, k + 1, spec.vocab), dtype=np.float64)
    for c in range(N):
        per_chain[:, c, 0] = logits[:, 0]
        per_chain[:, c, 1:] = logits[:, 1 + c * k: 1 + (c + 1) * k]
    S = B * N
    flat_logits = per_chain.reshape(S, k + 1, spec.vocab)
    flat_drafts = drafts.reshape(S, k)
    flat_lens = None if draft_lens is None else np.repeat(np.asarray(draft_lens), N)
    if verify_mode == GREEDY:
        v = verify_greedy(flat_logits, flat_drafts, flat_lens)
    elif verify_mode == MATCH:
        slot_u = np.repeat(np.asarray(uniforms)[:, :1, :], N, axis=1).reshape(S, k + 1)    # chain 0's row keys every chain
        v = verify_match(flat_logits, flat_drafts, slot_u, np.repeat(np.arange(B), N), temperature, sample_mode, flat_lens)
    else:
        flat_q = None if draft_probs is None else draft_probs.reshape(S, k, spec.vocab)
        stream = np.arange(S, dtype=np.uint64)          # b*N + chain
        v = verify_stochastic(flat_logits, flat_drafts, flat_q, uniforms.reshape(S, k + 1), stream,
                              temperature, sample_mode, flat_lens)

    ch_a = v.accepted.reshape(B, N)
    ch_y = v.token.reshape(B, N)
    best = np.argmax(ch_a, axis=1)                       # lowest chain id on ties
    a = ch_a[np.arange(B), best]
    out = np.full((B, k + 1), -1, dtype=np.int64)
    for b in range(B):
        out[b, :a[b]] = drafts[b, best[b], :a[b]]
        out[b, a[b]] = ch_y[b, best[b]]
        rollback(caches[b], int(best[b]), int(a[b]), k)
    return StepResult(a, out, best, logits, ch_a, ch_y, v.accept_margin.reshape(B, N),
                      v.draw_margin.reshape(B, N), v.zero_residual.reshape(B, N), margins)


def rollback(cache: M.SeqCache, best: int, a: int, k: int) -> None:
    """Step 5: after a pass that appended x0 and N chains of k drafts at slots L, L+1.., keep x0 and the `a`
    accepted drafts of chain `best` at slots L..L+a (chain c's draft i sits at slot L + 1 + c*k + (i-1)); the
    length becomes L + a + 1 and everything beyond it is dead."""
    L = cache.length
    for i in range(1, a + 1):
        src = L + 1 + best * k + (i - 1)
        for l in range(len(cache.k)):
            cache.k[l][L + i] = cache.k[l][src]
            cache.v[l][L + i] = cache.v[l][src]
    cache.length = L + a + 1


def prefill(spec: M.ModelSpec, weights: dict, cache: M.SeqCache, tokens: np.ndarray) -> np.ndarray:
    """Plain causal pass over a prompt; caches every token; returns logits [n, V]."""
    n = len(tokens)
    vis = np.tril(np.ones((n, n), dtype=bool))
    pos = cache.length + np.arange(n)
    logits = M.forward(spec, weights, [cache], np.asarray(tokens).reshape(1, n), pos.reshape(1, n),
                       vis.reshape(1, n, n))
    cache.length += n
    return logits[0]
