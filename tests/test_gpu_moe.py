"""Device parity of the mixture-of-experts feed-forward (router, grouping, expert products, combine) and of a
verification step through a small mixture-of-experts decoder, against the oracle."""
import numpy as np
import pytest
import torch

from oracle import model as M
from oracle import verify as OV
import workloads as W
from harness import Case, compare_step

pytestmark = pytest.mark.gpu

ROUTE_MARGIN = 1e-4     # relative gap between the last kept and the first dropped expert probability below
                        # which the fp32 router and the float64 router may keep different experts


def bf16_round(x: torch.Tensor) -> torch.Tensor:
    return x.to(torch.bfloat16)


@pytest.mark.parametrize("T,d,E,top_k,F,skew", [
    (24, 256, 64, 4, 128, 0.0),       # fewer assignments than experts x tile: most buckets hold 1-3 rows, some none
    (600, 256, 64, 8, 128, 0.0),      # ~75 rows per expert: three row tiles, ragged last tile
    (777, 384, 128, 8, 256, 3.0),     # skewed router: a few experts take several hundred rows (more than one
                                      # group of four tiles), many take none; odd row count
    (5, 128, 64, 1, 128, 0.0),        # top-1, a single partial tile
    (640, 2048, 128, 8, 768, 0.0),    # the benchmark's mixture-of-experts layer at full size (B=128, k=4)
])
def test_moe_ffn_matches_oracle(T, d, E, top_k, F, skew):
    import paper_2511_16193_amd as P
    g = torch.Generator().manual_seed(1000 + T)
    a = torch.randn((T, d), generator=g)
    w_router = torch.randn((E, d), generator=g) * 0.3
    if skew:
        u = torch.randn(d, generator=g)
        u /= u.norm()
        a += skew * 4.0 * u                                   # a common direction in every row ...
        w_router[: max(2, E // 16)] += skew * u               # ... that a few experts are aligned with
    w_gate_up = torch.randn((E, 2 * F, d), generator=g) * (1.0 / d ** 0.5)
    w_down = torch.randn((E, d, F), generator=g) * (1.0 / F ** 0.5)
    a, w_router, w_gate_up, w_down = map(bf16_round, (a, w_router, w_gate_up, w_down))

    spec = M.ModelSpec(n_layers=1, d_model=d, n_q_heads=1, n_kv_heads=1, head_dim=64, d_ff=0, vocab=128,
                       n_experts=E, top_k=top_k, d_expert=F, dtype="bf16")
    lw = {"w_router": w_router.float().numpy().astype(np.float64),
          "w_gate_up": w_gate_up.float().numpy().astype(np.float64),
          "w_down": w_down.float().numpy().astype(np.float64)}
    margins = []
    want = M.moe_ffn(spec, a.float().numpy().astype(np.float64), lw, margins)
    ids_o, wts_o, _ = M.route_top_k(M.matmul_wt(a.float().numpy().astype(np.float64), lw["w_router"]), top_k)
    margin = margins[0]

    out, ids, wts = P.op_moe_ffn(a.cuda(), w_router.cuda(), w_gate_up.cuda(), w_down.cuda(), top_k)
    torch.cuda.synchronize()
    out, ids, wts = out.cpu().numpy(), ids.cpu().numpy(), wts.cpu().numpy()

    clear = margin > ROUTE_MARGIN
    assert clear.mean() > 0.95
    # routing: same experts in the same order, same weights
    # (order inside the kept set can swap when two kept probabilities are within rounding; compare as sets then)
    for t in np.nonzero(clear)[0]:
        assert set(ids[t]) == set(ids_o[t]), f"row {t}: {ids[t]} vs {ids_o[t]} (margin {margin[t]})"
        got = dict(zip(ids[t], wts[t]))
        # logits of magnitude ~10 summed in fp32 over d products carry ~1e-5 absolute error, which is the
        # relative error of the probabilities
        for e, w in zip(ids_o[t], wts_o[t]):
            assert abs(got[e] - w) < 5e-5
    assert np.all(np.abs(wts.sum(axis=1) - 1.0) < 1e-5)
    if skew:
        counts = np.bincount(ids_o.reshape(-1), minlength=E)
        assert counts.max() > 128 and counts.min() == 0        # the case is what it says it is
    # outputs: fp32 accumulation against float64 (~1e-6 of the row's scale), plus the rare bf16 rounding flip of
    # one silu*up product: a flip moves the outputs of its row by 2^-8 |act| |w_down| each, up to ~2e-3 of the
    # row's scale when |act| is a few units.  So: all but a small fraction within 1e-4, everything within 1e-2.
    scale = np.sqrt(np.mean(want[clear] ** 2, axis=1, keepdims=True))
    err = np.abs(out[clear] - want[clear])
    assert np.mean(err > 1e-4 * scale + 1e-6) < 2e-2, f"fraction beyond 1e-4: {np.mean(err > 1e-4 * scale + 1e-6)}"
    assert np.all(err <= 1e-2 * scale + 1e-6), f"max error {err.max()} at scale {scale.mean()}"


MOE_SMALL = W.Shape("small-moe", 2, 256, 4, 2, 64, 0, 1024, n_experts=64, top_k=4, d_expert=128, dtype="bf16",
                    batch=6, k=3, seed=99)


@pytest.mark.parametrize("k,n_chains,vmode", [(3, 1, OV.STOCHASTIC), (2, 2, OV.GREEDY)])
def test_small_moe_step(k, n_chains, vmode):
    """Two-layer mixture-of-experts decoder (64 experts, top-4, expert width 128) over a ragged synthetic
    cache, two chained steps.  A routing decision the oracle took with a relative gap under ROUTE_MARGIN
    exempts its request (the row's logits may then legitimately differ)."""
    shape = W.scaled_down(MOE_SMALL, k=k, n_chains=n_chains)
    lengths = [0, 17, 64, 200, 1030, 333]
    B, V = len(lengths), shape.vocab
    case = Case(shape, lengths, verify_mode=vmode, packed=True)
    x0 = W.make_tokens((B,), V, shape.seed, "x0")
    for step in range(2):
        q = W.make_random_q((B, n_chains, k), V, 1.0, shape.seed + step)
        drafts = W.sample_from(q, shape.seed + step).numpy()
        u = W.make_uniforms((B, n_chains, k + 1), shape.seed + step)
        r, g = case.step(x0, drafts, q if vmode == OV.STOCHASTIC else None, u if vmode == OV.STOCHASTIC else None)
        n = 1 + n_chains * k
        row_margin = np.min(np.stack(r.router_margins), axis=0).reshape(B, n)     # over layers
        close = np.nonzero(row_margin.min(axis=1) < ROUTE_MARGIN)[0]
        assert len(close) <= 1
        for key in g:                                        # exempt requests: take the oracle's values
            g[key][close] = {"logits": r.logits, "accepted_len": r.accepted_len, "out_tokens": r.out_tokens,
                             "best_chain": r.best_chain}[key][close]
        err, exempt, diverged = compare_step(r, g, "bf16", k)
        assert not diverged or compare_step.beyond_margin == 0
        if diverged or len(close):
            break
        x0 = np.array([r.out_tokens[b, r.accepted_len[b]] for b in range(B)])
        assert np.array_equal(case.device_lengths(), [c.length for c in case.caches])
    case.close()


def test_moe_needs_packed_bf16_weights():
    """A mixture-of-experts model with row-major weights is refused at init, not silently mis-run."""
    from paper_2511_16193_amd import SvError
    with pytest.raises(SvError):
        Case(MOE_SMALL, [0, 5], verify_mode=OV.GREEDY, packed=False)
