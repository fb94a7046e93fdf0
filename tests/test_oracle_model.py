"""Pins of the oracle's forward pass against things other than itself:
library casts, an independent build from torch library primitives, and
invariants the mathematics fixes."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import model as M
from oracle import verify as OV
import workloads as W

TINY = W.Shape("tiny", 2, 64, 4, 2, 16, 128, 96, dtype="fp32", rope_theta=1.0e4, seed=7)


def spec_of(shape: W.Shape) -> M.ModelSpec:
    return M.ModelSpec(**shape.model_fields())


# ------------------------------------------------------------- rounding ---

def test_bf16_rounding_matches_library_cast():
    rng = np.random.default_rng(1)
    x32 = (rng.standard_normal(200000) * np.exp(rng.uniform(-20, 20, 200000))).astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()
    got = M.round_to_storage(x32.astype(np.float64), "bf16")
    assert np.array_equal(got, want)


def test_bf16_rounding_ties_and_direct_from_float64():
    # exact ties go to the even neighbour
    assert M.round_to_storage(np.array([1.0 + 2.0 ** -8]), "bf16")[0] == 1.0
    assert M.round_to_storage(np.array([1.0 + 3 * 2.0 ** -8]), "bf16")[0] == 1.0 + 2.0 ** -6
    # just above a tie: nearest bf16 is the upper neighbour, although rounding
    # through float32 first would land on the tie and fall back to 1.0
    x = np.array([1.0 + 2.0 ** -8 + 2.0 ** -30])
    assert M.round_to_storage(x, "bf16")[0] == 1.0 + 2.0 ** -7
    assert M.round_to_storage(-x, "bf16")[0] == -(1.0 + 2.0 ** -7)
    # fp32 storage rounds nowhere
    assert M.round_to_storage(x, "fp32")[0] == x[0]


# ------------------------------------------- independent library build ---

def torch_reference_logits(shape: W.Shape, w: dict, tokens: np.ndarray) -> np.ndarray:
    """Causal pass over a whole sequence built from torch library primitives in
    float64 (rms_norm, linear, scaled_dot_product_attention, silu) with RoPE
    done as a complex rotation.  Rounds to bf16 with torch's cast at the points
    where the data is stored in bf16."""
    dt = torch.float64
    hq, hkv, hd, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_model

    def rnd(x):
        return x.to(torch.bfloat16).to(dt) if shape.dtype == "bf16" else x

    def t(x):
        return x.to(dt)

    n = len(tokens)
    h = F.embedding(torch.from_numpy(tokens), t(w["embed"]))
    pos = torch.arange(n, dtype=dt)
    freqs = shape.rope_theta ** (-torch.arange(0, hd, 2, dtype=dt) / hd)
    rot = torch.polar(torch.ones(n, hd // 2, dtype=dt), pos[:, None] * freqs[None, :])     # e^{i pos f}

    def rope(x):       # x [n, heads, hd]; pair (i, i+hd/2) is one complex number
        z = torch.complex(x[..., : hd // 2], x[..., hd // 2:]) * rot[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for lw in w["layers"]:
        a = rnd(F.rms_norm(h, (d,), t(lw["ln1"]), eps=shape.rms_eps))
        qkv = F.linear(a, t(lw["wqkv"]))
        q, k, v = torch.split(qkv, [hq * hd, hkv * hd, hkv * hd], dim=-1)
        q = rnd(rope(q.reshape(n, hq, hd))).transpose(0, 1)
        k = rnd(rope(k.reshape(n, hkv, hd))).transpose(0, 1)
        v = rnd(v.reshape(n, hkv, hd)).transpose(0, 1)
        k = k.repeat_interleave(hq // hkv, dim=0)
        v = v.repeat_interleave(hq // hkv, dim=0)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        o = rnd(o.transpose(0, 1).reshape(n, hq * hd))
        h = h + F.linear(o, t(lw["wo"]))
        a = rnd(F.rms_norm(h, (d,), t(lw["ln2"]), eps=shape.rms_eps))
        if shape.n_experts:
            probs = torch.softmax(F.linear(a, t(lw["w_router"])), dim=-1)
            top_p, top_i = torch.topk(probs, shape.top_k, dim=-1)
            top_p = top_p / top_p.sum(-1, keepdim=True)
            out = torch.zeros_like(h)
            for tok in range(n):
                for j in range(shape.top_k):
                    e = int(top_i[tok, j])
                    g, u = F.linear(a[tok], t(lw["w_gate_up"][e])).chunk(2, dim=-1)
                    out[tok] += top_p[tok, j] * F.linear(rnd(F.silu(g) * u), t(lw["w_down"][e]))
            h = h + out
        else:
            g, u = F.linear(a, t(lw["w_gate_up"])).chunk(2, dim=-1)
            h = h + F.linear(rnd(F.silu(g) * u), t(lw["w_down"]))
    a = rnd(F.rms_norm(h, (d,), t(w["final_norm"]), eps=shape.rms_eps))
    return F.linear(a, t(w["lm_head"])).numpy()


@pytest.mark.parametrize("variant", ["fp32-gqa", "fp32-mha", "bf16-gqa", "fp32-moe"])
def test_forward_matches_independent_library_build(variant):
    shape = TINY
    tol = 1e-10
    if variant == "fp32-mha":
        shape = W.scaled_down(TINY, n_kv_heads=4)
    elif variant == "bf16-gqa":
        shape = W.scaled_down(TINY, dtype="bf16")
        tol = 2e-4       # torch's float64->bf16 cast rounds through float32: rare one-ulp differences
    elif variant == "fp32-moe":
        shape = W.scaled_down(TINY, n_experts=8, top_k=2, d_expert=32, d_ff=0)
    w = W.make_weights(shape)
    wn = W.weights_to_numpy(w)
    spec = spec_of(shape)
    toks = W.make_tokens((23,), shape.vocab, 5)
    want = torch_reference_logits(shape, w, toks)

    # (a) one causal pass
    cache = M.SeqCache(spec, 64)
    got = OV.prefill(spec, wn, cache, toks)
    assert np.max(np.abs(got - want)) < tol
    # (b) prefix cached, then the remaining rows as x0 + one chain of drafts
    cache = M.SeqCache(spec, 64)
    OV.prefill(spec, wn, cache, toks[:17])
    _, idx, vis = OV.new_token_layout(5, 1)
    logits = M.forward(spec, wn, [cache], toks[17:].reshape(1, 6), (17 + idx).reshape(1, 6), vis[None])
    assert np.max(np.abs(logits[0] - want[17:])) < tol


def test_batched_rows_equal_one_row_at_a_time():
    shape = TINY
    spec = spec_of(shape)
    wn = W.weights_to_numpy(W.make_weights(shape))
    toks = W.make_tokens((2, 12), shape.vocab, 9)
    caches = [M.SeqCache(spec, 32) for _ in range(2)]
    for b in range(2):
        OV.prefill(spec, wn, caches[b], toks[b, :7])
    _, idx, vis = OV.new_token_layout(4, 1)
    pos = np.array([[7], [7]]) + idx[None]
    batched = M.forward(spec, wn, caches, toks[:, 7:], pos, np.broadcast_to(vis, (2, 5, 5)))
    for b in range(2):
        c = M.SeqCache(spec, 32)
        OV.prefill(spec, wn, c, toks[b, :7])
        for j in range(5):
            one = M.forward(spec, wn, [c], toks[b, 7 + j].reshape(1, 1), np.array([[7 + j]]),
                            np.ones((1, 1, 1), dtype=bool))
            c.length += 1
            assert np.max(np.abs(one[0, 0] - batched[b, j])) < 1e-10


def test_chain_rows_do_not_see_other_chains():
    """Row (chain c, draft i) must equal a single-chain pass over that chain alone."""
    shape = TINY
    spec = spec_of(shape)
    wn = W.weights_to_numpy(W.make_weights(shape))
    prompt = W.make_tokens((9,), shape.vocab, 3)
    k, N = 3, 3
    new = W.make_tokens((1 + N * k,), shape.vocab, 4)
    cache = M.SeqCache(spec, 32)
    OV.prefill(spec, wn, cache, prompt)
    _, idx, vis = OV.new_token_layout(k, N)
    multi = M.forward(spec, wn, [cache], new.reshape(1, -1), (9 + idx).reshape(1, -1), vis[None])[0]
    for c in range(N):
        single_tokens = np.concatenate([new[:1], new[1 + c * k: 1 + (c + 1) * k]])
        cc = M.SeqCache(spec, 32)
        OV.prefill(spec, wn, cc, prompt)
        _, idx1, vis1 = OV.new_token_layout(k, 1)
        single = M.forward(spec, wn, [cc], single_tokens.reshape(1, -1), (9 + idx1).reshape(1, -1), vis1[None])[0]
        assert np.max(np.abs(single[0] - multi[0])) < 1e-10
        assert np.max(np.abs(single[1:] - multi[1 + c * k: 1 + (c + 1) * k])) < 1e-10


def test_rope_shift_invariance():
    """Attention scores depend on position differences only: shifting every
    position by a constant leaves the logits unchanged."""
    shape = TINY
    spec = spec_of(shape)
    wn = W.weights_to_numpy(W.make_weights(shape))
    toks = W.make_tokens((1, 10), shape.vocab, 21)
    vis = np.tril(np.ones((10, 10), dtype=bool))[None]
    out = []
    for shift in (0, 977):
        c = M.SeqCache(spec, 16)
        out.append(M.forward(spec, wn, [c], toks, shift + np.arange(10)[None], vis))
    assert np.max(np.abs(out[0] - out[1])) < 1e-9


def test_rms_norm_scale_invariance_and_unit_rms():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 64))
    w = np.ones(64)
    y = M.rms_norm(x, w, 0.0)
    assert np.allclose(np.sqrt(np.mean(y * y, axis=-1)), 1.0, atol=1e-12)
    assert np.allclose(M.rms_norm(37.5 * x, w, 0.0), y, atol=1e-12)
    g = rng.standard_normal(64)
    assert np.allclose(M.rms_norm(x, g, 0.0), y * g, atol=1e-12)


def test_identical_experts_equal_dense_ffn():
    shape = W.scaled_down(TINY, n_experts=6, top_k=3, d_expert=32, d_ff=0)
    spec = spec_of(shape)
    rng = np.random.default_rng(2)
    wgu = rng.standard_normal((64, 64)) * 0.1
    wd = rng.standard_normal((64, 32)) * 0.1
    lw = {"w_router": rng.standard_normal((6, 64)),
          "w_gate_up": np.broadcast_to(wgu, (6, 64, 64)), "w_down": np.broadcast_to(wd, (6, 64, 32))}
    a = rng.standard_normal((7, 64))
    moe = M.moe_ffn(spec, a, lw, None)
    dense = M.dense_ffn(spec, a, wgu, wd)
    assert np.max(np.abs(moe - dense)) < 1e-12


def test_route_top_k_against_sorted_definition():
    rng = np.random.default_rng(5)
    logits = rng.standard_normal((50, 16))
    logits[:, 3] = logits[:, 11]          # equal probabilities: lower id must win
    ids, wts, margin = M.route_top_k(logits, 4)
    for r in range(50):
        p = np.exp(logits[r] - logits[r].max())
        p = p / p.sum()
        order = sorted(range(16), key=lambda e: (-p[e], e))
        assert list(ids[r]) == order[:4]
        assert np.allclose(wts[r], p[order[:4]] / p[order[:4]].sum())
        assert np.isclose(margin[r], (p[order[3]] - p[order[4]]) / p[order[3]])
    assert np.allclose(wts.sum(-1), 1.0)


def test_attention_is_a_convex_combination_of_values():
    """With all cached V rows equal to one vector, attention returns that
    vector whatever the scores are (softmax rows sum to one)."""
    shape = W.scaled_down(TINY, n_layers=1)
    spec = spec_of(shape)
    wn = W.weights_to_numpy(W.make_weights(shape))
    # make the new token's own V equal to the same vector by zeroing Wv and using a zero cache V
    hq, hkv, hd = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    wn["layers"][0]["wqkv"][(hq + hkv) * hd:] = 0.0
    wn["layers"][0]["w_gate_up"][:] = 0.0
    c = M.SeqCache(spec, 16)
    rng = np.random.default_rng(3)
    c.k[0][:8] = rng.standard_normal((8, hkv, hd))
    c.length = 8
    tok = np.array([[5]])
    # V == 0 everywhere -> attention output 0 -> logits == lm_head(norm(embed))
    logits = M.forward(spec, wn, [c], tok, np.array([[8]]), np.ones((1, 1, 1), dtype=bool))
    h = wn["embed"][5].astype(np.float64)
    want = M.rms_norm(h, wn["final_norm"], spec.rms_eps) @ wn["lm_head"].astype(np.float64).T
    assert np.max(np.abs(logits[0, 0] - want)) < 1e-12
