"""Oracle forward pass of the target decoder (test infrastructure only).

The paper treats the trained model as a given (a Qwen-style decoder: Section
5.1 names Qwen2.5-32B and Qwen3-235B); what this step must compute is "one
parallel pass of the trained model over the drafted tokens of every request,
against that request's KV cache" (Section 3, "Opportunity" paragraph).  The
decoder written out here is the plain pre-norm decoder of that family:
RMSNorm, grouped-query attention with rotary position embedding (rotate-half
pairing), SwiGLU feed-forward or a softmax-routed top-k mixture of experts,
no biases, untied LM head.

Precision.  All arithmetic is float64.  A model whose storage type is bf16
additionally rounds (round-to-nearest-even, straight from float64) at the
points where the method's data lives in bf16: every matmul's left operand
(RMSNorm output, attention output, gated FFN activation), the rotated q and
k, and v.  Weights, embeddings and cached K/V are given as values already
representable in the storage type.  A model whose storage type is fp32 rounds
nowhere.

Pins (tests/test_oracle_model.py): bf16 rounding against the library cast;
the whole pass against an independent float64 build from library primitives
(scaled-dot-product attention, complex-rotation RoPE); batched rows against
one-row-at-a-time decoding; RoPE shift invariance; RMSNorm scale invariance;
identical experts == dense FFN; top-k routing weights against a sort-based
definition.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Sequence

import numpy as np


@dataclass(frozen=True)
class ModelSpec:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    n_experts: int = 0      # 0 = dense FFN
    top_k: int = 0
    d_expert: int = 0
    dtype: str = "bf16"     # storage type: "bf16" or "fp32"
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to the storage type; result stays float64.

    bf16 keeps 8 significant bits: drop the low 45 of float64's 52 fraction
    bits, ties to even.  (Exponent range is float32's; the values met here are
    far from overflow and from the subnormal range.)
    """
    x = np.asarray(x, dtype=np.float64)
    if dtype == "fp32":
        return x
    if dtype != "bf16":
        raise ValueError(dtype)
    bits = np.ascontiguousarray(x).view(np.uint64)
    keep_lsb = (bits >> np.uint64(45)) & np.uint64(1)
    bits = bits + (np.uint64((1 << 44) - 1) + keep_lsb)
    bits = bits & ~np.uint64((1 << 45) - 1)
    return bits.view(np.float64)


def matmul_wt(a: np.ndarray, w: np.ndarray, rows_per_chunk: int = 16384) -> np.ndarray:
    """a[n,K] @ w[N,K]^T in float64.  `w` may be float32 (exact storage values);
    it is widened a band of output columns at a time only to bound memory."""
    n_out = w.shape[0]
    if w.dtype == np.float64 or n_out <= rows_per_chunk:
        return a @ np.asarray(w, dtype=np.float64).T
    out = np.empty((a.shape[0], n_out), dtype=np.float64)
    for r0 in range(0, n_out, rows_per_chunk):
        r1 = min(n_out, r0 + rows_per_chunk)
        out[:, r0:r1] = a @ np.asarray(w[r0:r1], dtype=np.float64).T
    return out


def rms_norm(h: np.ndarray, weight: np.ndarray, eps: float) -> np.ndarray:
    """h * rsqrt(mean(h^2) + eps) * weight, over the last axis."""
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * np.asarray(weight, dtype=np.float64)


def rope(x: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: coordinates (i, i + hd/2) of each
    head are rotated by angle pos * theta^(-2i/hd).  x: [n, heads, hd]."""
    hd = x.shape[-1]
    half = hd // 2
    inv_freq = theta ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(positions, dtype=np.float64)[:, None] * inv_freq[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    x1 = x[..., :half]
    x2 = x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def softmax(x: np.ndarray, axis: int = -1) -> np.ndarray:
    m = np.max(x, axis=axis, keepdims=True)
    e = np.exp(x - m)
    return e / np.sum(e, axis=axis, keepdims=True)


def route_top_k(router_logits: np.ndarray, top_k: int):
    """Softmax over experts, keep the top_k largest probabilities (equal
    probabilities: the lower expert id wins), renormalise the kept ones to sum
    to one.  Returns (expert ids [n, top_k] in descending probability,
    weights [n, top_k], margin [n]) where margin is the relative gap between
    the last kept and the first dropped probability."""
    probs = softmax(router_logits, axis=-1)
    # stable sort of -probs keeps the lower id first among equals
    order = np.argsort(-probs, axis=-1, kind="stable")
    ids = order[:, :top_k]
    kept = np.take_along_axis(probs, ids, axis=-1)
    weights = kept / np.sum(kept, axis=-1, keepdims=True)
    if probs.shape[-1] > top_k:
        nxt = np.take_along_axis(probs, order[:, top_k:top_k + 1], axis=-1)[:, 0]
        margin = (kept[:, -1] - nxt) / kept[:, -1]
    else:
        margin = np.full(probs.shape[0], np.inf)
    return ids, weights, margin


class SeqCache:
    """Per-request KV cache: for every layer K and V of shape
    [capacity, n_kv_heads, head_dim]; `length` entries are live."""

    def __init__(self, spec: ModelSpec, capacity: int):
        store = np.float32 if spec.dtype == "bf16" else np.float64
        shape = (capacity, spec.n_kv_heads, spec.head_dim)
        self.k = [np.zeros(shape, dtype=store) for _ in range(spec.n_layers)]
        self.v = [np.zeros(shape, dtype=store) for _ in range(spec.n_layers)]
        self.length = 0
        self.capacity = capacity


def attend(q: np.ndarray, keys: np.ndarray, vals: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Grouped-query attention of n rows over m keys.  q [n, hq, hd]; keys, vals
    [m, hkv, hd]; mask bool [n, m] (True = row attends key).  Query head h uses
    kv head h // (hq/hkv).  softmax(q k^T / sqrt(hd)) v, float64.  -> [n, hq, hd]"""
    n, hq, hd = q.shape
    group = hq // keys.shape[1]
    out = np.empty((n, hq, hd), dtype=np.float64)
    for hh in range(hq):
        g = hh // group
        s = (q[:, hh, :] @ keys[:, g, :].T) / np.sqrt(hd)        # [n, m]
        s = np.where(mask, s, -np.inf)
        out[:, hh, :] = softmax(s, axis=-1) @ vals[:, g, :]
    return out


def dense_ffn(spec: ModelSpec, a: np.ndarray, w_gate_up: np.ndarray, w_down: np.ndarray) -> np.ndarray:
    """down( silu(gate(a)) * up(a) ); w_gate_up holds the gate rows first,
    then the up rows.  `a` is already rounded to the storage type."""
    f = w_gate_up.shape[0] // 2
    gu = matmul_wt(a, w_gate_up)
    act = round_to_storage(silu(gu[:, :f]) * gu[:, f:], spec.dtype)
    return matmul_wt(act, w_down)


def moe_ffn(spec: ModelSpec, a: np.ndarray, lw: dict, margins: list | None, trace: dict | None = None) -> np.ndarray:
    """Softmax router over all experts -> top-k -> renormalised weights ->
    weighted sum of the selected experts' SwiGLU FFNs."""
    ids, wts, margin = route_top_k(matmul_wt(a, lw["w_router"]), spec.top_k)
    if margins is not None:
        margins.append(margin)
    if trace is not None:
        trace.setdefault("routing", []).append((ids, wts, margin))
    out = np.zeros((a.shape[0], spec.d_model), dtype=np.float64)
    for e in np.unique(ids):
        tok, slot = np.nonzero(ids == e)
        y = dense_ffn(spec, a[tok], lw["w_gate_up"][e], lw["w_down"][e])
        out[tok] += wts[tok, slot][:, None] * y
    return out


def forward(spec: ModelSpec,
            weights: dict,
            caches: Sequence[SeqCache],
            tokens: np.ndarray,
            positions: np.ndarray,
            visible: np.ndarray,
            router_margins: list | None = None,
            trace: dict | None = None) -> np.ndarray:
    """One parallel pass over n new tokens of each of B requests.

    tokens, positions: int [B, n].  visible: bool [B, n, n]; visible[b, i, j]
    says new token i of request b attends new token j (every new token attends
    all `length` cached entries).  New token j's K/V are stored at cache slot
    `length + j`; `length` itself is left for the caller to advance.
    weights: {"embed" [V,d], "lm_head" [V,d], "final_norm" [d],
    "layers": sequence or callable l -> {"ln1","wqkv","wo","ln2", and either
    "w_gate_up","w_down" (dense) or "w_router","w_gate_up"[E],"w_down"[E]}}.
    wqkv rows: all q heads, then all k heads, then all v heads.
    Returns logits float64 [B, n, vocab].
    trace (observer only, changes nothing computed): if a dict, receives
    "hidden" = the residual stream [B*n, d] entering every layer, then the one
    leaving the last; "ffn_input" / "ffn_residual" = per layer the rounded
    normalised rows fed to the feed-forward block and the residual stream they
    are added to; and for mixture-of-experts models "routing" = per layer
    (expert ids, weights, margin).
    """
    B, n = tokens.shape
    hq, hkv, hd = spec.n_q_heads, spec.n_kv_heads, spec.head_dim
    layer_of: Callable[[int], dict] = (
        weights["layers"] if callable(weights["layers"]) else weights["layers"].__getitem__)

    h = np.asarray(weights["embed"], dtype=np.float64)[tokens.reshape(-1)]       # [B*n, d]
    pos_flat = positions.reshape(-1)

    for l in range(spec.n_layers):
        lw = layer_of(l)
        if trace is not None:
            trace.setdefault("hidden", []).append(h.copy())
        a = round_to_storage(rms_norm(h, lw["ln1"], spec.rms_eps), spec.dtype)
        qkv = matmul_wt(a, lw["wqkv"])
        q = qkv[:, : hq * hd].reshape(B * n, hq, hd)
        k = qkv[:, hq * hd: (hq + hkv) * hd].reshape(B * n, hkv, hd)
        v = qkv[:, (hq + hkv) * hd:].reshape(B * n, hkv, hd)
        q = round_to_storage(rope(q, pos_flat, spec.rope_theta), spec.dtype).reshape(B, n, hq, hd)
        k = round_to_storage(rope(k, pos_flat, spec.rope_theta), spec.dtype).reshape(B, n, hkv, hd)
        v = round_to_storage(v, spec.dtype).reshape(B, n, hkv, hd)

        attn = np.empty((B, n, hq, hd), dtype=np.float64)
        for b in range(B):
            c = caches[b]
            L = c.length
            c.k[l][L:L + n] = k[b]
            c.v[l][L:L + n] = v[b]
            keys = np.asarray(c.k[l][:L + n], dtype=np.float64)          # [L+n, hkv, hd]
            vals = np.asarray(c.v[l][:L + n], dtype=np.float64)
            mask = np.concatenate([np.ones((n, L), dtype=bool), visible[b]], axis=1)   # [n, L+n]
            attn[b] = attend(q[b], keys, vals, mask)
        attn = round_to_storage(attn.reshape(B * n, hq * hd), spec.dtype)
        h = h + matmul_wt(attn, lw["wo"])

        a = round_to_storage(rms_norm(h, lw["ln2"], spec.rms_eps), spec.dtype)
        if trace is not None:
            trace.setdefault("ffn_input", []).append(a.copy())
            trace.setdefault("ffn_residual", []).append(h.copy())
        if spec.n_experts:
            h = h + moe_ffn(spec, a, lw, router_margins, trace)
        else:
            h = h + dense_ffn(spec, a, lw["w_gate_up"], lw["w_down"])

    if trace is not None:
        trace.setdefault("hidden", []).append(h.copy())
    a = round_to_storage(rms_norm(h, weights["final_norm"], spec.rms_eps), spec.dtype)
    return matmul_wt(a, weights["lm_head"]).reshape(B, n, spec.vocab)
