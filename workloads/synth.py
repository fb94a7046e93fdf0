"""Seeded generators of weights, prefixes, cache contents, drafts and uniforms.

Everything is drawn with torch's generators on the requested device and cast
to the storage type with torch's own cast.  A tensor is keyed by (seed, name,
layer) so that any single tensor can be regenerated alone.  The CPU and the
GPU generators give different streams: a test that feeds both the oracle and
the device path generates once and hands the same values to both.
"""
from __future__ import annotations

import zlib

import numpy as np
import torch

from .configs import Shape

_TORCH_DTYPE = {"bf16": torch.bfloat16, "fp32": torch.float32}


def _gen(device, seed: int, *key) -> torch.Generator:
    g = torch.Generator(device=device)
    tag = zlib.crc32(repr(key).encode())
    g.manual_seed((int(seed) * 1_000_003 + tag) % (2 ** 63 - 1))
    return g


def _normal(shape, std, mean, dtype, device, seed, *key) -> torch.Tensor:
    g = _gen(device, seed, *key)
    x = torch.randn(shape, generator=g, device=device, dtype=torch.float32)
    return (x * std + mean).to(dtype)


def make_weights(s: Shape, device="cpu", seed: int | None = None) -> dict:
    """Matrices N(0, 0.02), norm gains 1 + N(0, 0.05), all in the storage type.
    Layout: matrices are [out_features, in_features] (in_features contiguous);
    wqkv rows = q heads, k heads, v heads; w_gate_up rows = gate then up."""
    seed = s.seed if seed is None else seed
    dt = _TORCH_DTYPE[s.dtype]
    d, hq, hkv, hd = s.d_model, s.n_q_heads, s.n_kv_heads, s.head_dim
    w = {
        "embed": _normal((s.vocab, d), 0.02, 0.0, dt, device, seed, "embed"),
        "lm_head": _normal((s.vocab, d), 0.02, 0.0, dt, device, seed, "lm_head"),
        "final_norm": _normal((d,), 0.05, 1.0, dt, device, seed, "final_norm"),
        "layers": [],
    }
    for l in range(s.n_layers):
        lw = {
            "ln1": _normal((d,), 0.05, 1.0, dt, device, seed, "ln1", l),
            "wqkv": _normal(((hq + 2 * hkv) * hd, d), 0.02, 0.0, dt, device, seed, "wqkv", l),
            "wo": _normal((d, hq * hd), 0.02, 0.0, dt, device, seed, "wo", l),
            "ln2": _normal((d,), 0.05, 1.0, dt, device, seed, "ln2", l),
        }
        if s.n_experts:
            lw["w_router"] = _normal((s.n_experts, d), 0.02, 0.0, dt, device, seed, "w_router", l)
            lw["w_gate_up"] = _normal((s.n_experts, 2 * s.d_expert, d), 0.02, 0.0, dt, device, seed, "w_gate_up", l)
            lw["w_down"] = _normal((s.n_experts, d, s.d_expert), 0.02, 0.0, dt, device, seed, "w_down", l)
        else:
            lw["w_gate_up"] = _normal((2 * s.d_ff, d), 0.02, 0.0, dt, device, seed, "w_gate_up", l)
            lw["w_down"] = _normal((d, s.d_ff), 0.02, 0.0, dt, device, seed, "w_down", l)
        w["layers"].append(lw)
    return w


def _np(t: torch.Tensor) -> np.ndarray:
    t = t.detach()
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)          # exact widening
    return t.cpu().numpy()


def weights_to_numpy(w: dict, lazy: bool = False) -> dict:
    """Same values as numpy float32 arrays (bf16 widened exactly).  With
    lazy=True the per-layer dicts are converted on access, one layer at a time
    (device -> host copy included), to bound host memory for large models."""
    out = {k: _np(v) for k, v in w.items() if k != "layers"}
    if lazy:
        layers = w["layers"]
        out["layers"] = lambda l: {k: _np(v) for k, v in layers[l].items()}
    else:
        out["layers"] = [{k: _np(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


def make_prefix_lengths(s: Shape, seed: int | None = None) -> np.ndarray:
    seed = s.seed if seed is None else seed
    rng = np.random.default_rng([seed, 11])
    return rng.integers(s.prefix_lo, s.prefix_hi + 1, size=s.batch).astype(np.int64)


def make_tokens(shape, vocab: int, seed: int, *key) -> np.ndarray:
    rng = np.random.default_rng([seed, 13, zlib.crc32(repr(key).encode())])
    return rng.integers(0, vocab, size=shape).astype(np.int64)


def make_uniforms(shape, seed: int, *key) -> np.ndarray:
    """float32 uniforms in [0, 1)."""
    rng = np.random.default_rng([seed, 17, zlib.crc32(repr(key).encode())])
    return rng.random(size=shape, dtype=np.float32)


def make_kv_block(s: Shape, seed: int, b: int, layer: int, length: int, device="cpu"):
    """Synthetic cache contents for one request and layer: K and V ~ N(0,1) in
    the storage type, shape [length, n_kv_heads, head_dim].  Stands in for a
    real prefill of the prefix, which the oracle cannot mirror at full size."""
    dt = _TORCH_DTYPE[s.dtype]
    shape = (length, s.n_kv_heads, s.head_dim)
    k = _normal(shape, 1.0, 0.0, dt, device, seed, "kvK", b, layer)
    v = _normal(shape, 1.0, 0.0, dt, device, seed, "kvV", b, layer)
    return k, v


def make_random_q(shape_prefix, vocab: int, sigma: float, seed: int, device="cpu", *key) -> torch.Tensor:
    """Draft distributions independent of the target: softmax(sigma * N(0,1)),
    float32 [*shape_prefix, vocab]."""
    g = _gen(device, seed, "randq", *key)
    z = torch.randn((*shape_prefix, vocab), generator=g, device=device, dtype=torch.float32) * sigma
    return torch.softmax(z, dim=-1)


def sample_from(q: torch.Tensor, seed: int, *key) -> torch.Tensor:
    """One categorical draw per row of q [..., V] (library multinomial)."""
    g = _gen(q.device, seed, "draw", *key)
    flat = q.reshape(-1, q.shape[-1])
    idx = torch.multinomial(flat, 1, generator=g)[:, 0]
    return idx.reshape(q.shape[:-1])
