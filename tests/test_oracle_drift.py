"""How far two correct implementations of the same numerics contract drift apart (CPU only).

The forward pass rounds its activations to bf16 at fixed points (every projection's left operand, q, k, v).  Two
implementations that agree on those points but accumulate differently -- the oracle in float64, a device kernel
in float32 in another order -- produce values that differ by ~1e-7 relative before a rounding, and a value
that close to a rounding boundary lands on different sides of it: one bf16 unit (2^-8 relative) in one entry of
a K-wide operand moves every output of the next projection by ~0.006 / sqrt(K) relative, which flips more
entries at the next rounding point, and so on, until the two residual streams differ by a few 1e-3 of each
block's output.  That noise is injected anew by every layer and adds up like a random walk.

Here the oracle runs twice on a deep, narrow bf16 model: as it is, and with its matrix product swapped (from
the test, the oracle's code is untouched) for one that multiplies and accumulates in float32 and walks the
reduction in another order.  Nothing else differs.  The tests show
  * with identical input a single layer stays inside the stated 2e-2 on logits (scaled to the logits' spread);
  * over 28 layers the two drift beyond that bound -- so no device kernel can be held to it end to end;
  * the drift grows like sqrt(layers) and stays below the fixed law the full-size device tests use
    (harness.DRIFT_RMS_PER_SQRT_LAYER, harness.DRIFT_MAX_OVER_RMS).
Measured with this file (rms of the logit difference / spread of the logits, 28 layers; SV_DRIFT_WIDE=1 runs
the widest): d_model 256: 4.6e-3, 512: 8.4e-3, 1024: 1.1e-2, 2048: 1.4e-2 (max 6.9e-2 absolute on logits of
spread 0.9); the device against the oracle at d_model 3584: 1.5e-2.
The first layer is the one exception to the single-layer statement: its input is the bare embedding (spread
0.02), so everything it emits is its own output and its logits carry the whole of its rounding noise.  At the
32B shape (d_model 5120, FFN 27648, vocabulary 152064, 50 rows; SV_DRIFT_WIDE=1) the oracle and its float32
copy differ there by 2.5e-2 at the worst of 7.6 million logits (rms 2.4e-3 of the spread): beyond 2e-2, inside
the one-layer value of the law, which is what the full-size device tests hold a first layer to.
"""
import os

import numpy as np
import pytest

from oracle import model as M
from oracle import verify as OV
import workloads as W
from harness import DRIFT_RMS_PER_SQRT_LAYER, DRIFT_MAX_OVER_RMS, LOGIT_TOL

FULL_SIZE_LOGIT_SPREAD = 1.2       # standard deviation of the 7B / 32B shapes' logits (0.02 * sqrt(d_model))


def float32_product(a, w, rows_per_chunk=None):
    """a @ w^T with float32 products and float32 accumulation, the reduction taken as four interleaved strides."""
    a32, w32 = np.asarray(a, dtype=np.float32), np.asarray(w, dtype=np.float32)
    acc = np.zeros((a32.shape[0], w32.shape[0]), dtype=np.float32)
    for s in range(4):
        acc += a32[:, s::4] @ w32[:, s::4].T
    return acc.astype(np.float64)


class Model:
    def __init__(self, d, heads, kv_heads, ff, layers, B=4, n=5, L=96, V=4096, seed=7):
        self.shape = W.Shape("drift", layers, d, heads, kv_heads, 128, ff, V, dtype="bf16", batch=B, k=n - 1, seed=seed)
        self.spec = M.ModelSpec(**self.shape.model_fields())
        self.wn = W.weights_to_numpy(W.make_weights(self.shape, "cpu"))
        self.B, self.n, self.L, self.V = B, n, L, V
        self.tokens = W.make_tokens((B, n), V, seed, "t")
        _, idx, vis = OV.new_token_layout(n - 1, 1)
        self.pos = L + np.broadcast_to(idx, (B, n))
        self.vis = np.broadcast_to(vis, (B, n, n))

    def caches(self, layers=None):
        out = []
        for b in range(self.B):
            c = M.SeqCache(self.spec if layers is None else M.ModelSpec(**{**self.shape.model_fields(), "n_layers": len(layers)}),
                           self.L + self.n + 1)
            for i, l in enumerate(range(self.shape.n_layers) if layers is None else layers):
                k, v = W.make_kv_block(self.shape, self.shape.seed, b, l, self.L, "cpu")
                c.k[i][:self.L] = k.float().numpy()
                c.v[i][:self.L] = v.float().numpy()
            c.length = self.L
            out.append(c)
        return out

    def logits(self, product=None, n_layers=None, trace=None):
        """Whole pass (or its first n_layers layers followed by the head)."""
        layers = list(range(self.shape.n_layers if n_layers is None else n_layers))
        spec = M.ModelSpec(**{**self.shape.model_fields(), "n_layers": len(layers)})
        return self._run(spec, self.wn["embed"], self.tokens, [self.wn["layers"][l] for l in layers], self.caches(layers), product, trace)

    def one_layer(self, layer, h_in, product=None):
        """Layer `layer` alone on the given residual rows, then the head: the rows enter through the embedding
        table (row t of the table is row t of h_in, token id t)."""
        spec = M.ModelSpec(**{**self.shape.model_fields(), "n_layers": 1})
        ids = np.arange(self.B * self.n).reshape(self.B, self.n)
        return self._run(spec, h_in, ids, [self.wn["layers"][layer]], self.caches([layer]), product, None)

    def _run(self, spec, embed, tokens, layers, caches, product, trace):
        w = {"embed": embed, "lm_head": self.wn["lm_head"], "final_norm": self.wn["final_norm"], "layers": layers}
        saved = M.matmul_wt
        if product is not None:
            M.matmul_wt = product
        try:
            return M.forward(spec, w, caches, tokens, self.pos, self.vis, trace=trace)
        finally:
            M.matmul_wt = saved


def drift(a, b):
    diff = np.abs(a - b)
    return float(np.sqrt(np.mean(diff ** 2)) / a.std()), float(diff.max() / a.std())


@pytest.fixture(scope="module")
def deep():
    m = Model(1024, 8, 2, 4096, 28)
    trace = {}
    ref = m.logits(trace=trace)
    return m, ref, trace["hidden"]


def test_single_layer_on_identical_input_stays_within_the_stated_logit_tolerance(deep):
    m, _, hidden = deep
    bound = LOGIT_TOL["bf16"] / FULL_SIZE_LOGIT_SPREAD            # 2e-2 on logits of spread 1.2
    for layer in (0, 1, 13, 27):
        a = m.one_layer(layer, hidden[layer])
        b = m.one_layer(layer, hidden[layer], float32_product)
        rms, mx = drift(a, b)
        assert mx < bound, (layer, mx)
        assert mx > 0.0                                           # the two products do differ


def test_the_hidden_trace_is_the_pass_itself(deep):
    """The one-layer harness reproduces the whole pass when chained with the oracle's own arithmetic: its output
    on the traced input of the last layer is the pass's logits (same operations on the same values)."""
    m, ref, hidden = deep
    assert len(hidden) == 29
    last = m.one_layer(27, hidden[27])
    assert np.max(np.abs(last - ref)) < 1e-12


def test_over_28_layers_two_correct_implementations_drift_beyond_the_per_layer_tolerance(deep):
    m, ref, _ = deep
    rms, mx = drift(ref, m.logits(float32_product))
    layers = m.shape.n_layers
    assert mx > LOGIT_TOL["bf16"] / FULL_SIZE_LOGIT_SPREAD, mx    # measured 5.3e-2 against 1.7e-2
    assert rms > 5e-3, rms                                        # measured 1.1e-2
    # ... and inside the fixed law the full-size device tests hold the device to
    assert rms < DRIFT_RMS_PER_SQRT_LAYER * np.sqrt(layers), rms
    assert mx < DRIFT_MAX_OVER_RMS * DRIFT_RMS_PER_SQRT_LAYER * np.sqrt(layers), mx


def test_drift_grows_like_the_square_root_of_the_depth():
    m = Model(512, 4, 2, 2048, 16, B=8)
    rms = {}
    for layers in (1, 4, 16):
        rms[layers], mx = drift(m.logits(n_layers=layers), m.logits(float32_product, n_layers=layers))
        assert rms[layers] < DRIFT_RMS_PER_SQRT_LAYER * np.sqrt(layers)
        assert mx < DRIFT_MAX_OVER_RMS * DRIFT_RMS_PER_SQRT_LAYER * np.sqrt(layers)
    assert rms[1] < rms[4] < rms[16]
    # a random walk: four times the layers, about twice the drift (measured 2.0; a systematic per-layer error
    # would give 4, a drift that is there from the first layer on 1)
    assert 1.3 < rms[16] / rms[4] < 3.0, rms


@pytest.mark.skipif(not os.environ.get("SV_DRIFT_WIDE"), reason="150 s: set SV_DRIFT_WIDE=1 (figures quoted in the module docstring)")
def test_wide_model_follows_the_same_law():
    m = Model(2048, 16, 4, 8192, 28, B=8)
    rms, mx = drift(m.logits(), m.logits(float32_product))
    print(f"d_model 2048, 28 layers: rms/spread {rms:.3e}, max/spread {mx:.3e}")
    assert 5e-3 < rms < DRIFT_RMS_PER_SQRT_LAYER * np.sqrt(28)
    assert mx < DRIFT_MAX_OVER_RMS * DRIFT_RMS_PER_SQRT_LAYER * np.sqrt(28)


@pytest.mark.skipif(not os.environ.get("SV_DRIFT_WIDE"), reason="170 s, 20 GB: set SV_DRIFT_WIDE=1 (figures quoted in the module docstring)")
def test_first_layer_of_the_32b_shape_exceeds_the_single_layer_tolerance():
    m = Model(5120, 40, 8, 27648, 1, B=2, n=25, L=2048, V=152064, seed=5000)
    ref = m.logits()
    rms, mx = drift(ref, m.logits(float32_product))
    print(f"32B shape, first layer alone: rms/spread {rms:.3e}, max {mx * ref.std():.3e} absolute")
    assert mx * ref.std() > LOGIT_TOL["bf16"]                    # measured 2.5e-2
    assert rms < DRIFT_RMS_PER_SQRT_LAYER and mx < DRIFT_MAX_OVER_RMS * DRIFT_RMS_PER_SQRT_LAYER
