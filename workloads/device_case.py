"""Full-size workload set-up on the GPU for the benchmark and the full-size parity test.

Builds, for one of the benchmark configurations: seeded weights, seeded prefix
lengths, a synthetic cache (N(0,1) K/V in the storage type, standing in for a
real prefill of the prefixes), x0, uniforms, and drafts.  Drafts follow the
configuration's recipe: draft i of a chain is sampled from
q_i = softmax(target logits + N(0, sigma^2) noise) at temperature 1, produced
one token at a time by plain decoding steps (k = 0) of the device library, after
which the cache lengths are put back.  Such drafts are inputs of the benchmark
only; a parity test that needs drafts for the oracle uses `independent_drafts`,
which does not involve the device library.
"""
from __future__ import annotations

import numpy as np
import torch

from .configs import Shape
from . import synth


class DeviceCase:
    def __init__(self, shape: Shape, *, k: int | None = None, n_chains: int | None = None, page_size: int = 64,
                 verify_mode: int | None = None, sample_mode: int = 1, packed: bool = True, keep_row_major=True,
                 max_chains: int | None = None, headroom_tokens: int = 0, device="cuda:0", log=None):
        from paper_2511_16193_amd import Verifier, pack_weights
        self.shape, self.device = shape, torch.device(device)
        self.k = shape.k if k is None else k
        self.N = shape.n_chains if n_chains is None else n_chains
        self.B = shape.batch
        self.log = log or (lambda *_: None)
        self.lengths = synth.make_prefix_lengths(shape)
        self.max_chains = max(self.N, max_chains or 1)       # the context may be sized for more chains than a step uses
        n = 1 + self.max_chains * self.k
        headroom = n + self.k + 2 + headroom_tokens            # headroom_tokens: room for steps that are not put back
        pages = [int((L + headroom + page_size - 1) // page_size) for L in self.lengths]
        self.log(f"weights for {shape.name} ...")
        self.weights = synth.make_weights(shape, self.device)           # row-major (what the oracle reads)
        # the library streams the projection matrices in its packed order (a one-off device-side reorder)
        self.weights_dev = pack_weights(self.weights) if packed and shape.dtype == "bf16" else self.weights
        packed_now = self.weights_dev is not self.weights
        if packed_now and keep_row_major == "host":       # the largest configurations have no room for both copies on
            cpu = {k: v.cpu() for k, v in self.weights.items() if k != "layers"}     # the device: the oracle's goes to the host
            cpu["layers"] = [{k: v.cpu() for k, v in lw.items()} for lw in self.weights["layers"]]
            self.weights = cpu
            torch.cuda.empty_cache()
        elif packed_now and not keep_row_major:
            self.weights = None
            torch.cuda.empty_cache()
        self.ver = Verifier(shape.model_fields(), self.weights_dev, packed=packed_now,
                            max_batch=self.B, max_k=max(self.k, 1),
                            max_chains=self.max_chains, max_seqs=self.B, page_size=page_size, num_pages=sum(pages) + 4,
                            max_pages_per_seq=max(pages) + 1,
                            verify_mode=shape.verify_mode if verify_mode is None else verify_mode,
                            sample_mode=sample_mode, temperature=1.0, device=device)
        self.log(f"synthetic cache: {int(self.lengths.sum())} tokens ...")
        for b in range(self.B):
            L = int(self.lengths[b])
            self.ver.seq_add(b, L)
            for l in range(shape.n_layers):
                kk, vv = synth.make_kv_block(shape, shape.seed, b, l, L, self.device)
                self.ver.kv_write(b, l, 0, kk, vv)
        self.ids = list(range(self.B))
        self.x0 = torch.from_numpy(synth.make_tokens((self.B,), shape.vocab, shape.seed, "x0")).to(
            device=self.device, dtype=torch.int32)
        self.uniforms = torch.from_numpy(synth.make_uniforms((self.B, self.N, self.k + 1), shape.seed, "u")).to(self.device)
        self.drafts = None
        self.draft_probs = None
        self.cur_lengths = [int(x) for x in self.lengths]      # the state reset() goes back to

    def kv_block(self, b: int, layer: int):
        """The synthetic cache contents of (request, layer), regenerated from the seed."""
        return synth.make_kv_block(self.shape, self.shape.seed, b, layer, int(self.lengths[b]), self.device)

    def reset(self):
        self.ver.seq_set_lens(self.ids, self.cur_lengths)

    def commit(self, accepted_len):
        """Make the state after a step (accepted_len: the step's output, read on the host) the one reset() goes
        back to: consecutive steps, each on the rolled-back cache of the one before."""
        self.cur_lengths = [L + int(a) + 1 for L, a in zip(self.cur_lengths, accepted_len)]

    def independent_drafts(self, sigma: float = 1.0):
        """Drafts sampled from q = softmax(sigma N(0,1)), unrelated to the target (random-weight targets are
        nearly flat, so about half of such drafts are still accepted)."""
        V = self.shape.vocab
        q = synth.make_random_q((self.B, self.N, self.k), V, sigma, self.shape.seed, self.device, "indep")
        d = synth.sample_from(q, self.shape.seed, "indep").to(torch.int32)
        self.drafts, self.draft_probs = d.contiguous(), q.contiguous()

    def one_hot_drafts(self):
        """Drafts without a distribution (what an n-gram or suffix-automaton drafter proposes): seeded token ids,
        draft_probs = None, i.e. q is one-hot on the draft."""
        self.independent_drafts(1.0)
        self.draft_probs = None

    def noisy_target_drafts(self, sigmas=None, x0=None):
        """The configuration's recipe (see module docstring), drafted from the state reset() goes back to."""
        V, B, N, k = self.shape.vocab, self.B, self.N, self.k
        if x0 is not None:
            self.x0 = x0.to(device=self.device, dtype=torch.int32).contiguous()
        sigmas = list(sigmas if sigmas is not None else self.shape.draft_sigma)
        drafts = torch.empty((B, N, k), dtype=torch.int32, device=self.device)
        q = torch.empty((B, N, k, V), dtype=torch.float32, device=self.device)
        u1 = torch.full((B, 1, 1), 0.5, dtype=torch.float32, device=self.device)
        for c in range(N):
            sigma = sigmas[c % len(sigmas)]
            tok = self.x0
            for i in range(k):
                out = self.ver.step(self.ids, tok, None, None, u1, want_logits=True)
                g = torch.Generator(device=self.device)
                g.manual_seed(self.shape.seed * 7919 + c * 131 + i)
                noise = torch.randn((B, V), generator=g, device=self.device, dtype=torch.float32) * sigma
                qi = torch.softmax(out["logits"][:, 0, :] + noise, dim=-1)
                q[:, c, i] = qi
                tok = torch.multinomial(qi, 1, generator=g)[:, 0].to(torch.int32).contiguous()
                drafts[:, c, i] = tok
            self.reset()
        self.drafts, self.draft_probs = drafts.contiguous(), q.contiguous()

    def step(self, want_logits: bool = False, out=None):
        return self.ver.step(self.ids, self.x0, self.drafts if self.k else None,
                             self.draft_probs if self.k else None, self.uniforms, want_logits=want_logits, out=out)

    def close(self):
        self.ver.close()
