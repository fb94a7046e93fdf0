"""Shared set-up for the device parity tests: builds the same seeded case for the
oracle (numpy) and for the HIP library (through the binding), and compares a
verification step's results under the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

from oracle import model as M
from oracle import verify as OV
import workloads as W

LOGIT_TOL = {"bf16": 2e-2, "fp32": 1e-4}      # absolute, on logits
MARGIN = 1e-3                                  # decisions closer than this are exempt from exact parity


def spec_of(shape: W.Shape) -> M.ModelSpec:
    return M.ModelSpec(**shape.model_fields())


def to_device(w: dict, device="cuda:0") -> dict:
    out = {k: v.to(device).contiguous() for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: v.to(device).contiguous() for k, v in lw.items()} for lw in w["layers"]]
    return out


class Case:
    """One workload instantiated on both sides."""

    def __init__(self, shape: W.Shape, lengths, *, verify_mode, sample_mode=OV.SAMPLE_EXP_RACE, temperature=1.0,
                 page_size=64, extra_tokens=64, synthetic_kv=True, packed=False, device="cuda:0"):
        from paper_2511_16193_amd import Verifier, pack_weights
        self.shape, self.device = shape, device
        self.spec = spec_of(shape)
        self.verify_mode, self.sample_mode, self.temperature = verify_mode, sample_mode, temperature
        w_cpu = W.make_weights(shape, "cpu")
        self.wn = W.weights_to_numpy(w_cpu)
        self.wd = to_device(w_cpu, device)
        if packed:                                   # projection weights in the library's streaming order
            self.wd = pack_weights(self.wd)
        self.lengths = np.asarray(lengths, dtype=np.int64)
        B = len(self.lengths)
        n = 1 + shape.n_chains * shape.k
        cap = int(self.lengths.max()) + extra_tokens + n
        pps = (cap + page_size - 1) // page_size + 1
        self.ver = Verifier(shape.model_fields(), self.wd, max_batch=B, max_k=shape.k, max_chains=shape.n_chains,
                            max_seqs=B, page_size=page_size, num_pages=B * pps + 2, max_pages_per_seq=pps,
                            verify_mode=verify_mode, sample_mode=sample_mode, temperature=temperature, packed=packed,
                            device=device)
        self.caches = [M.SeqCache(self.spec, cap) for _ in range(B)]
        for b in range(B):
            L = int(self.lengths[b])
            self.ver.seq_add(b, L if synthetic_kv else 0)
            if synthetic_kv:
                for l in range(shape.n_layers):
                    k, v = W.make_kv_block(shape, shape.seed, b, l, L, "cpu")
                    self.caches[b].k[l][:L] = k.float().numpy()
                    self.caches[b].v[l][:L] = v.float().numpy()
                    if L:
                        self.ver.kv_write(b, l, 0, k.to(device), v.to(device))
                self.caches[b].length = L

    def prefill(self, prompts: np.ndarray):
        """Real prefill on both sides; returns (oracle last-row logits, device last-row logits)."""
        lo, ld = [], []
        for b in range(len(prompts)):
            lo.append(OV.prefill(self.spec, self.wn, self.caches[b], prompts[b])[-1])
            ld.append(self.ver.prefill(b, torch.from_numpy(prompts[b]).to(torch.int32)).cpu().numpy())
        return np.stack(lo), np.stack(ld)

    def step(self, x0, drafts, draft_probs, uniforms, draft_lens=None):
        """Run one step on both sides.  draft_probs: torch fp32 cpu tensor or None."""
        dev = self.device
        B, N, k = drafts.shape
        r = OV.verify_step(self.spec, self.wn, self.caches, np.asarray(x0), np.asarray(drafts),
                           None if draft_probs is None else draft_probs.numpy(), uniforms,
                           verify_mode=self.verify_mode, sample_mode=self.sample_mode, temperature=self.temperature,
                           draft_lens=draft_lens)
        out = self.ver.step(
            list(range(B)), torch.as_tensor(np.asarray(x0), dtype=torch.int32, device=dev),
            torch.as_tensor(np.asarray(drafts), dtype=torch.int32, device=dev).contiguous() if k else None,
            None if draft_probs is None else draft_probs.to(dev).contiguous(),
            None if uniforms is None else torch.as_tensor(uniforms, dtype=torch.float32, device=dev).contiguous(),
            draft_lens=None if draft_lens is None else torch.as_tensor(draft_lens, dtype=torch.int32, device=dev),
            want_logits=True)
        torch.cuda.synchronize()
        return r, {k_: v.cpu().numpy() for k_, v in out.items()}

    def device_lengths(self):
        return np.array([self.ver.seq_len(b) for b in range(len(self.lengths))])

    def close(self):
        self.ver.close()


def compare_step(r: OV.StepResult, g: dict, dtype: str, k: int):
    """Logits within tolerance everywhere; accepted lengths, kept chains and emitted tokens identical,
    except for requests where a decision the oracle took was closer than the margin.  The margin is
    MARGIN (1e-3), widened to twice the logit error actually seen on that request's rows: two sets of
    logits that differ by e cannot be expected to agree on a decision whose margin is below 2e (both
    the compared logit and the log-sum-exp move).  Mismatches with a margin above 1e-3 are counted
    separately.  Returns (max logit error, number of exempted requests, requests that diverged)."""
    diff = np.abs(g["logits"].astype(np.float64) - r.logits)
    err = float(np.max(diff))
    assert err < LOGIT_TOL[dtype], f"logits differ by {err}"
    B = len(r.accepted_len)
    exempt, diverged = 0, []
    compare_step.beyond_margin = 0
    for b in range(B):
        same = (g["accepted_len"][b] == r.accepted_len[b] and g["best_chain"][b] == r.best_chain[b]
                and np.array_equal(g["out_tokens"][b], r.out_tokens[b]))
        assert 0 <= g["accepted_len"][b] <= k
        if same:
            continue
        margin = min(float(np.min(r.accept_margin[b])), float(np.min(r.draw_margin[b])))
        allowed = max(MARGIN, 2.0 * float(np.max(diff[b])))
        assert margin < allowed, (f"request {b}: device a={g['accepted_len'][b]} tokens={g['out_tokens'][b]} "
                                  f"chain={g['best_chain'][b]} vs oracle a={r.accepted_len[b]} "
                                  f"tokens={r.out_tokens[b]} chain={r.best_chain[b]}; smallest margin {margin}, "
                                  f"logit error on its rows {float(np.max(diff[b]))}")
        if margin >= MARGIN:
            compare_step.beyond_margin += 1
        exempt += 1
        diverged.append(b)
    return err, exempt, diverged


compare_step.beyond_margin = 0
