"""sv_op_sample_static (the sampler stage on the library's static scratch, for callers that cannot allocate)
against sv_op_sample (caller-provided scratch): identical accepted lengths, kept chains and tokens, on two
calls in a row of which the second is smaller (so that whatever the first call left in the shared array is
there when the second runs), and the limits of the static array are refused before anything is enqueued."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_case(B, N, k, V, seed, with_q):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((B, 1 + N * k, V)) * 1.2).astype(np.float32)
    q = W.make_random_q((B, N, k), V, 1.0, seed) if with_q else None
    drafts = (W.sample_from(q, seed).numpy() if with_q else rng.integers(0, V, (B, N, k))).astype(np.int64)
    per_chain = np.empty((B, N, k), dtype=np.int64)
    for c in range(N):                              # plant the target's argmax into a third of the slots
        rows = np.concatenate([logits[:, :1], logits[:, 1 + c * k: 1 + (c + 1) * k]], axis=1)[:, :k]
        per_chain[:, c] = np.argmax(rows, axis=-1)
    drafts = np.where(rng.random((B, N, k)) < 0.3, per_chain, drafts)
    u = W.make_uniforms((B, N, k + 1), seed)
    return (torch.from_numpy(logits).to(DEV), torch.from_numpy(drafts).to(torch.int32).to(DEV).contiguous(),
            None if q is None else q.to(DEV).contiguous(), torch.from_numpy(u).to(DEV))


@pytest.mark.parametrize("vmode,smode,with_q", [(1, 1, True), (1, 0, True), (0, 0, False), (2, 1, False), (1, 1, False)])
def test_static_scratch_sampler_equals_the_one_with_caller_scratch(vmode, smode, with_q):
    from paper_2511_16193_amd import op_sample
    from paper_2511_16193_amd.binding import op_sample_static
    # first call: 48 requests x 3 chains x 4 drafts over a ragged vocabulary; second: smaller in every dimension
    for (B, N, k, V, seed) in [(48, 3, 4, 4099, 11), (5, 1, 2, 2048, 12)]:
        logits, drafts, q, u = make_case(B, N, k, V, seed, with_q)
        want = [t.cpu().numpy() for t in op_sample(logits, drafts, q, u, verify_mode=vmode, sample_mode=smode)]
        acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        toks = torch.full((B, k + 1), -7, dtype=torch.int32, device=DEV)
        best = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        op_sample_static(logits, drafts, q, u, acc, toks, best, verify_mode=vmode, sample_mode=smode)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before           # torch's allocator was not touched either
        got = [acc.cpu().numpy(), toks.cpu().numpy(), best.cpu().numpy()]
        for g, w_ in zip(got, want):
            assert np.array_equal(g, w_), (B, N, k, V)
        assert want[0].max() > 0 or vmode == 2 or B < 48          # the large case exercises accepts as well


def test_static_scratch_sampler_refuses_sizes_beyond_its_array():
    from paper_2511_16193_amd import SvError
    from paper_2511_16193_amd.binding import op_sample_static
    B, N, k, V = 1024, 1, 4, 64                                   # 5120 logits rows > 4096
    logits = torch.zeros((B, 1 + N * k, V), dtype=torch.float32, device=DEV)
    drafts = torch.zeros((B, N, k), dtype=torch.int32, device=DEV)
    u = torch.zeros((B, N, k + 1), dtype=torch.float32, device=DEV)
    acc = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    toks = torch.full((B, k + 1), -7, dtype=torch.int32, device=DEV)
    best = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    with pytest.raises(SvError):
        op_sample_static(logits, drafts, None, u, acc, toks, best, verify_mode=1, sample_mode=1)
    torch.cuda.synchronize()
    assert int(acc.min()) == -7 and int(toks.min()) == -7         # nothing was enqueued
