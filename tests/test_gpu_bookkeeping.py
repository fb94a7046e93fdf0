"""Sequence bookkeeping and error behaviour of the C ABI on the device: cache round trips, page accounting,
rejected calls leave everything as it was, rollback to an earlier length replays a step exactly."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu

SHAPE = W.Shape("book-bf16", 2, 256, 4, 2, 64, 512, 1024, dtype="bf16", batch=3, k=3, seed=11)
SV_EINVAL, SV_ENOPAGES, SV_ENOSEQ = -1, -2, -3


def make_verifier(num_pages, max_pages_per_seq=8, max_batch=3, max_k=3):
    import paper_2511_16193_amd as P
    w = P.pack_weights(W.make_weights(SHAPE, "cuda:0"))
    return P.Verifier(SHAPE.model_fields(), w, packed=True, max_batch=max_batch, max_k=max_k, max_chains=1, max_seqs=4,
                      page_size=64, num_pages=num_pages, max_pages_per_seq=max_pages_per_seq, verify_mode=1, sample_mode=1,
                      temperature=1.0)


def step_inputs(B, k, seed):
    V = SHAPE.vocab
    x0 = torch.from_numpy(W.make_tokens((B,), V, seed, "x0")).to("cuda:0", torch.int32)
    q = W.make_random_q((B, 1, k), V, 1.0, seed, "cuda:0")
    d = W.sample_from(q, seed).to(torch.int32).contiguous()
    u = torch.from_numpy(W.make_uniforms((B, 1, k + 1), seed)).to("cuda:0")
    return x0, d, q.contiguous(), u


def test_cache_round_trip_across_pages():
    ver = make_verifier(num_pages=12)
    ver.seq_add(2, 150)                                    # three pages, the last partly used
    for layer in range(SHAPE.n_layers):
        k, v = W.make_kv_block(SHAPE, 5, 2, layer, 150, "cuda:0")
        ver.kv_write(2, layer, 0, k, v)
        for pos0, n in ((0, 150), (60, 10), (63, 2), (128, 22), (149, 1)):
            kk, vv = ver.kv_read(2, layer, pos0, n)
            assert torch.equal(kk, k[pos0:pos0 + n]) and torch.equal(vv, v[pos0:pos0 + n])
    assert ver.seq_len(2) == 150
    ver.close()


def test_rejected_calls_change_nothing():
    from paper_2511_16193_amd import SvError
    ver = make_verifier(num_pages=12)
    for b, L in enumerate((10, 70, 0)):
        ver.seq_add(b, L)
        for layer in range(SHAPE.n_layers):
            k, v = W.make_kv_block(SHAPE, 5, b, layer, L, "cuda:0")
            if L:
                ver.kv_write(b, layer, 0, k, v)
    x0, d, q, u = step_inputs(3, 3, 1)
    with pytest.raises(SvError) as e:                      # the same sequence twice in one batch
        ver.step([0, 1, 1], x0, d, q, u)
    assert e.value.code == SV_ENOSEQ
    with pytest.raises(SvError) as e:                      # a sequence that was never added
        ver.step([0, 1, 3], x0, d, q, u)
    assert e.value.code == SV_ENOSEQ
    x4, d4, q4, u4 = step_inputs(3, 4, 1)                  # more drafts than max_k
    with pytest.raises(SvError) as e:
        ver.step([0, 1, 2], x4, d4, q4, u4)
    assert e.value.code == SV_EINVAL
    with pytest.raises(SvError) as e:                      # stochastic verification without uniforms
        ver.step([0, 1, 2], x0, d, q, None)
    assert e.value.code == SV_EINVAL
    with pytest.raises(SvError):
        ver.seq_add(1, 5)                                  # already live
    with pytest.raises(SvError):
        ver.kv_read(0, 0, 60, 10)                          # beyond the pages the sequence holds
    assert [ver.seq_len(b) for b in range(3)] == [10, 70, 0]
    out = ver.step([0, 1, 2], x0, d, q, u)                 # and the context still works
    acc = out["accepted_len"].cpu().numpy()
    assert [ver.seq_len(b) for b in range(3)] == [10 + acc[0] + 1, 70 + acc[1] + 1, 0 + acc[2] + 1]
    ver.close()


def test_page_pool_exhaustion_and_reuse():
    from paper_2511_16193_amd import SvError
    ver = make_verifier(num_pages=4, max_pages_per_seq=4)
    ver.seq_add(0, 126)                                    # two pages
    ver.seq_add(1, 64)                                     # one page, full
    with pytest.raises(SvError) as e:
        ver.seq_add(2, 129)                                # would need three, one is free
    assert e.value.code == SV_ENOPAGES
    x0, d, q, u = step_inputs(2, 3, 2)
    # the step needs room for 4 more entries per request: request 0 crosses into a third page (126 + 4 > 128),
    # request 1 needs a second one -- two pages, one free: refused, nothing claimed
    with pytest.raises(SvError) as e:
        ver.step([0, 1], x0, d, q, u)
    assert e.value.code == SV_ENOPAGES
    assert ver.seq_len(0) == 126 and ver.seq_len(1) == 64
    ver.seq_remove(1)                                      # its page returns to the pool
    ver.seq_add(3, 10)
    out = ver.step([0, 3], x0, d, q, u)                    # now it fits: one new page for request 0
    acc = out["accepted_len"].cpu().numpy()
    assert ver.seq_len(0) == 127 + acc[0] and ver.seq_len(3) == 11 + acc[1]
    with pytest.raises(SvError) as e:
        ver.seq_set_len(3, 64 * 4 + 1)                     # beyond max_pages_per_seq
    assert e.value.code in (SV_ENOPAGES, SV_EINVAL)
    ver.close()


def test_rollback_to_saved_length_replays_the_step():
    ver = make_verifier(num_pages=12)
    lens = (33, 100, 7)
    for b, L in enumerate(lens):
        ver.seq_add(b, L)
        for layer in range(SHAPE.n_layers):
            k, v = W.make_kv_block(SHAPE, 9, b, layer, L, "cuda:0")
            ver.kv_write(b, layer, 0, k, v)
    x0, d, q, u = step_inputs(3, 3, 3)
    first = {k_: v.clone() for k_, v in ver.step([0, 1, 2], x0, d, q, u, want_logits=True).items()}
    assert any(ver.seq_len(b) != lens[b] for b in range(3))
    ver.seq_set_lens([0, 1, 2], list(lens))                # entries beyond are dead; the step rewrites them
    again = ver.step([0, 1, 2], x0, d, q, u, want_logits=True)
    for key in first:
        assert torch.equal(first[key], again[key]), key    # the step is deterministic, bit for bit
    ver.close()
