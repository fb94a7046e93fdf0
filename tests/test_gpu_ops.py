"""Device parity of single stages (through the C ABI) against the oracle."""
import numpy as np
import pytest
import torch

from oracle import model as M
from oracle import verify as OV
import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def bf16_cpu(shape, std, seed):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(torch.bfloat16)


@pytest.mark.parametrize("variant", [0, 1, 2])
@pytest.mark.parametrize("M_,N,K,splits", [(320, 512, 1024, 1), (37, 256, 512, 4), (129, 128, 64, 1), (1, 384, 2048, 8),
                                           (700, 640, 448, 1), (321, 768, 3584, 2), (320, 1024, 192, 1)])
def test_gemm_bf16_matches_float64_product(variant, M_, N, K, splits):
    """The row-major projection kernel: several tiles plus a ragged last row tile; every split count; the
    reduction in float64 on the same bf16 inputs is the reference.  fp32 accumulation of K <= 3584 products of
    magnitude ~0.02: absolute error far below 1e-4."""
    from paper_2511_16193_amd import op_gemm_bf16
    a = bf16_cpu((M_, K), 1.0, 1)
    w = bf16_cpu((N, K), 0.02, 2)
    want = M.matmul_wt(a.float().numpy().astype(np.float64), w.float().numpy())
    got = op_gemm_bf16(a.to(DEV), w.to(DEV), splits=splits, variant=variant)
    torch.cuda.synchronize()
    got = got.cpu().numpy().astype(np.float64).sum(axis=0)
    assert np.max(np.abs(got - want)) < 1e-4


@pytest.mark.parametrize("M_,N,K,splits,wide", [(320, 512, 1024, 1, True), (37, 256, 512, 4, True), (129, 128, 64, 1, False),
                                               (1, 384, 2048, 8, False), (700, 640, 448, 1, False),
                                               (321, 768, 3584, 2, True), (320, 1024, 192, 1, True),
                                               (64, 256, 2368, 1, True), (96, 256, 512, 2, True), (180, 384, 1024, 1, False),
                                               (513, 256, 256, 1, True)])
def test_gemm_weight_streaming_matches_float64_product(M_, N, K, splits, wide):
    """The weight-streaming kernel on packed operands: ragged row tiles (rows beyond M read as the last
    tile), both strip widths, fills of 8 and of 4 k-slices, every split count, every number of 32-row tiles per
    work-group (1 to 5; 513 rows: four groups of five tiles with 127 padding rows)."""
    from paper_2511_16193_amd import op_gemm_bf16_ws, op_pack_weight, op_pack_rows
    a = bf16_cpu((M_, K), 1.0, 1)
    w = bf16_cpu((N, K), 0.02, 2)
    want = M.matmul_wt(a.float().numpy().astype(np.float64), w.float().numpy())
    ap, wp = op_pack_rows(a.to(DEV)), op_pack_weight(w.to(DEV))
    for row_tiles in (0, 1, 2, 3, 4, 5):              # 0: the default choice; 1..5: 32-row tiles per work-group, as the plan may pick
        got = op_gemm_bf16_ws(ap, wp, M_, splits=splits, wide=wide, row_tiles=row_tiles)
        torch.cuda.synchronize()
        got = got.cpu().numpy().astype(np.float64).sum(axis=0)
        assert np.max(np.abs(got - want)) < 1e-4, row_tiles


@pytest.mark.parametrize("M_,N,K,splits", [(256, 256, 64, 1), (700, 512, 448, 1), (1, 256, 2048, 2), (1290, 768, 3584, 1),
                                           (513, 1024, 1536, 4)])
def test_gemm_256_tile_kernel_matches_float64_product(M_, N, K, splits):
    """The 256 x 256 kernel (both operands through LDS; row_tiles = 8 selects it): whole and ragged row blocks (rows
    beyond M read as the last tile and are never stored), one to many fills of four k-slices, split reductions."""
    from paper_2511_16193_amd import op_gemm_bf16_ws, op_pack_weight, op_pack_rows
    a = bf16_cpu((M_, K), 1.0, 1)
    w = bf16_cpu((N, K), 0.02, 2)
    want = M.matmul_wt(a.float().numpy().astype(np.float64), w.float().numpy())
    got = op_gemm_bf16_ws(op_pack_rows(a.to(DEV)), op_pack_weight(w.to(DEV)), M_, splits=splits, wide=True, row_tiles=8)
    torch.cuda.synchronize()
    got = got.cpu().numpy().astype(np.float64).sum(axis=0)
    assert np.max(np.abs(got - want)) < 1e-4


@pytest.mark.parametrize("k,n_chains,group", [(0, 1, 7), (1, 1, 7), (2, 1, 7), (4, 1, 7), (8, 1, 7), (4, 1, 8), (3, 3, 4),
                                              (8, 3, 5)])
def test_attention_bf16_matches_oracle(k, n_chains, group):
    """Verify attention alone: n = 1 + N*k rows per request over a paged bf16 cache, with the head
    grouping of the benchmark shapes (7, 8, 5 q heads per kv head) and lengths that put the new rows
    at the start, in the middle and at the end of a 32-key tile, of a page and of a 1024-key chunk,
    plus empty and multi-chunk caches.  The output is rounded to bf16 (half a unit in the last place) and the
    MFMA path also rounds the softmax weights to bf16 before the PV product (up to another unit when a row has
    only a few keys, relative to the weighted mean of |v|): |got - want| <= 2^-8 (|want| + sum_j p_j |v_j|)."""
    import paper_2511_16193_amd as P
    hkv, hd = 2, 128
    hq = hkv * group
    n = 1 + n_chains * k
    lengths = [0, 1, 31, 32, 63, 64, 1023, 1024, 1029, 2047, 3100]
    B = len(lengths)
    model = dict(n_layers=1, d_model=256, n_q_heads=hq, n_kv_heads=hkv, head_dim=hd, d_ff=512, vocab=2048,
                 dtype="bf16", rope_theta=1e6, rms_eps=1e-6)
    wd = W.make_weights(W.Shape("attn", 1, 256, hq, hkv, hd, 512, 2048), DEV)
    ver = P.Verifier(model, wd, max_batch=B, max_k=max(k, 1), max_chains=n_chains, max_seqs=B, page_size=64,
                     num_pages=B * 52, max_pages_per_seq=51, verify_mode=0)
    q = bf16_cpu((B * n, hq, hd), 1.0, 3)
    ks, vs = [], []
    for b, L in enumerate(lengths):
        ver.seq_add(b, L)
        ks.append(bf16_cpu((L + n, hkv, hd), 1.0, 10 + b))
        vs.append(bf16_cpu((L + n, hkv, hd), 1.0, 50 + b))
    ids = list(range(B))
    ver.op_attention(ids, n, k, 0, q.to(DEV))          # reserves the pages of the new rows
    for b in range(B):
        ver.kv_write(b, 0, 0, ks[b].to(DEV), vs[b].to(DEV))
    _, _, vis = OV.new_token_layout(k, n_chains)
    # the MFMA kernel with at most 3 (default), 4, 2 and 1 row tiles per work-group (more stacked rows go to row
    # groups), then the generic kernel
    for generic, max_tiles in ((0, 3), (0, 4), (0, 2), (0, 1), (1, 3)):
        ver.set_option(P.SV_OPT_ATTN_GENERIC, generic)
        ver.set_option(P.SV_OPT_ATTN_MAX_ROW_TILES, max_tiles)
        got = ver.op_attention(ids, n, k, 0, q.to(DEV))
        torch.cuda.synchronize()
        got = got.float().cpu().numpy().reshape(B, n, hq, hd)
        for b, L in enumerate(lengths):
            mask = np.concatenate([np.ones((n, L), dtype=bool), vis], axis=1)
            want = M.attend(q[b * n:(b + 1) * n].double().numpy(), ks[b].double().numpy(), vs[b].double().numpy(), mask)
            spread = M.attend(q[b * n:(b + 1) * n].double().numpy(), ks[b].double().numpy(),
                              np.abs(vs[b].double().numpy()), mask)
            tol = 2.0 ** -8 * (np.abs(want) + spread) + 1e-6
            assert np.all(np.abs(got[b] - want) <= tol), (generic, max_tiles, b, L, float(np.max(np.abs(got[b] - want))))
    ver.close()


@pytest.mark.parametrize("k,n_chains,group,max_tiles", [(4, 1, 7, 4), (8, 3, 5, 4), (8, 3, 5, 3), (8, 1, 7, 2)])
def test_attention_with_scores_that_keep_growing(k, n_chains, group, max_tiles):
    """Keys aligned with the queries and growing along the cache, so that the largest score so far rises by
    some 80 log2 units over each request: the kernels' lazily moved softmax reference has to move several times
    in mid-stream (in the skewed kernel with PV products of the previous tile still pending), where random keys
    move it on the first tile only.  Both MFMA kernels (up to 48 stacked rows; more rows / several row groups)."""
    import paper_2511_16193_amd as P
    hkv, hd = 2, 128
    hq = hkv * group
    n = 1 + n_chains * k
    lengths = [700, 2047, 3100, 95]
    B = len(lengths)
    model = dict(n_layers=1, d_model=256, n_q_heads=hq, n_kv_heads=hkv, head_dim=hd, d_ff=512, vocab=2048,
                 dtype="bf16", rope_theta=1e6, rms_eps=1e-6)
    wd = W.make_weights(W.Shape("attn", 1, 256, hq, hkv, hd, 512, 2048), DEV)
    ver = P.Verifier(model, wd, max_batch=B, max_k=k, max_chains=n_chains, max_seqs=B, page_size=64,
                     num_pages=B * 52, max_pages_per_seq=51, verify_mode=0)
    g = torch.Generator().manual_seed(4)
    u = torch.sign(torch.randn(hd, generator=g))                       # |u|^2 = 128
    q = (u[None, None, :] * (0.5 + torch.rand((B * n, hq, 1), generator=g)) + 0.3 * torch.randn((B * n, hq, hd), generator=g)).to(torch.bfloat16)
    ks, vs = [], []
    for b, L in enumerate(lengths):
        ver.seq_add(b, L)
        ramp = torch.linspace(0.0, 5.0, L + n)[:, None, None] * (1.0 if b % 2 == 0 else -1.0) + (0.0 if b % 2 == 0 else 5.0)
        ks.append((ramp * u[None, None, :] + 0.3 * torch.randn((L + n, hkv, hd), generator=g)).to(torch.bfloat16))
        vs.append(bf16_cpu((L + n, hkv, hd), 1.0, 50 + b))
    ids = list(range(B))
    ver.set_option(P.SV_OPT_ATTN_MAX_ROW_TILES, max_tiles)
    ver.op_attention(ids, n, k, 0, q.to(DEV))
    for b in range(B):
        ver.kv_write(b, 0, 0, ks[b].to(DEV), vs[b].to(DEV))
    _, _, vis = OV.new_token_layout(k, n_chains)
    got = ver.op_attention(ids, n, k, 0, q.to(DEV))
    torch.cuda.synchronize()
    got = got.float().cpu().numpy().reshape(B, n, hq, hd)
    for b, L in enumerate(lengths):
        mask = np.concatenate([np.ones((n, L), dtype=bool), vis], axis=1)
        qb = q[b * n:(b + 1) * n].double().numpy()
        want = M.attend(qb, ks[b].double().numpy(), vs[b].double().numpy(), mask)
        spread = M.attend(qb, ks[b].double().numpy(), np.abs(vs[b].double().numpy()), mask)
        tol = 2.0 ** -8 * (np.abs(want) + spread) + 1e-6
        assert np.all(np.isfinite(got[b]))
        assert np.all(np.abs(got[b] - want) <= tol), (b, L, float(np.max(np.abs(got[b] - want))))
    ver.close()


def random_case(B, N, k, V, seed, sigma_q=1.0, with_q=True):
    rng = np.random.default_rng(seed)
    logits = (rng.standard_normal((B, 1 + N * k, V)) * 1.2).astype(np.float32)
    q = W.make_random_q((B, N, k), V, sigma_q, seed) if with_q and k else None
    if k:
        drafts = (W.sample_from(q, seed).numpy() if q is not None else rng.integers(0, V, (B, N, k))).astype(np.int64)
        # make a good share of drafts likely: copy the target's argmax into some slots
        per_chain = np.empty((B, N, k), dtype=np.int64)
        for c in range(N):
            rows = np.concatenate([logits[:, :1], logits[:, 1 + c * k: 1 + (c + 1) * k]], axis=1)[:, :k]
            per_chain[:, c] = np.argmax(rows, axis=-1)
        take = rng.random((B, N, k)) < 0.3
        drafts = np.where(take, per_chain, drafts)
    else:
        drafts = np.zeros((B, N, 0), dtype=np.int64)
    u = W.make_uniforms((B, N, k + 1), seed)
    return logits, drafts, q, u


def oracle_sample(logits, drafts, q, u, verify_mode, sample_mode, temperature, draft_lens=None):
    from harness import decide
    return decide(logits, drafts, None if q is None else q.numpy(), u, verify_mode, sample_mode, temperature, draft_lens)


CASES = [
    # B, N, k, V, verify_mode, sample_mode, temperature, with_q, ragged
    (7, 1, 4, 2048, OV.GREEDY, 0, 1.0, False, False),
    (9, 1, 4, 2048, OV.STOCHASTIC, OV.SAMPLE_INVERSE_CDF, 1.0, True, False),
    (9, 1, 4, 2048, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 1.0, True, False),
    (5, 3, 8, 4099, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 0.7, True, False),
    (5, 3, 8, 4099, OV.GREEDY, 0, 1.0, False, True),
    (6, 1, 4, 3001, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 1.0, False, False),       # one-hot drafts
    (6, 1, 4, 3001, OV.STOCHASTIC, OV.SAMPLE_INVERSE_CDF, 1.3, False, True),
    (4, 1, 0, 2048, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 1.0, False, False),       # k = 0: plain decoding
    (16, 1, 4, 152064, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 1.0, True, False),     # full vocabulary
    (8, 1, 4, 152064, OV.STOCHASTIC, OV.SAMPLE_INVERSE_CDF, 1.0, True, False),
    (16, 1, 4, 152064, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 1.0, False, False),    # one-hot drafts at the full vocabulary
    (12, 3, 8, 152064, OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, 1.0, False, True),     # the same with three chains, ragged windows
    (1, 1, 1, 16, OV.STOCHASTIC, OV.SAMPLE_INVERSE_CDF, 1.0, True, False),       # degenerate sizes
]


@pytest.mark.parametrize("B,N,k,V,vmode,smode,temp,with_q,ragged", CASES)
def test_sampler_matches_oracle_on_given_logits(B, N, k, V, vmode, smode, temp, with_q, ragged):
    """Identical fp32 logits on both sides: accepted lengths, kept chain and tokens must be identical
    except where the oracle's own decision margin is below 1e-5 (fp32 vs fp64 evaluation of exp/log)."""
    from paper_2511_16193_amd import op_sample
    logits, drafts, q, u = random_case(B, N, k, V, 100 + B + k + V % 7, with_q=with_q)
    lens = np.random.default_rng(5).integers(0, k + 1, B) if ragged else None
    a, out, best, margin = oracle_sample(logits, drafts, q, u, vmode, smode, temp, lens)
    ga, gout, gbest = op_sample(
        torch.from_numpy(logits).to(DEV), torch.from_numpy(drafts).to(torch.int32).to(DEV).contiguous(),
        None if q is None else q.to(DEV).contiguous(), torch.from_numpy(u).to(DEV),
        verify_mode=vmode, sample_mode=smode, temperature=temp,
        draft_lens=None if lens is None else torch.from_numpy(lens).to(torch.int32).to(DEV))
    torch.cuda.synchronize()
    ga, gout, gbest = ga.cpu().numpy(), gout.cpu().numpy(), gbest.cpu().numpy()
    bad = [b for b in range(B) if not (ga[b] == a[b] and gbest[b] == best[b] and np.array_equal(gout[b], out[b]))]
    for b in bad:
        assert margin[b] < 1e-5, (b, ga[b], a[b], gout[b], out[b], margin[b])
    assert len(bad) <= max(1, B // 8)
    assert a.max() > 0 or k == 0 or not with_q or ragged


@pytest.mark.parametrize("B,N,k,V,smode,temp,ragged", [
    (6, 3, 4, 2048, OV.SAMPLE_EXP_RACE, 1.0, False),
    (6, 3, 4, 2048, OV.SAMPLE_INVERSE_CDF, 0.8, True),
    (5, 1, 8, 4099, OV.SAMPLE_EXP_RACE, 1.0, True),
    (4, 1, 0, 2048, OV.SAMPLE_EXP_RACE, 1.0, False),            # k = 0: plain sampling of one token
    (8, 2, 4, 152064, OV.SAMPLE_EXP_RACE, 1.0, False),          # full vocabulary
])
def test_sampler_match_mode_on_given_logits(B, N, k, V, smode, temp, ragged):
    """Sampled exact match on identical fp32 logits: the tokens the oracle draws for the slots are planted into
    the drafts with probability 0.6, so chains agree with them for a while; accepted lengths, kept chain and tokens
    must be identical except where the oracle's own draw margin is below 1e-5."""
    from paper_2511_16193_amd import op_sample
    logits, drafts, _, u = random_case(B, N, k, V, 300 + B + k + V % 5, with_q=False)
    rng = np.random.default_rng(9)
    if k:
        # the token of every row under the (request, slot) key
        n = 1 + N * k
        p = M.softmax(logits.astype(np.float64) / temp, axis=-1).reshape(B * n, V)
        slot = np.array([0] + [i + 1 for _ in range(N) for i in range(k)])           # slot index - 1 served by row j
        uu = u[:, 0, :][:, slot].reshape(-1)
        if smode == OV.SAMPLE_INVERSE_CDF:
            t, _ = OV.draw_inverse_cdf(p, uu.astype(np.float64))
        else:
            t, _ = OV.draw_exp_race(p, uu.astype(np.float32), np.repeat(np.arange(B, dtype=np.uint64), n))
        t = t.reshape(B, n)
        for c in range(N):
            rows = np.concatenate([t[:, :1], t[:, 1 + c * k: 1 + (c + 1) * k]], axis=1)[:, :k]
            drafts[:, c] = np.where(rng.random((B, k)) < 0.6, rows, drafts[:, c])
    lens = rng.integers(0, k + 1, B) if ragged else None
    a, out, best, margin = oracle_sample(logits, drafts, None, u, OV.MATCH, smode, temp, lens)
    ga, gout, gbest = op_sample(
        torch.from_numpy(logits).to(DEV), torch.from_numpy(drafts).to(torch.int32).to(DEV).contiguous(), None,
        torch.from_numpy(u).to(DEV), verify_mode=OV.MATCH, sample_mode=smode, temperature=temp,
        draft_lens=None if lens is None else torch.from_numpy(lens).to(torch.int32).to(DEV))
    torch.cuda.synchronize()
    ga, gout, gbest = ga.cpu().numpy(), gout.cpu().numpy(), gbest.cpu().numpy()
    bad = [b for b in range(B) if not (ga[b] == a[b] and gbest[b] == best[b] and np.array_equal(gout[b], out[b]))]
    for b in bad:
        assert margin[b] < 1e-5, (b, ga[b], a[b], gout[b], out[b], margin[b])
    assert len(bad) <= max(1, B // 8)
    assert k == 0 or a.max() > 0


def test_sampler_zero_residual_falls_back_to_target():
    """p and q one-hot on the same token (all other logits -inf) and a draft elsewhere: p(x) = q(x) = 0, so
    u*q(x) < p(x) fails and the draft is rejected, yet max(p - q, 0) is identically zero: the draw must fall
    back to p."""
    from paper_2511_16193_amd import op_sample
    V = 64
    logits = np.full((1, 2, V), -np.inf, dtype=np.float32)
    logits[0, 0, 7] = 20.0                          # p = one-hot(7) to fp32 precision
    logits[0, 1, 9] = 20.0
    q = np.zeros((1, 1, 1, V), dtype=np.float32)
    q[0, 0, 0, 7] = 1.0                             # q = one-hot(7): p - q == 0 everywhere
    drafts = np.array([[[3]]])                      # the draft itself is a token with p = q = 0 -> rejected (u*0 < 0 false)
    u = np.array([[[0.5, 0.25]]], dtype=np.float32)
    for smode in (OV.SAMPLE_INVERSE_CDF, OV.SAMPLE_EXP_RACE):
        v = OV.verify_stochastic(logits.astype(np.float64), drafts.reshape(1, 1), q.reshape(1, 1, V), u.reshape(1, 2),
                                 np.zeros(1, np.uint64), 1.0, smode)
        assert v.accepted[0] == 0 and v.zero_residual[0] and v.token[0] == 7
        ga, gout, _ = op_sample(torch.from_numpy(logits).to(DEV), torch.from_numpy(drafts).to(torch.int32).to(DEV),
                                torch.from_numpy(q).to(DEV), torch.from_numpy(u).to(DEV),
                                verify_mode=OV.STOCHASTIC, sample_mode=smode)
        torch.cuda.synchronize()
        assert int(ga[0]) == 0 and int(gout[0, 0]) == 7


@pytest.mark.parametrize("vmode,smode,with_q", [(OV.GREEDY, 0, False), (OV.STOCHASTIC, OV.SAMPLE_EXP_RACE, True),
                                                (OV.STOCHASTIC, OV.SAMPLE_INVERSE_CDF, False), (OV.MATCH, OV.SAMPLE_EXP_RACE, False)])
def test_sampler_rejects_draft_ids_outside_the_vocabulary(vmode, smode, with_q):
    """Draft ids arrive in device memory from the drafter's process and cannot be checked on the host.  An id
    below 0 or >= vocab is rejected without being used as an index, and the token supplied for its slot is drawn
    from the target's distribution of that slot (q taken as zero): exactly what a draft window that ends just
    before that slot gives, which is how the oracle states the expectation."""
    from paper_2511_16193_amd import op_sample
    B, N, k, V = 8, 1, 4, 2048
    logits, drafts, q, u = random_case(B, N, k, V, 77, with_q=with_q)
    # make every draft acceptable up to the planted slot: greedy / match need the target's own token there
    if vmode == OV.GREEDY:
        drafts[:, 0] = np.argmax(logits[:, :k], axis=-1)
    if vmode == OV.MATCH:
        p = M.softmax(logits.astype(np.float64), axis=-1).reshape(B * (k + 1), V)
        t, _ = OV.draw_exp_race(p, u[:, 0, :].reshape(-1).astype(np.float32), np.repeat(np.arange(B, dtype=np.uint64), k + 1))
        drafts[:, 0] = t.reshape(B, k + 1)[:, :k]
    bad_slot = np.array([0, 1, 2, 3, 0, 1, 2, 3])                 # 0-based slot of the planted id
    bad_id = np.array([-1, V, V + 12345, -2**31, 2**31 - 1, -5, V, V + 1])
    planted = drafts.copy()
    planted[np.arange(B), 0, bad_slot] = bad_id
    a, out, best, margin = oracle_sample(logits, drafts, q, u, vmode, smode, 1.0, bad_slot.copy())
    ga, gout, gbest = op_sample(
        torch.from_numpy(logits).to(DEV), torch.from_numpy(planted).to(torch.int32).to(DEV).contiguous(),
        None if q is None else q.to(DEV).contiguous(), torch.from_numpy(u).to(DEV),
        verify_mode=vmode, sample_mode=smode, temperature=1.0)
    torch.cuda.synchronize()
    ga, gout = ga.cpu().numpy(), gout.cpu().numpy()
    assert np.all(ga <= bad_slot)                                 # never past the planted id
    for b in range(B):
        assert 0 <= gout[b, ga[b]] < V                            # the supplied token is a valid one
        if margin[b] >= 1e-5:
            assert ga[b] == a[b] and np.array_equal(gout[b], out[b]), (b, ga[b], a[b], gout[b], out[b])
    assert (a == bad_slot).sum() >= 2                             # some walks did reach the planted id


@pytest.mark.parametrize("dtype,hd,N,k", [("bf16", 128, 3, 8), ("bf16", 128, 2, 3), ("fp32", 64, 3, 4), ("bf16", 128, 1, 4)])
def test_rollback_moves_the_kept_chain_next_to_x0(dtype, hd, N, k):
    """The rollback stage alone on given verdicts, against the oracle's rollback on the same cache contents:
    lengths that put the moved entries across 32-key tiles and 64-key pages, every kept chain and accepted
    length, a verdict that keeps chain 0 (nothing moves) and two that are out of range (nothing moves, nothing
    is touched); afterwards every slot of every layer is compared bit for bit -- moved entries, entries that
    had to stay, and the dead ones beyond."""
    import paper_2511_16193_amd as P
    hkv, layers = 2, 3
    n = 1 + N * k
    lengths = [0, 5, 30, 31, 56, 60, 63, 64, 100, 127, 1000]
    B = len(lengths)
    shape = W.Shape("rb", layers, 256, 2 * hkv, hkv, hd, 512, 2048, dtype=dtype)
    spec = M.ModelSpec(**shape.model_fields())
    wd = W.make_weights(shape, DEV)
    ver = P.Verifier(shape.model_fields(), wd, max_batch=B, max_k=k, max_chains=N, max_seqs=B, page_size=64,
                     num_pages=B * 18, max_pages_per_seq=18, verify_mode=0)
    rng = np.random.default_rng(3)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    caches = []
    for b, L in enumerate(lengths):
        ver.seq_add(b, L + n)                                  # a pass has appended its n rows
        c = M.SeqCache(spec, L + n)
        for l in range(layers):
            kk = torch.from_numpy(rng.standard_normal((L + n, hkv, hd)).astype(np.float32)).to(tdt)
            vv = torch.from_numpy(rng.standard_normal((L + n, hkv, hd)).astype(np.float32)).to(tdt)
            ver.kv_write(b, l, 0, kk.to(DEV), vv.to(DEV))
            c.k[l][:] = kk.float().numpy()
            c.v[l][:] = vv.float().numpy()
        c.length = L
        caches.append(c)
    ver.seq_set_lens(list(range(B)), lengths)                  # live lengths back to before the pass
    best = rng.integers(0, N, B).astype(np.int32)
    acc = rng.integers(0, k + 1, B).astype(np.int32)
    best[0], acc[0] = N - 1, k                                 # the longest move there is
    best[1], acc[1] = 0, k                                     # chain 0 already sits in place
    dev_best, dev_acc = best.copy(), acc.copy()
    if N > 1:
        dev_best[2], dev_acc[3] = N + 5, k + 7                 # out of range: must move nothing
        best[2], acc[3] = 0, 0                                 # (what the oracle is told instead)
        acc[2] = dev_acc[2]
        best[3] = dev_best[3]
    ver.op_rollback(list(range(B)), N, k, torch.from_numpy(dev_acc).to(DEV), torch.from_numpy(dev_best).to(DEV), commit=False)
    torch.cuda.synchronize()
    for b, L in enumerate(lengths):                            # (reading a length back would release the pages beyond it)
        OV.rollback(caches[b], int(best[b]), int(acc[b]), k)
        for l in range(layers):
            kd, vd = ver.kv_read(b, l, 0, L + n)
            assert np.array_equal(kd.float().cpu().numpy(), caches[b].k[l][:L + n]), (b, l)
            assert np.array_equal(vd.float().cpu().numpy(), caches[b].v[l][:L + n]), (b, l)
    # with commit the lengths advance by a + 1 (out-of-range verdicts aside, which the step never produces); without, not
    ver.op_rollback(list(range(B)), N, k, torch.from_numpy(acc).to(DEV), torch.from_numpy(best).to(DEV), commit=False)
    ver.op_rollback(list(range(B)), N, k, torch.from_numpy(acc).to(DEV), torch.from_numpy(best).to(DEV), commit=True)
    assert [ver.seq_len(b) for b in range(B)] == [L + int(a) + 1 for L, a in zip(lengths, acc)]
    ver.close()
