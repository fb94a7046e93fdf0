"""Graph replay of the verification step (SV_OPT_GRAPH): the same steps through a captured HIP graph and through
plain launches must give identical results, replay after replay, with the lengths changing in between."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu

SHAPE = W.Shape("graph-bf16", 3, 256, 8, 2, 128, 512, 2048, dtype="bf16", batch=6, k=4, prefix_lo=40, prefix_hi=2600,
                seed=321)


def run_steps(graph: bool, steps: int):
    """Six requests, k = 4, stochastic verification; the cache advances by the accepted tokens after every step
    (no reset), every third step the lengths are put back, so the item list of the attention and the lengths
    differ between replays.  Returns everything a step produces, per step."""
    import paper_2511_16193_amd as P
    from workloads.device_case import DeviceCase
    stream = torch.cuda.Stream()                      # graph capture needs a stream of its own
    res = []
    with torch.cuda.stream(stream):
        case = DeviceCase(SHAPE)
        case.independent_drafts(1.0)
        if graph:
            case.ver.set_option(P.SV_OPT_GRAPH, 1)
        B, N, k, V = case.B, case.N, case.k, SHAPE.vocab
        out = {"accepted_len": torch.empty(B, dtype=torch.int32, device=case.device),
               "out_tokens": torch.empty((B, k + 1), dtype=torch.int32, device=case.device),
               "best_chain": torch.empty(B, dtype=torch.int32, device=case.device),
               "logits": torch.empty((B, 1 + N * k, V), dtype=torch.float32, device=case.device)}
        for s in range(steps):
            if s % 3 == 0 and s:
                case.reset()                          # plain launches between replays
            case.step(out=out)                        # same buffers every step: one graph serves them all
            stream.synchronize()
            res.append({key: v.cpu().numpy().copy() for key, v in out.items()})
            res[-1]["lens"] = np.array([case.ver.seq_len(b) for b in range(B)])
            # the supplied token becomes the next x0 (device-side copy, plain torch work between replays)
            idx = out["accepted_len"].long()
            case.x0.copy_(out["out_tokens"].gather(1, idx[:, None])[:, 0])
        case.close()
    return res


def test_graph_replay_matches_plain_launches():
    plain = run_steps(False, 8)
    graph = run_steps(True, 8)            # step 0 plain (first of its kind), step 1 captured, steps 2.. replayed
    for s, (p, g) in enumerate(zip(plain, graph)):
        for key in p:
            assert np.array_equal(p[key], g[key]), f"step {s}: {key} differs between plain launches and graph replay"
    assert any(r["accepted_len"].sum() > 0 for r in plain)
    assert not np.array_equal(plain[1]["lens"], plain[2]["lens"])     # the replays did see different lengths


def test_graph_needs_own_stream():
    import paper_2511_16193_amd as P
    from workloads.device_case import DeviceCase
    case = DeviceCase(W.scaled_down(SHAPE, batch=2))      # created on the null stream
    with pytest.raises(P.SvError):
        case.ver.set_option(P.SV_OPT_GRAPH, 1)
    case.close()
