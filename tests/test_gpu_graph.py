"""The decode step under HIP graph capture (how bench.py launches it): replays, with eager work and
synchronisation in between, must reproduce the eager results bit for bit; the append variant restores
the sequence lengths before every step, as a serving loop that reuses a graph for a fixed shape would."""
import numpy as np
import pytest
import torch

import workloads as W

pytestmark = pytest.mark.gpu


def capture(body):
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        body()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        body()
    return graph


@pytest.mark.parametrize("append,context", [(False, 20000), (True, 20000), (False, 40000), (True, 40000)])
def test_graph_replays_equal_eager(append, context):
    """20000 tokens: ENCODE-Q + SCORE + TOPK in one launch; 40000: the two-launch select, and with an append the
    launch that the append shares with the query encoder."""
    import paper_2412_14468_amd as ha
    from paper_2412_14468_amd import runner
    cfg = W.scaled(W.c1(context=context, k=context // 32, batch=3), name="graph", append=append)
    t = W.device_tensors(cfg, W.BASE_SEED + 99, extra_rows=4)
    s = runner.layer_from_tensors(t)
    ctx = ha.Context(cfg.n_q_heads, cfg.n_kv_heads, cfg.batch, t["n_max"], s.k_max)
    runner.build_key_codes(ctx, s)
    lens0 = s.seq_lens.clone()
    max0 = s.cache.max_seq_len

    def step():
        if append:
            s.seq_lens.copy_(lens0)
            s.cache.max_seq_len = max0
        runner.decode_step(ctx, s, append=append)

    step()
    torch.cuda.synchronize()
    ref = (s.idx.clone(), s.count.clone(), s.out.clone(), s.seq_lens.clone(), s.q_codes.clone())
    g = capture(step)
    scratch = torch.empty(1 << 22, dtype=torch.float32, device="cuda:0")
    for i in range(4):
        s.idx.fill_(-1); s.count.fill_(-1); s.out.zero_(); s.q_codes.zero_()
        scratch.normal_()                                    # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(s.count, ref[1]), f"replay {i}: counts"
        assert torch.equal(s.idx, ref[0]), f"replay {i}: index sets"
        assert torch.equal(s.out.view(torch.int16), ref[2].view(torch.int16)), f"replay {i}: outputs"
        assert torch.equal(s.seq_lens, ref[3]) and torch.equal(s.q_codes, ref[4])
        float(scratch.sum())                                 # a library reduction and a host sync in between
    if append:
        assert s.seq_lens.cpu().tolist() == (lens0 + 1).cpu().tolist()


def test_two_contexts_on_two_streams():
    """Each context owns its scratch: steps of two contexts issued on two streams at the same time give
    what each gives alone."""
    import paper_2412_14468_amd as ha
    from paper_2412_14468_amd import runner
    states, ctxs, refs = [], [], []
    for i, (n, k, batch) in enumerate(((30000, 900, 2), (9000, 300, 5))):
        cfg = W.scaled(W.c1(context=n, k=k, batch=batch), name=f"pair{i}")
        t = W.device_tensors(cfg, W.BASE_SEED + 200 + i)
        s = runner.layer_from_tensors(t)
        ctx = ha.Context(cfg.n_q_heads, cfg.n_kv_heads, cfg.batch, t["n_max"], s.k_max)
        runner.build_key_codes(ctx, s)
        runner.decode_step(ctx, s)
        torch.cuda.synchronize()
        refs.append((s.idx.clone(), s.count.clone(), s.out.clone()))
        states.append(s)
        ctxs.append(ctx)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for s in states:
        s.idx.fill_(-1); s.count.fill_(-1); s.out.zero_()
    torch.cuda.synchronize()
    for _ in range(3):                                        # interleaved submissions, no waits in between
        for ctx, s, st in zip(ctxs, states, streams):
            with torch.cuda.stream(st):
                runner.decode_step(ctx, s)
    torch.cuda.synchronize()
    for s, (idx, count, out) in zip(states, refs):
        assert torch.equal(s.count, count) and torch.equal(s.idx, idx)
        assert torch.equal(s.out.view(torch.int16), out.view(torch.int16))
