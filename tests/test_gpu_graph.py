"""ist_subnet_steps only enqueues kernels on the caller's stream (no allocation, no host
synchronisation, no memset nodes), so a caller can record it into a HIP graph: replays of the
captured steps must leave exactly the parameters that the same calls leave when issued eagerly."""
import numpy as np
import pytest
import torch

import ist_harness as H
from test_gpu_parity import SHAPES

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["cfg1", "ragged-bf16", "cfg5-small"])
def test_graph_replays_equal_eager_steps(name):
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev="cuda:0")
    k, reps = 2, 3
    eager, graphed = P.context(), P.context()
    eager.partition(P.dW, P.db, P.dperm)
    graphed.partition(P.dW, P.db, P.dperm)
    torch.cuda.synchronize()
    for _ in range(reps):
        P.gpu_steps(eager, k=k, loss=False)
    torch.cuda.synchronize()
    want = H.export_all(eager, cfg)

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            P.gpu_steps(graphed, k=k, loss=False)
    torch.cuda.current_stream().wait_stream(side)
    for r in range(reps):
        g.replay()
        torch.cuda.synchronize()          # the program's own synchronisation between replays
        _ = P.dy.sum().item()             # and eager work of its own
    got = H.export_all(graphed, cfg)
    for s in range(cfg.S):
        for l in range(cfg.t):
            assert np.array_equal(H.bits(got[s][0][l]), H.bits(want[s][0][l])), (name, s, l)
            assert np.array_equal(H.bits(got[s][1][l]), H.bits(want[s][1][l])), (name, s, l, "bias")
    eager.close()
    graphed.close()


@pytest.mark.parametrize("name", ["cfg1", "ragged-bf16", "uneven-S3-f32", "cfg5-small"])
def test_graph_replays_of_a_whole_round_equal_eager_rounds(name):
    """ist_partition, ist_subnet_steps and ist_merge of one round recorded into one graph (unchecked
    mode: nothing synchronises): every replay is a round on the network the previous one merged, and
    after each of them the full network must hold exactly the bits that eager rounds leave."""
    cfg = SHAPES[name]
    P = H.Problem(cfg, dev="cuda:0")
    k, reps = 2, 3
    eager, graphed = P.context(), P.context()
    We, be = [w.clone() for w in P.dW], [b.clone() for b in P.db]
    Wg, bg = [w.clone() for w in P.dW], [b.clone() for b in P.db]

    def round_(ctx, W, b):
        ctx.partition(W, b, P.dperm)
        P.gpu_steps(ctx, k=k, loss=False)
        ctx.merge(W, b)

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            round_(graphed, Wg, bg)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for w0, w in zip(P.dW, Wg):           # (capturing runs nothing: the network is still the initial one)
        assert torch.equal(w0, w)
    for r in range(reps):
        round_(eager, We, be)
        g.replay()
        torch.cuda.synchronize()          # the program's own synchronisation between replays
        _ = P.dy.sum().item()             # and eager work of its own
        for l in range(cfg.t):
            assert np.array_equal(H.bits(Wg[l]), H.bits(We[l])), (name, r, l)
            assert np.array_equal(H.bits(bg[l]), H.bits(be[l])), (name, r, l, "bias")
    assert not torch.equal(We[0], P.dW[0])    # the rounds did train
    eager.close()
    graphed.close()
