"""The whole layer can be recorded into a HIP graph and replayed: every call only enqueues kernels on
the caller's stream (no allocation, no synchronisation, no memset nodes), so a replay must give
the results of the eager run bit for bit -- on every replay, with eager work and synchronisations
in between."""
import numpy as np
import pytest
import torch

from paper_2603_18636_amd import svoo, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

NAMES = ("labels_q", "labels_k", "cq", "ck", "counts_q", "counts_k", "perm_q", "perm_k", "q_offsets", "k_offsets",
         "block_count", "bitmap", "out")


@pytest.mark.parametrize("partitioner", ["cocluster", "kmeans"])
def test_layer_replays_from_a_graph(partitioner):
    cfg = synth.CONFIGS[1]
    heads = [0, 5]
    data = [synth.make_layer(cfg, layer, heads=heads, workers=8) for layer in (0, 1)]
    bh = len(heads)
    layer = svoo.Layer(bh, cfg.n, cfg.d, torch.bfloat16, cfg.kq, cfg.kk, H.DEV)
    static = {k: H.to_dev(data[0][k], "bf16") for k in "qkv"}
    static.update({k: H.to_dev(data[0][k]) for k in ("init_q_idx", "init_k_idx")})
    keep = H.to_dev(np.full(bh, 0.25, dtype=np.float32))

    def step():
        layer.run(static["q"], static["k"], static["v"], static["init_q_idx"], static["init_k_idx"], cfg.iters, keep,
                  0.95, 0.1, partitioner=partitioner)

    def load(d):
        for k in "qkv":
            static[k].copy_(H.to_dev(d[k], "bf16"))
        for k in ("init_q_idx", "init_k_idx"):
            static[k].copy_(H.to_dev(d[k]))

    def snapshot():
        torch.cuda.synchronize()
        return {name: getattr(layer, name).clone() for name in NAMES}

    eager = []
    for d in data:
        load(d)
        step()
        eager.append(snapshot())
    assert not torch.equal(eager[0]["labels_q"], eager[1]["labels_q"])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    torch.cuda.synchronize()

    for which in (0, 1, 1, 0):
        load(data[which])
        for name in NAMES:                       # eager work between replays; stale results must not survive
            getattr(layer, name).zero_()
        torch.cuda.synchronize()
        graph.replay()
        got = snapshot()
        for name in NAMES:
            assert torch.equal(got[name], eager[which][name]), (which, name)


def test_two_layers_on_two_streams_with_workspaces_of_their_own():
    """The binding's cached workspace is one buffer per device; layers whose calls may overlap on the
    GPU take ``own_workspace=True``.  Two such layers, each on a stream of its own, must give what the
    same layers give one after the other."""
    cfg = synth.CONFIGS[1]
    heads = [[0, 1], [2, 3]]
    data = [synth.make_layer(cfg, 0, heads=h, workers=4) for h in heads]
    layers = [svoo.Layer(2, cfg.n, cfg.d, torch.bfloat16, cfg.kq, cfg.kk, H.DEV, own_workspace=True) for _ in heads]
    assert layers[0].ws.data_ptr() != layers[1].ws.data_ptr()
    dev = [{k: H.to_dev(d[k], "bf16") for k in "qkv"} for d in data]
    for t, d in zip(dev, data):
        t.update({k: H.to_dev(d[k]) for k in ("init_q_idx", "init_k_idx")})
    keep = H.to_dev(np.full(2, 0.3, dtype=np.float32))

    def step(g):
        layers[g].run(dev[g]["q"], dev[g]["k"], dev[g]["v"], dev[g]["init_q_idx"], dev[g]["init_k_idx"], cfg.iters,
                      keep, 0.95, 0.1)

    serial = []
    for g in range(2):
        step(g)
        torch.cuda.synchronize()
        serial.append({name: getattr(layers[g], name).clone() for name in NAMES})
    streams = [torch.cuda.Stream() for _ in heads]
    for rep in range(3):
        for g in range(2):
            streams[g].wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(streams[g]):
                step(g)
        for g in range(2):
            torch.cuda.current_stream().wait_stream(streams[g])
        torch.cuda.synchronize()
        for g in range(2):
            for name in NAMES:
                assert torch.equal(getattr(layers[g], name), serial[g][name]), (rep, g, name)
