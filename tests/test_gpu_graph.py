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
