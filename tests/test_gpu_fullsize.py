"""GPU parity at the benchmark's full size and launch configuration (configs[2]: 12 heads x
75,600 tokens, d = 128, bf16, 256 + 256 clusters, 3 iterations).  The oracle cannot run a whole
layer at this size in seconds, so: one head is checked end to end (labels, mask, sampled attention
rows), and every head is checked step by step on sampled outputs with the GPU's own inputs to
that step (rows of attention and tokens of the assignment are independent, so sampling is exact
per sample)."""
import math

import numpy as np
import pytest
import torch

from oracle import svoo_oracle as so
from paper_2603_18636_amd import svoo, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

CFG = synth.CONFIGS[2]
ROWS_PER_HEAD = H.ROWS_PER_HEAD


@pytest.fixture(scope="module")
def full_layer():
    data = synth.make_layer(CFG, 0, workers=8)
    keep = float(synth.layer_keeps(CFG)[0])
    layer = svoo.Layer(CFG.heads, CFG.n, CFG.d, torch.bfloat16, CFG.kq, CFG.kk, H.DEV)
    dev = {k: H.to_dev(data[k], "bf16") for k in "qkv"}
    dev["init_q_idx"] = H.to_dev(data["init_q_idx"])
    dev["init_k_idx"] = H.to_dev(data["init_k_idx"])
    keep_dev = H.to_dev(np.full(CFG.heads, keep, dtype=np.float32))
    out = layer.run(dev["q"], dev["k"], dev["v"], dev["init_q_idx"], dev["init_k_idx"], CFG.iters, keep_dev, 1.0, 0.0)
    torch.cuda.synchronize()
    got = {name: H.to_np(getattr(layer, name)) for name in
           ("labels_q", "labels_k", "cq", "ck", "counts_q", "counts_k", "perm_q", "perm_k", "q_offsets", "k_offsets",
            "block_count", "block_list", "bitmap")}
    got["out"] = H.to_np(out)
    return data, dev, keep, layer, got


def test_fullsize_head0_end_to_end(full_layer):
    """Head 0 through the oracle end to end: labels of every half-step (a difference must be a proven
    near-tie, after which the oracle follows the GPU), centroids, mask, >= 4096 stratified attention rows."""
    data, dev, keep, layer, got = full_layer
    b = 0
    scale = H.scale_of(CFG.d)
    q, k, v = data["q"][b], data["k"][b], data["v"][b]
    one = {name: dev[name][b:b + 1] for name in ("q", "k", "init_q_idx", "init_k_idx")}
    steps, _ = H.gpu_cocluster_steps(one["q"], one["k"], one["init_q_idx"], one["init_k_idx"], CFG.iters)
    assert (steps[(CFG.iters - 1, "q")][0] == got["labels_q"][b]).all()     # heads are independent problems
    assert (steps[(CFG.iters - 1, "k")][0] == got["labels_k"][b]).all()
    ref = H.resync_cocluster(q, k, data["init_q_idx"][b], data["init_k_idx"][b], CFG.iters, H.slice_steps(steps, 0),
                             what="configs[2] head 0")
    assert (got["labels_q"][b] == ref["labels_q"]).all() and (got["labels_k"][b] == ref["labels_k"]).all()
    np.testing.assert_array_equal(got["cq"][b], ref["cq"].astype(np.float32))
    np.testing.assert_array_equal(got["ck"][b], ref["ck"].astype(np.float32))
    cq32, ck32 = ref["cq"].astype(np.float32), ref["ck"].astype(np.float32)
    mask = so.block_mask(cq32, ck32, ref["counts_q"], ref["counts_k"], np.float32(keep), 1.0, 0.0, scale)
    margins = so.selection_margins(cq32, ck32, ref["counts_q"], ref["counts_k"], np.float32(keep), 1.0, 0.0, scale)
    H.compare_mask(got["bitmap"][b], mask, margins, "configs[2] head 0")
    rows = H.stratified_rows(ref["labels_q"], ref["counts_q"], ROWS_PER_HEAD, np.random.default_rng(0))
    assert rows.size >= ROWS_PER_HEAD
    out_ref = so.sparse_attention(q, k, v, ref["labels_q"], ref["labels_k"], mask, scale, rows=rows)
    H.assert_attn_close(got["out"][b][rows], out_ref, "bf16", "full-size head 0")


def test_fullsize_every_head_stepwise(full_layer):
    data, dev, keep, layer, got = full_layer
    scale = H.scale_of(CFG.d)
    rng = np.random.default_rng(1)
    worst = (0.0, 0.0)
    for b in range(CFG.heads):
        lq, lk = got["labels_q"][b], got["labels_k"][b]
        # sizes, offsets and the permutation follow from the labels (bit-exact)
        assert (np.bincount(lq, minlength=CFG.kq) == got["counts_q"][b]).all()
        assert (np.bincount(lk, minlength=CFG.kk) == got["counts_k"][b]).all()
        for labels, perm, off, kk in ((lq, got["perm_q"][b], got["q_offsets"][b], CFG.kq),
                                      (lk, got["perm_k"][b], got["k_offsets"][b], CFG.kk)):
            p_ref, o_ref = so.stable_permutation(labels, kk)
            assert (perm == p_ref).all() and (off == o_ref).all()
        # centroids are the float32-rounded member means (sampled clusters)
        for j in rng.integers(0, CFG.kk, 8):
            if got["counts_k"][b][j] > 0:
                mean = data["k"][b][lk == j].astype(np.float64).mean(axis=0)
                np.testing.assert_allclose(got["ck"][b][j], mean, rtol=1e-6, atol=1e-7)
        # the mask from the GPU's centroids and sizes (bit-exact away from near-ties)
        mask = so.block_mask(got["cq"][b], got["ck"][b], got["counts_q"][b], got["counts_k"][b], np.float32(keep), 1.0,
                             0.0, scale)
        margins = so.selection_margins(got["cq"][b], got["ck"][b], got["counts_q"][b], got["counts_k"][b],
                                       np.float32(keep), 1.0, 0.0, scale)
        gpu_mask = got["bitmap"][b].astype(bool)
        H.compare_mask(gpu_mask, mask, margins, f"configs[2] head {b}")
        assert (got["block_count"][b] == gpu_mask.sum(1)).all()
        # sampled attention rows with the GPU's labels and the GPU's mask
        rows = H.stratified_rows(lq, got["counts_q"][b], ROWS_PER_HEAD, rng)
        assert rows.size >= ROWS_PER_HEAD
        out_ref = so.sparse_attention(data["q"][b], data["k"][b], data["v"][b], lq, lk, gpu_mask, scale, rows=rows)
        e = H.assert_attn_close(got["out"][b][rows], out_ref, "bf16", f"full-size head {b}")
        worst = (max(worst[0], e[0]), max(worst[1], e[1]))
    print(f"worst sampled attention error over heads: max_abs={worst[0]:.3e} rel_l2={worst[1]:.3e}")


def test_fullsize_assign_teacher_forced_sampled(full_layer):
    """svoo_assign on all 12 heads at full N with the layer's final centroids; the oracle decides a
    sample of 4096 tokens per head from the same float32 centroids."""
    data, dev, keep, layer, got = full_layer
    rng = np.random.default_rng(2)
    labels = H.to_np(svoo.assign(dev["k"], layer.ck, layer.cq))
    near = 0
    for b in range(CFG.heads):
        sample = np.sort(rng.choice(CFG.n, 4096, replace=False))
        ref, best, second = H.oracle_assign(data["k"][b][sample], got["ck"][b], got["cq"][b])
        near += H.compare_labels(labels[b][sample], ref, best, second)
    print(f"near-tie label differences in the sample: {near}")


def test_fullsize_dense_sampled(full_layer):
    data, dev, keep, layer, got = full_layer
    scale = H.scale_of(CFG.d)
    out = H.to_np(layer.dense(dev["q"], dev["k"], dev["v"], scale))
    rng = np.random.default_rng(3)
    for b in (0, 5, 11):
        rows = np.sort(rng.choice(CFG.n, 256, replace=False))
        rows[0], rows[-1] = 0, CFG.n - 1
        ref = so.dense_attention(data["q"][b], data["k"][b], data["v"][b], scale, rows=rows, chunk=128)
        H.assert_attn_close(out[b][rows], ref, "bf16", f"dense head {b}")
