"""GPU parity of the independent k-means partitioner (ablation "w/o On") and of the attention-recall
diagnostic built on the kernels' log-sum-exp outputs, against the fp64 oracle."""
import math

import numpy as np
import pytest
import torch

from oracle import svoo_oracle as so
from paper_2603_18636_amd import svoo, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu


def small_head(layer=0, head=0, grid=(6, 12, 20), n_seeds=24, kq=24, kk=20, d=128, dtype="bf16"):
    return synth.make_head(synth.CONFIGS[1], layer, head, grid=grid, n_seeds=n_seeds, kq=kq, kk=kk, d=d, dtype=dtype)


def run_and_check(xd, x, init_idx, iters, b=0, what="k-means"):
    """svoo_kmeans on device tensor xd [bh, n, d] next to the oracle on slice b, iteration by iteration:
    a label difference must be a proven near-tie of that iteration, after which the oracle follows the
    GPU, so counts and centroids are always compared.  Returns the number of near-tie differences."""
    steps, _ = H.gpu_kmeans_steps(xd, H.to_dev(init_idx), iters)
    out = svoo.kmeans(xd, H.to_dev(init_idx), iters, want_inertia=True)
    assert (H.to_np(out["labels"]) == steps[iters - 1]).all()
    ref = H.resync_kmeans(x, init_idx[b], iters, H.slice_steps(steps, b), what=what)
    assert (H.to_np(out["labels"])[b] == ref["labels"]).all()
    assert (H.to_np(out["counts"])[b] == ref["counts"]).all()
    np.testing.assert_array_equal(H.to_np(out["c"])[b], ref["c"].astype(np.float32))
    inertia = H.to_np(out["inertia"])[b]
    for it, j_ref in enumerate(ref["inertia"]):
        if j_ref is None or sum(ref["near_steps"][:it]) > 0:
            continue              # a moved label changes the sums from there on
        np.testing.assert_allclose(inertia[it], j_ref, rtol=1e-9)
    return ref["near"]


@pytest.mark.parametrize("dtype,d,iters", [("bf16", 128, 3), ("f32", 64, 5), ("bf16", 64, 2), ("f32", 128, 1)])
def test_kmeans_matches_oracle(dtype, d, iters):
    h = small_head(d=d, dtype=dtype)
    for side, idx in (("k", "init_k_idx"), ("q", "init_q_idx")):
        x = h[side]
        run_and_check(H.to_dev(x[None], dtype), x, h[idx][None], iters)


def test_kmeans_heads_are_independent_and_k_1024():
    """Three heads in one call; 1024 clusters on 5000 tokens (32-centroid blocks, many near-empty)."""
    cfg = synth.CONFIGS[1]
    heads = [synth.make_head(cfg, 0, hd, grid=(5, 25, 40), n_seeds=64, kq=1024, kk=1000) for hd in range(3)]
    x = np.stack([h["k"] for h in heads])
    for name, k in (("init_q_idx", 1024), ("init_k_idx", 1000)):
        idx = np.stack([h[name] for h in heads])
        for b in range(3):
            run_and_check(H.to_dev(x, "bf16"), x[b], idx, 2, b)


def test_kmeans_warm_start_duplicates_and_far_centroid():
    h = small_head(dtype="bf16")
    k = h["k"]
    c0 = k[h["init_k_idx"]].astype(np.float32)
    c0[5] = c0[2]                      # duplicate: ties go to the lower index, cluster 5 stays empty
    c0[7] = 300.0                      # far from every token: empty, must keep its centroid
    for iters in (1, 2):   # after the first update cluster 2 has moved and cluster 5 may win tokens
        out = svoo.kmeans(H.to_dev(k[None], "bf16"), None, iters, init_c=H.to_dev(c0[None]))
        ref = so.kmeans(k, None, iters, init_c=c0)
        assert (H.to_np(out["labels"])[0] == ref["labels"]).all()
        counts = H.to_np(out["counts"])[0]
        assert counts[7] == 0 and (counts == ref["counts"]).all()
        got_c = H.to_np(out["c"])[0]
        assert (got_c[7] == 300.0).all()
        if iters == 1:
            assert counts[5] == 0 and (got_c[5] == c0[2]).all()
        np.testing.assert_array_equal(got_c, ref["c"].astype(np.float32))


def test_kmeans_full_size_head_of_config2():
    """One head at the real shape (75,600 tokens, 256 clusters, d = 128), two iterations."""
    cfg = synth.CONFIGS[2]
    h = synth.make_head(cfg, 0, 1)
    for side, idx in (("q", "init_q_idx"), ("k", "init_k_idx")):
        near = run_and_check(H.to_dev(h[side][None], "bf16"), h[side], h[idx][None], 2,
                             what=f"configs[2] k-means({side})")
        print(f"config 2 k-means({side}): {near} near-tie label differences of {cfg.n}")


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_layer_with_kmeans_partitioner_and_recall(dtype, d):
    """Whole path with the independent partitioner, then the recall diagnostic from the two
    log-sum-exp outputs against the oracle's dense-softmax definition."""
    h = small_head(d=d, dtype=dtype, layer=3)
    q, k, v = h["q"], h["k"], h["v"]
    kq, kk, iters, keep = 24, 20, 2, 0.3
    scale = H.scale_of(d)
    dev = {n: H.to_dev(h[n][None], dtype) for n in "qkv"}
    layer = svoo.Layer(1, q.shape[0], d, H.torch_dtype(dtype), kq, kk, H.DEV)
    keep_dev = H.to_dev(np.array([keep], dtype=np.float32))
    out = layer.run(dev["q"], dev["k"], dev["v"], H.to_dev(h["init_q_idx"][None]), H.to_dev(h["init_k_idx"][None]),
                    iters, keep_dev, 1.0, 0.0, scale, partitioner="kmeans")
    ref = so.layer(q, k, v, h["init_q_idx"], h["init_k_idx"], iters, float(np.float32(keep)), 1.0, 0.0, scale,
                   partitioner="kmeans")
    assert (H.to_np(layer.labels_q)[0] == ref["labels_q"]).all()
    assert (H.to_np(layer.labels_k)[0] == ref["labels_k"]).all()
    assert (H.to_np(layer.bitmap)[0].astype(bool) == ref["mask"]).all()
    H.assert_attn_close(H.to_np(out)[0], ref["out"], dtype, "k-means layer")
    rec = H.to_np(layer.row_recall(dev["q"], dev["k"], dev["v"], scale))[0]
    rec_ref = so.row_recall(q, k, ref["labels_q"], ref["labels_k"], ref["mask"], scale, np.arange(q.shape[0]))
    tol = 3e-2 if dtype == "bf16" else 1e-4
    assert np.abs(rec - rec_ref).max() <= tol
    assert abs(rec.mean() - rec_ref.mean()) <= tol / 5
    assert 0.0 < rec_ref.mean() < 1.0
