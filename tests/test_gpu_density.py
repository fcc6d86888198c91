"""GPU parity of svoo_attention_density (offline profiling, attention density of Sec. 4.1) against
the fp64 oracle.  Prefix lengths are integers decided by floating point: a length must equal the
oracle's unless the oracle's cumulative sum passes tau by less than SLACK on one side of the
crossing (float32 logits and masses on the GPU against float64); then it may differ by a few."""
import math

import numpy as np
import pytest
import torch

from oracle import svoo_oracle as so
from paper_2603_18636_amd import svoo, synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

SLACK = 2e-5        # float32 logits: relative error ~1e-6 on |s| ~ 10 -> masses good to ~1e-5


def compare_prefix(got, ref, max_near=None):
    diff = np.nonzero(got != ref["prefix_len"])[0]
    bad = diff[ref["slack"][diff] > SLACK]
    assert bad.size == 0, f"{bad.size} rows differ beyond rounding; first {bad[0]}: {got[bad[0]]} vs {ref['prefix_len'][bad[0]]}"
    if diff.size:
        rel = np.abs(got[diff] - ref["prefix_len"][diff]) / ref["prefix_len"][diff]
        assert (np.abs(got[diff] - ref["prefix_len"][diff]) <= 2 + 1e-3 * ref["prefix_len"][diff]).all(), rel.max()
    if max_near is not None:
        assert diff.size <= max_near
    return int(diff.size)


@pytest.mark.parametrize("dtype,d,grid,tau", [("bf16", 128, (6, 12, 20), 0.95), ("bf16", 64, (3, 3, 37), 0.5),
                                              ("f32", 64, (4, 16, 16), 0.95), ("f32", 128, (1, 3, 43), 0.9),
                                              ("bf16", 128, (1, 1, 64), 0.99), ("bf16", 64, (1, 1, 2), 0.95)])
def test_density_matches_oracle(dtype, d, grid, tau):
    cfg = synth.CONFIGS[1]
    heads = [synth.make_head(cfg, 2, hd, grid=grid, n_seeds=8, kq=1, kk=1, d=d, dtype=dtype) for hd in range(2)]
    q = np.stack([h["q"] for h in heads])
    k = np.stack([h["k"] for h in heads])
    n = q.shape[1]
    scale, tau32 = H.scale_of(d), float(np.float32(tau))
    plen, dens = svoo.attention_density(H.to_dev(q, dtype), H.to_dev(k, dtype), tau32, scale)
    plen, dens = H.to_np(plen), H.to_np(dens)
    for b in range(2):
        ref = so.attention_density(q[b], k[b], scale, tau32)
        near = compare_prefix(plen[b], ref, max_near=max(2, n // 100))
        assert abs(dens[b] - plen[b].mean() / n) < 1e-15
        if near == 0:     # same integers; only the order of the divisions differs
            assert abs(dens[b] - ref["density"]) <= 1e-14


@pytest.mark.parametrize("d,grid,copies", [(128, (6, 12, 20), 12), (128, (6, 12, 20), 24), (64, (3, 3, 37), 45),
                                           (64, (3, 3, 37), 90), (128, (1, 3, 43), 300)])
def test_density_in_every_launch_shape(d, grid, copies):
    """The bf16 kernel splits the keys 4, 2 or 1 ways inside a workgroup depending on how many
    workgroups the launch has (<= 256, <= 512, more); the small cases above all take the 4-way shape.
    Here two heads are repeated ``copies`` times so that the same data runs through the other shapes
    (n = 1440: 12 workgroups per head -> 288 and 576; n = 333, ragged last tile: 3 per head -> 270 and
    540; n = 129: 2 per head, three 64-key tiles of which the last holds one key -> 1200), each
    compared with the oracle, and every copy must equal the first."""
    cfg = synth.CONFIGS[1]
    heads = [synth.make_head(cfg, 7, hd, grid=grid, n_seeds=8, kq=1, kk=1, d=d, dtype="bf16") for hd in range(2)]
    q = np.tile(np.stack([h["q"] for h in heads]), (copies, 1, 1))
    k = np.tile(np.stack([h["k"] for h in heads]), (copies, 1, 1))
    n = q.shape[1]
    wgs = (n + 127) // 128 * 2 * copies
    assert wgs > 256
    scale, tau32 = H.scale_of(d), float(np.float32(0.95))
    plen, dens, passes = svoo.attention_density(H.to_dev(q, "bf16"), H.to_dev(k, "bf16"), tau32, scale, want_passes=True)
    plen, dens, passes = H.to_np(plen), H.to_np(dens), H.to_np(passes)
    for b in range(2):
        ref = so.attention_density(q[b], k[b], scale, tau32)
        compare_prefix(plen[b], ref, max_near=max(2, n // 100))
        assert (plen[b::2] == plen[b]).all() and (dens[b::2] == dens[b]).all() and (passes[b::2] == passes[b]).all()
    # the 4-way shape on the same two heads
    plen4, _ = svoo.attention_density(H.to_dev(q[:2], "bf16"), H.to_dev(k[:2], "bf16"), tau32, scale)
    differ = int((H.to_np(plen4) != plen[:2]).sum())
    print(f"{wgs} workgroups: {differ} of {2 * n} prefix lengths differ from the 4-way launch")
    assert differ <= max(2, n // 100)


def test_density_row_subset_and_order():
    h = synth.make_head(synth.CONFIGS[1], 5, 0, grid=(6, 12, 20), n_seeds=8, kq=1, kk=1)
    q, k, n = h["q"][None], h["k"][None], h["q"].shape[0]
    rows = np.array([n - 1, 0, 17, 17, 700, 129], dtype=np.int32)        # any order, repeats allowed
    plen, dens = svoo.attention_density(H.to_dev(q, "bf16"), H.to_dev(k, "bf16"), 0.95, H.scale_of(128),
                                        rows=H.to_dev(rows))
    ref = so.attention_density(q[0], k[0], H.scale_of(128), float(np.float32(0.95)), rows=rows)
    compare_prefix(H.to_np(plen)[0], ref, max_near=0)
    assert abs(H.to_np(dens)[0] - ref["prefix_len"].mean() / n) <= 1e-14


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_density_single_key(dtype):
    x = synth.round_to_bf16(np.random.default_rng(0).standard_normal((3, 1, 128)).astype(np.float32))
    plen, dens = svoo.attention_density(H.to_dev(x, dtype), H.to_dev(x, dtype))       # default tau and scale
    assert (H.to_np(plen) == 1).all() and (H.to_np(dens) == 1.0).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_density_ties_uniform_and_geometric(dtype):
    """Zero queries: every key ties, the prefix is ceil(tau n).  Keys -j ln2 / scale on one axis
    against a unit query: p_j ~ 2^-j, so the prefix for tau is ceil(log2(1 / (1 - tau)))."""
    n, d, scale = 200, 64, 0.25
    rng = np.random.default_rng(1)
    k = synth.round_to_bf16(rng.standard_normal((1, n, d)).astype(np.float32))
    q0 = np.zeros((1, n, d), dtype=np.float32)
    for tau in (0.95, 0.5, 1.0):
        plen, _ = svoo.attention_density(H.to_dev(q0, dtype), H.to_dev(k, dtype), tau, scale)
        assert (H.to_np(plen) == math.ceil(float(np.float32(tau)) * n)).all()
    # pairs of identical keys: ties inside the prefix are taken one at a time
    kd = np.repeat(k[:, : n // 2], 2, axis=1)
    qd = synth.round_to_bf16(rng.standard_normal((1, n, d)).astype(np.float32))
    plen, _ = svoo.attention_density(H.to_dev(qd, dtype), H.to_dev(kd, dtype), 0.9, scale)
    ref = so.attention_density(qd[0], kd[0], scale, float(np.float32(0.9)))
    compare_prefix(H.to_np(plen)[0], ref, max_near=2)
    kg = np.zeros((1, n, d), dtype=np.float32)
    kg[0, :, 0] = -np.arange(n) * 4.0                     # bf16-exact; scale ln2 / 4 makes p_j ~ 2^-j
    qg = np.zeros((1, n, d), dtype=np.float32)
    qg[0, :, 0] = 1.0
    sc = float(np.float32(math.log(2.0) / 4.0))
    for tau, want in ((0.9, 4), (0.6, 2), (0.99, 7)):
        plen, dens = svoo.attention_density(H.to_dev(qg, dtype), H.to_dev(kg, dtype), tau, sc)
        assert (H.to_np(plen) == want).all()
        assert abs(H.to_np(dens)[0] - want / n) < 1e-15


def test_density_full_size_head_of_config2():
    """One head at the real shape (75,600 keys), 1,024 sampled query rows, tau = 0.95."""
    cfg = synth.CONFIGS[2]
    h = synth.make_head(cfg, 0, 2)
    rows = np.sort(np.random.default_rng(3).choice(cfg.n, 1024, replace=False)).astype(np.int32)
    scale = H.scale_of(cfg.d)
    plen, dens, passes = svoo.attention_density(H.to_dev(h["q"][None], "bf16"), H.to_dev(h["k"][None], "bf16"), 0.95,
                                                scale, rows=H.to_dev(rows), want_passes=True)
    torch.cuda.synchronize()
    assert 3 <= int(H.to_np(passes)[0]) <= 40
    ref = so.attention_density(h["q"], h["k"], scale, float(np.float32(0.95)), rows=rows, chunk=256)
    plen = H.to_np(plen)[0]
    near = compare_prefix(plen, ref)
    d_gpu, d_ref = H.to_np(dens)[0], ref["density"]
    print(f"config 2 density: gpu {d_gpu:.6f} oracle {d_ref:.6f}, {near} of 1024 prefix lengths differ within rounding")
    assert abs(d_gpu - d_ref) <= 1e-4 * d_ref
