"""Shared helpers of the GPU parity tests (marshalling and comparison only)."""
import math
import os

import numpy as np
import torch

from oracle import svoo_oracle as so

DEV = "cuda:0"

# Acceptance bars (floating point): bf16 inputs -> max-abs 2e-2 and relative L2 5e-3; fp32 -> 1e-5.
TOL = {"bf16": (2e-2, 5e-3), "f32": (1e-5, 1e-5)}
NEAR_TIE = 1e-6


def torch_dtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def to_dev(x, dtype_name=None):
    """numpy -> device tensor.  Floating inputs hold dtype-exact values, so the cast is lossless."""
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype_name is not None:
        t = t.to(torch_dtype(dtype_name))
    return t.to(DEV).contiguous()


def to_np(t):
    t = t.detach()
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.cpu().numpy()


def attn_errors(got, ref):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    max_abs = float(np.abs(got - ref).max()) if got.size else 0.0
    rel_l2 = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)) if got.size else 0.0
    return max_abs, rel_l2


def assert_attn_close(got, ref, dtype_name, what=""):
    max_abs, rel_l2 = attn_errors(got, ref)
    tol_abs, tol_rel = TOL[dtype_name]
    assert max_abs <= tol_abs and rel_l2 <= tol_rel, f"{what}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}"
    return max_abs, rel_l2


def compare_labels(gpu_labels, oracle_labels, best, second):
    """Labels must be bit-exact except where the oracle's best and second-best squared distances
    differ by less than 1e-6 relative.  Returns the number of such near-tie differences."""
    gpu_labels = np.asarray(gpu_labels)
    diff = np.nonzero(gpu_labels != oracle_labels)[0]
    if diff.size == 0:
        return 0
    gap = (second[diff] - best[diff]) / np.maximum(np.abs(second[diff]), 1e-300)
    bad = diff[gap >= NEAR_TIE]
    assert bad.size == 0, (f"{bad.size} labels differ beyond near-ties; first token {bad[0]}: gpu "
                           f"{gpu_labels[bad[0]]} oracle {oracle_labels[bad[0]]} rel gap {gap[gap >= NEAR_TIE][0]:.3e}")
    return int(diff.size)


def oracle_assign(x, c_own32, c_opp32):
    """Oracle assignment from float32 centroids (what crosses the library boundary)."""
    x = np.asarray(x, np.float64)
    dist = so.affinity_distances(x, np.asarray(c_own32, np.float64), np.asarray(c_opp32, np.float64), "l2")
    labels = so.argmin_lowest(dist)
    best = dist[np.arange(x.shape[0]), labels]
    if dist.shape[1] > 1:
        dist[np.arange(x.shape[0]), labels] = np.inf
        second = dist.min(axis=1)
    else:
        second = np.full_like(best, np.inf)
    return labels, best, second


def scale_of(d):
    """1/sqrt(d) as the float32 that crosses the boundary."""
    return float(np.float32(1.0 / math.sqrt(d)))


# the paper's intuition example for query-key coupling (fixture tests/golden/query_dependent_key_partition.txt)
def load_coupling_example():
    pts, parts = {}, {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "query_dependent_key_partition.txt")):
        line = line.split("#")[0].strip()
        if not line:
            continue
        name, rest = line.split(None, 1)
        if name.startswith("partition_"):
            parts[name[len("partition_"):]] = {frozenset(int(t) for t in grp.split()) for grp in rest.split("|")}
        else:
            pts[name] = [float(t) for t in rest.split()]
    return pts, parts


def embed(rows, d):
    out = np.zeros((len(rows), d))
    out[:, :2] = np.asarray(rows)
    return out
