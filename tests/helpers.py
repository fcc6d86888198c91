"""Shared helpers of the GPU parity tests (marshalling and comparison only)."""
import math
import os
import warnings

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


def report_near_ties(what, count, total):
    """Near-tie differences are allowed but must be seen: a quiet pytest run prints warnings."""
    if count:
        warnings.warn(f"{what}: {count} label(s) of {total} differ from the oracle at near-ties "
                      f"(oracle distance gap < {NEAR_TIE:g} relative)")


def compare_mask(gpu_mask, oracle_mask, margins, what="", max_near_tie_rows=0):
    """EVERY block-mask row is compared with the oracle's, bit for bit.  A row that differs is an
    error unless its selection hangs on a margin below 1e-6 relative (two weights at the cut, or a
    cumulative weight at tau: ``oracle.selection_margins``); such rows are counted, reported and
    bounded (both sides decide in float64, so none is expected: the default bound is 0).  Returns
    (rows equal, rows that differ at a near-tie)."""
    gpu_mask = np.asarray(gpu_mask).astype(bool)
    oracle_mask = np.asarray(oracle_mask).astype(bool)
    differ = (gpu_mask != oracle_mask).any(axis=1)
    near = np.asarray(margins) < NEAR_TIE
    wrong = np.nonzero(differ & ~near)[0]
    assert wrong.size == 0, f"{what}: mask rows {wrong[:8]} differ from the oracle's (margins {np.asarray(margins)[wrong[:8]]})"
    flipped = int((differ & near).sum())
    assert flipped <= max_near_tie_rows, f"{what}: {flipped} mask rows differ at near-ties (allowed {max_near_tie_rows})"
    if flipped:
        warnings.warn(f"{what}: {flipped} block-mask row(s) differ from the oracle's at near-ties "
                      f"(selection margin < {NEAR_TIE:g} relative)")
    return int((~differ).sum()), flipped


def resync_cocluster(q, k, init_q_idx, init_k_idx, iters, gpu_steps, init_cq=None, init_ck=None, what=""):
    """Algorithm 1 by the oracle, half-step by half-step, next to the labels the GPU produced at the
    same half-step (gpu_steps[(it, side)], side "k" = Step A, "q" = Step B).  At every half-step the
    GPU labels must equal the oracle's except at proven near-ties (``compare_labels`` with the
    oracle's own best / second-best distances of THAT half-step); where they differ the oracle
    continues from the GPU's labels (its centroids are recomputed from them), so every later
    comparison stays exact.  Returns the oracle's result dict in step with the GPU, with
    ``near`` = total near-tie differences and ``near_steps`` = per half-step counts."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    cq = np.array(init_cq, np.float64) if init_cq is not None else q[np.asarray(init_q_idx)].copy()
    ck = np.array(init_ck, np.float64) if init_ck is not None else k[np.asarray(init_k_idx)].copy()
    near_steps = []
    lq = lk = nq = nk = None
    for it in range(iters):
        for side in ("k", "q"):
            x, c_own, c_opp = (k, ck, cq) if side == "k" else (q, cq, ck)
            labels, c_new, counts, _, best, second = so.half_step(x, c_own, c_opp)
            gpu = np.asarray(gpu_steps[(it, side)])
            near = compare_labels(gpu, labels, best, second)
            if near:
                labels = gpu.astype(np.int32)
                c_new, counts = so.update_centroids(x, labels, c_own)
            near_steps.append(near)
            if side == "k":
                lk, ck, nk = labels, c_new, counts
            else:
                lq, cq, nq = labels, c_new, counts
    total = int(sum(near_steps))
    report_near_ties(what or "co-clustering", total, 2 * iters * q.shape[0])
    return {"labels_q": lq, "labels_k": lk, "cq": cq, "ck": ck, "counts_q": nq, "counts_k": nk,
            "near": total, "near_steps": near_steps}


def resync_kmeans(x, init_idx, iters, gpu_steps, init_c=None, what=""):
    """The same for the independent partitioner: gpu_steps[it] = GPU labels after iteration it."""
    x = np.asarray(x, np.float64)
    c = np.array(init_c, np.float64) if init_c is not None else x[np.asarray(init_idx)].copy()
    near_steps, inertia = [], []
    labels = counts = None
    for it in range(iters):
        one = so.kmeans(x, None, 1, init_c=c)
        tr = one["trace"][0]
        labels, c_new, counts = one["labels"], one["c"], one["counts"]
        gpu = np.asarray(gpu_steps[it])
        near = compare_labels(gpu, labels, tr["best"], tr["second"])
        if near:
            labels = gpu.astype(np.int32)
            c_new, counts = so.update_centroids(x, labels, c)
        near_steps.append(near)
        inertia.append(tr["inertia"] if not near else None)
        c = c_new
    total = int(sum(near_steps))
    report_near_ties(what or "k-means", total, iters * x.shape[0])
    return {"labels": labels, "c": c, "counts": counts, "near": total, "near_steps": near_steps, "inertia": inertia}


def gpu_cocluster_steps(qd, kd, init_q_idx, init_k_idx, iters, init_cq=None, init_ck=None):
    """Labels of every half-step of svoo_cocluster, [bh, n] each: the call with t iterations ends
    with Step A and Step B of iteration t, and the library is deterministic, so the calls with
    t = 1 .. iters expose every intermediate labelling of the full run.  Returns (steps, last call's
    outputs)."""
    from paper_2603_18636_amd import svoo
    steps, out = {}, None
    for t in range(1, iters + 1):
        out = svoo.cocluster(qd, kd, init_q_idx, init_k_idx, t, init_cq=init_cq, init_ck=init_ck)
        steps[(t - 1, "k")] = to_np(out["labels_k"])
        steps[(t - 1, "q")] = to_np(out["labels_q"])
    return steps, out


def gpu_kmeans_steps(xd, init_idx, iters, init_c=None):
    from paper_2603_18636_amd import svoo
    steps, out = {}, None
    for t in range(1, iters + 1):
        out = svoo.kmeans(xd, init_idx, t, init_c=init_c)
        steps[t - 1] = to_np(out["labels"])
    return steps, out


def slice_steps(steps, b):
    return {key: val[b] for key, val in steps.items()}


ROWS_PER_HEAD = 4096      # stratified attention rows checked per head at the full-size workloads (rows are
                          # independent problems, so a sampled row is checked exactly)


def stratified_rows(labels_q, counts_q, n_rows, rng):
    """Sample rows covering the smallest and the largest query clusters and every cluster once."""
    rows = []
    live = np.nonzero(counts_q > 0)[0]
    order = live[np.argsort(counts_q[live])]
    for r in list(order[:4]) + list(order[-4:]):
        members = np.nonzero(labels_q == r)[0]
        rows.extend(members[[0, len(members) // 2, len(members) - 1]])
    for r in live:
        members = np.nonzero(labels_q == r)[0]
        rows.append(members[rng.integers(0, len(members))])
    rows = np.unique(np.array(rows, dtype=np.int64))
    rest = np.setdiff1d(np.arange(labels_q.shape[0]), rows)
    extra = rng.choice(rest, max(0, min(rest.size, n_rows - rows.size)), replace=False)
    return np.unique(np.concatenate([rows, extra]))


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
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "query_dependent_key_partition.txt")).read().splitlines():
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
