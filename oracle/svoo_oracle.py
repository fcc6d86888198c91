"""Plain fp64 CPU oracle for the online stage of SVOO (one attention layer, one head at a time).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file; it exists so that
the HIP kernels can be compared against a slow, obviously-correct implementation written from the
paper.  It shares no code with the GPU path and never imports it.  NumPy/SciPy, float64
throughout, original token order (it never permutes anything).

What follows the paper and where:

* ``half_step`` / ``cocluster``  -- Algorithm 1 (bidirectional co-clustering): Step A (query-aware
  key partition) and Step B (key-aware query partition), in the printed order, with the printed
  centroid versions (Step B uses the *new* key centroids and the *old* query centroids).
* ``block_weights`` / ``select_blocks`` / ``block_mask`` -- paragraph "Top Block-Pair Selection":
  coarse estimate from centroids, recall threshold tau, budget s, switch threshold theta.
* ``sparse_attention`` / ``dense_attention`` -- softmax(q K^T / sqrt(d')) V as defined in
  Sec. 4.1 (definition of z_i), restricted to the kept (query block, key block) pairs.
* ``kmeans`` -- the independent K-means partitioner of the ablation "w/o On" and of the prior work
  the paper contrasts itself with ("Difference from SVG2"): textbook Lloyd iterations per side.
* ``minimal_prefix`` / ``attention_density`` / ``sparsity_schedule`` -- the offline profiling
  module of Sec. 4.1: attention density (minimal fraction of entries covering a share tau of each
  row's mass) and the Gaussian upper-quantile schedule built on it.
* ``row_recall`` / ``attention_recall`` -- the attention-recall measure of the clustering
  comparison section, read as the dense softmax mass on kept keys.

Readings taken where the paper is silent (each is listed in the design notes of this build):
Norm(.) is row-wise L2 normalisation with a 1e-12 floor; argmin ties go to the lowest index; an
empty cluster keeps its previous centroid; the budget s is a *keep ratio*; the block estimate is
scaled by 1/sqrt(d), soft-maxed over key clusters with key-cluster sizes as weights; Recall is
the minimal descending-sorted prefix reaching cumulative weight tau, per query cluster; the
number of kept blocks is rounded up and at least one; softmax in the sparse attention is
normalised over the kept keys only.

Pins (tests/, CPU only): dense attention against a library routine, keep-everything == dense,
permutation invariance, one Lloyd iteration against scikit-learn when the affinity is the
identity, cosine-distance argmin against SciPy, block selection against brute-force block sums of
the exact attention matrix on zero-variance clusters, hand-computed selection cases; k-means
against SciPy's and scikit-learn's Lloyd iterations from the same start; recall against the
log-sum-exp identity, the uniform-attention closed form and explicit loops; density against
uniform and geometric rows (closed forms), hand cases at the tau boundary and explicit loops.  Whether the
paper's authors' code would produce the same labels is *parity unpinned*: Norm, the weighting of
the block estimate, Recall and the meaning of s cannot be confirmed from the text alone.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
from scipy.spatial.distance import cdist

NORM_FLOOR = 1e-12


# --------------------------------------------------------------------------------------------
# Algorithm 1: bidirectional co-clustering
# --------------------------------------------------------------------------------------------
def normalize_rows(p: np.ndarray, norm: str) -> np.ndarray:
    """Norm(.) of Algorithm 1.  "l2": every row divided by max(its 2-norm, 1e-12).  "none": as is."""
    if norm == "none":
        return p
    if norm != "l2":
        raise ValueError(norm)
    nrm = np.sqrt(np.sum(p * p, axis=1, keepdims=True))
    return p / np.maximum(nrm, NORM_FLOOR)


def affinity_distances(x: np.ndarray, c_own: np.ndarray, c_opp: np.ndarray, norm: str) -> np.ndarray:
    """D[i, j] = || Norm(x_i C_opp^T) - Norm(c_own_j C_opp^T) ||_2^2  (Algorithm 1, assignment lines).

    The squared 2-norm is summed term by term (SciPy's ``sqeuclidean``), not expanded.
    """
    p = normalize_rows(x @ c_opp.T, norm)
    p_bar = normalize_rows(c_own @ c_opp.T, norm)
    return cdist(p, p_bar, metric="sqeuclidean")


def argmin_lowest(dist: np.ndarray) -> np.ndarray:
    """Row-wise argmin; numpy returns the first (lowest-index) minimum."""
    return np.argmin(dist, axis=1).astype(np.int32)


def update_centroids(x: np.ndarray, labels: np.ndarray, c_prev: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Mean(X via L): mean of the member rows; an empty cluster keeps its previous centroid."""
    k = c_prev.shape[0]
    c_new = c_prev.copy()
    counts = np.zeros(k, dtype=np.int32)
    for j in range(k):
        members = x[labels == j]
        counts[j] = members.shape[0]
        if members.shape[0] > 0:
            c_new[j] = members.sum(axis=0) / members.shape[0]
    return c_new, counts


def half_step(x: np.ndarray, c_own: np.ndarray, c_opp: np.ndarray, norm: str = "l2"):
    """One of Step A / Step B: assign every row of x, then recompute the own-side centroids.

    Returns labels, new centroids, counts, J_assign = sum_i D[i, L_i] in the anchor space that
    produced the labels, and the per-row best and second-best distances (for near-tie accounting).
    """
    dist = affinity_distances(x, c_own, c_opp, norm)
    labels = argmin_lowest(dist)
    best = dist[np.arange(dist.shape[0]), labels]
    if dist.shape[1] > 1:
        tmp = dist.copy()
        tmp[np.arange(dist.shape[0]), labels] = np.inf
        second = tmp.min(axis=1)
    else:
        second = np.full_like(best, np.inf)
    c_new, counts = update_centroids(x, labels, c_own)
    return labels, c_new, counts, float(best.sum()), best, second


def cocluster(q: np.ndarray, k: np.ndarray, init_q_idx: Optional[np.ndarray], init_k_idx: Optional[np.ndarray],
              iters: int, norm: str = "l2", init_cq: Optional[np.ndarray] = None,
              init_ck: Optional[np.ndarray] = None) -> Dict[str, object]:
    """Algorithm 1 on one head.  q, k: [N, d].  Initial centroids are the anchor tokens at the given
    indices (Sample(.) is an input here), or the given warm-start centroids."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    cq = np.array(init_cq, dtype=np.float64) if init_cq is not None else q[np.asarray(init_q_idx)].copy()
    ck = np.array(init_ck, dtype=np.float64) if init_ck is not None else k[np.asarray(init_k_idx)].copy()
    trace: List[Dict[str, object]] = []
    lq = lk = None
    nq = nk = None
    for it in range(iters):
        # Step A: keys against query anchors C_q^(i-1); own centroids C_k^(i-1).
        lk, ck_new, nk, j_a, best_a, second_a = half_step(k, ck, cq, norm)
        trace.append({"iter": it, "side": "k", "labels": lk, "c_own_in": ck, "c_opp_in": cq,
                      "c_out": ck_new, "counts": nk, "J": j_a, "best": best_a, "second": second_a})
        ck = ck_new
        # Step B: queries against the NEW key anchors C_k^(i); own centroids are the OLD C_q^(i-1).
        lq, cq_new, nq, j_b, best_b, second_b = half_step(q, cq, ck, norm)
        trace.append({"iter": it, "side": "q", "labels": lq, "c_own_in": cq, "c_opp_in": ck,
                      "c_out": cq_new, "counts": nq, "J": j_b, "best": best_b, "second": second_b})
        cq = cq_new
    return {"labels_q": lq, "labels_k": lk, "cq": cq, "ck": ck, "counts_q": nq, "counts_k": nk,
            "trace": trace}


# --------------------------------------------------------------------------------------------
# Independent partitioner (ablation "w/o On"; the K-means block partitioning the paper contrasts
# its co-clustering with in "Difference from SVG2")
# --------------------------------------------------------------------------------------------
def kmeans(x: np.ndarray, init_idx: Optional[np.ndarray], iters: int,
           init_c: Optional[np.ndarray] = None) -> Dict[str, object]:
    """Lloyd's k-means on the raw rows of x [N, d], one side at a time, no coupling to the other
    side.  Per iteration: labels = argmin_j ||x_i - c_j||_2^2 (summed term by term, lowest j on
    ties), then c_j = mean of its rows (an empty cluster keeps its centroid).  Returned centroids
    are the means of the returned labels, as in Algorithm 1."""
    x = np.asarray(x, dtype=np.float64)
    c = np.array(init_c, dtype=np.float64) if init_c is not None else x[np.asarray(init_idx)].copy()
    trace: List[Dict[str, object]] = []
    labels = counts = None
    for it in range(iters):
        dist = cdist(x, c, metric="sqeuclidean")
        labels = argmin_lowest(dist)
        best = dist[np.arange(dist.shape[0]), labels]
        if dist.shape[1] > 1:
            tmp = dist.copy()
            tmp[np.arange(dist.shape[0]), labels] = np.inf
            second = tmp.min(axis=1)
        else:
            second = np.full_like(best, np.inf)
        c_new, counts = update_centroids(x, labels, c)
        trace.append({"iter": it, "labels": labels, "c_in": c, "c_out": c_new, "counts": counts,
                      "inertia": float(best.sum()), "best": best, "second": second})
        c = c_new
    return {"labels": labels, "c": c, "counts": counts, "trace": trace}


# --------------------------------------------------------------------------------------------
# Top block-pair selection
# --------------------------------------------------------------------------------------------
def block_weights(cq: np.ndarray, ck: np.ndarray, counts_k: np.ndarray, scale: float) -> np.ndarray:
    """Coarse block estimate A_bar = C_q C_k^T, scaled, soft-maxed over key clusters per query
    cluster with the key-cluster sizes as weights; empty key clusters get weight 0."""
    a_bar = scale * (np.asarray(cq, np.float64) @ np.asarray(ck, np.float64).T)
    nk = np.asarray(counts_k, dtype=np.float64)
    live = nk > 0
    w = np.zeros_like(a_bar)
    if not live.any():
        return w
    row_max = np.max(np.where(live[None, :], a_bar, -np.inf), axis=1, keepdims=True)
    e = np.where(live[None, :], nk[None, :] * np.exp(a_bar - row_max), 0.0)
    z = e.sum(axis=1, keepdims=True)
    return e / z


BUDGET_SNAP = 1e-6


def budget_blocks(keep: float, kk: int) -> int:
    """Number of key clusters the budget s allows: keep * K_k rounded up.  The keep ratio reaches
    the library as a float32, so a decimal ratio whose product with K_k is an integer (0.3 * 20)
    arrives a hair above it; a product within 1e-6 * K_k of an integer is therefore taken as that
    integer before rounding up."""
    x = float(keep) * kk
    nearest = round(x)
    if abs(x - nearest) <= BUDGET_SNAP * kk:
        return int(nearest)
    return int(math.ceil(x))


def select_blocks(w_row: np.ndarray, live: np.ndarray, keep: float, tau: float, theta: float) -> np.ndarray:
    """Kept key clusters of one query cluster (boolean [K_k]) from its weight row.

    Order the live key clusters by weight, descending, equal weights by lower index first.  m =
    length of the shortest prefix whose cumulative weight reaches tau (all live clusters when tau
    >= 1).  b = ceil(keep * K_k) (``budget_blocks``).  The number kept is min(m, b) if keep > theta,
    max(m, b) otherwise (the threshold-dependent rule of the selection paragraph), clamped to
    [1, #live].
    """
    kk = w_row.shape[0]
    n_live = int(live.sum())
    kept = np.zeros(kk, dtype=bool)
    if n_live == 0:
        return kept
    idx = np.nonzero(live)[0]
    order = idx[np.argsort(-w_row[idx], kind="stable")]
    if tau >= 1.0:
        m = n_live
    else:
        csum = np.cumsum(w_row[order])
        reach = np.nonzero(csum >= tau)[0]
        m = int(reach[0]) + 1 if reach.size else n_live
    b = budget_blocks(keep, kk)
    n_keep = min(m, b) if float(keep) > float(theta) else max(m, b)
    n_keep = max(1, min(n_keep, n_live))
    kept[order[:n_keep]] = True
    return kept


def block_mask(cq: np.ndarray, ck: np.ndarray, counts_q: np.ndarray, counts_k: np.ndarray, keep: float,
               tau: float, theta: float, scale: float) -> np.ndarray:
    """Boolean [K_q, K_k] block mask.  Empty query clusters keep nothing."""
    w = block_weights(cq, ck, counts_k, scale)
    live = np.asarray(counts_k) > 0
    out = np.zeros(w.shape, dtype=bool)
    for r in range(w.shape[0]):
        if counts_q[r] > 0:
            out[r] = select_blocks(w[r], live, keep, tau, theta)
    return out


def selection_margins(cq, ck, counts_q, counts_k, keep, tau, theta, scale) -> np.ndarray:
    """Per query cluster, how close the selection is to flipping: the smaller of (a) the relative
    weight gap between the last kept and the first dropped key cluster and (b) the relative distance
    of the cumulative weight from tau at the cut.  Used only to account for near-ties in parity."""
    w = block_weights(cq, ck, counts_k, scale)
    live = np.asarray(counts_k) > 0
    kq = w.shape[0]
    out = np.full(kq, np.inf)
    idx = np.nonzero(live)[0]
    for r in range(kq):
        if counts_q[r] == 0 or idx.size == 0:
            continue
        order = idx[np.argsort(-w[r, idx], kind="stable")]
        ws = w[r, order]
        n_keep = int(select_blocks(w[r], live, keep, tau, theta).sum())
        gap = np.inf
        if n_keep < ws.size:
            gap = (ws[n_keep - 1] - ws[n_keep]) / max(ws[n_keep - 1], 1e-300)
        csum = np.cumsum(ws)
        tgap = np.inf
        if tau < 1.0:
            tgap = float(np.min(np.abs(csum - tau))) / tau
        out[r] = min(gap, tgap)
    return out


# --------------------------------------------------------------------------------------------
# Attention
# --------------------------------------------------------------------------------------------
def _softmax_rows(s: np.ndarray) -> np.ndarray:
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def dense_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float,
                    rows: Optional[np.ndarray] = None, chunk: int = 1024) -> np.ndarray:
    """softmax(scale * q K^T) V for the given query rows (all by default)."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows)
    out = np.empty((rows.shape[0], v.shape[1]), dtype=np.float64)
    for a in range(0, rows.shape[0], chunk):
        sel = rows[a:a + chunk]
        out[a:a + chunk] = _softmax_rows(scale * (q[sel] @ k.T)) @ v
    return out


def sparse_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, labels_q: np.ndarray, labels_k: np.ndarray,
                     mask: np.ndarray, scale: float, rows: Optional[np.ndarray] = None,
                     chunk: int = 1024) -> np.ndarray:
    """Block-sparse attention in token order: query i (cluster r = labels_q[i]) attends to key t iff
    mask[r, labels_k[t]]; softmax normalised over those keys only.  A query with no kept key gets a
    zero row (cannot happen for masks made by ``block_mask``)."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    v = np.asarray(v, np.float64)
    rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows)
    out = np.zeros((rows.shape[0], v.shape[1]), dtype=np.float64)
    row_cluster = np.asarray(labels_q)[rows]
    for r in np.unique(row_cluster):
        key_sel = np.nonzero(mask[r][np.asarray(labels_k)])[0]
        if key_sel.size == 0:
            continue
        pos = np.nonzero(row_cluster == r)[0]
        kk, vv = k[key_sel], v[key_sel]
        for a in range(0, pos.size, chunk):
            p = pos[a:a + chunk]
            out[p] = _softmax_rows(scale * (q[rows[p]] @ kk.T)) @ vv
    return out


# --------------------------------------------------------------------------------------------
# Layout helpers of the library boundary (definitions, not kernels)
# --------------------------------------------------------------------------------------------
def stable_permutation(labels: np.ndarray, n_clusters: int) -> Tuple[np.ndarray, np.ndarray]:
    """perm[p] = token at sorted position p (clusters ascending, token index ascending inside a
    cluster); offsets[j] = first sorted position of cluster j, offsets[n_clusters] = N."""
    labels = np.asarray(labels)
    perm = np.argsort(labels, kind="stable").astype(np.int32)
    counts = np.bincount(labels, minlength=n_clusters)
    offsets = np.zeros(n_clusters + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    return perm, offsets


def kept_fraction(mask: np.ndarray, counts_q: np.ndarray, counts_k: np.ndarray) -> float:
    """phi = sum over kept blocks of n_r * n_j / N^2 (fraction of the dense score matrix computed)."""
    nq = np.asarray(counts_q, np.float64)
    nk = np.asarray(counts_k, np.float64)
    return float((nq[:, None] * nk[None, :] * mask).sum() / (nq.sum() * nk.sum()))


def row_recall(q, k, labels_q, labels_k, mask, scale, rows) -> np.ndarray:
    """Per given query row, the exact softmax mass (dense softmax over all keys) that falls on
    the keys of its kept key blocks.  Attention recall of the clustering comparison section is
    read as the mean of this over rows; the paper's own definition sits in an appendix that is
    not in the text."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    rows = np.asarray(rows)
    a = _softmax_rows(scale * (q[rows] @ k.T))
    kept = mask[np.asarray(labels_q)[rows]][:, np.asarray(labels_k)]
    return (a * kept).sum(axis=1)


def attention_recall(q, k, v_unused, labels_q, labels_k, mask, scale, rows) -> float:
    """Mean of ``row_recall`` over the given rows (diagnostic)."""
    return float(row_recall(q, k, labels_q, labels_k, mask, scale, rows).mean())


# --------------------------------------------------------------------------------------------
# Offline profiling: attention density (Sec. 4.1, the offline profiling module)
# --------------------------------------------------------------------------------------------
def minimal_prefix(a: np.ndarray, tau: float) -> Tuple[np.ndarray, np.ndarray]:
    """Per row of the probability matrix a: entries sorted in descending order, the length of the
    shortest prefix whose sum reaches tau (a prefix whose sum equals tau exactly is long enough),
    capped at the row length.  Also returns how far the cumulative sum is from tau on either
    side of the crossing (small = the length hangs on rounding)."""
    a = np.asarray(a, np.float64)
    n = a.shape[1]
    c = np.cumsum(-np.sort(-a, axis=1), axis=1)
    length = np.minimum((c < tau).sum(axis=1) + 1, n)
    idx = np.arange(a.shape[0])
    above = c[idx, length - 1] - tau
    below = np.where(length > 1, tau - c[idx, np.maximum(length - 2, 0)], np.inf)
    return length.astype(np.int64), np.minimum(np.abs(above), below)


def attention_density(q, k, scale: float, tau: float, rows: Optional[np.ndarray] = None,
                      chunk: int = 512) -> Dict[str, object]:
    """Density of one head's attention map: for every (given) query row the minimal fraction of
    the n post-softmax entries that covers a share tau of the row's mass, averaged over rows
    (the equation defining d_{l,h}; the paper sets tau = 0.95).  The softmax is the dense one of
    Sec. 4.1 over all n keys."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    n = k.shape[0]
    rows = np.arange(q.shape[0]) if rows is None else np.asarray(rows)
    lengths = np.empty(rows.shape[0], dtype=np.int64)
    slack = np.empty(rows.shape[0])
    for a0 in range(0, rows.shape[0], chunk):
        r = rows[a0:a0 + chunk]
        lengths[a0:a0 + chunk], slack[a0:a0 + chunk] = minimal_prefix(_softmax_rows(scale * (q[r] @ k.T)), tau)
    return {"prefix_len": lengths, "slack": slack, "density": float((lengths / n).mean())}


def sparsity_schedule(densities: np.ndarray, alpha: float = 0.95) -> float:
    """From the densities of one (layer, head) over the calibration inputs to its sparsity:
    Gaussian fit (mean, standard deviation of the samples), upper alpha-quantile as the
    conservative density, s = 1 - that (the two equations after the density definition).  The
    standard deviation is the maximum-likelihood one (divide by m); the text does not say which."""
    from scipy.stats import norm as gaussian
    d = np.asarray(densities, np.float64)
    d_hat = d.mean() + gaussian.ppf(alpha) * d.std()
    return float(1.0 - d_hat)


def layer(q, k, v, init_q_idx, init_k_idx, iters, keep, tau, theta, scale=None, norm="l2",
          rows: Optional[np.ndarray] = None, centroid_dtype=np.float32,
          partitioner: str = "cocluster") -> Dict[str, object]:
    """The whole online stage for one head.  Centroids cross the library boundary as float32, so
    they are rounded to that type between clustering and selection (``centroid_dtype=None`` keeps
    float64).  ``partitioner="kmeans"`` replaces Algorithm 1 by two independent k-means runs (the
    "w/o On" ablation); everything after the partition is unchanged."""
    d = q.shape[1]
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    if partitioner == "cocluster":
        cc = cocluster(q, k, init_q_idx, init_k_idx, iters, norm)
    elif partitioner == "kmeans":
        kq_, kk_ = kmeans(q, init_q_idx, iters), kmeans(k, init_k_idx, iters)
        cc = {"labels_q": kq_["labels"], "labels_k": kk_["labels"], "cq": kq_["c"], "ck": kk_["c"],
              "counts_q": kq_["counts"], "counts_k": kk_["counts"], "trace": [kq_["trace"], kk_["trace"]]}
    else:
        raise ValueError(partitioner)
    cq, ck = cc["cq"], cc["ck"]
    if centroid_dtype is not None:
        cq = cq.astype(centroid_dtype).astype(np.float64)
        ck = ck.astype(centroid_dtype).astype(np.float64)
    mask = block_mask(cq, ck, cc["counts_q"], cc["counts_k"], keep, tau, theta, scale)
    out = sparse_attention(q, k, v, cc["labels_q"], cc["labels_k"], mask, scale, rows=rows)
    res = dict(cc)
    res.update({"mask": mask, "out": out, "cq_boundary": cq, "ck_boundary": ck})
    return res
