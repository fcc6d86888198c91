"""Seeded synthetic video-shaped Q/K/V for one DiT attention layer.

This module only *draws inputs*: it holds none of the method's arithmetic (no clustering, no
mask, no attention) and is the one piece shared by the CPU oracle's tests and the HIP path's
tests and benchmark.  NumPy only; nothing here touches the GPU.

The tensors stand in for the per-head query/key/value activations of a video Diffusion
Transformer whose tokens are the flattened (t, h, w) latent grid (paper, Sec. 1 and the
experimental setup: 720p, 81 or 129 frames).  Each of Q and K is the sum of three terms:

* a *region prototype*: the grid is cut into Voronoi regions around random seed points and every
  token carries its region's prototype vector, pushed through a random linear map that differs
  between Q and K (so Q and K share cluster structure without being equal);
* a smooth *positional* term: random Fourier features of the normalised 3-D position through a
  random projection;
* i.i.d. Gaussian noise with standard deviation 0.3.

The sum is rescaled so that the average row-variance of the logits Q K^T / sqrt(d) equals 9
("std about 3"), using the trace identity of the paper's appendix (variance computation, the boxed
average row-wise variance) rewritten on Q and K directly.  V is i.i.d. N(0, 1).  Values are
rounded once to the configuration's dtype (bf16 or fp32) and returned as float32 arrays holding
exactly those values, so that both consumers see identical numbers.
"""
from __future__ import annotations

import dataclasses
import math
import threading
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 18636 * 1000


@dataclasses.dataclass(frozen=True)
class Config:
    """One workload.  ``grid`` is (T, H, W); ``n_seeds`` the number of Voronoi regions."""

    name: str
    cfg_id: int
    heads: int
    d: int
    grid: Tuple[int, int, int]
    n_seeds: int
    kq: int
    kk: int
    iters: int
    dtype: str  # "bf16" | "f32"
    keep: float
    n_layers: int = 1
    keep_range: Optional[Tuple[float, float]] = None
    keep_sweep: Optional[Tuple[float, ...]] = None
    dirichlet_alpha: Optional[float] = None

    @property
    def n(self) -> int:
        t, h, w = self.grid
        return t * h * w


CONFIGS: Dict[int, Config] = {
    0: Config("tiny_fp32", 0, 1, 64, (4, 16, 16), 16, 16, 16, 5, "f32", 0.3),
    1: Config("wan1.3b_480p", 1, 12, 128, (21, 30, 52), 128, 128, 128, 3, "bf16", 0.2),
    2: Config("wan1.3b_720p", 2, 12, 128, (21, 45, 80), 256, 256, 256, 3, "bf16", 0.2,
              n_layers=30, keep_range=(0.08, 0.45)),
    3: Config("wide_14b_720p", 3, 40, 128, (21, 45, 80), 256, 256, 256, 3, "bf16", 0.2,
              keep_sweep=(0.1, 0.2, 0.4, 1.0)),
    4: Config("long_seq_skewed", 4, 24, 128, (33, 45, 80), 384, 512, 512, 3, "bf16", 0.15,
              dirichlet_alpha=0.3),
    # not a BASELINE workload: the hyper-parameters of the paper's own experiments (Sec. 5.1
    # "Implementations": K_q = 256, K_k = 1024, two co-clustering iterations) on the 720p grid
    5: Config("paper_hparams_720p", 5, 12, 128, (21, 45, 80), 256, 256, 1024, 2, "bf16", 0.2),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result is float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    u = (u + bias) & np.uint32(0xFFFF0000)  # finite inputs well below the float32 maximum: no wrap-around
    return u.view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable (uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    assert not np.any(u & 0xFFFF), "values are not bf16-representable"
    return (u >> 16).astype(np.uint16).reshape(x.shape)


def layer_seed(cfg_id: int, layer: int) -> int:
    return BASE_SEED + 100 * cfg_id + layer


def layer_keeps(cfg: Config) -> np.ndarray:
    """Per-layer keep ratios (float32).  A sweep config draws them uniformly from its range."""
    if cfg.keep_range is None:
        return np.full(cfg.n_layers, cfg.keep, dtype=np.float32)
    rng = np.random.default_rng([layer_seed(cfg.cfg_id, 0), 777])
    lo, hi = cfg.keep_range
    return rng.uniform(lo, hi, size=cfg.n_layers).astype(np.float32)


# Heads may be drawn by several threads at once (make_layer), and the draw must not depend on that.  A
# BLAS product of a tall matrix does: OpenBLAS splits the rows among however many of its workers are
# free at that moment, rows that fall into a remainder panel are summed in another order (differences
# of a few 1e-14), and the single rounding to bf16 turns some of those into different inputs.  So the
# tall products (N rows, inner dimension 3, 16 or d) are written as a fixed-order sum of rank-1 terms
# (`_rowmix`), and only the two d x d Gram matrices of the scale computation go through BLAS, whose
# reduction over the N rows is done by one thread per output element in a fixed blocking (`_mm`; the
# lock keeps concurrent callers from sharing the worker pool all the same).
_MATMUL_LOCK = threading.Lock()


def _mm(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    with _MATMUL_LOCK:
        return a @ b


def _rowmix(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """a @ b for a tall a [N, c] and a small inner dimension c, as sum_c a[:, c] b[c] added in index order:
    every row is computed the same way whatever else runs at the same time."""
    out = a[:, 0:1] * b[0]
    for c in range(1, a.shape[1]):
        out += a[:, c:c + 1] * b[c]
    return out


def grid_positions(grid: Tuple[int, int, int]) -> np.ndarray:
    """Normalised (t, h, w) position of every token, token index = (t*H + h)*W + w."""
    t, h, w = grid
    tt, hh, ww = np.meshgrid(np.arange(t), np.arange(h), np.arange(w), indexing="ij")
    u = np.stack([tt.ravel() / max(t - 1, 1), hh.ravel() / max(h - 1, 1),
                  ww.ravel() / max(w - 1, 1)], axis=1)
    return u.astype(np.float64)


def voronoi_regions(u: np.ndarray, seeds: np.ndarray, weights: Optional[np.ndarray]) -> np.ndarray:
    """Region id of every position: nearest seed, lowest id on ties.

    With ``weights`` the squared distance to seed s is divided by (S*weights[s] + 1e-9)^(2/3) so
    that a region's volume grows roughly in proportion to its weight (skewed region sizes).
    """
    n, s = u.shape[0], seeds.shape[0]
    out = np.empty(n, dtype=np.int64)
    step = 16384
    denom = None
    if weights is not None:
        denom = (s * weights + 1e-9) ** (2.0 / 3.0)
    for a in range(0, n, step):
        ua = u[a:a + step]
        d2 = np.zeros((ua.shape[0], s))
        for c in range(3):
            diff = ua[:, c:c + 1] - seeds[None, :, c]
            d2 += diff * diff
        if denom is not None:
            d2 /= denom[None, :]
        out[a:a + step] = np.argmin(d2, axis=1)
    return out


def logit_row_variance(q: np.ndarray, k: np.ndarray) -> float:
    """Mean over query rows of the variance (over keys) of q_i . k_j / sqrt(d), in O(N d^2).

    Equals (1/d) * tr(Sigma_K * Q^T Q / N) with Sigma_K the (biased) sample covariance of the key
    rows: the paper's boxed average row-wise variance with x_i M replaced by q_i and X by K.
    """
    n, d = q.shape
    mu = k.mean(axis=0, keepdims=True)
    kc = k - mu
    sigma_k = _mm(kc.T, kc) / k.shape[0]
    gram_q = _mm(q.T, q) / n
    return float(np.trace(_mm(sigma_k, gram_q)) / d)


def sample_distinct(rng: np.random.Generator, n: int, k: int) -> np.ndarray:
    """k distinct indices in [0, n) by a partial Fisher-Yates shuffle (int32)."""
    idx = np.arange(n, dtype=np.int64)
    for i in range(k):
        j = int(rng.integers(i, n))
        idx[i], idx[j] = idx[j], idx[i]
    return idx[:k].astype(np.int32)


def make_head(cfg: Config, layer: int, head: int, grid: Optional[Tuple[int, int, int]] = None,
              n_seeds: Optional[int] = None, kq: Optional[int] = None, kk: Optional[int] = None,
              d: Optional[int] = None, dtype: Optional[str] = None) -> Dict[str, np.ndarray]:
    """Q, K, V and initial anchor indices of one head.  Overrides shrink a config for tests."""
    grid = grid or cfg.grid
    d = d or cfg.d
    n_seeds = n_seeds or cfg.n_seeds
    kq = kq or cfg.kq
    kk = kk or cfg.kk
    dtype = dtype or cfg.dtype
    rng = np.random.default_rng([layer_seed(cfg.cfg_id, layer), head])
    u = grid_positions(grid)
    n = u.shape[0]
    seeds = rng.uniform(0.0, 1.0, size=(n_seeds, 3))
    weights = None
    if cfg.dirichlet_alpha is not None:
        weights = rng.dirichlet(np.full(n_seeds, cfg.dirichlet_alpha))
    region = voronoi_regions(u, seeds, weights)
    z = rng.standard_normal((n_seeds, d))
    m_q = rng.standard_normal((d, d)) / math.sqrt(d)
    m_k = rng.standard_normal((d, d)) / math.sqrt(d)
    freqs = rng.standard_normal((8, 3)) * 2.0
    f_q = rng.standard_normal((16, d)) / 4.0
    f_k = rng.standard_normal((16, d)) / 4.0
    ang = 2.0 * math.pi * _rowmix(u, freqs.T)
    phi = np.concatenate([np.sin(ang), np.cos(ang)], axis=1)
    q = _rowmix(z, m_q)[region] + _rowmix(phi, f_q) + 0.3 * rng.standard_normal((n, d))
    k = _rowmix(z, m_k)[region] + _rowmix(phi, f_k) + 0.3 * rng.standard_normal((n, d))
    v = rng.standard_normal((n, d))
    var = logit_row_variance(q, k)
    gamma = (9.0 / var) ** 0.25
    q *= gamma
    k *= gamma
    init_q = sample_distinct(rng, n, kq)
    init_k = sample_distinct(rng, n, kk)
    q32, k32, v32 = (a.astype(np.float32) for a in (q, k, v))
    if dtype == "bf16":
        q32, k32, v32 = round_to_bf16(q32), round_to_bf16(k32), round_to_bf16(v32)
    elif dtype != "f32":
        raise ValueError(dtype)
    return {"q": q32, "k": k32, "v": v32, "init_q_idx": init_q, "init_k_idx": init_k,
            "region": region.astype(np.int32)}


def make_layer(cfg: Config, layer: int = 0, heads: Optional[List[int]] = None, workers: int = 1,
               **overrides) -> Dict[str, np.ndarray]:
    """Stack ``make_head`` over heads: q/k/v [BH, N, d] float32, init_*_idx [BH, K] int32.
    ``workers`` > 1 draws the heads in a thread pool (every head has its own generator state)."""
    heads = list(range(cfg.heads)) if heads is None else list(heads)
    if workers > 1 and len(heads) > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as pool:
            parts = list(pool.map(lambda h: make_head(cfg, layer, h, **overrides), heads))
    else:
        parts = [make_head(cfg, layer, h, **overrides) for h in heads]
    out = {key: np.stack([p[key] for p in parts], axis=0) for key in parts[0]}
    out["keep"] = np.full(len(heads), layer_keeps(cfg)[layer % cfg.n_layers], dtype=np.float32)
    return out
