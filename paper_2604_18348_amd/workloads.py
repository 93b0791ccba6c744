"""Seeded synthetic Q/K/V generators for the five benchmark configurations.

This module holds none of the method's arithmetic: it only draws inputs.  The
tests feed the same arrays to the CPU oracle and to the HIP library.  Real DiT
activations (the paper's HunyuanVideo / Wan / CogVideoX runs) are not available
offline; these mixtures stand in for them with the paper's shapes (token counts
of the resolution table, 64/128-wide heads, 65 query clusters, hundreds of key
clusters).

Recipe per head (component = a spatio-temporal Voronoi blob of the video grid):
  * M sites drawn uniformly in the (T,H,W) box; a token's component is its
    nearest site (ties to the lowest id); extra text tokens get 8 components of
    their own, assigned round-robin.
  * Q and K means per component are independent draws: N(0,I_d), or, for the
    "lognormal-norm" configs, r*sqrt(d)*u with u uniform on the sphere and
    r ~ LogNormal(0, 0.5).
  * token = mean[component] + sigma * N(0,I);  a Bernoulli fraction of tokens is
    replaced by isotropic N(0,I) outliers;  V ~ N(0,1).
  * "diffuse" heads are pure N(0,I) (no structure); "near-isotropic" heads use
    sigma = 1 and means scaled by 0.25.
Random numbers come from numpy's counter-based Philox generator keyed by
(seed, head, tensor), so any head can be generated on its own.
"""
from __future__ import annotations

import numpy as np
from scipy.spatial import cKDTree

# run parameters mirror the fields of the C params struct
CONFIGS = {
    "c1": dict(dtype="f32", H=1, grid=(16, 16, 16), text=0, d=64, M=32, sigma=0.3,
               outlier=0.0, lognorm=False, diffuse_heads=(), neariso_heads=(), seed=0,
               params=dict(q_clusters=32, q_iters=3, k_iters=3, k_m0=16, k_m_min=4,
                           k_max_clusters=128, k_max_stages=10, tau_abs=0.0, tau_factor=1.5,
                           min_unassigned_frac=0.0, score_mode=0, select_mode=0, topk=8,
                           top_p=0.9)),
    "c2": dict(dtype="bf16", H=30, grid=(13, 30, 45), text=226, d=64, M=256, sigma=0.3,
               outlier=0.02, lognorm=False, diffuse_heads=tuple(range(24, 30)),
               neariso_heads=(), seed=2000,
               params=dict(q_clusters=65, q_iters=3, k_iters=3, k_m0=128, k_m_min=16,
                           k_max_clusters=512, k_max_stages=10, tau_abs=0.0, tau_factor=1.5,
                           min_unassigned_frac=0.03, score_mode=0, select_mode=0, topk=64,
                           top_p=0.9)),
    "c3": dict(dtype="bf16", H=12, grid=(21, 30, 52), text=0, d=128, M=512, sigma=0.3,
               outlier=0.0, lognorm=True, diffuse_heads=(), neariso_heads=(), seed=3000,
               params=dict(q_clusters=65, q_iters=3, k_iters=3, k_m0=256, k_m_min=16,
                           k_max_clusters=1024, k_max_stages=10, tau_abs=0.0, tau_factor=1.5,
                           min_unassigned_frac=0.03, score_mode=0, select_mode=1, topk=64,
                           top_p=0.9)),
    "c4": dict(dtype="bf16", H=30, grid=(21, 45, 80), text=0, d=64, M=1024, sigma=(0.2, 0.6),
               outlier=0.02, lognorm=False, diffuse_heads=(), neariso_heads=(), seed=4000,
               params=dict(q_clusters=65, q_iters=3, k_iters=3, k_m0=512, k_m_min=16,
                           k_max_clusters=2048, k_max_stages=10, tau_abs=0.0, tau_factor=1.5,
                           min_unassigned_frac=0.03, score_mode=0, select_mode=0, topk=64,
                           top_p=0.9)),
    "c5": dict(dtype="bf16", H=24, grid=(50, 45, 80), text=0, d=128, M=2048, sigma=0.3,
               outlier=0.0, lognorm=True, diffuse_heads=(), neariso_heads=tuple(range(16, 24)),
               seed=5000,
               params=dict(q_clusters=65, q_iters=3, k_iters=3, k_m0=1024, k_m_min=16,
                           k_max_clusters=4096, k_max_stages=10, tau_abs=0.0, tau_factor=1.5,
                           min_unassigned_frac=0.03, score_mode=0, select_mode=0, topk=64,
                           top_p=0.9)),
}


def n_tokens(cfg):
    t, h, w = cfg["grid"]
    return t * h * w + cfg["text"]


def round_bf16_f32(a):
    """float32 array -> float32 array holding bfloat16-representable values (RNE)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _rng(seed, head, tensor):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(head) * 16 + int(tensor)]))


def _components(cfg, head, M):
    t, h, w = cfg["grid"]
    g = _rng(cfg["seed"], head, 0)
    sites = g.random((M, 3)) * np.array([t, h, w], dtype=np.float64)
    tt, hh, ww = np.meshgrid(np.arange(t), np.arange(h), np.arange(w), indexing="ij")
    pts = np.stack([tt.ravel(), hh.ravel(), ww.ravel()], axis=1).astype(np.float64) + 0.5
    _, comp = cKDTree(sites).query(pts, k=1)
    comp = comp.astype(np.int64)
    if cfg["text"]:
        comp = np.concatenate([comp, M + (np.arange(cfg["text"]) % 8)])
    return comp


def _means(cfg, g, n_comp, d, scale):
    if cfg["lognorm"]:
        u = g.standard_normal((n_comp, d))
        u /= np.linalg.norm(u, axis=1, keepdims=True)
        r = np.exp(0.5 * g.standard_normal(n_comp))
        mu = r[:, None] * np.sqrt(d) * u
    else:
        mu = g.standard_normal((n_comp, d))
    return (scale * mu).astype(np.float32)


def make_head(cfg, head, M=None, aligned=False):
    """Q, K, V float32 [N,d] of one head (bf16 configs: already bf16-rounded).  aligned: the queries of a
    component are drawn around the KEY mean of that component, so that attention concentrates on the
    component's own keys (the default draws the two means independently: diffuse attention)."""
    d = cfg["d"]
    N = n_tokens(cfg)
    M = int(M if M is not None else cfg["M"])
    if head in cfg["diffuse_heads"]:
        Q = _rng(cfg["seed"], head, 1).standard_normal((N, d), dtype=np.float32)
        K = _rng(cfg["seed"], head, 2).standard_normal((N, d), dtype=np.float32)
    else:
        comp = _components(cfg, head, M)
        n_comp = M + (8 if cfg["text"] else 0)
        gm = _rng(cfg["seed"], head, 4)
        near = head in cfg["neariso_heads"]
        mscale = 0.25 if near else 1.0
        sig = cfg["sigma"]
        if isinstance(sig, tuple):
            sig = float(sig[0] + (sig[1] - sig[0]) * gm.random())
        if near:
            sig = 1.0
        muq = _means(cfg, gm, n_comp, d, mscale)
        muk = _means(cfg, gm, n_comp, d, mscale)
        if aligned:
            muq = muk
        Q = muq[comp] + np.float32(sig) * _rng(cfg["seed"], head, 1).standard_normal((N, d), dtype=np.float32)
        K = muk[comp] + np.float32(sig) * _rng(cfg["seed"], head, 2).standard_normal((N, d), dtype=np.float32)
        if cfg["outlier"] > 0:
            go = _rng(cfg["seed"], head, 5)
            oq = go.random(N) < cfg["outlier"]
            ok = go.random(N) < cfg["outlier"]
            Q[oq] = go.standard_normal((int(oq.sum()), d), dtype=np.float32)
            K[ok] = go.standard_normal((int(ok.sum()), d), dtype=np.float32)
    V = _rng(cfg["seed"], head, 3).standard_normal((N, d), dtype=np.float32)
    if cfg["dtype"] == "bf16":
        Q, K, V = round_bf16_f32(Q), round_bf16_f32(K), round_bf16_f32(V)
    return Q, K, V


def make_qkv(name, heads=None):
    """Q, K, V float32 [H',N,d] for config `name` (optionally a subset of heads)."""
    cfg = CONFIGS[name]
    hs = list(range(cfg["H"])) if heads is None else list(heads)
    N, d = n_tokens(cfg), cfg["d"]
    Q = np.empty((len(hs), N, d), dtype=np.float32)
    K = np.empty_like(Q)
    V = np.empty_like(Q)
    for i, h in enumerate(hs):
        Q[i], K[i], V[i] = make_head(cfg, h)
    return Q, K, V


def make_small(seed, N, d, M, sigma=0.3, dtype="f32", H=1, grid=None):
    """A small mixture with the same recipe, for tests at sizes the oracle finishes fast."""
    if grid is None:
        t = max(1, int(round(N ** (1 / 3))))
        h = max(1, int(round((N / t) ** 0.5)))
        w = max(1, N // (t * h))
        grid = (t, h, w)
    text = N - grid[0] * grid[1] * grid[2]
    assert text >= 0
    cfg = dict(dtype=dtype, H=H, grid=grid, text=text, d=d, M=M, sigma=sigma, outlier=0.0,
               lognorm=False, diffuse_heads=(), neariso_heads=(), seed=seed)
    Q = np.empty((H, N, d), dtype=np.float32)
    K = np.empty_like(Q)
    V = np.empty_like(Q)
    for h in range(H):
        Q[h], K[h], V[h] = make_head(cfg, h)
    return Q, K, V
