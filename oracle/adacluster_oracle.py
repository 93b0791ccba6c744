"""CPU oracle for the AdaCluster clustered sparse-attention call.

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, fp64 numpy statement of
what the attention-layer replacement of the paper computes (Algorithm 3:
query clustering, Algorithm 1 multi-stage key clustering, Algorithm 2 / Eq. 1-2
cluster scores, arg-top-k selection, attention over the selected clusters).
Only the tests, the smoke check and the benchmark's cpu_baseline leg may import
it; the product path never does, and this file imports nothing from the
product.  It shares no code, table or helper with the HIP kernels.

Every function follows the algorithm's steps in the paper's order; there is no
blocking, fusion or reordering.  All arithmetic is IEEE double precision.

Pins (tests/test_oracle_*.py): brute-force dense softmax attention and its
closed forms, select-all == dense, argmin / member-mean invariants recomputed
by explicit loops, the structural invariants of Algorithm 1, Eq. 1 written as
loops against its GEMM form, brute-force sorting for the selections, and one
eight-token call of the whole algorithm worked out by hand
(tests/test_oracle_hand_worked.py).
The end-to-end numbers of the whole call have no printed example in the paper:
they are pinned only through those properties and that hand calculation
("parity unpinned by a worked example of the paper's").

Conventions used where the paper is silent (each is a stated reading):
  * k-means: deterministic strided initialisation over the current point list,
    a fixed number of assignment passes, ties to the lowest centre index,
    empty clusters keep their previous centre.
  * A Lloyd run with `n_iters` passes does: assign, update, assign, update, ...,
    assign.  It returns the centres used by the LAST assignment (so that every
    label is exactly the arg-min / arg-max to a returned centre).
  * `round_fn`, if given, is applied to the centres before every assignment
    (the HIP path stores assignment centres in the I/O dtype); None = exact.
"""
from __future__ import annotations

import math
import numpy as np

F64 = np.float64
NEG_INF = -np.inf


# --------------------------------------------------------------------------
# small helpers
# --------------------------------------------------------------------------
def round_to_bf16(x):
    """Round to the nearest bfloat16 (ties to even), result held in float64.

    Done as float64 -> float32 (numpy, RNE) -> keep the top 16 bits with RNE on
    the dropped half, which is what a device converting its fp32 centre does.
    """
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    u = (u + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = u.astype(np.uint32).view(np.float32)
    return out.astype(F64).reshape(np.shape(x))


def normalize_rows(X, eps=1e-12):
    """x / max(||x||_2, eps) per row (Sec. 3.1: queries are put on the unit sphere)."""
    X = np.asarray(X, dtype=F64)
    n = np.sqrt(np.sum(X * X, axis=1))
    return X / np.maximum(n, eps)[:, None]


def strided_indices(n, m):
    """Deterministic initial sample: index floor((j + 1/2) * n / m), j = 0..m-1."""
    j = np.arange(m, dtype=np.int64)
    return ((2 * j + 1) * int(n)) // (2 * int(m))


# --------------------------------------------------------------------------
# dense attention (the plain definition everything reduces to)
# --------------------------------------------------------------------------
def dense_attention(Q, K, V, scale=None):
    """softmax(scale * Q K^T) V for one head, Q [Nq,d], K,V [Nk,d]."""
    Q = np.asarray(Q, dtype=F64)
    K = np.asarray(K, dtype=F64)
    V = np.asarray(V, dtype=F64)
    if scale is None:
        scale = 1.0 / math.sqrt(Q.shape[1])
    S = scale * (Q @ K.T)
    S = S - S.max(axis=1, keepdims=True)
    P = np.exp(S)
    return (P @ V) / P.sum(axis=1, keepdims=True)


# --------------------------------------------------------------------------
# query clustering: k-means on normalised queries (Alg. 3 line 1, Sec. 3.1)
# --------------------------------------------------------------------------
def _spherical_update(Xn, labels, C_old):
    C = C_old.copy()
    m = C_old.shape[0]
    sizes = np.bincount(labels, minlength=m)
    for j in range(m):
        if sizes[j] == 0:
            continue
        s = Xn[labels == j].sum(axis=0)
        nrm = math.sqrt(float(s @ s))
        if nrm < 1e-12:
            continue
        C[j] = s / nrm
    return C, sizes


def query_kmeans(Q, n_clusters, n_iters, init_centroids=None, round_fn=None, normalize=True):
    """Clustering of the queries (Sec. 3.1; Alg. 3 line 1: KMeans(Normalize(Q))).

    normalize=True (the method): points are the unit-normalised queries; label =
    arg-max cosine to a unit centre; update = re-normalised member sum.
    normalize=False (the "w/o Norm" row of the component ablation): the same Lloyd
    iterations as `euclid_kmeans` on the raw queries, centres = member means.
    Returns a dict with
      labels            int64 [N]
      assign_centroids  [Cq,d]  centres the labels are the arg-max (arg-min) of
      centroids         [Cq,d]  normalised member means (member means) under `labels`
      sizes             int64 [Cq]
      mean_norm         [Cq]    mean ||q|| of the members (1 without normalisation; 0 when empty)
    """
    Q = np.asarray(Q, dtype=F64)
    N = Q.shape[0]
    if not normalize:
        if init_centroids is None:
            C = Q[strided_indices(N, n_clusters)].copy()
        else:
            C = np.asarray(init_centroids, dtype=F64).copy()
        labels = None
        Ca = C
        for it in range(n_iters):
            Ca = round_fn(C) if round_fn is not None else C
            labels = euclid_assign(Q, Ca)
            if it < n_iters - 1:
                C, _ = _mean_update(Q, labels, C)
        cent, sizes = _mean_update(Q, labels, C)
        return dict(labels=labels.astype(np.int64), assign_centroids=Ca.copy(), centroids=cent,
                    sizes=sizes.astype(np.int64), mean_norm=(sizes > 0).astype(F64))
    Xn = normalize_rows(Q)
    if init_centroids is None:
        C = Xn[strided_indices(N, n_clusters)].copy()
    else:
        C = np.asarray(init_centroids, dtype=F64).copy()
    labels = None
    Ca = C
    for it in range(n_iters):
        Ca = round_fn(C) if round_fn is not None else C
        labels = np.argmax(Xn @ Ca.T, axis=1)
        if it < n_iters - 1:
            C, _ = _spherical_update(Xn, labels, C)
    cent, sizes = _spherical_update(Xn, labels, C)
    qn = np.sqrt(np.sum(Q * Q, axis=1))
    mean_norm = np.zeros(n_clusters, dtype=F64)
    for j in range(n_clusters):
        if sizes[j] > 0:
            mean_norm[j] = qn[labels == j].mean()
    return dict(labels=labels.astype(np.int64), assign_centroids=Ca.copy(),
                centroids=cent, sizes=sizes.astype(np.int64), mean_norm=mean_norm)


# --------------------------------------------------------------------------
# Euclidean k-means (the KMeans(U, m_t) call inside Alg. 1)
# --------------------------------------------------------------------------
def euclid_assign(X, C):
    """labels = arg-min_j ||x - c_j||^2, evaluated as ||c_j||^2 - 2 x.c_j (ties lowest j)."""
    cn = np.sum(C * C, axis=1)
    G = cn[None, :] - 2.0 * (X @ C.T)
    return np.argmin(G, axis=1)


def _mean_update(X, labels, C_old):
    C = C_old.copy()
    m = C_old.shape[0]
    sizes = np.bincount(labels, minlength=m)
    for j in range(m):
        if sizes[j] > 0:
            C[j] = X[labels == j].mean(axis=0)
    return C, sizes


def euclid_kmeans(X, m, n_iters, init_centroids=None, round_fn=None):
    """Lloyd iterations on the rows of X with m centres.

    Returns (labels, centres used by the last assignment, squared distance of
    every row to its assigned centre)."""
    X = np.asarray(X, dtype=F64)
    n = X.shape[0]
    if init_centroids is None:
        C = X[strided_indices(n, m)].copy()
    else:
        C = np.asarray(init_centroids, dtype=F64).copy()
    Ca = C
    labels = None
    for it in range(n_iters):
        Ca = round_fn(C) if round_fn is not None else C
        labels = euclid_assign(X, Ca)
        if it < n_iters - 1:
            C, _ = _mean_update(X, labels, C)
    diff = X - Ca[labels]
    d2 = np.sum(diff * diff, axis=1)
    return labels.astype(np.int64), Ca.copy(), d2


# --------------------------------------------------------------------------
# Algorithm 1: multi-stage (threshold-wise adaptive) k-means on the keys
# --------------------------------------------------------------------------
def stage_cluster_count(n_unassigned, n_total, m0, m_min):
    """m_t: m0 at the first stage, shrinking with the unassigned share afterwards."""
    m = -((-int(m0) * int(n_unassigned)) // int(n_total))      # ceil(m0*|U|/N)
    m = max(int(m_min), min(int(m0), m))
    return min(int(n_unassigned), m)


def min_unassigned_count(frac, n_total):
    """Largest |U| at which staging stops early: floor(float32(frac) * N)."""
    return int(math.floor(float(np.float32(frac)) * int(n_total)))


def stage0_distances(K, m0, n_iters, round_fn=None):
    """Token-to-centre distances of the first stage (used to set tau, Sec. 4.1)."""
    K = np.asarray(K, dtype=F64)
    m = stage_cluster_count(K.shape[0], K.shape[0], m0, 1)
    _, _, d2 = euclid_kmeans(K, m, n_iters, round_fn=round_fn)
    return np.sqrt(d2)


def tau_from_factor(K_heads, tau_factor, m0, n_iters, round_fn=None):
    """tau = factor x mean distance over all heads and tokens after stage 0."""
    tot = 0.0
    cnt = 0
    for K in K_heads:
        d = stage0_distances(K, m0, n_iters, round_fn)
        tot += float(d.sum())
        cnt += d.shape[0]
    return float(np.float32(tau_factor)) * tot / cnt


def multistage_kmeans(K, tau, n_max, m0, m_min=1, n_iters=3, max_stages=10,
                      min_unassigned_frac=0.0, round_fn=None):
    """Algorithm 1 for one head.

    Returns a dict:
      labels           final assignment: nearest centre among ALL stage centres
      assign_centroids [|C|,d] union of the stage centres, in stage order
      centroids        [|C|,d] member means under `labels` (empty -> stage centre)
      sizes            [|C|]
      box_min/box_max  [|C|,d] per-dimension member extremes (empty -> 0)
      full_flag        True iff the loop stopped on |C| >= n_max with U non-empty
      stage_offs       [stages+1] running centre count
      stage_of         [N] stage at which a token was removed (-1: never)
      n_unassigned     [stages+1] |U| entering each stage, last = what is left
    """
    K = np.asarray(K, dtype=F64)
    N, d = K.shape
    tau2 = float(tau) * float(tau)
    u_min = min_unassigned_count(min_unassigned_frac, N)
    U = np.arange(N, dtype=np.int64)
    stage_c = []
    stage_offs = [0]
    n_un = [N]
    stage_of = np.full(N, -1, dtype=np.int64)
    full = False
    t = 0
    n_c = 0
    while U.size > 0:
        if n_c >= n_max:
            full = True
            break
        if t >= max_stages or U.size <= u_min:
            break
        m_t = stage_cluster_count(U.size, N, m0, m_min)
        _, C_t, d2 = euclid_kmeans(K[U], m_t, n_iters, round_fn=round_fn)
        removed = d2 < tau2
        stage_of[U[removed]] = t
        U = U[~removed]
        stage_c.append(C_t)
        n_c += m_t
        stage_offs.append(n_c)
        n_un.append(int(U.size))
        t += 1
    C = np.concatenate(stage_c, axis=0) if stage_c else np.zeros((0, d))
    labels = euclid_assign(K, C).astype(np.int64)
    cent, sizes = _mean_update(K, labels, C)
    bmin = np.zeros_like(C)
    bmax = np.zeros_like(C)
    for j in range(C.shape[0]):
        if sizes[j] > 0:
            mem = K[labels == j]
            bmin[j] = mem.min(axis=0)
            bmax[j] = mem.max(axis=0)
    return dict(labels=labels, assign_centroids=C, centroids=cent,
                sizes=sizes.astype(np.int64), box_min=bmin, box_max=bmax,
                full_flag=bool(full), stage_offs=np.asarray(stage_offs, dtype=np.int64),
                stage_of=stage_of, n_unassigned=np.asarray(n_un, dtype=np.int64))


def warm_key_clustering(K, prev_centroids, n_iters, round_fn=None):
    """Later denoising steps (Sec. 3.2.2, "Efficient initialization"): the number of clusters is
    fixed, the previous step's centres initialise k-means, `n_iters` assignment passes are run.
    Returns the same fields as multistage_kmeans (one stage, nothing staged)."""
    K = np.asarray(K, dtype=F64)
    prev = np.asarray(prev_centroids, dtype=F64)
    labels, Ca, _ = euclid_kmeans(K, prev.shape[0], n_iters, init_centroids=prev, round_fn=round_fn)
    cent, sizes, bmin, bmax = finalize_key_clusters(K, labels, Ca)
    return dict(labels=labels, assign_centroids=Ca, centroids=cent, sizes=sizes, box_min=bmin, box_max=bmax)


def finalize_key_clusters(K, labels, assign_centroids):
    """Member means, sizes and boxes for given labels (second half of Alg. 1's output)."""
    K = np.asarray(K, dtype=F64)
    C = np.asarray(assign_centroids, dtype=F64)
    cent, sizes = _mean_update(K, np.asarray(labels, dtype=np.int64), C)
    bmin = np.zeros_like(C)
    bmax = np.zeros_like(C)
    for j in range(C.shape[0]):
        if sizes[j] > 0:
            mem = K[labels == j]
            bmin[j] = mem.min(axis=0)
            bmax[j] = mem.max(axis=0)
    return cent, sizes.astype(np.int64), bmin, bmax


def compactness_mse(K, labels, centroids):
    """Mean squared reconstruction error of one head (Sec. 3.2.1): the mean over tokens of
    ||k - c(k)||^2, c(k) the centre of the token's cluster.  The layer score of the paper is
    Comp = 1 / (mean of this over the heads)."""
    K = np.asarray(K, dtype=F64)
    C = np.asarray(centroids, dtype=F64)
    lab = np.asarray(labels, dtype=np.int64)
    diff = K - C[lab]
    return float(np.mean(np.sum(diff * diff, axis=1)))


def compactness_score(mse_per_head):
    """Comp = 1 / mean_h MSE_h (Sec. 3.2.1)."""
    return 1.0 / float(np.mean(np.asarray(mse_per_head, dtype=F64)))


# --------------------------------------------------------------------------
# cluster scores (Eq. 1, Eq. 2 / Alg. 2, and the mean-based ablation)
# --------------------------------------------------------------------------
SCORE_TQ, SCORE_BOX, SCORE_DOT = 0, 1, 2


def _two_part_score(Qc, Rpos, Rneg):
    """matmul(Q+, Rpos^T) + matmul(Q-, Rneg^T) with the contraction summed in
    ascending dimension order, one rounded multiply and one rounded add per term
    (so that a device can reproduce every bit)."""
    Qc = np.asarray(Qc, dtype=F64)
    Qp = np.maximum(Qc, 0.0)
    Qm = np.minimum(Qc, 0.0)
    sp = np.zeros((Qc.shape[0], Rpos.shape[0]), dtype=F64)
    sn = np.zeros_like(sp)
    for dd in range(Qc.shape[1]):
        sp = sp + Qp[:, dd][:, None] * Rpos[:, dd][None, :]
        sn = sn + Qm[:, dd][:, None] * Rneg[:, dd][None, :]
    return sp + sn


def score_tensorquest(Qc, Kc):
    """Alg. 2 applied to centroids: Q+ (K+)^T + Q- (K-)^T."""
    Kc = np.asarray(Kc, dtype=F64)
    return _two_part_score(Qc, np.maximum(Kc, 0.0), np.minimum(Kc, 0.0))


def score_box(Qc, box_min, box_max):
    """Eq. 1 in GEMM form: Q+ (max K)^T + Q- (min K)^T over each cluster's box."""
    return _two_part_score(Qc, np.asarray(box_max, dtype=F64), np.asarray(box_min, dtype=F64))


def score_dot(Qc, Kc):
    """Mean-based score (the 'w/o Quest' ablation): plain centroid dot product."""
    Qc = np.asarray(Qc, dtype=F64)
    Kc = np.asarray(Kc, dtype=F64)
    s = np.zeros((Qc.shape[0], Kc.shape[0]), dtype=F64)
    for dd in range(Qc.shape[1]):
        s = s + Qc[:, dd][:, None] * Kc[:, dd][None, :]
    return s


def quest_upper_bound_loops(q, page):
    """Eq. 1 literally: sum_d max(q_d * max_i K_id, q_d * min_i K_id)."""
    q = np.asarray(q, dtype=F64)
    page = np.asarray(page, dtype=F64)
    tot = 0.0
    for dd in range(q.shape[0]):
        hi = max(page[i, dd] for i in range(page.shape[0]))
        lo = min(page[i, dd] for i in range(page.shape[0]))
        tot += max(q[dd] * hi, q[dd] * lo)
    return tot


def cluster_scores(mode, Qc, Kc, box_min, box_max, sizes):
    """Score matrix [Cq,Ck]; empty key clusters score -inf."""
    if mode == SCORE_TQ:
        S = score_tensorquest(Qc, Kc)
    elif mode == SCORE_BOX:
        S = score_box(Qc, box_min, box_max)
    elif mode == SCORE_DOT:
        S = score_dot(Qc, Kc)
    else:
        raise ValueError("score mode")
    S = S.copy()
    S[:, np.asarray(sizes) == 0] = NEG_INF
    return S


# --------------------------------------------------------------------------
# selection (Alg. 3 line 8: argtopk; plus the top-p budget of the benchmark)
# --------------------------------------------------------------------------
def select_topk(S, topk):
    """Per row: the min(topk, #finite) largest scores, ties to the lowest index,
    returned as ascending index lists."""
    out = []
    for i in range(S.shape[0]):
        row = S[i]
        valid = np.flatnonzero(row > NEG_INF)
        order = sorted(valid.tolist(), key=lambda j: (-row[j], j))
        out.append(np.asarray(sorted(order[:min(int(topk), len(order))]), dtype=np.int64))
    return out


_EXP_COEF = [1.0 / float(math.factorial(n)) for n in range(14)]
_LOG2E = 1.4426950408889634
_LN2_HI = 0.693147180369123816490
_LN2_LO = 1.90821492927058770002e-10


def exp_det(x):
    """exp(x) for x <= 0 from +,*,rint,ldexp only, every step separately rounded:
    k = rint(x*log2e); r = (x - k*ln2_hi) - k*ln2_lo; degree-13 Taylor polynomial
    by Horner; result scaled by 2^k.  Below -700 the result is 0."""
    x = np.asarray(x, dtype=F64)
    xs = np.where(x < -700.0, 0.0, x)
    k = np.rint(xs * _LOG2E)
    r = (xs - k * _LN2_HI) - k * _LN2_LO
    p = np.full_like(r, _EXP_COEF[13])
    for n in range(12, -1, -1):
        p = p * r + _EXP_COEF[n]
    out = np.ldexp(p, k.astype(np.int64))
    return np.where(x < -700.0, 0.0, out)


def select_topp(S, sizes, alpha, top_p):
    """Per row i: weights w_j = n_j * exp(alpha_i * (S_ij - max_j S_ij)); clusters
    sorted by w descending (ties lowest j); the shortest prefix whose running sum
    reaches float32(top_p) * total (total = sum in ascending j); at least one
    cluster; top_p >= 1 selects every non-empty cluster.  Ascending index lists."""
    sizes = np.asarray(sizes, dtype=np.int64)
    p = float(np.float32(top_p))
    out = []
    for i in range(S.shape[0]):
        row = S[i]
        valid = np.flatnonzero((row > NEG_INF) & (sizes > 0))
        if valid.size == 0:
            out.append(np.zeros(0, dtype=np.int64))
            continue
        if p >= 1.0:
            out.append(valid.astype(np.int64))
            continue
        mx = row[valid].max()
        a = float(alpha[i])
        w = np.zeros(row.shape[0], dtype=F64)
        w[valid] = sizes[valid].astype(F64) * exp_det(a * (row[valid] - mx))
        total = 0.0
        for j in range(row.shape[0]):
            total = total + w[j]
        order = sorted(valid.tolist(), key=lambda j: (-w[j], j))
        target = p * total
        cum = 0.0
        take = len(order)
        for r_, j in enumerate(order):
            cum = cum + w[j]
            if cum >= target:
                take = r_ + 1
                break
        out.append(np.asarray(sorted(order[:take]), dtype=np.int64))
    return out


# --------------------------------------------------------------------------
# attention over the selected clusters (Alg. 3 lines 9-10)
# --------------------------------------------------------------------------
def selection_matrix(sel_lists, n_kclusters):
    M = np.zeros((len(sel_lists), n_kclusters), dtype=bool)
    for i, s in enumerate(sel_lists):
        M[i, np.asarray(s, dtype=np.int64)] = True
    return M


def sparse_attention_mask(Q, K, V, q_labels, k_labels, sel_lists, scale=None, n_kclusters=None):
    """Definition by masking: query n attends key m iff the cluster of m is
    selected for the cluster of n.  O(N^2) memory: small inputs only."""
    Q = np.asarray(Q, dtype=F64)
    K = np.asarray(K, dtype=F64)
    V = np.asarray(V, dtype=F64)
    if scale is None:
        scale = 1.0 / math.sqrt(Q.shape[1])
    if n_kclusters is None:
        n_kclusters = int(np.max(k_labels)) + 1
        for s in sel_lists:
            if len(s):
                n_kclusters = max(n_kclusters, int(np.max(s)) + 1)
    n_kc = int(n_kclusters)
    M = selection_matrix(sel_lists, n_kc)
    allow = M[np.asarray(q_labels)][:, np.asarray(k_labels)]
    S = scale * (Q @ K.T)
    S = np.where(allow, S, NEG_INF)
    mx = S.max(axis=1, keepdims=True)
    mx = np.where(np.isfinite(mx), mx, 0.0)
    P = np.exp(S - mx)
    den = P.sum(axis=1, keepdims=True)
    O = P @ V
    return np.where(den > 0, O / np.where(den > 0, den, 1.0), 0.0)


def sparse_attention_gather(Q, K, V, q_labels, k_labels, sel_lists, scale=None, rows=None):
    """Same result by gathering K*, V* per query cluster (Alg. 3 line 9).  `rows`
    restricts the computation to a subset of query rows (others are left 0)."""
    Q = np.asarray(Q, dtype=F64)
    K = np.asarray(K, dtype=F64)
    V = np.asarray(V, dtype=F64)
    q_labels = np.asarray(q_labels)
    k_labels = np.asarray(k_labels)
    if scale is None:
        scale = 1.0 / math.sqrt(Q.shape[1])
    O = np.zeros((Q.shape[0], V.shape[1]), dtype=F64)
    row_mask = None
    if rows is not None:
        row_mask = np.zeros(Q.shape[0], dtype=bool)
        row_mask[np.asarray(rows)] = True
    order = np.argsort(k_labels, kind="stable")
    sorted_lab = k_labels[order]
    for i, sel in enumerate(sel_lists):
        qi = q_labels == i
        if row_mask is not None:
            qi = qi & row_mask
        qidx = np.flatnonzero(qi)
        if qidx.size == 0 or len(sel) == 0:
            continue
        sel = np.asarray(sel, dtype=np.int64)
        lo = np.searchsorted(sorted_lab, sel, side="left")
        hi = np.searchsorted(sorted_lab, sel, side="right")
        kidx = np.concatenate([order[a:b] for a, b in zip(lo, hi)]) if sel.size else np.zeros(0, int)
        if kidx.size == 0:
            continue
        O[qidx] = dense_attention(Q[qidx], K[kidx], V[kidx], scale)
    return O


# --------------------------------------------------------------------------
# Algorithm 3 end to end, all heads
# --------------------------------------------------------------------------
def adacluster_attention(Q, K, V, *, q_clusters, q_iters, k_iters, k_m0, k_m_min,
                         k_max_clusters, k_max_stages=10, tau_abs=0.0, tau_factor=1.5,
                         min_unassigned_frac=0.0, score_mode=SCORE_TQ, select_mode=0,
                         topk=64, top_p=0.9, softmax_scale=None, round_fn=None,
                         use_gather=False, q_no_norm=0):
    """Q,K,V [H,N,d].  Returns (O [H,N,d], per-head info list, tau)."""
    Q = np.asarray(Q, dtype=F64)
    K = np.asarray(K, dtype=F64)
    V = np.asarray(V, dtype=F64)
    H, N, d = Q.shape
    scale = softmax_scale if (softmax_scale is not None and softmax_scale > 0) else 1.0 / math.sqrt(d)
    if tau_abs > 0:
        tau = float(np.float32(tau_abs))
    else:
        tau = tau_from_factor(K, tau_factor, k_m0, k_iters, round_fn)
    O = np.zeros_like(Q)
    infos = []
    for h in range(H):
        qc = query_kmeans(Q[h], q_clusters, q_iters, round_fn=round_fn, normalize=not q_no_norm)
        kc = multistage_kmeans(K[h], tau, k_max_clusters, k_m0, k_m_min, k_iters,
                               k_max_stages, min_unassigned_frac, round_fn)
        if kc["full_flag"]:
            sel = None
            O[h] = dense_attention(Q[h], K[h], V[h], scale)
        else:
            S = cluster_scores(score_mode, qc["centroids"], kc["centroids"],
                               kc["box_min"], kc["box_max"], kc["sizes"])
            if select_mode == 0:
                sel = select_topk(S, topk)
            else:
                sel = select_topp(S, kc["sizes"], qc["mean_norm"] * scale, top_p)
            fn = sparse_attention_gather if use_gather else sparse_attention_mask
            O[h] = fn(Q[h], K[h], V[h], qc["labels"], kc["labels"], sel, scale)
        infos.append(dict(q=qc, k=kc, sel=sel))
    return O, infos, tau
