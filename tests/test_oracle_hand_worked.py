"""A whole call (Algorithm 3) small enough to work out with pencil and paper.

One head, eight tokens in two dimensions.  Every expected number below was derived by hand from the
algorithm's steps (the derivation is in the comments), not produced by the code under test, so a
mistake in how the oracle strings the steps together - the wrong centres fed to the scores, the
stage rule of Algorithm 1, the sign split of Eq. 2, the softmax scale, a selected cluster dropped -
changes one of them."""
import math

import numpy as np

from oracle import adacluster_oracle as orc

S2 = 1.0 / math.sqrt(2.0)

# Keys.  The strided initial sample of 8 points with 2 centres is rows 2 and 6.
K = np.array([[4, 0], [4, 2], [4, 1], [6, 1],            # right-hand group, row 2 seeds centre 0
              [-4, 0], [-4, 2], [-4, 1], [-12, 5]],      # left-hand group, row 6 seeds centre 1; row 7 is far out
             dtype=np.float64)
# Queries: unit directions (0.6,0.8), (0.8,0.6) and their mirror images, with norms 5, 10, 10, 5.
Q = np.array([[3, 4], [8, 6], [6, 8], [4, 3],
              [-3, 4], [-8, 6], [-6, 8], [-4, 3]], dtype=np.float64)
# Values mark the key cluster a row ends up in: cluster 0 -> (1,0), cluster 2 -> (0,1), cluster 1 -> (100,100).
V = np.array([[1, 0]] * 4 + [[100, 100]] * 3 + [[0, 1]], dtype=np.float64)

PARAMS = dict(q_clusters=2, q_iters=2, k_iters=2, k_m0=2, k_m_min=1, k_max_clusters=4, tau_abs=3.0,
              topk=2, softmax_scale=math.log(2.0) / 2.0)      # softmax weights become 2^(q.k/2)


def run(score_mode):
    O, info, tau = orc.adacluster_attention(Q[None], K[None], V[None], score_mode=score_mode, **PARAMS)
    assert tau == 3.0
    return O[0], info[0]


def test_key_clustering_by_hand():
    # Stage 0, pass 1: centres (4,1) and (-4,1) split the rows 0-3 | 4-7.  Means: (18/4, 4/4) = (4.5,1)
    # and (-24/4, 8/4) = (-6,2).  Pass 2 assigns to those; squared distances are
    # 1.25, 1.25, 0.25, 2.25 | 8, 4, 5, 45.  With tau = 3 (tau^2 = 9) only row 7 stays unassigned.
    # Stage 1: |U| = 1, m_1 = ceil(2*1/8) = 1; its centre is row 7 itself, distance 0, U is empty.
    _, info = run(orc.SCORE_TQ)
    k = info["k"]
    assert k["stage_offs"].tolist() == [0, 2, 3]
    assert k["n_unassigned"].tolist() == [8, 1, 0]
    assert k["stage_of"].tolist() == [0, 0, 0, 0, 0, 0, 0, 1]
    assert not k["full_flag"]
    assert np.array_equal(k["assign_centroids"], np.array([[4.5, 1], [-6, 2], [-12, 5]]))
    # Final labels: nearest of the three stage centres.  Rows 4-6 are 8, 4, 5 from (-6,2) and >= 73 from
    # (-12,5).  The reported centroids are the member means: (-4,1) for cluster 1, not the stage centre.
    assert k["labels"].tolist() == [0, 0, 0, 0, 1, 1, 1, 2]
    assert k["sizes"].tolist() == [4, 3, 1]
    assert np.array_equal(k["centroids"], np.array([[4.5, 1], [-4, 1], [-12, 5]]))
    assert np.array_equal(k["box_min"], np.array([[4, 0], [-4, 0], [-12, 5]]))
    assert np.array_equal(k["box_max"], np.array([[6, 2], [-4, 2], [-12, 5]]))


def test_query_clustering_by_hand():
    # Seeds are the directions of rows 2 and 6: (0.6,0.8) and (-0.6,0.8).  cos((0.8,0.6),(0.6,0.8)) = 0.96
    # against 0 for the mirrored seed, so rows 0-3 | 4-7.  Member sums (2.8,2.8) and (-2.8,2.8) normalise to
    # (1,1)/sqrt2 and (-1,1)/sqrt2; the second pass changes nothing.  Mean norms (5+10+10+5)/4 = 7.5.
    _, info = run(orc.SCORE_TQ)
    q = info["q"]
    assert q["labels"].tolist() == [0, 0, 0, 0, 1, 1, 1, 1]
    assert np.allclose(q["centroids"], [[S2, S2], [-S2, S2]], atol=1e-14)
    assert np.allclose(q["mean_norm"], [7.5, 7.5], atol=1e-14)
    assert q["sizes"].tolist() == [4, 4]


def test_scores_and_selection_by_hand():
    # Eq. 2 on the centroids, q_A = (s,s), q_B = (-s,s), s = 1/sqrt2; K+ = max(K,0), K- = min(K,0):
    #   c0 = (4.5,1): A: s(4.5+1) = 5.5s          B: s*1 + (-s)*0    = s
    #   c1 = (-4,1):  A: s(0+1)   = s             B: s*1 + (-s)(-4)  = 5s
    #   c2 = (-12,5): A: s(0+5)   = 5s            B: s*5 + (-s)(-12) = 17s
    _, info = run(orc.SCORE_TQ)
    S = orc.cluster_scores(orc.SCORE_TQ, info["q"]["centroids"], info["k"]["centroids"], None, None,
                           info["k"]["sizes"])
    assert np.allclose(S, S2 * np.array([[5.5, 1, 5], [1, 5, 17]]), atol=1e-13)
    assert [s.tolist() for s in info["sel"]] == [[0, 2], [1, 2]]
    # Plain centroid products: A: 5.5s, (-4+1)s, (-12+5)s -> {0,1};  B: -3.5s, 5s, 17s -> {1,2}.
    _, info = run(orc.SCORE_DOT)
    assert [s.tolist() for s in info["sel"]] == [[0, 1], [1, 2]]
    # Eq. 1 on the boxes: A takes the per-dimension maxima: s(6+2), s(-4+2), s(-12+5) -> {0,1};
    # B takes max in y and min in x: 2s-4s, 2s+4s, 5s+12s -> {1,2}.
    _, info = run(orc.SCORE_BOX)
    Sb = orc.cluster_scores(orc.SCORE_BOX, info["q"]["centroids"], None, info["k"]["box_min"],
                            info["k"]["box_max"], info["k"]["sizes"])
    assert np.allclose(Sb, S2 * np.array([[8, -2, -7], [-2, 6, 17]]), atol=1e-13)
    assert [s.tolist() for s in info["sel"]] == [[0, 1], [1, 2]]


def test_attention_rows_by_hand():
    O, _ = run(orc.SCORE_TQ)
    # Row 0, q = (3,4), attends clusters {0,2} = key rows 0,1,2,3,7 with q.k = 12, 20, 16, 22, -16:
    # weights 2^6 + 2^10 + 2^8 + 2^11 = 3392 on value (1,0) and 2^-8 on value (0,1).
    den = 3392 + 2.0 ** -8
    assert np.allclose(O[0], [3392 / den, 2.0 ** -8 / den], rtol=1e-12, atol=0)
    # Row 4, q = (-3,4), attends clusters {1,2} = key rows 4,5,6,7 with q.k = 12, 20, 16, 56:
    # weights 2^6 + 2^10 + 2^8 = 1344 on value (100,100) and 2^28 on value (0,1).
    den = 1344 + 2.0 ** 28
    assert np.allclose(O[4], [100 * 1344 / den, (100 * 1344 + 2.0 ** 28) / den], rtol=1e-12, atol=0)
    # Rows of query cluster A never see cluster 1: their two components are the two weights of a convex
    # combination of (1,0) and (0,1).
    assert np.allclose(O[:4].sum(axis=1), 1.0, atol=1e-14)
    # Rows of B never see cluster 0: y - x is the weight of row 7 alone, in (0,1].
    w7 = O[4:, 1] - O[4:, 0]
    assert np.all((w7 > 0) & (w7 <= 1.0))
    assert np.allclose(O[4:, 0], 100 * (1 - w7), rtol=1e-12)
