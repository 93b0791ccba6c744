"""Writes tests/golden/oracle_digest.txt: a digest of what the CPU oracle returns today on three seeded
inputs, so that a later edit that changes the oracle's arithmetic cannot go unnoticed (the test that
reads the file fails until the file is written again, and the commit that does so has to say which
passage of the paper justifies the change).

The paper prints no numeric worked example, so this folder holds no value taken from it; every value
in the digest comes from oracle/ alone - this script calls nothing else that computes (the input
generator only draws numbers).

    python tests/golden/make_oracle_digest.py            # rewrite the file
    python tests/golden/make_oracle_digest.py --print    # show what would be written
"""
import hashlib
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import adacluster_oracle as orc                       # noqa: E402
from paper_2604_18348_amd import workloads as wl                  # noqa: E402

CASES = {
    # name: (seed, N, d, mixture components, heads, oracle keyword arguments)
    "topk_tensorquest_d64": (71, 1500, 64, 12, 2, dict(
        q_clusters=13, q_iters=3, k_iters=3, k_m0=20, k_m_min=4, k_max_clusters=80, tau_factor=1.5,
        min_unassigned_frac=0.03, score_mode=orc.SCORE_TQ, select_mode=0, topk=6)),
    "topp_box_d128": (72, 900, 128, 9, 1, dict(
        q_clusters=7, q_iters=2, k_iters=2, k_m0=12, k_m_min=2, k_max_clusters=60, tau_factor=1.2,
        min_unassigned_frac=0.0, score_mode=orc.SCORE_BOX, select_mode=1, top_p=0.8)),
    "topk_dot_unnormalised_queries_bf16_centres": (73, 1100, 64, 10, 1, dict(
        q_clusters=9, q_iters=3, k_iters=3, k_m0=16, k_m_min=4, k_max_clusters=64, tau_abs=2.8,
        min_unassigned_frac=0.02, score_mode=orc.SCORE_DOT, select_mode=0, topk=4, q_no_norm=1,
        round_fn=orc.round_to_bf16)),
}


def sha(a):
    return hashlib.sha256(np.ascontiguousarray(np.asarray(a, dtype=np.int64)).tobytes()).hexdigest()[:16]


def digest_lines():
    lines = []
    for name, (seed, N, d, M, H, kw) in CASES.items():
        Q, K, V = wl.make_small(seed, N, d, M, dtype="bf16", H=H)
        O, infos, tau = orc.adacluster_attention(Q, K, V, use_gather=True, **kw)
        lines.append(f"case {name}")
        lines.append(f"tau {tau:.12e}")
        for h, info in enumerate(infos):
            k, q = info["k"], info["q"]
            sel = info["sel"] if info["sel"] is not None else []
            flat = np.concatenate([np.append(s, -1) for s in sel]) if len(sel) else np.zeros(0)
            lines.append(f"head {h} full {int(k['full_flag'])} stage_offs {' '.join(map(str, k['stage_offs']))}")
            lines.append(f"head {h} unassigned {' '.join(map(str, k['n_unassigned']))}")
            lines.append(f"head {h} q_labels {sha(q['labels'])} k_labels {sha(k['labels'])} "
                         f"k_sizes {sha(k['sizes'])} sel {sha(flat)}")
            lines.append(f"head {h} sum {float(O[h].sum()):.10e} sumsq {float((O[h] ** 2).sum()):.10e} "
                         f"centroid_sumsq {float((k['centroids'] ** 2).sum()):.10e}")
    return lines


if __name__ == "__main__":
    text = "\n".join(digest_lines()) + "\n"
    if "--print" in sys.argv:
        sys.stdout.write(text)
    else:
        with open(os.path.join(HERE, "oracle_digest.txt"), "w") as f:
            f.write(text)
