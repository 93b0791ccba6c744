"""Measured variants of the clustered sparse-attention call (the paper's ablations, Sec. 4.3 and
App. A.5, restated on synthetic inputs): for each variant the time of a call, the executed density,
the mean key-cluster count, the per-layer compactness score (Sec. 3.2.1), the share of the dense soft-max
mass that the selection keeps (sampled queries) and the error of the output against dense attention
computed by the same library (relative L2 and max-abs; the paper reports PSNR/SSIM of generated videos,
which need the models).

    python -m paper_2604_18348_amd.ablate --config c2

Variants: the adaptive call as configured; Eq. 1 scoring on the per-cluster box instead of Alg. 2 on
centroids; mean-based scoring ("w/o Quest"); a fixed cluster count equal to the mean adaptive count
("AvgClus": one plain k-means stage); query clustering without normalisation ("w/o Norm"); half and
twice the top-k.  Prints one JSON line per variant.
Runs on the GPU only (there is no CPU path)."""
import argparse
import dataclasses
import json
import sys
import time

import numpy as np


def attention_mass_kept(torch, Q, K, outs, p, scale, per_head=128, seed=0):
    """Share of the dense soft-max mass that falls on the selected keys, averaged over `per_head` sampled
    queries of every head: what a selection keeps of the attention it approximates, whatever V holds.
    Evaluation only (plain torch on the device; not part of the call)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    H, N, _ = Q.shape
    cap = outs["sel_idx"].shape[2]
    tot = 0.0
    for h in range(H):
        idx = torch.randperm(N, generator=g)[:min(per_head, N)].to(Q.device)
        logits = (Q[h, idx].float() @ K[h].float().T) * scale
        P = torch.softmax(logits, dim=1)
        cnt = outs["sel_cnt"][h].long()                                       # [Cq]
        pos = torch.arange(cap, device=Q.device)[None, :] < cnt[:, None]      # valid entries of sel_idx
        mask = torch.zeros((p.q_clusters, cap + 1), dtype=torch.bool, device=Q.device)
        mask.scatter_(1, torch.where(pos, outs["sel_idx"][h].long(), torch.full_like(pos, cap, dtype=torch.long)), True)
        allowed = mask[:, :cap][outs["q_labels"][h, idx].long()][:, outs["k_labels"][h].long()]   # [S, N]
        tot += float((P * allowed).sum(dim=1).mean())
    return tot / H


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--aligned", action="store_true",
                    help="queries drawn around the key mean of their component: concentrated attention")
    a = ap.parse_args()

    import torch
    from . import harness
    from paper_2604_18348_amd import binding as B
    from paper_2604_18348_amd import workloads as wl
    B.load_library()
    torch.cuda.set_device(0)
    cfg, Q, K, V = harness.device_inputs(a.config, aligned=a.aligned)
    H, N, d = Q.shape
    dtype = B.BF16 if cfg["dtype"] == "bf16" else B.F32
    base = B.Params(H=H, N=N, d=d, dtype=dtype, **cfg["params"])

    scale = base.softmax_scale if base.softmax_scale > 0 else 1.0 / float(d) ** 0.5
    dense = B.adacluster_dense_attn(base, Q, K, V).float()
    torch.cuda.synchronize()
    dense_norm = float(torch.linalg.vector_norm(dense))

    def run(name, p):
        ws = B.workspace(p)
        outs = B.alloc_outputs(p, "cuda", want_box=(p.score_mode == B.SCORE_BOX), want_stage=False)
        O = torch.empty_like(Q)
        for _ in range(3):
            B.adacluster_attn(p, Q, K, V, outs=outs, out=O, ws=ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            B.adacluster_attn(p, Q, K, V, outs=outs, out=O, ws=ws)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / a.steps
        pairs = harness.executed_pairs(outs, p)
        mse = B.adacluster_compactness(p, K, outs["k_labels"], outs["k_centroids"], ws=ws).cpu().numpy()
        diff = O.float() - dense
        rec = {"variant": name, "config": a.config, "aligned": bool(a.aligned), "ms_per_call": ms,
               "density": pairs / (H * float(N) * float(N)),
               "k_clusters_mean": float(outs["k_count"].float().mean()),
               "heads_full_attention": int(outs["full_flag"].sum()),
               "compactness": float(1.0 / np.mean(mse)),
               "attention_mass_kept": attention_mass_kept(torch, Q, K, outs, p, scale),
               "rel_l2_vs_dense": float(torch.linalg.vector_norm(diff)) / dense_norm,
               "max_abs_vs_dense": float(diff.abs().max())}
        print(json.dumps(rec), flush=True)
        return rec

    first = run("adaptive", base)
    run("box_scores_eq1", dataclasses.replace(base, score_mode=B.SCORE_BOX))
    run("mean_scores_no_quest", dataclasses.replace(base, score_mode=B.SCORE_DOT))
    avg = max(1, min(int(round(first["k_clusters_mean"])), base.k_max_clusters))
    run("fixed_count_avgclus", dataclasses.replace(base, k_m0=avg, k_m_min=min(base.k_m_min, avg), k_max_stages=1,
                                                   tau_abs=1e30))
    run("queries_not_normalised", dataclasses.replace(base, q_no_norm=1))
    if base.select_mode == B.SELECT_TOPK:
        run("topk_half", dataclasses.replace(base, topk=max(1, base.topk // 2)))
        run("topk_double", dataclasses.replace(base, topk=base.topk * 2))


if __name__ == "__main__":
    sys.exit(main())
