"""Choice of N_max (the paper's k_max) from one calibration call.

Sec. 4.1 sets k_max "such that the top 15 % of layers use full attention": the units whose keys need
the most clusters are the ones where clustering pays least, and they are sent to the dense branch by
the flag F of Algorithm 1.  A unit is a layer in the paper; here it is whatever the caller collects
rows for - the heads of one call, or the heads of the calls of several layers.

How the flag depends on N_max is read off one run of Algorithm 1 with the cap out of reach.  The loop
tests |C| >= N_max at the head of a stage, while U is not empty, so with stage heads at the counts
offs[0] < offs[1] < ... the flag is set exactly when N_max <= theta, where theta is the count at the
last stage head that still had unassigned keys: offs[T-1] for a run of T stages that emptied U, and
offs[T] (the final count) when the stage limit or the left-over limit stopped it with keys left.
Nothing before that head depends on N_max, so the prediction is exact, not an estimate.

    python -m paper_2604_18348_amd.calibrate --config c2 --dense-fraction 0.15

runs the calibration call on the synthetic workload, picks N_max, runs the key clustering again with
it and prints what was predicted and what came out (GPU only; the two functions below are plain numpy).
"""
import argparse
import json

import numpy as np


def flag_thresholds(stage_offs, k_count, left_over):
    """theta per unit: the largest N_max at which Algorithm 1 sets the flag F for it.

    stage_offs [U, S+1] running centre counts as the library exports them (entries past the last stage
    repeat the final count), k_count [U] final counts, left_over [U] true where the run ended with
    unassigned keys (some k_stage_of == -1).  The run must not have been stopped by its own cap."""
    offs = np.asarray(stage_offs, dtype=np.int64)
    kc = np.asarray(k_count, dtype=np.int64)
    left = np.asarray(left_over, dtype=bool)
    theta = np.zeros(kc.shape[0], dtype=np.int64)
    for u in range(kc.shape[0]):
        n_stage = int(np.searchsorted(offs[u], kc[u]))        # first index whose count is the final one
        theta[u] = kc[u] if left[u] else (offs[u, n_stage - 1] if n_stage >= 1 else 0)
    return theta


def choose_n_max(theta, dense_fraction, n_min=1):
    """N_max that flags the round(dense_fraction * U) units with the largest theta (more on ties, fewer
    when their theta lies below n_min, the smallest N_max the caller can use: k_m0).  Returns
    (n_max, flags predicted for it)."""
    theta = np.asarray(theta, dtype=np.int64)
    want = int(round(float(dense_fraction) * theta.shape[0]))
    if want <= 0:
        n_max = int(theta.max()) + 1 if theta.size else int(n_min)
    else:
        n_max = int(np.sort(theta)[::-1][want - 1])
    n_max = max(n_max, int(n_min), 1)
    return n_max, theta >= n_max


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--dense-fraction", type=float, default=0.15)
    ap.add_argument("--aligned", action="store_true",
                    help="queries drawn around the key mean of their component: concentrated attention")
    a = ap.parse_args()

    import dataclasses
    import torch
    from . import harness
    from paper_2604_18348_amd import binding as B
    from paper_2604_18348_amd import workloads as wl
    B.load_library()
    torch.cuda.set_device(0)
    cfg, Q, K, V = harness.device_inputs(a.config, aligned=a.aligned)
    H, N, d = K.shape
    dtype = B.BF16 if cfg["dtype"] == "bf16" else B.F32
    base = B.Params(H=H, N=N, d=d, dtype=dtype, **cfg["params"])
    # the cap out of reach: every stage adds at most k_m0 centres
    free = dataclasses.replace(base, k_max_clusters=min(7168 - base.k_m0, base.k_m0 * (base.k_max_stages + 1)))
    cal = B.adacluster_kcluster(free, K, want_box=False)
    torch.cuda.synchronize()
    assert int(cal["full_flag"].sum()) == 0
    left = (cal["k_stage_of"] == -1).any(dim=1).cpu().numpy()
    theta = flag_thresholds(cal["k_stage_offs"].cpu().numpy(), cal["k_count"].cpu().numpy(), left)
    n_max, predicted = choose_n_max(theta, a.dense_fraction, n_min=base.k_m0)
    capped = dataclasses.replace(base, k_max_clusters=n_max, tau_abs=float(cal["tau_used"][0]))
    out = B.adacluster_kcluster(capped, K, want_box=False)
    torch.cuda.synchronize()
    got = out["full_flag"].cpu().numpy().astype(bool)
    print(json.dumps({"config": a.config, "dense_fraction_asked": a.dense_fraction, "n_max": n_max,
                      "theta": theta.tolist(), "flags_predicted": predicted.astype(int).tolist(),
                      "flags_measured": got.astype(int).tolist(),
                      "dense_fraction_measured": float(got.mean()),
                      "k_count_uncapped": cal["k_count"].cpu().numpy().tolist(),
                      "prediction_exact": bool(np.array_equal(got, predicted))}))


if __name__ == "__main__":
    main()
