#!/usr/bin/env python3
"""Benchmark of the clustered sparse-attention call on one MI355X.

A step is one adacluster_attn call (query clustering, Algorithm 1, selection, permutation, block-sparse
attention) over one synthetic Q/K/V batch, inputs resident in HBM.  The default workload is the largest
configuration (config 5: 180 000 tokens, 24 heads of width 128).  Prints ONE JSON line: the call's latency,
its stage times, the dense call beside it, the attention kernel against the bf16 MFMA peak (useful and issued
FLOPs), the HBM-bound passes against the HBM peak, a register-only MFMA yardstick, the 75.6K-token
configuration as a second block, and the CPU oracle timed on the host.
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM-side traffic of one attention-kernel launch, bytes: FETCH_SIZE (divided by the 0.50 the counter
# reads for a plain copy of known size) + WRITE_SIZE of the two rocprofv3 --pmc passes summarised in
# profiles/attn_pipeline_<config>.txt.  A counter cannot be read from inside this script, so the
# figures are stored; a config without a profile reports null.
PROFILED_ATTN_TRAFFIC_BYTES = {"c2": 960.3e6, "c3": 293.2e6, "c4": 3100.6e6, "c5": 4493.1e6}


def cpu_baseline(name, wl, target_s=15.0):
    """The oracle, as it stands, on a bounded sample of the workload.  Small configurations: the whole call
    on as many heads as fit about `target_s` seconds.  Large ones (a head alone takes longer): the steps of
    the call on head 0 one by one, each in full except the attention, which runs on every `stride`-th query
    row and is scaled back; the sum is scaled by H."""
    from oracle import adacluster_oracle as orc
    cfg = wl.CONFIGS[name]
    P = cfg["params"]
    rf = orc.round_to_bf16 if cfg["dtype"] == "bf16" else None
    H, N, d = cfg["H"], wl.n_tokens(cfg), cfg["d"]
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1

    if float(N) * N * d < 2e12:
        def timed(heads):
            Q, K, V = wl.make_qkv(name, heads=heads)
            t0 = time.perf_counter()
            orc.adacluster_attention(Q, K, V, use_gather=True, round_fn=rf, **P)
            return time.perf_counter() - t0
        heads = [0]
        dt = timed(heads)
        more = min(H, int(target_s / max(dt, 1e-3)))
        if more > 1:
            heads = list(range(more))
            dt = timed(heads)
        return dict(value=dt * 1e3 * H / len(heads), unit="ms/call", cores=int(cores), kind="oracle",
                    sample="fp64 numpy oracle, full call on %d of %d heads (%.1f s measured), scaled by H"
                           % (len(heads), H, dt))

    scale = 1.0 / math.sqrt(d)

    def one_head(head, stride):
        """every step of the call on one head; stride None: sized by a probe.  -> (step seconds, stride, head seconds)"""
        Q, K, V = wl.make_qkv(name, heads=[head])
        Q, K, V = Q[0].astype(np.float64), K[0].astype(np.float64), V[0].astype(np.float64)
        t = [time.perf_counter()]
        tau = float(np.float32(P["tau_abs"])) if P["tau_abs"] > 0 else orc.tau_from_factor(K[None], P["tau_factor"], P["k_m0"], P["k_iters"], rf)
        t.append(time.perf_counter())
        qc = orc.query_kmeans(Q, P["q_clusters"], P["q_iters"], round_fn=rf)
        t.append(time.perf_counter())
        kc = orc.multistage_kmeans(K, tau, P["k_max_clusters"], P["k_m0"], P["k_m_min"], P["k_iters"], P["k_max_stages"],
                                   P["min_unassigned_frac"], rf)
        t.append(time.perf_counter())
        S = orc.cluster_scores(P["score_mode"], qc["centroids"], kc["centroids"], kc["box_min"], kc["box_max"], kc["sizes"])
        sel = orc.select_topk(S, P["topk"]) if P["select_mode"] == 0 else orc.select_topp(S, kc["sizes"], qc["mean_norm"] * scale, P["top_p"])
        t.append(time.perf_counter())

        def attention(st):
            t0 = time.perf_counter()
            rows = np.arange(0, N, st)
            orc.sparse_attention_gather(Q, K, V, qc["labels"], kc["labels"], sel, scale, rows=rows)
            return time.perf_counter() - t0, len(rows)

        if stride is None:
            # a probe on every 512th query row sizes the stride so that the sample takes about two thirds of
            # the time asked for; the probe's time is partly per-cluster overhead, so one refinement follows
            probe_s, _ = attention(512)
            stride = int(min(512, max(1, math.ceil(probe_s * 512 / (target_s * 0.67)))))
            ta, nrows = attention(stride)
            if stride > 1 and ta < 0.3 * target_s:
                stride = int(max(1, math.floor(stride * ta / (target_s * 0.67))))
                ta, nrows = attention(stride)
        else:
            ta, nrows = attention(stride)
        dt = [b - a for a, b in zip(t[:-1], t[1:])] + [ta]
        return dt, stride, dt[0] + dt[1] + dt[2] + dt[3] + dt[4] * (N / nrows)

    # head 0, then further heads (spread over the head range) while less than about 10 s have been measured
    dts, stride, hs = one_head(0, None)
    measured, heads, head_secs = sum(dts), [0], [hs]
    for head in (H // 2, H - 1, H // 4):
        if measured >= 10.0 or head in heads:
            break
        d2, _, h2 = one_head(head, stride)
        measured += sum(d2); heads.append(head); head_secs.append(h2)
    head_s = float(np.mean(head_secs))
    return dict(value=head_s * 1e3 * H, unit="ms/call", cores=int(cores), kind="oracle",
                sample="fp64 numpy oracle on head%s %s of %d, step by step; head 0: threshold pass %.1f s, query clustering "
                       "%.1f s, Algorithm 1 %.1f s, selection %.1f s (all in full), attention on every %dth query row "
                       "%.1f s (scaled by %d); %.1f s measured in all, a head's mean %.1f s scaled by H"
                       % ("s" if len(heads) > 1 else "", ", ".join(map(str, heads)), H, dts[0], dts[1], dts[2], dts[3], stride,
                          dts[4], stride, measured, head_s))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--spinup-ms", type=float, default=500.0,
                    help="untimed calls before the warm-up, until the GPU clock has left its idle state")
    ap.add_argument("--config", default="c5", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--also", default="c4", help="a second configuration reported as an extra block ('' for none)")
    ap.add_argument("--dense-steps", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (heads would shard over GPUs without any "
              "communication, but nothing here launches a second one); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2604_18348_amd import binding as B
    from paper_2604_18348_amd import harness as hz
    from paper_2604_18348_amd import workloads as wl
    B.load_library()
    torch.cuda.set_device(0)

    # a plain device copy of known size (256 MiB read + 256 MiB written): the calibration kernel
    # for the FETCH_SIZE / WRITE_SIZE counters of a profiler run of this same command
    calib_src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    del calib_src, calib_dst

    dense_steps = 0 if a.no_dense else a.dense_steps
    m = hz.measure(a.config, a.steps, a.warmup, a.spinup_ms, dense_steps)
    probe = hz.mfma_microbench_tflops(B)

    out = {
        "metric": "clustered sparse attention ms/call (adacluster_attn, 1 MI355X)",
        "value": m["ms"], "unit": "ms", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "spinup_ms": a.spinup_ms,
        "ms_per_step": m["ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": m["dtype"], "data": "synthetic",
        "config": {"workload": m["workload"]},
    }
    for k in ("stage_ms", "warm_start_ms", "warm_start_stage_ms", "density", "executed_tflop", "issued_tflop",
              "k_clusters_mean", "stages_mean", "heads_full_attention", "dense_ms", "dense_attn_kernel_ms",
              "speedup_vs_dense", "warm_speedup_vs_dense", "dense_tflops", "call_effective_tflops", "hbm"):
        if k in m:
            out[k] = m[k]
    out["mfma_microbench_tflops"] = probe
    out["roofline"] = {"kernel": m["kernel"], "bound": m["bound"], "achieved": m["attn_tflops"], "peak": m["peak_tflops"],
                       "unit": "TFLOP/s", "frac": m["attn_frac_of_peak"],
                       "issued_frac": m["attn_issued_frac_of_peak"],
                       "frac_of_microbench": m["attn_tflops"] / probe if m["bound"] == "mfma" else None,
                       "meets_0.40_target": bool(m["attn_frac_of_peak"] >= 0.40),
                       "traffic": PROFILED_ATTN_TRAFFIC_BYTES.get(a.config),
                       "traffic_unit": "bytes per launch (rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE, see profiles/)"}
    if a.also and a.also != a.config:
        x = hz.measure(a.also, max(5, a.steps), a.warmup, 200.0, dense_steps)
        out["also"] = {k: x[k] for k in ("workload", "ms", "stage_ms", "warm_start_ms", "density", "executed_tflop",
                                         "issued_tflop", "k_clusters_mean", "heads_full_attention", "dense_ms",
                                         "speedup_vs_dense", "warm_speedup_vs_dense", "dense_tflops", "attn_kernel_ms",
                                         "attn_tflops", "attn_frac_of_peak", "hbm") if k in x}
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a.config, wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
