#!/usr/bin/env python3
"""Benchmark of the clustered sparse-attention call on one MI355X.

A step is one adacluster_attn call (query clustering, Algorithm 1, selection, permutation,
block-sparse attention) over one synthetic Q/K/V batch of the chosen configuration, inputs
resident in HBM.  Prints ONE JSON line: the call's latency, its stage times, the dense call beside
it, the attention kernel against the bf16 MFMA peak, and the CPU oracle timed on the host.
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
FP32_VALU_PEAK_TFLOPS = 157.3


# HBM-side traffic of one attention-kernel launch, bytes: FETCH_SIZE (divided by the 0.504 the counter
# reads for a plain copy of known size) + WRITE_SIZE of the two rocprofv3 --pmc passes summarised in
# profiles/attn_pipeline_<config>.txt.  A counter cannot be read from inside this script, so the
# figures are stored; a config without a profile reports null.
PROFILED_ATTN_TRAFFIC_BYTES = {"c2": 707.7e6, "c3": 289.0e6, "c4": 2670.6e6, "c5": 4324.2e6}


def gen_inputs(name, torch, B, wl):
    cfg = wl.CONFIGS[name]
    H, N, d = cfg["H"], wl.n_tokens(cfg), cfg["d"]
    dt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    Q = torch.empty((H, N, d), dtype=dt, device="cuda")
    K = torch.empty_like(Q)
    V = torch.empty_like(Q)

    def one(h):
        return h, wl.make_head(cfg, h)

    with ThreadPoolExecutor(max_workers=min(16, H)) as ex:
        for h, (q, k, v) in ex.map(one, range(H)):
            Q[h].copy_(torch.from_numpy(q).to(dt))
            K[h].copy_(torch.from_numpy(k).to(dt))
            V[h].copy_(torch.from_numpy(v).to(dt))
    return cfg, Q, K, V


def executed_pairs(outs, p):
    """sum over heads and query clusters of n_q(i) * sum_{j in sel(i)} n_k(j)."""
    import torch
    tot = 0
    qs = outs["q_sizes"].cpu().numpy().astype(np.int64)
    ks = outs["k_sizes"].cpu().numpy().astype(np.int64)
    si = outs["sel_idx"].cpu().numpy()
    sc = outs["sel_cnt"].cpu().numpy()
    for h in range(p.H):
        for i in range(p.q_clusters):
            tot += int(qs[h, i]) * int(ks[h, si[h, i, :sc[h, i]]].sum())
    return tot


def cpu_baseline(name, wl, target_s=15.0):
    """The oracle, as it stands, on a bounded sample of the workload: the whole call on the first
    heads.  One head is timed first; if that leaves room, as many heads as fit about `target_s`
    seconds are then run in one call (tau is then the mean over those heads) and that run is the
    one reported."""
    from oracle import adacluster_oracle as orc
    cfg = wl.CONFIGS[name]
    rf = orc.round_to_bf16 if cfg["dtype"] == "bf16" else None

    def timed(heads):
        Q, K, V = wl.make_qkv(name, heads=heads)
        t0 = time.perf_counter()
        orc.adacluster_attention(Q, K, V, use_gather=True, round_fn=rf, **cfg["params"])
        return time.perf_counter() - t0

    heads = [0]
    dt = timed(heads)
    more = min(cfg["H"], int(target_s / max(dt, 1e-3)))
    if more > 1:
        heads = list(range(more))
        dt = timed(heads)
    try:
        from threadpoolctl import threadpool_info
        cores = max([i.get("num_threads", 1) for i in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return dict(value=dt * 1e3 * cfg["H"] / len(heads), unit="ms/call", cores=int(cores), kind="oracle",
                sample="fp64 numpy oracle, full call on %d of %d heads (%.1f s measured), scaled by H"
                       % (len(heads), cfg["H"], dt))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--spinup-ms", type=float, default=500.0,
                    help="untimed calls before the warm-up, until the GPU clock has left its idle state")
    ap.add_argument("--config", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
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
    from paper_2604_18348_amd import workloads as wl
    B.load_library()
    torch.cuda.set_device(0)

    cfg, Q, K, V = gen_inputs(a.config, torch, B, wl)
    H, N, d = Q.shape
    dtype = B.BF16 if cfg["dtype"] == "bf16" else B.F32
    p = B.Params(H=H, N=N, d=d, dtype=dtype, **cfg["params"])
    ws = B.workspace(p)
    outs = B.alloc_outputs(p, "cuda", want_box=False, want_stage=False)
    O = torch.empty_like(Q)

    # a plain device copy of known size (256 MiB read + 256 MiB written): the calibration kernel
    # for the FETCH_SIZE / WRITE_SIZE counters of a profiler run of this same command
    calib_src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    calib_dst = torch.empty_like(calib_src)
    calib_dst.copy_(calib_src)
    del calib_src, calib_dst

    # The shader clock takes a few hundred milliseconds of load to climb from its idle level; calls
    # made before that run up to 20 % slower.  Spin up first (untimed, outside warm-up and steps).
    t_spin = time.perf_counter()
    while (time.perf_counter() - t_spin) * 1e3 < a.spinup_ms:
        B.adacluster_attn(p, Q, K, V, outs=outs, out=O, ws=ws)
        torch.cuda.synchronize()

    B.adacluster_profile_enable(True)
    for _ in range(a.warmup):
        B.adacluster_attn(p, Q, K, V, outs=outs, out=O, ws=ws)
    torch.cuda.synchronize()
    stage_acc = {}
    t0 = time.perf_counter()
    for _ in range(a.steps):
        B.adacluster_attn(p, Q, K, V, outs=outs, out=O, ws=ws)
        for k, v in B.adacluster_profile_read().items():
            stage_acc[k] = stage_acc.get(k, 0.0) + v
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / a.steps
    stage_ms = {k: v / a.steps for k, v in stage_acc.items()}

    pairs = executed_pairs(outs, p)
    flops = 4.0 * d * pairs
    dense_flops = 4.0 * d * H * float(N) * float(N)
    attn_ms = stage_ms["attention"]
    peak = BF16_PEAK_TFLOPS if dtype == B.BF16 else FP32_VALU_PEAK_TFLOPS
    attn_tflops = flops / (attn_ms * 1e-3) / 1e12
    kc = outs["k_count"].cpu().numpy()
    ff = outs["full_flag"].cpu().numpy()

    # later denoising steps (Sec. 3.2.2): cluster counts fixed, previous centres as the start
    import dataclasses
    pw = dataclasses.replace(p, q_init_mode=1, k_init_mode=1, q_iters=2, k_iters=2)
    B.adacluster_attn(pw, Q, K, V, outs=outs, out=O, ws=ws)
    torch.cuda.synchronize()
    wacc = {}
    t2 = time.perf_counter()
    for _ in range(a.steps):
        B.adacluster_attn(pw, Q, K, V, outs=outs, out=O, ws=ws)
        for k, v in B.adacluster_profile_read().items():
            wacc[k] = wacc.get(k, 0.0) + v
    torch.cuda.synchronize()
    warm_ms = (time.perf_counter() - t2) * 1e3 / a.steps
    warm_stage_ms = {k: v / a.steps for k, v in wacc.items()}

    dense_ms = None
    dense_attn_ms = None
    if not a.no_dense:
        B.adacluster_dense_attn(p, Q, K, V, out=O, ws=ws)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        acc = 0.0
        for _ in range(a.dense_steps):
            B.adacluster_dense_attn(p, Q, K, V, out=O, ws=ws)
            acc += B.adacluster_profile_read()["attention"]
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - t1) * 1e3 / a.dense_steps
        dense_attn_ms = acc / a.dense_steps
    B.adacluster_profile_enable(False)

    out = {
        "metric": "clustered sparse attention ms/call (adacluster_attn, 1 MI355X)",
        "value": ms, "unit": "ms", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "spinup_ms": a.spinup_ms,
        "ms_per_step": ms, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": "%s: %s H=%d N=%d d=%d, Cq=%d m0=%d Nmax=%d %s" % (
            a.config, cfg["dtype"], H, N, d, p.q_clusters, p.k_m0, p.k_max_clusters,
            ("top-p %.2f" % p.top_p) if p.select_mode else ("top-k %d" % p.topk))},
        "stage_ms": stage_ms,
        "warm_start_ms": warm_ms, "warm_start_stage_ms": warm_stage_ms,
        "density": flops / dense_flops,
        "executed_tflop": flops / 1e12,
        "k_clusters_mean": float(kc.mean()), "heads_full_attention": int(ff.sum()),
        "dense_ms": dense_ms, "dense_attn_kernel_ms": dense_attn_ms,
        "speedup_vs_dense": (dense_ms / ms) if dense_ms else None,
        "warm_speedup_vs_dense": (dense_ms / warm_ms) if dense_ms else None,
        "dense_tflops": (dense_flops / (dense_attn_ms * 1e-3) / 1e12) if dense_attn_ms else None,
        "call_effective_tflops": flops / (ms * 1e-3) / 1e12,
        "roofline": {"kernel": "attn_mfma" if dtype == B.BF16 else "attn_f32",
                     "bound": "mfma" if dtype == B.BF16 else "alu",
                     "achieved": attn_tflops, "peak": peak, "unit": "TFLOP/s",
                     "frac": attn_tflops / peak, "traffic": PROFILED_ATTN_TRAFFIC_BYTES.get(a.config),
                     "traffic_unit": "bytes per launch (rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE, see profiles/)"},
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(a.config, wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
