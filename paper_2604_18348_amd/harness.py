"""Measurement harness shared by bench.py and the package's measurement scripts: synthetic inputs on the
device, timing of the fused call and of its parts, and the figures derived from them.  Argument handling
and timing only: every step of the method runs in the library."""
from __future__ import annotations

import dataclasses
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

BF16_PEAK_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
FP32_VALU_PEAK_TFLOPS = 157.3  # MI355X fp32 vector, published
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published


def device_inputs(name, aligned=False):
    """Q, K, V of benchmark configuration `name` as device tensors [H,N,d] (heads drawn on host threads)."""
    import torch
    from . import workloads as wl
    cfg = wl.CONFIGS[name]
    H, N, d = cfg["H"], wl.n_tokens(cfg), cfg["d"]
    dt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    Q = torch.empty((H, N, d), dtype=dt, device="cuda")
    K = torch.empty_like(Q)
    V = torch.empty_like(Q)

    def one(h):
        return h, wl.make_head(cfg, h, aligned=aligned)

    with ThreadPoolExecutor(max_workers=min(16, H)) as ex:
        for h, (q, k, v) in ex.map(one, range(H)):
            Q[h].copy_(torch.from_numpy(q).to(dt))
            K[h].copy_(torch.from_numpy(k).to(dt))
            V[h].copy_(torch.from_numpy(v).to(dt))
    return cfg, Q, K, V


def executed_pairs(outs, p):
    """sum over heads and query clusters of n_q(i) * sum_{j in sel(i)} n_k(j), from a call's outputs."""
    qs = outs["q_sizes"].cpu().numpy().astype(np.int64)
    ks = outs["k_sizes"].cpu().numpy().astype(np.int64)
    si = outs["sel_idx"].cpu().numpy()
    sc = outs["sel_cnt"].cpu().numpy()
    tot = 0
    cols = np.arange(si.shape[2])[None, :]
    for h in range(p.H):
        live = cols < sc[h][:, None]                       # entries past a list's count are not written
        keys = np.where(live, ks[h][np.where(live, si[h], 0)], 0).sum(axis=1)
        tot += int((qs[h] * keys).sum())
    return tot


def _timed_calls(fn, steps):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def _profiled(fn, B, reps):
    """mean stage times (ms) over `reps` profiled calls (events recorded by the library on its own streams)."""
    acc = {}
    for _ in range(reps):
        fn()
        for k, v in B.adacluster_profile_read().items():
            acc[k] = acc.get(k, 0.0) + v
    return {k: v / reps for k, v in acc.items()}


def mfma_microbench_tflops(B, iters=20000):
    """bf16 TFLOP/s of a register-only MFMA loop on every SIMD (what the matrix cores sustain here)."""
    import torch
    sink = torch.empty(1024, dtype=torch.float32, device="cuda")
    B.adacluster_mfma_probe(iters, sink)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    flops = B.adacluster_mfma_probe(iters, sink)
    e1.record()
    torch.cuda.synchronize()
    return flops / (e0.elapsed_time(e1) * 1e-3) / 1e12


def measure(name, steps, warmup, spinup_ms=500.0, dense_steps=3, profile_reps=None, want_hbm=True):
    """One configuration, end to end: the fused call cold and warm-started, its stage times, the dense call
    on the same kernel, the attention kernel against the bf16 MFMA peak, and the HBM-bound passes (label
    sorts, segmented reduction, and for fp32 inputs the K/V row gather) against the HBM peak.  Returns a
    dict of plain numbers."""
    import torch
    from . import binding as B
    from . import workloads as wl
    cfg, Q, K, V = device_inputs(name)
    H, N, d = Q.shape
    dtype = B.BF16 if cfg["dtype"] == "bf16" else B.F32
    es = 2 if dtype == B.BF16 else 4
    p = B.Params(H=H, N=N, d=d, dtype=dtype, **cfg["params"])
    ws = B.workspace(p)
    outs = B.alloc_outputs(p, "cuda", want_box=False, want_stage=False)
    O = torch.empty_like(Q)
    call = lambda: B.adacluster_attn(p, Q, K, V, outs=outs, out=O, ws=ws)
    reps = profile_reps or max(3, min(steps, 10))

    # The shader clock takes a few hundred milliseconds of load to climb from its idle level; calls made
    # before that run up to 20 % slower.  Spin up first (untimed, outside warm-up and steps).
    t_spin = time.perf_counter()
    while (time.perf_counter() - t_spin) * 1e3 < spinup_ms:
        call()
        torch.cuda.synchronize()
    for _ in range(warmup):
        call()
    ms = _timed_calls(call, steps)                      # the headline: profiling off, one wait at the end
    B.adacluster_profile_enable(True)
    stage_ms = _profiled(call, B, reps)
    stats = B.adacluster_stats_fetch(p, ws)
    B.adacluster_profile_enable(False)
    pairs = sum(s["executed_pairs"] for s in stats)
    issued = sum(s["issued_pairs"] for s in stats)
    flops, issued_flops = 4.0 * d * pairs, 4.0 * d * issued
    dense_flops = 4.0 * d * H * float(N) * float(N)
    attn_ms = stage_ms["attention"]
    peak = BF16_PEAK_TFLOPS if dtype == B.BF16 else FP32_VALU_PEAK_TFLOPS
    attn_tflops = flops / (attn_ms * 1e-3) / 1e12

    # later denoising steps (Sec. 3.2.2): cluster counts fixed, previous centres as the start
    pw = dataclasses.replace(p, q_init_mode=1, k_init_mode=1, q_iters=2, k_iters=2)
    warm = lambda: B.adacluster_attn(pw, Q, K, V, outs=outs, out=O, ws=ws)
    warm()
    warm_ms = _timed_calls(warm, steps)
    B.adacluster_profile_enable(True)
    warm_stage_ms = _profiled(warm, B, reps)
    B.adacluster_profile_enable(False)

    out = {
        "workload": "%s: %s H=%d N=%d d=%d, Cq=%d m0=%d Nmax=%d %s" % (
            name, cfg["dtype"], H, N, d, p.q_clusters, p.k_m0, p.k_max_clusters,
            ("top-p %.2f" % p.top_p) if p.select_mode else ("top-k %d" % p.topk)),
        "dtype": cfg["dtype"], "ms": ms, "stage_ms": stage_ms,
        "warm_start_ms": warm_ms, "warm_start_stage_ms": warm_stage_ms,
        "density": flops / dense_flops, "executed_tflop": flops / 1e12, "issued_tflop": issued_flops / 1e12,
        "k_clusters_mean": float(np.mean([s["k_count"] for s in stats])),
        "stages_mean": float(np.mean([s["stages"] for s in stats])),
        "heads_full_attention": int(sum(s["full_flag"] for s in stats)),
        "call_effective_tflops": flops / (ms * 1e-3) / 1e12,
        "attn_kernel_ms": attn_ms, "attn_tflops": attn_tflops, "attn_frac_of_peak": attn_tflops / peak,
        "attn_issued_frac_of_peak": issued_flops / (attn_ms * 1e-3) / 1e12 / peak,
        "peak_tflops": peak, "bound": "mfma" if dtype == B.BF16 else "alu",
        "kernel": "attn_mfma" if dtype == B.BF16 else "attn_f32",
    }

    if dense_steps > 0:
        dense = lambda: B.adacluster_dense_attn(p, Q, K, V, out=O, ws=ws)
        dense()
        dense_ms = _timed_calls(dense, dense_steps)
        B.adacluster_profile_enable(True)
        dense_attn_ms = _profiled(dense, B, 1)["attention"]
        B.adacluster_profile_enable(False)
        out.update({"dense_ms": dense_ms, "dense_attn_kernel_ms": dense_attn_ms,
                    "speedup_vs_dense": dense_ms / ms, "warm_speedup_vs_dense": dense_ms / warm_ms,
                    "dense_tflops": dense_flops / (dense_attn_ms * 1e-3) / 1e12})

    if want_hbm:
        # The HBM-bound passes, each timed where nothing else shares the GPU: the stand-alone entry points
        # run them on one stream (in the fused call they overlap other work and their times stretch).
        B.adacluster_profile_enable(True)
        kc = B.adacluster_kcluster(p, K, want_box=False, ws=ws)
        t_red = B.adacluster_profile_read().get("kreduce")
        B.adacluster_sparse_attn(p, Q, K, V, outs["q_labels"], outs["k_labels"], outs["k_count"], outs["sel_idx"],
                                 outs["sel_cnt"], out=O, ws=ws)
        pr = B.adacluster_profile_read()
        B.adacluster_profile_enable(False)
        del kc
        rows = float(H) * N
        cap = p.k_max_clusters + p.k_m0
        q_passes, k_passes = -(-max(1, (p.q_clusters - 1).bit_length()) // 7), -(-max(1, (cap - 1).bit_length()) // 7)
        hbm = {}

        def entry(key, ms_, nbytes, what):
            if ms_ and ms_ > 0:
                gbs = nbytes / (ms_ * 1e-3) / 1e9
                hbm[key] = {"ms": ms_, "bytes": nbytes, "GB/s": gbs, "frac": gbs / HBM_PEAK_GBS, "what": what}
        entry("gather_rows2", pr.get("permute"), 4.0 * rows * d * es + 4.0 * rows,
              "K and V rows read and written once, permutation read")
        sort_bytes = lambda passes: (16.0 + 20.0 * (passes - 1)) * rows
        entry("label_sorts", pr.get("select"), sort_bytes(q_passes) + sort_bytes(k_passes),
              "query labels (%d radix pass) and key labels (%d): per item and pass 4 B read to count, 4 B (first "
              "pass) or 8 B read and 8 B written to scatter" % (q_passes, k_passes))
        entry("seg_reduce", t_red, rows * d * es + 4.0 * rows, "K rows and the permutation read once")
        out["hbm"] = hbm
    del Q, K, V, O, ws, outs
    torch.cuda.empty_cache()
    return out
