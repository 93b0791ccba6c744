"""A sequence of calls on slowly drifting inputs: what re-using the clustering across denoising steps
saves and what it costs in accuracy (Sec. 3.2.2, "Efficient initialization"; Sec. 4.1: the centres of the
previous step are reused for all later steps).

    python -m paper_2604_18348_amd.denoise_sequence --config c2 --steps 10 --drift 0.05

Step 0 is a cold call (Algorithm 1 decides the cluster counts).  Every later step first moves the inputs,
x <- x + drift * N(0, I) (rounded to the I/O type; the paper's consecutive denoising steps change the
activations a little), then makes a warm-start call: counts fixed, the previous step's centres as the
start, two assignment passes.  Beside it, for comparison only, the same inputs go through a cold call
with buffers of its own.  For both the line gives the time of the call (HIP events around it), the
executed density, the share of the dense soft-max mass that the selection keeps (sampled queries) and
the error of the output against dense attention by the same library on the same inputs (relative L2).  Prints one JSON line per step and a summary line.  GPU only."""
import argparse
import dataclasses
import json


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--drift", type=float, default=0.05)
    ap.add_argument("--aligned", action="store_true",
                    help="queries drawn around the key mean of their component: concentrated attention")
    a = ap.parse_args()

    import torch
    from . import harness
    from paper_2604_18348_amd import binding as B
    from paper_2604_18348_amd import workloads as wl
    from paper_2604_18348_amd.ablate import attention_mass_kept
    B.load_library()
    torch.cuda.set_device(0)
    cfg, Q, K, V = harness.device_inputs(a.config, aligned=a.aligned)
    H, N, d = Q.shape
    dtype = B.BF16 if cfg["dtype"] == "bf16" else B.F32
    cold_p = B.Params(H=H, N=N, d=d, dtype=dtype, **cfg["params"])
    warm_p = dataclasses.replace(cold_p, q_init_mode=1, k_init_mode=1, q_iters=2, k_iters=2)
    scale = cold_p.softmax_scale if cold_p.softmax_scale > 0 else 1.0 / float(d) ** 0.5
    ws = B.workspace(cold_p)
    seq = B.alloc_outputs(cold_p, "cuda", want_box=False, want_stage=False)      # carried from step to step
    ref = B.alloc_outputs(cold_p, "cuda", want_box=False, want_stage=False)      # the cold call beside it
    O = torch.empty_like(Q)
    O_ref = torch.empty_like(Q)
    O_dense = torch.empty_like(Q)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg["seed"] + 77)

    def timed(p, outs, out):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.adacluster_attn(p, Q, K, V, outs=outs, out=out, ws=ws)
        e1.record()
        e1.synchronize()
        return e0.elapsed_time(e1)

    def rel_l2(x):
        return float(torch.linalg.vector_norm(x.float() - O_dense.float()) / torch.linalg.vector_norm(O_dense.float()))

    def drift(x):
        noise = torch.randn(x.shape, generator=gen, device="cuda", dtype=torch.float32)
        return (x.float() + a.drift * noise).to(x.dtype)

    for _ in range(20):                       # clock spin-up on a scratch set of buffers
        B.adacluster_attn(cold_p, Q, K, V, outs=ref, out=O_ref, ws=ws)
    torch.cuda.synchronize()

    rows = []
    for t in range(a.steps):
        if t > 0:
            Q, K, V = drift(Q), drift(K), drift(V)
        B.adacluster_dense_attn(cold_p, Q, K, V, out=O_dense, ws=ws)
        ms = timed(cold_p if t == 0 else warm_p, seq, O)
        ms_ref = timed(cold_p, ref, O_ref)
        row = {"step": t, "call": "cold" if t == 0 else "warm", "ms": ms,
               "density": harness.executed_pairs(seq, cold_p) / (H * float(N) * float(N)),
               "k_clusters_mean": float(seq["k_count"].float().mean()),
               "attention_mass_kept": attention_mass_kept(torch, Q, K, seq, cold_p, scale),
               "rel_l2_vs_dense": rel_l2(O),
               "cold_beside": {"ms": ms_ref, "density": harness.executed_pairs(ref, cold_p) / (H * float(N) * float(N)),
                               "k_clusters_mean": float(ref["k_count"].float().mean()),
                               "attention_mass_kept": attention_mass_kept(torch, Q, K, ref, cold_p, scale),
                               "rel_l2_vs_dense": rel_l2(O_ref)}}
        rows.append(row)
        print(json.dumps(row), flush=True)
    warm = rows[1:]
    if warm:
        print(json.dumps({"config": a.config, "steps": a.steps, "drift": a.drift,
                          "cold_ms_mean": sum(r["cold_beside"]["ms"] for r in rows) / len(rows),
                          "warm_ms_mean": sum(r["ms"] for r in warm) / len(warm),
                          "cold_mass_kept_mean": sum(r["cold_beside"]["attention_mass_kept"] for r in rows) / len(rows),
                          "warm_mass_kept_mean": sum(r["attention_mass_kept"] for r in warm) / len(warm),
                          "cold_rel_l2_mean": sum(r["cold_beside"]["rel_l2_vs_dense"] for r in rows) / len(rows),
                          "warm_rel_l2_mean": sum(r["rel_l2_vs_dense"] for r in warm) / len(warm),
                          "warm_rel_l2_last": warm[-1]["rel_l2_vs_dense"]}))


if __name__ == "__main__":
    main()
