"""Timing of the two forms of the Quest score (the paper's Sec. 4.3, "TensorQuest reformulation
benefits", restated on synthetic inputs): Eq. 1 with vector arithmetic against Eq. 2 / Algorithm 2 on
the matrix cores, for query rows of the five workloads' token counts against cluster boxes of their
typical cluster counts.

    python -m paper_2604_18348_amd.quest_timing

Prints one JSON line per shape: milliseconds of both forms, their ratio, and the rate of the
matrix-core form in TFLOP/s (4*Lq*Lk*d flops).  bf16 inputs; H heads per call as listed.  Runs on the
GPU only (there is no CPU path)."""
import json
import sys

SHAPES = [  # name, H, Lq (tokens), Lk (key clusters), d
    ("c1-like", 4, 4096, 64, 64),
    ("c2-like", 4, 17776, 173, 64),
    ("c3-like", 4, 32760, 300, 128),
    ("c4-like", 2, 75600, 450, 64),
    ("c5-like", 1, 180000, 1171, 128),
    ("centroids c5", 24, 65, 1171, 128),
]


def main():
    import torch
    from paper_2604_18348_amd import binding as B
    B.load_library()
    torch.cuda.set_device(0)
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    for name, H, Lq, Lk, d in SHAPES:
        Q = torch.randn((H, Lq, d), device="cuda", generator=g).to(torch.bfloat16)
        C = torch.randn((H, Lk, d), device="cuda", generator=g)
        spread = torch.randn((H, Lk, d), device="cuda", generator=g).abs()
        lo, hi = (C - spread).to(torch.bfloat16), (C + spread).to(torch.bfloat16)
        S = torch.empty((H, Lq, Lk), dtype=torch.float32, device="cuda")
        ms = {}
        for form, key in ((B.QUEST_ALU, "alu_ms"), (B.QUEST_MFMA, "mfma_ms")):
            for _ in range(3):
                B.adacluster_quest_scores(Q, hi, lo, form, out=S)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 10
            e0.record()
            for _ in range(reps):
                B.adacluster_quest_scores(Q, hi, lo, form, out=S)
            e1.record()
            torch.cuda.synchronize()
            ms[key] = e0.elapsed_time(e1) / reps
        flops = 4.0 * H * Lq * Lk * d
        print(json.dumps({"shape": name, "H": H, "Lq": Lq, "Lk": Lk, "d": d, **ms,
                          "alu_over_mfma": ms["alu_ms"] / ms["mfma_ms"],
                          "mfma_tflops": flops / ms["mfma_ms"] / 1e9,
                          "score_bytes_mb": H * Lq * Lk * 4 / 1e6}), flush=True)
        del Q, C, spread, lo, hi, S


if __name__ == "__main__":
    sys.exit(main())
