"""Benchmark of the layout-elided hot path on one MI355X.

Workload (benchmark configs[1]): Swin stage-3 chain, bf16, B=32, 14x14
tokens, C=384, 12 heads, window 7, 6 blocks alternating shift 0/3, MLP ratio 4;
seeded synthetic inputs resident in HBM before the timed region.  One step =
one pass of the whole chain (13 kernels in elided mode: per block window attention and one kernel for
proj + residual + LayerNorm + MLP + residual + the next block's LayerNorm and QKV, plus the first block's LayerNorm +
QKV kernel; the explicit chain runs 30 + 30 copies) over one batch.

Prints ONE JSON line: whole-job throughput (images/s) of the elided chain, the
explicit-transpose baseline chain timed the same way, per-kernel durations
measured with HIP events on the launch stream, the roofline of the dominant
kernel, and the CPU oracle timed on the host cores.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM = 8.0e12          # B/s, MI355X published
PEAK_BF16 = 2.5e15         # FLOP/s dense bf16 MFMA, MI355X published

# HBM traffic per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (bytes, scaled by the
# calibration against an identity copy of known size, --calibrate-copy); filled from profiles/, None = not measured.
MEASURED_TRAFFIC = {
    # profiles/swin_stage3_chain_b32_hbm_counters.md: (FETCH_SIZE KiB x 2.000 + WRITE_SIZE KiB x 1.000) x 1024
    "proj+ln+mlp_bf16[6272,1536,384]+ln+qkv": int((18726.1 * 2.0 + 18816.1) * 1024),
    "proj+ln+mlp_bf16[6272,1536,384]": int((15194.2 * 2.0 + 4704.0) * 1024),
    "ln+mlp_bf16[6272,1536,384]": int((11666.8 * 2.0 + 4704.0) * 1024),
    "ln+pgemm_bf16[6272,1152,384]": int((5892.6 * 2.0 + 14115.9) * 1024),
    "gemm_bf16[6272,1152,384]": int((6443.5 * 2.0 + 14114.2) * 1024),
    "gemm_bf16[6272,384,384]+res": int((3784.5 * 2.0 + 4704.0) * 1024),
    "attention_window_bf16[128,12,49,49,32]": int((7137.5 * 2.0 + 4704.0) * 1024),
    "layernorm_bf16[6272,384]+scatter": int((2432.1 * 2.0 + 4704.0) * 1024),
    "layernorm_bf16[6272,384]": int((2432.1 * 2.0 + 4704.0) * 1024),
}


def kernel_model(label, e=2):
    """Algorithmic bytes and flops of one launch, from the kernel label (tensor reads + writes at
    kernel-per-op granularity with fused epilogues; weights and bias included)."""
    m = re.match(r"(proj\+)?(ln\+)?mlp_\w+\[(\d+),(\d+),(\d+)\](\+ln)?(\+qkv)?", label)
    if m:      # fused MLP: X and the residual read, Y written, both weights, biases (and the norm's vectors);
        #        with the projection in front: its [C, C] weight and bias as well (A, x0 read, Y written);
        #        "+ln": the next block's LayerNorm as a second output
        M, Hd, C = int(m.group(3)), int(m.group(4)), int(m.group(5))
        by = 3 * M * C + 2 * Hd * C + Hd + C + (2 * C if m.group(2) else 0) + (C * C + C if m.group(1) else 0)
        by += (M * C + 2 * C) if m.group(6) and not m.group(7) else 0
        fl = 4.0 * M * Hd * C + (2.0 * M * C * C if m.group(1) else 0.0)
        if m.group(7):      # ... and the next block's QKV Linear on that norm: its weight, bias and [M, 3C] output
            by += 2 * C + 3 * C * C + 3 * C + 3 * M * C
            fl += 6.0 * M * C * C
        return by * e, fl
    m = re.match(r"(?:ln\+|rms\+)?p?gemm_\w+\[(\d+),(\d+),(\d+)\](.*)", label)
    if m:
        M, N, K = int(m.group(1)), int(m.group(2)), int(m.group(3))
        n_out = N // 2 if "+glu" in m.group(4) else N
        by = (M * K + N * K + N + M * n_out + (M * n_out if "+res" in m.group(4) else 0)) * e
        return by, 2.0 * M * N * K
    m = re.match(r"(layernorm|rmsnorm)_\w+\[(\d+),(\d+)\]", label)
    if m:
        R, C = int(m.group(2)), int(m.group(3))
        return (2 * R * C + 2 * C) * e, 8.0 * R * C
    m = re.match(r"attention_(\w+)_\w+\[(\d+),(\d+),(\d+),(\d+),(\d+)\]", label)
    if m:
        nb, h, nq, nk, d = [int(m.group(i)) for i in range(2, 7)]
        fl = 4.0 * nb * h * nq * nk * d * (0.5 if m.group(1) == "causal" else 1.0)
        return nb * h * (2 * nq + 2 * nk) * d * e, fl
    m = re.match(r"copy_\w+\[(\d+)\](.*)", label)
    if m:
        n = int(m.group(1))
        return (3 if "+add" in m.group(2) else 2) * n * e, 0.0
    return 0, 0.0


def fold_microbench(sm, torch, steps, warmup):
    """A transposition between two MatMuls, T = X . W1^T then Y = T^T . W2^T, three ways (the paper's micro-experiment
    "version a optimises reads, version b optimises writes", Sec. 3.2.2, for the MatMul operator):
    write_fold: the producer stores T transposed (strided stores), the consumer reads K-contiguous rows;
    read_fold:  the producer stores T as it comes, the consumer reads it transposed in place (K-strided loads);
    explicit:   the producer stores T as it comes, a copy kernel transposes it, the consumer reads the copy."""
    dt = torch.bfloat16
    out = {"experiment": "read- versus write-side folding of a transposition between two Linears (bf16)", "cases": []}
    for (M, N, K, N2) in ((2048, 2048, 512, 512), (6272, 1536, 384, 384)):
        g = torch.Generator().manual_seed(7)
        X = torch.randn(M, K, generator=g).to(dt).cuda()
        W1 = (torch.randn(N, K, generator=g) * K ** -0.5).to(dt).cuda()
        W2 = (torch.randn(N2, M, generator=g) * M ** -0.5).to(dt).cuda()
        T = torch.empty(M * N, dtype=dt, device="cuda")
        T2 = torch.empty(N, M, dtype=dt, device="cuda")
        Y = torch.empty(N, N2, dtype=dt, device="cuda")
        tmap = sm.Map.create((M, N), [("permute", (1, 0))])          # view [N, M] of T [M, N]

        def write_fold():
            sm.linear(X, W1, c_transposed_batch=M, out=T)             # T stored as [N, M]
            sm.linear(T, W2, out=Y, M=N)

        def read_fold():
            sm.linear(X, W1, out=T)
            sm.linear(T, W2, a_map=tmap, out=Y, M=N)

        def explicit():
            sm.linear(X, W1, out=T)
            tmap.gather(T.view(M, N), out=T2)
            sm.linear(T2, W2, out=Y, M=N)

        res, ref = {}, None
        for name, fn in (("write_fold", write_fold), ("read_fold", read_fold), ("explicit", explicit)):
            for _ in range(warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            res[name + "_us"] = round((time.perf_counter() - t0) / steps * 1e6, 2)
            y = Y.float().clone()
            ref = y if ref is None else ref
            res[name + "_max_diff"] = float((y - ref).abs().max())
        res.update(shape={"M": M, "N": N, "K": K, "N2": N2},
                   read_over_write=round(res["read_fold_us"] / res["write_fold_us"], 3),
                   explicit_over_write=round(res["explicit_us"] / res["write_fold_us"], 3))
        out["cases"].append(res)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run an identity sm_gather_mapped copy of 256 MiB three times (counter calibration for rocprofv3 --pmc)")
    ap.add_argument("--fold-microbench", action="store_true",
                    help="instead of the chain: the read-versus-write folding micro-experiment of Sec. 3.2.2 on the mapped Linear")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus %d refused)" % a.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2404_13528_amd import binding as sm, workloads as Wl

    if a.fold_microbench:
        print(json.dumps(fold_microbench(sm, torch, a.steps, a.warmup)))
        return

    B, H, W, C, h, w, depth = 32, 14, 14, 384, 12, 7, 6
    dtype = torch.bfloat16
    x, blocks = Wl.swin_stage_case(B, H, W, C, h, w, depth)
    dev_blocks = [{k: v.to(dtype).cuda() for k, v in p.items()} for p in blocks]
    xd = x.to(dtype).cuda()
    chains = {name: sm.SwinChain(B, [(C, h, depth, H, W)], w, {"stages": [dev_blocks]}, dtype, mode)
              for name, mode in (("elided", sm.SM_ELIDED), ("explicit", sm.SM_EXPLICIT))}
    y = torch.empty_like(xd)
    stream = torch.cuda.current_stream()

    def timed(chain):
        for _ in range(a.warmup):
            chain(xd, out=y, stream=stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            chain(xd, out=y, stream=stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / a.steps

    def kernels(chain):
        sm.timing_enable(True)
        for _ in range(a.steps):
            chain(xd, out=y, stream=stream)
        sm.timing_calibrate(64, stream=stream)        # what an event pair adds to a kernel's own run time
        torch.cuda.synchronize()
        rep = sm.timing_report()
        sm.timing_enable(False)
        n, ms = rep.pop("empty_kernel")
        n2, ms2 = rep.pop("empty_pair")
        return rep, {"empty_kernel_us": round(ms / n * 1e3, 3), "empty_pair_us": round(ms2 / n2 * 1e3, 3)}

    if a.calibrate_copy:
        n = 128 * 1024 * 1024                         # bf16 elements: 256 MiB read + 256 MiB written per launch
        src = torch.zeros(n, dtype=dtype, device="cuda")
        ident = sm.Map.create((n // 1024, 1024), [])
        for _ in range(3):
            ident.gather(src.view(n // 1024, 1024), stream=stream)
        torch.cuda.synchronize()
        del src

    sec = {name: timed(c) for name, c in chains.items()}
    rep, overhead_us = {}, {}
    for name, c in chains.items():
        rep[name], overhead_us[name] = kernels(c)

    def table(r):
        # avg_us: HIP-event time around each launch on the launch stream.  It contains the dispatch and the event
        # records themselves: a profiler's kernel duration is 2.5 to 3 us shorter (see event_calibration below for
        # what an event pair measures around an empty kernel and around nothing)
        rows = []
        for label, (n, ms) in r.items():
            by, fl = kernel_model(label)
            us = ms / n * 1e3
            rows.append({"kernel": label, "launches_per_step": n // a.steps, "avg_us": round(us, 3),
                         "alg_bytes": by, "flops": fl,
                         "GBps": round(by / us * 1e-3, 1), "TFLOPs": round(fl / us * 1e-6, 1)})
        return rows

    tab = table(rep["elided"])
    dom = max(tab, key=lambda r: r["avg_us"] * r["launches_per_step"])
    t_hbm, t_mfma = dom["alg_bytes"] / PEAK_HBM, dom["flops"] / PEAK_BF16
    if t_mfma >= t_hbm:
        roof = {"bound": "mfma", "achieved": dom["TFLOPs"], "peak": PEAK_BF16 * 1e-12, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": dom["GBps"], "peak": PEAK_HBM * 1e-9, "unit": "GB/s"}
    roof["frac"] = round(roof["achieved"] / roof["peak"], 4)
    roof["traffic"] = MEASURED_TRAFFIC.get(dom["kernel"])
    roof["kernel"] = dom["kernel"]
    roof["avg_us"] = dom["avg_us"]

    alg_bytes = {name: sum(kernel_model(l)[0] * (n // a.steps) for l, (n, _) in r.items()) for name, r in rep.items()}
    kern_us = {name: sum(ms for _, ms in r.values()) / a.steps * 1e3 for name, r in rep.items()}

    out = {
        "metric": "Swin/attention block images(tokens)/s + HBM bytes vs explicit-transpose chain",
        "value": round(B / sec["elided"], 1), "unit": "images/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(sec["elided"] * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: Swin stage-3 chain, B=32, 14x14 tokens, C=384, 12 heads, window 7, "
                               "6 blocks shift 0/3, MLP 4x", "mode": "elided", "global_batch": B},
        "explicit_chain": {"images_per_s": round(B / sec["explicit"], 1), "ms_per_step": round(sec["explicit"] * 1e3, 4),
                           "alg_bytes_per_step": alg_bytes["explicit"], "kernel_us_per_step": round(kern_us["explicit"], 2)},
        "elided_chain": {"alg_bytes_per_step": alg_bytes["elided"], "kernel_us_per_step": round(kern_us["elided"], 2),
                         "speedup_vs_explicit": round(sec["explicit"] / sec["elided"], 3),
                         "bytes_ratio_explicit_over_elided": round(alg_bytes["explicit"] / alg_bytes["elided"], 3)},
        "roofline": roof,
        "event_calibration": overhead_us["elided"],
        "kernels": tab,
    }

    if not a.no_cpu_baseline:
        from oracle import swin
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            cores = os.cpu_count()
        xn = x.double().numpy()
        pn = [{k: v.double().numpy() for k, v in p.items()} for p in blocks]
        reps, t0 = 0, time.perf_counter()
        while reps < 2 or time.perf_counter() - t0 < 10.0:          # about 10 s of host work
            swin.swin_stage(xn, pn, H, W, w, h)
            reps += 1
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(B * reps / dt, 2), "unit": "images/s", "cores": cores, "kind": "oracle",
                               "sample": "the full workload %d times (32 images through 6 blocks each), float64 numpy, %.2f s" % (reps, dt)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
