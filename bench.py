#!/usr/bin/env python3
"""Throughput of the RDK redistribute + verify path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic inputs that already sit in HBM:
redistribution with the top-k sparse kernel (Alg. 1 steps 1-2) and verification (Alg. 4), through the fused
entry point rdk_redistribute_verify (default) or as rdk_redistribute_linear -> rdk_verify_sample.
Prints ONE JSON line: positions/s, the roofline of the dominant kernel (timed live with HIP events
inside the library), and the CPU oracle timed on a bounded sample of the same workload.

  python bench.py [--steps K] [--warmup W] [--mode sparse|taylor] [--path fused|twocall] [--workload NAME] [--no-cpu]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16, published


def algorithmic_bytes(kernel, w, B, kk, fused, esz):
    """Bytes one launch of a kernel must move for B positions (inputs read once, outputs written once).
    esz = bytes per input element (4: fp32, 2: bf16 logits).  In the fused path the product / Eq. 3 kernels
    read p instead of writing q'."""
    N, n = w.N, w.n
    tables = 8 * (N - n) * kk + 4 * n + 4 * N                               # neighbour rows, diagonal, id maps: once
    return {
        "verify_stream_kernel": B * (esz + 4) * N,                          # read p and q'
        "sparse_product_kernel": B * ((esz if fused else 4) * N + 4 * n) + tables,   # read q^T, p (fused) or write q'
        "taylor_stats_kernel": B * esz * (N + n) + 4 * N,                   # read p, q, slot table
        "taylor_write_kernel": B * (esz * (N + n) + (0 if fused else 4 * N)) + 4 * N,
        "q_transpose_kernel": B * (esz + 4) * n,
        "row_stats_kernel": B * esz * n,
        "verify_finalize_kernel": B * 3 * 4 * ((N + 1023) // 1024),
    }.get(kernel)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--mode", default="sparse", choices=["sparse", "taylor"])
    ap.add_argument("--path", default="fused", choices=["fused", "twocall"],
                    help="fused: rdk_redistribute_verify (q' never stored); twocall: rdk_redistribute_linear + rdk_verify_sample")
    ap.add_argument("--workload", default=None)
    ap.add_argument("--copies", type=int, default=4, help="input/output buffer sets rotated through (defeats the 256 MB cache)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle baseline")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build is a one-GPU library (positions are independent: shard the batch); run with --gpus 1")

    import torch
    from paper_2506_03206_amd import rdk, synth

    wname = args.workload or "llama3"
    w = synth.WORKLOADS[wname]
    B = w.B
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    t0 = time.time()
    bias, kept, E, rng = synth.make_vocab(w)
    batch = synth.make_batch(w, bias, kept, rng)
    gen_s = time.time() - t0

    kept_d = torch.from_numpy(kept).to(dev)
    t0 = time.time()
    if args.mode == "sparse":
        kern = rdk.rdk_build_kernel(w.N, kept_d, rdk.SPARSE_TOPK, embeddings=torch.from_numpy(E).to(dev), tau=w.tau, k=w.k)
    else:
        kern = rdk.rdk_build_kernel(w.N, kept_d, rdk.IDENTITY)
    torch.cuda.synchronize()
    build_s = time.time() - t0

    if w.logits_bf16:
        p_host = torch.from_numpy(batch["z_p"]).to(torch.bfloat16)
        q_host = torch.from_numpy(batch["z_q"]).to(torch.bfloat16)
        kind = "logit"
    else:
        p_host, q_host, kind = torch.from_numpy(batch["p"]), torch.from_numpy(batch["q_hat"]), "prob"
    C = max(1, args.copies)
    ps = [p_host.to(dev) for _ in range(C)]
    qs = [q_host.to(dev) for _ in range(C)]
    outs = [torch.empty((B, w.N), dtype=torch.float32, device=dev) for _ in range(C)] if args.path == "twocall" else None
    vout = rdk.VerifyOutputs(B, w.N, w.gamma, dev)
    kern.workspace(B)
    mode = rdk.LINEAR_SPARSE if args.mode == "sparse" else rdk.LINEAR_TAYLOR

    fused = args.path == "fused"

    def step(i):
        c = i % C
        if fused:
            rdk.rdk_redistribute_verify(kern, mode, ps[c], qs[c], seed=2506, offset=i * B, gamma=w.gamma, p_kind=kind,
                                        q_kind=kind, outputs=vout)
        else:
            rdk.rdk_redistribute_linear(kern, mode, qs[c], kind, p=ps[c] if args.mode == "taylor" else None, p_kind=kind,
                                        out=outs[c])
            rdk.rdk_verify_sample(ps[c], outs[c], seed=2506, offset=i * B, gamma=w.gamma, p_kind=kind, outputs=vout)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    # which kernel dominates?  a short pass with every kernel bracketed by events
    names = ["row_stats_kernel", "q_transpose_kernel", "sparse_product_kernel", "taylor_stats_kernel", "taylor_write_kernel",
             "verify_stream_kernel", "verify_finalize_kernel"]
    rdk.rdk_timing_select("*")
    for i in range(20):
        step(i)
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    per_kernel = {}
    for nm in names:
        cnt, ms = rdk.rdk_timing_read(nm)
        if cnt:
            per_kernel[nm] = {"launches_per_step": cnt / 20.0, "avg_us": 1e3 * ms / cnt}
    dominant = max(per_kernel, key=lambda k: per_kernel[k]["avg_us"] * per_kernel[k]["launches_per_step"])

    # the timed region: K steps, the dominant kernel's launches bracketed by events on the launch stream
    rdk.rdk_timing_select(dominant)
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for i in range(args.steps):
        step(args.warmup + i)
    stop.record()
    torch.cuda.synchronize()
    rdk.rdk_timing_select(None)
    total_ms = start.elapsed_time(stop)
    cnt, kms = rdk.rdk_timing_read(dominant)
    ms_per_step = total_ms / args.steps
    value = B / (ms_per_step * 1e-3)

    kk = (max(w.k, 1) + 15) // 16 * 16
    esz = 2 if w.logits_bf16 else 4
    alg = algorithmic_bytes(dominant, w, B, kk, fused, esz)
    avg_s = kms / cnt * 1e-3
    achieved = alg / avg_s / 1e9
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None, "avg_launch_us": round(avg_s * 1e6, 2),
                "algorithmic_bytes_per_launch": alg}
    # whole-step compulsory bytes: fused = read p and q once; two calls = q read, q' written then read, p read (twice for Eq. 3)
    if fused:
        step_bytes = B * esz * (w.N + w.n) + (8 * (w.N - w.n) * kk if args.mode == "sparse" else 0)
    else:
        step_bytes = B * (esz * (w.n + w.N) + 8 * w.N) + (8 * (w.N - w.n) * kk if args.mode == "sparse" else B * esz * w.N)
    extra = {"kernels": {k: {"avg_us": round(v["avg_us"], 2), "per_step": v["launches_per_step"]} for k, v in per_kernel.items()},
             "step_algorithmic_GBs": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
             "step_frac_of_hbm_peak": round(step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
             "kernel_build_s": round(build_s, 3), "input_gen_s": round(gen_s, 2),
             "accept_rate": float(vout.accept.float().mean().item()), "mean_alpha": float(vout.alpha.mean().item())}

    cpu = None
    if not args.no_cpu:
        cpu = cpu_baseline(args, w, batch, kept)

    line = {"metric": "redistribute+verify positions/sec at N=%d, n=%d" % (w.N, w.n), "value": round(value, 1),
            "unit": "positions/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": "%s: N=%d n=%d B=%d (%d seqs x %d drafts) k=%d, %s linear RDK + verify/sample, %s inputs"
                       % (w.name, w.N, w.n, B, w.seqs, w.gamma, w.k, args.mode, "bf16 logit" if w.logits_bf16 else "fp32 prob"),
                       "mode": args.mode, "path": args.path, "N": w.N, "n": w.n, "B": B, "k": w.k},
            "roofline": roofline, "cpu_baseline": cpu, "extra": extra}
    print(json.dumps(line))


def cpu_baseline(args, w, batch, kept):
    """The oracle, as it stands, on the host: same pipeline, same batch, repeated until ~cpu_seconds have passed."""
    import oracle
    from paper_2506_03206_amd import synth
    B = w.B
    p = batch["p"] if not w.logits_bf16 else None
    sp = synth.random_sparse_kernel(np.random.default_rng(1), w.N, kept, w.k) if args.mode == "sparse" else None
    done, t0 = 0, time.time()
    rows = 0
    while True:
        for b0 in range(0, B, 32):
            sl = slice(b0, min(B, b0 + 32))
            if w.logits_bf16:
                pr = oracle.probs_from(batch["z_p"][sl], "logit")
                qr = oracle.probs_from(batch["z_q"][sl], "logit")
            else:
                pr, qr = p[sl], batch["q_hat"][sl]
            if args.mode == "sparse":
                qp = oracle.redistribute_batch("sparse", qr, kept, w.N, sparse=sp)
            else:
                qp = oracle.redistribute_batch("taylor", qr, kept, w.N, p=pr)
            oracle.verify_batch(pr, qp, 2506, done * B + b0, gamma=w.gamma)
            rows += sl.stop - sl.start
            if time.time() - t0 > args.cpu_seconds:
                break
        done += 1
        if time.time() - t0 > args.cpu_seconds:
            break
    el = time.time() - t0
    return {"value": round(rows / el, 1), "unit": "positions/s", "cores": 1, "kind": "oracle",
            "sample": "%d positions of the same batch (TLI -> %s redistribution -> accept/residual/sample), %.1f s, "
                      "single thread, fp64; the sparse kernel is a random top-k kernel of the same shape" % (rows, args.mode, el)}


if __name__ == "__main__":
    main()
